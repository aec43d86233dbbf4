#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

Workload: batch 64, 12 query / 2 KV heads, head_dim 128, bf16,
prompt 256, 4096 generated tokens, c = 16.  One *step* is one pass of the hot path over one
batch for one attention layer: append the token's K/V, decode attention over
[prompt | beacons | window], beacon append + eviction on the sequences that are due.
The model is represented by `--layers` independent cache instances visited round-robin
(as the layers of a model are), so consecutive steps touch different memory and the caches
(together larger than the 256 MB Infinity Cache) are read from HBM, not from cache.
The timed region is the last `--steps` layer-steps of the rollout, the warm-up the ones
before it; by default the two cover the whole 4096-token rollout.

Prints ONE JSON line: value = algorithmic KV bytes read by decode
attention per second over the whole timed region (all kernels and launch gaps included).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def stored_traffic():
    """HBM bytes per launch of the decode kernel as measured by the committed rocprofv3 PMC runs
    (FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size); None if absent.
    bench.py cannot run the profiler around itself, so it reports the stored measurement."""
    path = os.path.join(ROOT, "profiles", "decode_batch64_c16_hbm_traffic.txt")
    try:
        vals = {}
        with open(path) as f:
            for line in f:
                line = line.split("#")[0]
                if "=" in line:
                    k, v = line.split("=")
                    vals[k.strip()] = float(v)
        return {"bytes_per_launch": int(vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"]),
                "algorithmic_bytes_per_launch": int(vals["algorithmic_kv_bytes_per_launch"]),
                "ratio": vals["traffic_over_algorithmic"],
                "source": "profiles/decode_batch64_c16_hbm_traffic.txt (tokens 3825..4096 of the rollout)"}
    except (OSError, KeyError, ValueError):
        return None


def stored_value(key):
    """One `key = value` figure from profiles/prefill_config5_hbm_traffic.txt (measured HBM-side bytes of
    the prefill and distillation kernels, same method as stored_traffic); None if absent."""
    try:
        with open(os.path.join(ROOT, "profiles", "prefill_config5_hbm_traffic.txt")) as f:
            for line in f:
                line = line.split("#")[0]
                if "=" in line and line.split("=")[0].strip() == key:
                    return int(float(line.split("=")[1]))
    except (OSError, ValueError):
        pass
    return None


def kv_bytes_per_step(wl, t):
    """Algorithmic K+V bytes decode attention reads at token-step t: every resident row once."""
    es = 2 if wl.dtype == "bf16" else 4
    c = int(wl.c[0])
    L = (wl.P + ((t - 1) // c + (t - 1) % c + 1 if c > 0 else t)).astype(np.int64)
    return int(L.sum()) * wl.Hkv * wl.d * 2 * es


def cpu_baseline(wl, budget_s=12.0):
    """Oracle decode attention timed on the host cores, on a bounded sample of the workload:
    repeated decode steps over the end-of-rollout cache state (all sequences, all heads)."""
    import psutil
    from oracle import attention as OA
    rng = np.random.default_rng(1)
    c = int(wl.c[0])
    G = int(wl.G[0])
    L = int(wl.P[0]) + (G // c + G % c if c > 0 else G)
    K = [rng.standard_normal((L, wl.Hkv, wl.d)).astype(np.float32) for _ in range(wl.B)]
    V = [rng.standard_normal((L, wl.Hkv, wl.d)).astype(np.float32) for _ in range(wl.B)]
    proc = psutil.Process()
    cpu0 = proc.cpu_times()
    t0 = time.perf_counter()
    steps = 0
    while time.perf_counter() - t0 < budget_s:
        q = rng.standard_normal((wl.B, wl.Hq, wl.d)).astype(np.float32)
        for s in range(wl.B):
            OA.decode_attention(q[s], K[s], V[s], wl.scale)
        steps += 1
    wall = time.perf_counter() - t0
    cpu1 = proc.cpu_times()
    cpu = (cpu1.user - cpu0.user) + (cpu1.system - cpu0.system)
    nbytes = steps * wl.B * L * wl.Hkv * wl.d * 2 * 2
    return {"value": nbytes / wall / 1e9, "unit": "GB/s", "cores": max(1, int(round(cpu / wall))),
            "kind": "oracle", "steps_per_sec": steps / wall,
            "sample": "%d decode steps at the end-of-rollout state (L=%d), all %d sequences x %d heads, "
                      "fp64 NumPy oracle, %.1f s" % (steps, L, wl.B, wl.Hq, wall)}


def uncompressed_control(dev, NL=4, reps=10):
    """The same shapes without compression (c = infinity) at the end of the rollout: every sequence
    holds P + G = 4352 entries.  Decode attention alone (the tables do not change), NL cache
    instances round-robin (2.3 GB > Infinity Cache), graph replay, HIP events."""
    import torch
    from paper_2510_13797_amd import bc, workloads
    wl = workloads.batch64(c=0)
    G = int(wl.G[0])
    layers = []
    for _ in range(NL):
        rt = bc.Runtime(wl.B, wl.Hq, wl.Hkv, wl.d, wl.dtype, wl.scale, wl.P, wl.c, wl.capacity(), dev)
        rt.k_slab.normal_()
        rt.v_slab.normal_()
        rt.set_tables(np.zeros(wl.B, np.int32), np.full(wl.B, G, np.int32))
        layers.append(rt)
    q = torch.randn(wl.B, wl.Hq, wl.d, device=dev).to(torch.bfloat16)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for rt in layers:
            rt.decode_attn(q)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for rt in layers:
                rt.decode_attn(q)
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            graph.replay()
        e1.record(stream)
        stream.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * NL)
    L = int(wl.P[0]) + G
    nbytes = wl.B * L * wl.Hkv * wl.d * 2 * 2
    assert torch.isfinite(layers[0].out).all()
    return {"workload": "same shapes, c=inf, end of rollout: L=%d entries per sequence" % L,
            "kv_bytes_per_step": nbytes, "us_per_step": round(us, 2),
            "GBps": round(nbytes / us / 1e3, 1), "pct_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS * 100, 1)}


def visible_pairs(S, P, c):
    """Number of (query row, visible key) pairs of one trajectory: sum over rows of |vis(r)|."""
    r = np.arange(S, dtype=np.int64)
    if c <= 0:
        return int((r + 1).sum())
    u = np.maximum(r - P, 0)
    resp = P + u // (c + 1) + u % (c + 1) + 1
    return int(np.where(r < P, r + 1, resp).sum())


def bench_prefill(args):
    """Config 5: beacon-masked prefill attention forward, B=16, 12/2 heads, d=128, bf16,
    8192 tokens (256 prompt) + one beacon per 16 response tokens = 8688 rows per trajectory."""
    import torch
    from paper_2510_13797_amd import bc, workloads
    bc.load()
    dev = torch.device("cuda:0")
    pw = workloads.prefill_train()
    S = int(pw.S[0])
    R = int(pw.S.sum())
    off = np.zeros(pw.B + 1, np.int64)
    off[1:] = np.cumsum(pw.S)
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    q = torch.randn(R, pw.Hq, pw.d, generator=gen, device=dev).to(torch.bfloat16)
    k = torch.randn(R, pw.Hkv, pw.d, generator=gen, device=dev).to(torch.bfloat16)
    v = torch.randn(R, pw.Hkv, pw.d, generator=gen, device=dev).to(torch.bfloat16)
    shape = bc.bc_shape(pw.B, pw.Hq, pw.Hkv, pw.d, bc.BC_BF16, pw.scale)
    offd = torch.from_numpy(off).to(dev)
    Pd = torch.from_numpy(pw.P).to(dev)
    cd = torch.from_numpy(pw.c).to(dev)
    out = torch.empty(R, pw.Hq, pw.d, dtype=torch.float32, device=dev)
    lse = torch.empty(R, pw.Hq, dtype=torch.float32, device=dev)
    import ctypes as C
    ptr = lambda t: C.c_void_p(t.data_ptr())
    stream = torch.cuda.current_stream()

    def step():
        st = bc.bc_prefill_attn(shape, ptr(q), ptr(k), ptr(v), ptr(offd), ptr(Pd), ptr(cd), S, ptr(out),
                                ptr(lse), C.c_void_p(stream.cuda_stream))
        assert st == 0, st

    W_ = args.warmup if args.warmup >= 0 else 3
    K_ = args.steps if args.steps >= 0 else 20
    for _ in range(W_):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    e0.record(stream)
    for _ in range(K_):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms = max(e0.elapsed_time(e1), wall * 1e3) / K_
    assert torch.isfinite(out).all()
    pairs = sum(visible_pairs(int(pw.S[b]), int(pw.P[b]), int(pw.c[b])) for b in range(pw.B))
    flops = 4.0 * pw.d * pairs * pw.Hq               # q.k and p.v, 2 flop per multiply-add
    tflops = flops / (ms * 1e-3) / 1e12
    hbm_bytes = R * (pw.Hq * pw.d * 2 + 2 * pw.Hkv * pw.d * 2 + pw.Hq * pw.d * 4 + pw.Hq * 4)
    rec = {"metric": "prefill_attn_TFLOPs", "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": K_, "warmup": W_, "ms_per_step": round(ms, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "beacon-masked prefill forward: B=16, Hq=12, Hkv=2, d=128, bf16, "
                                  "8192 tokens (P=256) + 496 beacons = 8688 rows, c=16",
                      "algorithmic_GFLOP": round(flops / 1e9, 1),
                      # q, k, v read once (bf16), out (fp32) and lse written once
                      "algorithmic_MB": round(hbm_bytes / 1e6, 1),
                      "algorithmic_GBps": round(hbm_bytes / (ms * 1e-3) / 1e9, 1)},
           "roofline": {"bound": "mfma", "kernel": "bc::prefill_kernel<3>", "achieved": round(tflops, 2),
                        "peak": 2500.0, "unit": "TFLOP/s", "frac": round(tflops / 2500.0, 4),
                        "traffic": stored_value("prefill_fwd_traffic_bytes")}}
    print(json.dumps(rec))


def bench_prefill_bwd(args):
    """Config 5, backward of the beacon-masked attention (dq, dk, dv), after one forward."""
    import ctypes as C
    import torch
    from paper_2510_13797_amd import bc, workloads
    bc.load()
    dev = torch.device("cuda:0")
    pw = workloads.prefill_train()
    S = int(pw.S[0])
    R = int(pw.S.sum())
    off = np.zeros(pw.B + 1, np.int64)
    off[1:] = np.cumsum(pw.S)
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    mk = lambda h: torch.randn(R, h, pw.d, generator=gen, device=dev).to(torch.bfloat16)
    q, k, v, do = mk(pw.Hq), mk(pw.Hkv), mk(pw.Hkv), mk(pw.Hq)
    out, lse = bc.prefill_attn(q, k, v, off, pw.P, pw.c, pw.Hq, pw.Hkv, pw.d, pw.scale, True)
    shape = bc.bc_shape(pw.B, pw.Hq, pw.Hkv, pw.d, bc.BC_BF16, pw.scale)
    offd = torch.from_numpy(off).to(dev)
    Pd, cd = torch.from_numpy(pw.P).to(dev), torch.from_numpy(pw.c).to(dev)
    dq = torch.empty(R, pw.Hq, pw.d, dtype=torch.float32, device=dev)
    dk = torch.empty(R, pw.Hkv, pw.d, dtype=torch.float32, device=dev)
    dv = torch.empty_like(dk)
    ws_bytes = int(bc.bc_prefill_bwd_workspace_bytes(shape, R))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    stream = torch.cuda.current_stream()

    def step():
        st = bc.bc_prefill_attn_bwd(shape, ptr(q), ptr(k), ptr(v), ptr(out), ptr(lse), ptr(do), ptr(offd),
                                    ptr(Pd), ptr(cd), S, R, ptr(dq), ptr(dk), ptr(dv), ptr(ws), ws_bytes,
                                    C.c_void_p(stream.cuda_stream))
        assert st == 0, st

    W_ = args.warmup if args.warmup >= 0 else 2
    K_ = args.steps if args.steps >= 0 else 10
    for _ in range(W_):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    e0.record(stream)
    for _ in range(K_):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms = max(e0.elapsed_time(e1), wall * 1e3) / K_
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()
    pairs = sum(visible_pairs(int(pw.S[b]), int(pw.P[b]), int(pw.c[b])) for b in range(pw.B))
    flops = 10.0 * pw.d * pairs * pw.Hq              # recompute q.k, dO.v; dv, dq, dk: 5 products
    tflops = flops / (ms * 1e-3) / 1e12
    print(json.dumps({"metric": "prefill_attn_bwd_TFLOPs", "value": round(tflops, 2), "unit": "TFLOP/s",
                      "n_gpus": 1, "steps": K_, "warmup": W_, "ms_per_step": round(ms, 4),
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
                      "data": "synthetic",
                      "config": {"workload": "backward of the beacon-masked prefill attention, config 5 shape",
                                 "algorithmic_GFLOP": round(flops / 1e9, 1)},
                      "roofline": {"bound": "mfma", "kernel": "bc::prefill_bwd_dq_kernel + bc::prefill_bwd_dkv_kernel",
                                   "achieved": round(tflops, 2), "peak": 2500.0, "unit": "TFLOP/s",
                                   "frac": round(tflops / 2500.0, 4),
                                   "traffic": stored_value("prefill_bwd_traffic_bytes")}}))


def bench_distill(args):
    """Distillation loss at the paper's shape: T=4096 tokens x 151,936 logits (bf16), top-100
    teacher.  Forward and backward are timed separately; both are single streaming passes."""
    import ctypes as C
    import torch
    from paper_2510_13797_amd import bc
    bc.load()
    dev = torch.device("cuda:0")
    T, V, k = 4096, 151936, 100
    gen = torch.Generator(device=dev).manual_seed(1234)
    z = (2.0 * torch.randn((T, V), generator=gen, device=dev)).to(torch.bfloat16)
    tl = torch.empty((T, k), dtype=torch.float32, device=dev)
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    for t0 in range(0, T, 512):
        top = torch.topk(z[t0:t0 + 512].float() + torch.randn((512, V), generator=gen, device=dev), k, dim=1)
        tl[t0:t0 + 512] = top.values
        idx[t0:t0 + 512] = top.indices.to(torch.int32)
    loss = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev)
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    dz = torch.empty_like(z)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)

    def fwd():
        st = bc.bc_topk_kl_loss(T, V, k, ptr(z), bc.BC_BF16, ptr(tl), ptr(idx), ptr(loss), ptr(lse), ptr(mean), sp)
        assert st == 0, st

    def bwd():
        st = bc.bc_topk_kl_loss_bwd(T, V, k, ptr(z), bc.BC_BF16, ptr(tl), ptr(idx), ptr(lse), 1.0 / T, ptr(dz), sp)
        assert st == 0, st

    W_ = args.warmup if args.warmup >= 0 else 3
    K_ = args.steps if args.steps >= 0 else 20

    def timed(fn):
        for _ in range(W_):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(K_):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / K_

    ms_f, ms_b = timed(fwd), timed(bwd)
    assert torch.isfinite(mean).all() and torch.isfinite(dz[:8].float()).all()
    bytes_f = T * V * 2 + T * k * 10              # logits once; teacher logits + ids; gathered logits
    bytes_b = 2 * T * V * 2 + T * k * 8
    gbs_f, gbs_b = bytes_f / (ms_f * 1e-3) / 1e9, bytes_b / (ms_b * 1e-3) / 1e9
    ms = ms_f + ms_b
    print(json.dumps({"metric": "distill_loss_tokens_per_s", "value": round(T / (ms * 1e-3), 1), "unit": "tokens/s",
                      "n_gpus": 1, "steps": K_, "warmup": W_, "ms_per_step": round(ms, 4),
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
                      "data": "synthetic",
                      "config": {"workload": "top-100 KL distillation loss, forward + backward: T=4096 tokens, "
                                             "V=151936 logits (bf16)",
                                 "ms_forward": round(ms_f, 4), "ms_backward": round(ms_b, 4),
                                 "forward_GBps": round(gbs_f, 1), "backward_GBps": round(gbs_b, 1)},
                      "roofline": {"bound": "hbm", "kernel": "bc::topk_kl_bwd_kernel<bf16_t, true>",
                                   "achieved": round(gbs_b, 1), "peak": 8000.0, "unit": "GB/s",
                                   "frac": round(gbs_b / 8000.0, 4),
                                   "traffic": stored_value("distill_bwd_traffic_bytes")}}))


def bench_copy(args):
    """Plain device copy of known size: calibrates the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    dev = torch.device("cuda:0")
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    reps = 8
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"workload": "copy", "bytes_read_per_copy": n, "bytes_written_per_copy": n,
                      "copies": reps}))


def bench_readfloor(args):
    """What a read-only kernel of the decode step's size costs: bc_diag_stream_read over 33.5 MB
    (the K/V bytes of one step at L = 512) from 16 rotating buffers, with the decode grid's 128
    workgroups and with larger grids, as back-to-back launches replayed from a HIP graph."""
    import torch
    from paper_2510_13797_amd import bc
    bc.load()
    dev = torch.device("cuda:0")
    nbytes = 64 * 512 * 2 * 128 * 2 * 2                 # B x L x Hkv x d x 2 bytes x (K and V)
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(16)]
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    st = torch.cuda.Stream()
    n_launch, reps = 256, 8

    def timed(nb, wgs):
        with torch.cuda.stream(st):
            sp = st.cuda_stream

            def run():
                for i in range(n_launch):
                    rc = bc.bc_diag_stream_read(bufs[i % 16].data_ptr() if nb else None, nb, wgs,
                                                sink.data_ptr(), sp)
                    assert rc == 0, rc
            run()
            st.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                run()
            g.replay()
            st.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(reps):
                g.replay()
            e1.record(st)
            st.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * n_launch)

    empty_us = timed(0, 128)
    res = []
    for wgs in (128, 256, 512, 1024, 2048):
        us = timed(nbytes, wgs)
        res.append({"workgroups": wgs, "us_per_launch": round(us, 3), "GBps": round(nbytes / us / 1e3, 1)})
    print(json.dumps({"workload": "readfloor", "bytes_per_launch": nbytes, "launches_per_graph": n_launch,
                      "empty_kernel_us": round(empty_us, 3), "results": res}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="decode", choices=["decode", "prefill", "prefill_bwd", "distill", "copy", "readfloor"])
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=-1)
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--layers", type=int, default=16, help="cache instances visited round-robin")
    ap.add_argument("--c", type=int, default=16, help="compression ratio (0: uncompressed control)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--beacon-attn", action="store_true",
                    help="also run the beacon token's own attention (bc_beacon_step) at every window end "
                         "instead of handing the beacon K/V to the token step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-control", action="store_true", help="skip the uncompressed (c=inf) control measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU sharding is a design "
              "note in the design document, not an implemented path", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_13797_amd import bc, workloads
    bc.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "prefill":
        return bench_prefill(args)
    if args.workload == "prefill_bwd":
        return bench_prefill_bwd(args)
    if args.workload == "distill":
        return bench_distill(args)
    if args.workload == "copy":
        return bench_copy(args)
    if args.workload == "readfloor":
        return bench_readfloor(args)

    wl = workloads.batch64(c=args.c)
    NL = args.layers
    G = int(wl.G[0])
    c = int(wl.c[0])
    cyc_tokens = c if c > 0 else 16
    cycle = cyc_tokens * NL                     # layer-steps per captured graph
    total = G * NL
    W = args.warmup if args.warmup >= 0 else cycle
    K = args.steps if args.steps >= 0 else total - W
    use_graph = not args.no_graph and K % cycle == 0 and W % cycle == 0
    if K < 1 or K + W > total:
        print("bench.py: steps must be at least 1 and steps + warmup at most %d (one rollout of %d "
              "tokens through %d layers)" % (total, G, NL), file=sys.stderr)
        sys.exit(2)
    # the run ends at the end of the rollout; a count that is not a multiple of --layers simply
    # stops part-way through the last token's layers (every layer-step is a step of its own cache)
    t0 = G - (K + W + NL - 1) // NL             # tokens already generated when the warm-up starts

    # --- state: NL cache instances fast-forwarded to token t0, inputs resident in HBM ---------
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    tdt = torch.bfloat16
    layers = []
    for _ in range(NL):
        rt = bc.Runtime(wl.B, wl.Hq, wl.Hkv, wl.d, wl.dtype, wl.scale, wl.P, wl.c, wl.capacity(), dev)
        rt.k_slab.copy_(torch.randn(rt.k_slab.shape, generator=gen, device=dev, dtype=torch.float32))
        rt.v_slab.copy_(torch.randn(rt.v_slab.shape, generator=gen, device=dev, dtype=torch.float32))
        if c > 0:
            rt.set_tables(np.full(wl.B, t0 // c, np.int32), np.full(wl.B, t0 % c, np.int32))
        else:
            rt.set_tables(np.zeros(wl.B, np.int32), np.full(wl.B, t0, np.int32))
        layers.append(rt)
    n_pool = 64

    def rnd(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(tdt)

    pool = [dict(k=rnd(wl.B, wl.Hkv, wl.d), v=rnd(wl.B, wl.Hkv, wl.d), q=rnd(wl.B, wl.Hq, wl.d),
                 bk=rnd(wl.B, wl.Hkv, wl.d), bv=rnd(wl.B, wl.Hkv, wl.d)) for _ in range(n_pool)]

    faithful = args.beacon_attn and c > 0
    if faithful and (K % NL or W % NL):
        print("bench.py: with --beacon-attn steps and warmup must be multiples of --layers", file=sys.stderr)
        sys.exit(2)

    def layer_step(i):
        """i-th layer-step of the rollout (counted from the warm-up start)."""
        rt = layers[i % NL]
        x = pool[i % n_pool]
        if not faithful:
            rt.decode_step(x["k"], x["v"], x["q"], x["bk"] if c > 0 else None, x["bv"] if c > 0 else None)
            return
        # the window's last token is followed by the beacon token's own pass through all layers
        rt.decode_step(x["k"], x["v"], x["q"], None, None)
        if (t0 + i // NL + 1) % c == 0 and i % NL == NL - 1:
            for li in range(NL):
                y = pool[(i + 1 + li) % n_pool]
                layers[li].beacon_step(y["bk"], y["bv"], y["q"])

    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        if use_graph:
            # the first cycle of the warm-up runs eagerly, the rest of it and all timed steps as
            # replays of one captured cycle (window position and pool index repeat every cycle)
            done = 0
            if W > 0:
                for i in range(cycle):
                    layer_step(i)
                done = cycle
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            saved = [(rt.nb.clone(), rt.w.clone()) for rt in layers]
            with torch.cuda.graph(graph, stream=stream):
                for i in range(cycle):
                    layer_step(i)
            for rt, (nb, w) in zip(layers, saved):      # capture does not run; restore anyway
                rt.nb.copy_(nb); rt.w.copy_(w)
            for _ in range((W - done) // cycle):
                graph.replay()
        else:
            for i in range(W):
                layer_step(i)
            if not args.no_graph and K <= 16384:
                # counts that are not whole 16-token cycles: the K timed steps as one graph
                stream.synchronize()
                saved = [(rt.nb.clone(), rt.w.clone()) for rt in layers]
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for i in range(W, W + K):
                        layer_step(i)
                # one untimed replay (the first replay of a graph pays for its upload), then the
                # tables go back: the timed replay rewrites the same rows with the same values
                graph.replay()
                stream.synchronize()
                for rt, (nb, w) in zip(layers, saved):
                    rt.nb.copy_(nb); rt.w.copy_(w)
        stream.synchronize()

        # --- timed region: exactly K layer-steps ------------------------------------------------
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        ev0.record(stream)
        if use_graph:
            for _ in range(K // cycle):
                graph.replay()
        elif graph is not None:
            graph.replay()
        else:
            for i in range(W, W + K):
                layer_step(i)
        ev1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
    gpu_ms = ev0.elapsed_time(ev1)
    elapsed = max(wall, gpu_ms / 1e3)

    err = max(rt.tables()[2] for rt in layers)
    nb_end, w_end, _ = layers[0].tables()
    t_end = t0 + (W + K + NL - 1) // NL         # tokens the first layer's cache has seen
    want = (t_end // c, t_end % c) if c > 0 else (0, t_end)
    assert err == 0 and (int(nb_end[0]), int(w_end[0])) == want, (err, nb_end[0], w_end[0], want)
    assert torch.isfinite(layers[0].out).all()

    tok_first = t0 + W // NL + 1
    step_bytes = [kv_bytes_per_step(wl, t) for t in range(tok_first, t_end + 1)]
    # layer-step i (counted from the warm-up start) belongs to token t0 + i // NL + 1
    total_bytes = sum(step_bytes[(i // NL) - (W // NL)] for i in range(W, W + K))
    launches = K
    if faithful:     # the beacon steps read the full window plus the beacon itself
        row = wl.B * wl.Hkv * wl.d * 2 * 2
        beacon_tokens = [t for t in range(tok_first, t_end + 1) if t % c == 0]
        total_bytes += sum(kv_bytes_per_step(wl, t) + row for t in beacon_tokens) * NL
        launches += len(beacon_tokens) * NL
    value = total_bytes / elapsed / 1e9

    # --- dominant kernel: the fused step kernel (append + attention + eviction in one launch),
    # timed by HIP event pairs on the launch stream, over the same token range of the rollout.
    n_samp = 0
    samp_bytes = 0
    samp_ms = 0.0
    with torch.cuda.stream(stream):
        for rt in layers:
            t_s = tok_first - 1
            if c > 0:
                rt.set_tables(np.full(wl.B, t_s // c, np.int32), np.full(wl.B, t_s % c, np.int32))
            else:
                rt.set_tables(np.zeros(wl.B, np.int32), np.full(wl.B, t_s, np.int32))
        n_tok = t_end - tok_first + 1
        stride = max(1, n_tok // 256)
        pairs = []
        for j in range(n_tok):
            for li, rt in enumerate(layers):
                x = pool[(j * NL + li) % n_pool]
                sampled = j % stride == 0 and li == (j // stride) % NL
                if sampled:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                rt.decode_step(x["k"], x["v"], x["q"], x["bk"] if c > 0 else None,
                               x["bv"] if c > 0 else None)
                if sampled:
                    e1.record(stream)
                    pairs.append((e0, e1, step_bytes[j]))
        stream.synchronize()
    for e0, e1, nbytes in pairs:
        samp_ms += e0.elapsed_time(e1)
        samp_bytes += nbytes
        n_samp += 1
    achieved = samp_bytes / (samp_ms / 1e3) / 1e9 if samp_ms > 0 else 0.0
    avg_launch_us = samp_ms * 1e3 / max(n_samp, 1)
    method = "HIP event pair around each of %d sampled launches (eager)" % n_samp
    if graph is not None:
        # The timed region is K back-to-back launches of this one kernel and nothing else, so the
        # region's own event pair gives the average launch duration without per-pair event cost.
        avg_launch_us = gpu_ms * 1e3 / launches
        achieved = total_bytes / (gpu_ms / 1e3) / 1e9
        method = "HIP events over the timed region / %d launches (graph replay, one kernel per step)" % launches

    rec = {
        "metric": "decode_attn_kv_GBps", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(elapsed * 1e3 / K, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "steps_per_sec": round(K / elapsed, 1),
        "token_steps_per_sec_%d_layers" % NL: round(K / NL / elapsed, 1),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "config": {"workload": "batch64 rollout: B=64, Hq=12, Hkv=2, d=128, bf16, P=256, G=4096, c=%s; "
                               "tokens %d..%d of the rollout" % (c if c > 0 else "inf", tok_first, t_end),
                   "layers_round_robin": NL, "hip_graph": graph is not None, "beacon_token_attention": bool(faithful),
                   "uniform_layout_promise": bool(layers[0].cache.uniform_P > 0),
                   "step": "bc_decode_step for one layer: append_kv + decode_attn + compress_evict, one launch",
                   "kv_bytes_per_step_mean": int(np.mean(step_bytes))},
        "roofline": {"bound": "hbm", "kernel": "bc::decode_lds_kernel<false, 1, 128, 2, 12> (bc_decode_step: append + attention + eviction)",
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": (stored_traffic() or {}).get("bytes_per_launch"),
                     "traffic_detail": stored_traffic(),
                     "avg_launch_us": round(avg_launch_us, 3), "method": method,
                     "avg_launch_us_event_pairs_eager": round(samp_ms * 1e3 / max(n_samp, 1), 3),
                     "bytes_per_launch_mean": int(total_bytes / launches)},
    }
    if c > 0 and not args.no_control:
        del layers, pool
        torch.cuda.empty_cache()
        rec["uncompressed_control"] = uncompressed_control(dev)
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
