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


def stored_profile(name):
    """HBM bytes per launch of a decode kernel as measured by a committed rocprofv3 PMC run
    (FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size); None if absent.
    bench.py cannot run the profiler around itself, so it reports the stored measurement and
    says so."""
    path = os.path.join(ROOT, "profiles", name)
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
                "source": "stored measurement: profiles/" + name}
    except (OSError, KeyError, ValueError):
        return None


def stored_traffic():
    return stored_profile("decode_batch64_c16_hbm_traffic.txt")


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

    # default: bc_prefill_attn (weights in two bf16 parts, the form whose output also feeds the
    # backward); --workspace-prefill: bc_prefill_attn_ws (V copied to half precision by a conversion
    # pass inside the timed call, weights in one half-precision part when V allows it, as N(0,1) does)
    use_ws = args.workspace_prefill
    ws_bytes = int(bc.bc_prefill_workspace_bytes(shape, R)) if use_ws else 0
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def step():
        if use_ws:
            st = bc.bc_prefill_attn_ws(shape, ptr(q), ptr(k), ptr(v), ptr(offd), ptr(Pd), ptr(cd), S, R, ptr(out),
                                       ptr(lse), ptr(ws), ws_bytes, C.c_void_p(stream.cuda_stream))
        else:
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
           "roofline": {"bound": "mfma",
                        "kernel": "bc::prefill_kernel<3, 128, %s>" % ("true" if use_ws else "false"),
                        "entry_point": "bc_prefill_attn_ws (conversion pass included)" if use_ws else "bc_prefill_attn",
                        "achieved": round(tflops, 2),
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
    (the K/V bytes of one step at L = 512) from 16 rotating buffers, with the decode grid's
    workgroup counts and with larger grids, by register loads (mode 0) and by LDS-DMA with up to
    48 KB in flight per wave (mode 1), as back-to-back launches replayed from a HIP graph."""
    import torch
    from paper_2510_13797_amd import bc
    bc.load_diag()
    dev = torch.device("cuda:0")
    nbytes = 64 * 512 * 2 * 128 * 2 * 2                 # B x L x Hkv x d x 2 bytes x (K and V)
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(16)]
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    st = torch.cuda.Stream()
    n_launch, reps = 256, 8

    def timed(nb, wgs, mode):
        with torch.cuda.stream(st):
            sp = st.cuda_stream

            def run():
                for i in range(n_launch):
                    rc = bc.bc_diag_stream_read(bufs[i % 16].data_ptr() if nb else None, nb, wgs, mode,
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

    empty_us = timed(0, 128, 0)
    res = []
    for mode, what in ((0, "register loads"), (1, "LDS-DMA")):
        for wgs in (128, 256, 512, 1024, 2048):
            us = timed(nbytes, wgs, mode)
            res.append({"mode": what, "workgroups": wgs, "us_per_launch": round(us, 3),
                        "GBps": round(nbytes / us / 1e3, 1)})
    print(json.dumps({"workload": "readfloor", "bytes_per_launch": nbytes, "launches_per_graph": n_launch,
                      "empty_kernel_us": round(empty_us, 3), "results": res}))


# ---------------------------------------------------------------------------
# CPU baseline: the oracle on the host cores, in worker processes that are started before anything
# touches the GPU (a process that has initialised the GPU is never forked).
# ---------------------------------------------------------------------------
def host_cores():
    """Cores this process may use: its affinity mask, and at most the 16 a one-GPU machine grants."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def _cpu_worker(job):
    """One worker's share: decode steps of the oracle over its sequences until the time is up.
    job = (lengths of its sequences, Hq, Hkv, d, scale, seconds, seed)."""
    lengths, Hq, Hkv, d, scale, seconds, seed = job
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)         # one thread per worker: the workers are the cores
    except Exception:                                 # pragma: no cover
        limiter = None
    from oracle import attention as OA
    rng = np.random.default_rng(seed)
    K = [rng.standard_normal((L, Hkv, d)).astype(np.float32) for L in lengths]
    V = [rng.standard_normal((L, Hkv, d)).astype(np.float32) for L in lengths]
    t0 = time.perf_counter()
    steps = 0
    while time.perf_counter() - t0 < seconds:
        q = rng.standard_normal((len(lengths), Hq, d)).astype(np.float32)
        for s in range(len(lengths)):
            OA.decode_attention(q[s], K[s], V[s], scale)
        steps += 1
    del limiter
    return steps, time.perf_counter() - t0


def cpu_baseline(pool, ncores, wl, lengths, what, budget_s=12.0):
    """Oracle decode attention timed on the host cores, on a bounded sample of the workload: the
    sequences of the state `lengths` (resident rows per sequence) are dealt round-robin to the
    workers, each of which repeats decode steps over its share for `budget_s` seconds."""
    lengths = [int(x) for x in lengths]
    shares = [lengths[i::ncores] for i in range(ncores)]
    shares = [sh for sh in shares if sh]
    jobs = [(sh, wl.Hq, wl.Hkv, wl.d, wl.scale, budget_s, 100 + i) for i, sh in enumerate(shares)]
    t0 = time.perf_counter()
    res = pool.map(_cpu_worker, jobs)
    wall = time.perf_counter() - t0
    row = wl.Hkv * wl.d * 2 * 2                   # bytes of one resident entry (K and V) in the GPU's format
    nbytes = sum(steps * sum(sh) * row for (steps, _), sh in zip(res, shares))
    seq_steps = sum(steps * len(sh) for (steps, _), sh in zip(res, shares))
    span = max(el for _, el in res)
    return {"value": nbytes / span / 1e9, "unit": "GB/s", "cores": len(shares), "host_nproc": os.cpu_count(),
            "kind": "oracle", "steps_per_sec": seq_steps / len(lengths) / span,
            "sample": "%s: %d sequences x %d heads dealt to %d worker processes (one thread each), fp64 NumPy "
                      "oracle repeated for %.1f s (%.1f s with start-up)" % (what, len(lengths), wl.Hq,
                                                                           len(shares), span, wall)}


# ---------------------------------------------------------------------------
# decode workloads
# ---------------------------------------------------------------------------
def tables_at(wl, t):
    """(nb, w) after t generated tokens per sequence (t: scalar or [B])."""
    t = np.broadcast_to(np.asarray(t, dtype=np.int64), (wl.B,))
    cc = np.maximum(wl.c, 1).astype(np.int64)
    nb = np.where(wl.c > 0, t // cc, 0)
    w = np.where(wl.c > 0, t % cc, t)
    return nb.astype(np.int32), w.astype(np.int32)


def rows_seen(wl, t):
    """Resident rows per sequence that the attention of decode step t reads (t: scalar or [B])."""
    t = np.broadcast_to(np.asarray(t, dtype=np.int64), (wl.B,))
    cc = np.maximum(wl.c, 1).astype(np.int64)
    gen = np.where(wl.c > 0, (t - 1) // cc + (t - 1) % cc + 1, t)
    return wl.P.astype(np.int64) + gen


class DecodeBench:
    """NL cache instances of one workload (the layers of a model, visited round-robin so that every
    step reads its K/V from HBM), their tables in one tensor so that one small kernel restores
    them, a pool of resident inputs, and the fused step of one layer."""

    def __init__(self, wl, NL, dev, t_start, sort=False, plan=0):
        import torch
        from paper_2510_13797_amd import bc
        self.torch, self.bc, self.wl, self.NL, self.dev = torch, bc, wl, NL, dev
        gen = torch.Generator(device=dev)
        gen.manual_seed(20251013)
        self.gen = gen
        cap = wl.capacity()
        self.tab = torch.zeros(NL, 2, wl.B, dtype=torch.int32, device=dev)
        self.layers = []
        for li in range(NL):
            rt = bc.Runtime(wl.B, wl.Hq, wl.Hkv, wl.d, wl.dtype, wl.scale, wl.P, wl.c, cap, dev)
            rt.k_slab.copy_(torch.randn(rt.k_slab.shape, generator=gen, device=dev, dtype=torch.float32))
            rt.v_slab.copy_(torch.randn(rt.v_slab.shape, generator=gen, device=dev, dtype=torch.float32))
            rt.nb, rt.w = self.tab[li, 0], self.tab[li, 1]           # the tables live in the shared tensor
            rt.cache.nb, rt.cache.w = rt.nb.data_ptr(), rt.w.data_ptr()
            rt.cache.plan = plan
            self.layers.append(rt)
        self.set_state(t_start)
        if sort:
            for rt in self.layers:
                rt.sort_by_length()
        n_pool = 64
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        rnd = lambda *shape: torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        self.pool = [dict(k=rnd(wl.B, wl.Hkv, wl.d), v=rnd(wl.B, wl.Hkv, wl.d), q=rnd(wl.B, wl.Hq, wl.d),
                          bk=rnd(wl.B, wl.Hkv, wl.d), bv=rnd(wl.B, wl.Hkv, wl.d)) for _ in range(n_pool)]
        self.saved = torch.empty_like(self.tab)
        self.compress = bool((wl.c > 0).any())

    def set_state(self, t):
        nb, w = tables_at(self.wl, t)
        host = np.stack([nb, w])[None].repeat(self.NL, axis=0)
        self.tab.copy_(self.torch.from_numpy(np.ascontiguousarray(host)))

    def save(self):
        self.saved.copy_(self.tab)

    def restore(self):
        """One elementwise kernel (no memset or memcpy node when captured)."""
        self.torch.add(self.saved, 0, out=self.tab)

    def step(self, i, token=None):
        """Layer-step i (token: the decode step it belongs to)."""
        rt = self.layers[i % self.NL]
        x = self.pool[i % len(self.pool)]
        rt.decode_step(x["k"], x["v"], x["q"], x["bk"] if self.compress else None,
                       x["bv"] if self.compress else None)

    def beacon_step(self, li, i):
        y = self.pool[i % len(self.pool)]
        self.layers[li].beacon_step(y["bk"], y["bv"], y["q"])

    def kernel(self):
        st, text = self.bc.bc_decode_plan_describe(self.layers[0].shape, self.layers[0].cache)
        assert st == 0, st
        return text

    def check(self):
        err = max(rt.tables()[2] for rt in self.layers)
        assert err == 0, "device error bits %d" % err
        assert self.torch.isfinite(self.layers[0].out).all()


def replay_timed(stream, graph, replays):
    """(mean, min, median) microseconds per replay of a captured graph: one event pair around all
    replays for the mean, then one pair per replay for the spread."""
    import torch
    with torch.cuda.stream(stream):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        e0.record(stream)
        for _ in range(replays):
            graph.replay()
        e1.record(stream)
        stream.synchronize()
        wall = time.perf_counter() - wall0
        pairs = []
        for _ in range(replays):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            graph.replay()
            b.record(stream)
            pairs.append((a, b))
        stream.synchronize()
    each = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
    return e0.elapsed_time(e1) * 1e3 / replays, wall * 1e6 / replays, each[0], each[len(each) // 2]


def decode_record(wl, what, K, W, us_step, us_step_wall, step_bytes, extra_cfg, roof_extra, kernel, traffic):
    """The standard JSON line of a decode workload.  us_step: event time per step, us_step_wall:
    host clock per step; step_bytes: algorithmic K+V bytes of the timed steps."""
    total = float(sum(step_bytes))
    n = len(step_bytes)
    slow = max(us_step, us_step_wall)
    value = total / n / slow / 1e3
    achieved = total / n / us_step / 1e3
    rec = {"metric": "decode_attn_kv_GBps", "value": round(value, 2), "unit": "GB/s", "n_gpus": 1,
           "steps": K, "warmup": W, "ms_per_step": round(slow / 1e3, 6), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "steps_per_sec": round(1e6 / slow, 1), "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
           "config": dict({"workload": what,
                           "step": "bc_decode_step for one layer: append_kv + decode_attn + compress_evict, one launch",
                           "kv_bytes_per_step_mean": int(total / n)}, **extra_cfg),
           "roofline": dict({"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 2),
                             "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                             "traffic": (traffic or {}).get("bytes_per_launch"), "traffic_detail": traffic,
                             "avg_launch_us": round(us_step, 3), "bytes_per_launch_mean": int(total / n)},
                            **roof_extra)}
    return rec


def run_replayed(db, K, W, replays, first_token, tokens_per_step=None):
    """Warm up W layer-steps eagerly, then time the unit [restore tables, K layer-steps]: a small
    kernel at its head puts the tables back, so every execution of the unit does the same K
    steps.  One graph holds several units back to back (about 256 launches: the pause between two
    graph launches is then a small part of it) and is replayed until the unit has run at least
    `replays` times.  Returns timing per unit and the token index of each timed layer-step."""
    import torch
    stream = torch.cuda.Stream()
    NL = db.NL
    units = max(1, 256 // (K + 1))
    launches = (replays + units - 1) // units
    tok = (lambda i: first_token + i // NL) if first_token is not None else (lambda i: None)
    with torch.cuda.stream(stream):
        for i in range(W):
            db.step(i, tok(i))
        stream.synchronize()
        db.save()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(units):
                db.restore()
                for i in range(W, W + K):
                    db.step(i, tok(i))
        for _ in range(3):                      # untimed: the first replay of a graph pays for its upload
            graph.replay()
        stream.synchronize()
    after = db.tab.clone()
    us_ev, us_wall, us_min, us_med = replay_timed(stream, graph, launches)
    assert torch.equal(after, db.tab), "a replay did not end in the state of the one before"
    db.check()
    tokens = [first_token + i // NL for i in range(W, W + K)] if first_token is not None else []
    return {"us_replay_mean": us_ev / units, "us_replay_wall": us_wall / units, "us_replay_min": us_min / units,
            "us_replay_median": us_med / units, "tokens": tokens, "stream": stream,
            "units_run": launches * units, "units_per_graph": units}


def bench_decode(args, pool, ncores):
    """Config 2 (the headline): batch 64, 12/2 heads, d 128, bf16, P 256, G 4096, c 16.

    Without --steps/--warmup: the whole rollout (tokens 17..4096 through --layers cache instances),
    replayed as HIP graphs of one 16-token cycle.  With them (the driver's form): the last K
    layer-steps of the rollout, captured once behind a kernel that restores the tables and replayed
    --replays times between one event pair."""
    import torch
    from paper_2510_13797_amd import workloads
    dev = torch.device("cuda:0")
    wl = workloads.batch64(c=args.c)
    NL, G, c = args.layers, int(wl.G[0]), int(wl.c[0])
    what = "batch64 rollout: B=64, Hq=12, Hkv=2, d=128, bf16, P=256, G=4096, c=%s" % (c if c > 0 else "inf")
    cyc_tokens = c if c > 0 else 16
    cycle = cyc_tokens * NL
    total = G * NL
    if args.steps < 0 and args.warmup < 0 and not args.beacon_attn:
        # ---- the whole rollout --------------------------------------------------------------
        W, K = cycle, total - cycle
        db = DecodeBench(wl, NL, dev, 0, plan=args.plan)
        ncycles = K // cycle
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for i in range(cycle):
                db.step(i, 1 + i // NL)
            stream.synchronize()
            db.save()
            # one graph of a cycle (window position and input pool index repeat every cycle),
            # captured before the clock starts (capturing runs nothing)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(cycle):
                    db.step(i, cyc_tokens + 1 + i // NL)
            graphs = [(g, ncycles)]
            db.restore()                       # put the tables back where the warm-up left them
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            wall0 = time.perf_counter()
            e0.record(stream)
            for g, n in graphs:
                for _ in range(n):
                    g.replay()
            e1.record(stream)
            stream.synchronize()
            wall = time.perf_counter() - wall0
        db.check()
        nb_end, w_end, _ = db.layers[0].tables()
        want = (G // c, G % c) if c > 0 else (0, G)
        assert (int(nb_end[0]), int(w_end[0])) == want, (nb_end[0], w_end[0], want)
        tokens = [cyc_tokens + 1 + i // NL for i in range(K)]
        step_bytes = [kv_bytes_per_step(wl, t) for t in tokens]
        rec = decode_record(wl, what + "; tokens %d..%d of the rollout" % (tokens[0], tokens[-1]), K, W,
                            e0.elapsed_time(e1) * 1e3 / K, wall * 1e6 / K, step_bytes,
                            {"layers_round_robin": NL, "hip_graph": True, "replays": K // cycle,
                             "uniform_layout_promise": bool(db.layers[0].cache.uniform_P > 0)},
                            {"method": "HIP events over the timed region / %d launches (replays of one graph of a "
                                       "%d-token cycle, one kernel per step)" % (K, cyc_tokens)},
                            db.kernel(), stored_traffic())
        rec["token_steps_per_sec_%d_layers" % NL] = round(rec["steps_per_sec"] / NL, 1)
    else:
        # ---- the last K layer-steps of the rollout, replayed ----------------------------------
        W = args.warmup if args.warmup >= 0 else 5
        K = args.steps if args.steps >= 0 else 20
        if K < 1 or K + W > total:
            print("bench.py: steps must be at least 1 and steps + warmup at most %d" % total, file=sys.stderr)
            sys.exit(2)
        if args.beacon_attn and (c <= 0 or K % NL or W % NL):
            print("bench.py: --beacon-attn needs c > 0 and steps and warmup that are multiples of --layers",
                  file=sys.stderr)
            sys.exit(2)
        t0 = G - (K + W + NL - 1) // NL             # tokens already generated when the warm-up starts
        db = DecodeBench(wl, NL, dev, t0, plan=args.plan)
        launches = [K]
        if args.beacon_attn:
            # the beacon token's own pass through all layers follows the window's last token
            plain = db.step

            def faithful(i, token=None):
                rt, x = db.layers[i % NL], db.pool[i % len(db.pool)]
                rt.decode_step(x["k"], x["v"], x["q"], None, None)
                if (t0 + i // NL + 1) % c == 0 and i % NL == NL - 1:
                    for li in range(NL):
                        db.beacon_step(li, i + 1 + li)
                    if i >= W:
                        launches[0] += NL
            db.step = faithful
        r = run_replayed(db, K, W, args.replays, t0 + 1)
        step_bytes = [kv_bytes_per_step(wl, t) for t in r["tokens"]]
        if args.beacon_attn:
            row = wl.B * wl.Hkv * wl.d * 2 * 2
            step_bytes += [kv_bytes_per_step(wl, t) + row for t in sorted(set(r["tokens"])) if t % c == 0
                           for _ in range(NL)]
        n = len(step_bytes)
        rec = decode_record(wl, what + "; tokens %d..%d of the rollout" % (r["tokens"][0], r["tokens"][-1]), K, W,
                            r["us_replay_mean"] / n, r["us_replay_wall"] / n, step_bytes,
                            {"layers_round_robin": NL, "hip_graph": True, "replays": r["units_run"],
                             "units_per_graph": r["units_per_graph"],
                             "beacon_token_attention": bool(args.beacon_attn),
                             "uniform_layout_promise": bool(db.layers[0].cache.uniform_P > 0)},
                            {"method": "HIP events around %d executions of the unit [restore tables, %d steps], %d units "
                                       "per graph; per launch = unit / %d (the restore kernel's share included)"
                                       % (r["units_run"], K, r["units_per_graph"], n),
                             "min_launch_us": round(r["us_replay_min"] / n, 3),
                             "median_launch_us": round(r["us_replay_median"] / n, 3)},
                            db.kernel(), stored_traffic())
        rec["token_steps_per_sec_%d_layers" % NL] = round(rec["steps_per_sec"] / NL, 1)
    lengths = rows_seen(wl, G)
    del db
    torch.cuda.empty_cache()
    if c > 0 and not args.no_control:
        rec["uncompressed_control"] = uncompressed_control(dev, args)
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(pool, ncores, wl, lengths,
                                           "decode steps at the end-of-rollout state (L=%d)" % int(lengths[0]))
    print(json.dumps(rec))


def uncompressed_control(dev, args, NL=4, K=8, replays=25):
    """The same shapes without compression (c = infinity) at the end of the rollout: every sequence
    holds P + G = 4352 entries.  Fused steps (append + attention, no eviction), NL cache
    instances round-robin (2.3 GB > Infinity Cache), replayed like the main measurement."""
    from paper_2510_13797_amd import workloads
    wl = workloads.batch64(c=0)
    G = int(wl.G[0])
    db = DecodeBench(wl, NL, dev, G - (K + NL - 1) // NL - 1, plan=args.plan)
    r = run_replayed(db, K, NL, replays, G - (K + NL - 1) // NL)
    step_bytes = [kv_bytes_per_step(wl, t) for t in r["tokens"]]
    us = r["us_replay_mean"] / K
    nbytes = float(np.mean(step_bytes))
    out = {"workload": "same shapes, c=inf, end of rollout: L=%d entries per sequence" % int(rows_seen(wl, G)[0]),
           "kernel": db.kernel(), "kv_bytes_per_step": int(nbytes), "us_per_step": round(us, 2),
           "GBps": round(nbytes / us / 1e3, 1), "pct_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS * 100, 1)}
    del db
    return out


def bench_long(args, pool, ncores):
    """Config 4: long reasoning rollouts, batch 32, 32/8 heads, d 128, bf16, P 512, G 32768, c 32;
    the last K layer-steps of the rollout (L = 1536 and up), fused step."""
    import torch
    from paper_2510_13797_amd import workloads
    dev = torch.device("cuda:0")
    wl = workloads.long_reasoning()
    NL = args.layers if args.layers != 16 else 4        # 205 MB of K/V per instance
    G = int(wl.G[0])
    W = args.warmup if args.warmup >= 0 else NL
    K = args.steps if args.steps >= 0 else 32
    t0 = G - (K + W + NL - 1) // NL
    db = DecodeBench(wl, NL, dev, t0, plan=args.plan)
    r = run_replayed(db, K, W, args.replays, t0 + 1)
    step_bytes = [kv_bytes_per_step(wl, t) for t in r["tokens"]]
    rec = decode_record(wl, "long reasoning rollout: B=32, Hq=32, Hkv=8, d=128, bf16, P=512, G=32768, c=32; "
                            "tokens %d..%d of the rollout (L=%d..%d)" % (r["tokens"][0], r["tokens"][-1],
                                                                        int(rows_seen(wl, r["tokens"][0])[0]),
                                                                        int(rows_seen(wl, r["tokens"][-1])[0])),
                        K, W, r["us_replay_mean"] / K, r["us_replay_wall"] / K, step_bytes,
                        {"layers_round_robin": NL, "hip_graph": True, "replays": r["units_run"],
                         "units_per_graph": r["units_per_graph"]},
                        {"method": "HIP events around %d executions of the unit [restore tables, %d steps], %d units per graph"
                                   % (r["units_run"], K, r["units_per_graph"]),
                         "min_launch_us": round(r["us_replay_min"] / K, 3),
                         "median_launch_us": round(r["us_replay_median"] / K, 3)},
                        db.kernel(), stored_profile("decode_long_c32_hbm_traffic.txt"))
    lengths = rows_seen(wl, G)[:8]
    del db
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(pool, ncores, wl, np.repeat(lengths, 2),
                                           "decode steps at the end-of-rollout state (L=%d), 16 of the 32 sequences"
                                           % int(lengths[0]))
    print(json.dumps(rec))


def bench_ragged(args, pool, ncores):
    """Config 3: ragged batch of 256 sequences (P ~ U[64,512], G ~ U[1024,16384], c from
    {2,4,8,16,32}) around the snapshot step T drawn from the seed: the K timed fused steps end
    in the state in which sequence s has generated min(T, G_s) tokens (every sequence advances, the
    finished ones over the last tokens of their own rollout), with the dispatch order of
    bc_sort_by_length attached (refreshed once, before the capture) unless --no-sort."""
    import torch
    from paper_2510_13797_amd import workloads
    dev = torch.device("cuda:0")
    wl = workloads.ragged256()
    NL = args.layers if args.layers != 16 else 2          # about 0.5 GB of K/V per instance
    T = int(wl.extra["T"])
    W = args.warmup if args.warmup >= 0 else NL
    K = args.steps if args.steps >= 0 else 16
    # the timed steps end at the snapshot: sequence s goes from t_s - n to t_s = min(T, G_s) tokens
    t_start = np.minimum(T, wl.G).astype(np.int64) - (K + W + NL - 1) // NL
    db = DecodeBench(wl, NL, dev, t_start, sort=not args.no_sort, plan=args.plan)
    r = run_replayed(db, K, W, args.replays, None)
    # layer-step i (from the warm-up start) is decode step t_start + i // NL + 1 of every sequence
    step_bytes = [int(rows_seen(wl, t_start + i // NL + 1).sum()) * wl.Hkv * wl.d * 2 * 2 for i in range(W, W + K)]
    Ls = rows_seen(wl, np.minimum(T, wl.G))
    rec = decode_record(wl, "ragged batch: 256 sequences, Hq=12, Hkv=2, d=128, bf16, P~U[64,512], G~U[1024,16384], "
                            "c in {2,4,8,16,32}; the %d steps that end at the snapshot T=%d (resident rows %d..%d, %d in all)"
                            % (K, T, int(Ls.min()), int(Ls.max()), int(Ls.sum())),
                        K, W, r["us_replay_mean"] / K, r["us_replay_wall"] / K, step_bytes,
                        {"layers_round_robin": NL, "hip_graph": True, "replays": r["units_run"],
                         "units_per_graph": r["units_per_graph"],
                         "dispatch_order": "bc_sort_by_length, once before the capture" if not args.no_sort else "index order"},
                        {"method": "HIP events around %d executions of the unit [restore tables, %d steps], %d units per graph"
                                   % (r["units_run"], K, r["units_per_graph"]),
                         "min_launch_us": round(r["us_replay_min"] / K, 3),
                         "median_launch_us": round(r["us_replay_median"] / K, 3)},
                        db.kernel(), stored_profile("decode_ragged256_hbm_traffic.txt"))
    del db
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(pool, ncores, wl, Ls[:64],
                                           "decode steps at the snapshot state, the first 64 of the 256 sequences")
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="decode",
                    choices=["decode", "ragged256", "long", "prefill", "prefill_bwd", "distill", "copy", "readfloor"])
    ap.add_argument("--workspace-prefill", action="store_true",
                    help="prefill workload: time bc_prefill_attn_ws (half-precision value product) instead of bc_prefill_attn")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=-1)
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--replays", type=int, default=200,
                    help="executions of the timed steps (decode workloads with --steps), at least")
    ap.add_argument("--layers", type=int, default=16, help="cache instances visited round-robin")
    ap.add_argument("--c", type=int, default=16, help="compression ratio (0: uncompressed control)")
    ap.add_argument("--beacon-attn", action="store_true",
                    help="also run the beacon token's own attention (bc_beacon_step) at every window end "
                         "instead of handing the beacon K/V to the token step")
    ap.add_argument("--no-sort", action="store_true", help="ragged256: dispatch in index order")
    ap.add_argument("--plan", type=int, default=0, help="bc_cache::plan bits for the decode calls (measurements)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-control", action="store_true", help="skip the uncompressed (c=inf) control measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU sharding is a design "
              "note in the design document, not an implemented path", file=sys.stderr)
        sys.exit(2)

    # the CPU baseline's worker processes start here, before this process initialises the GPU
    pool = ncores = None
    if args.workload in ("decode", "ragged256", "long") and not args.no_cpu_baseline:
        import multiprocessing as mp
        ncores = host_cores()
        pool = mp.get_context("fork").Pool(ncores)

    import torch
    from paper_2510_13797_amd import bc
    bc.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(torch.device("cuda:0"))
    try:
        if args.workload == "decode":
            bench_decode(args, pool, ncores)
        elif args.workload == "ragged256":
            bench_ragged(args, pool, ncores)
        elif args.workload == "long":
            bench_long(args, pool, ncores)
        elif args.workload == "prefill":
            bench_prefill(args)
        elif args.workload == "prefill_bwd":
            bench_prefill_bwd(args)
        elif args.workload == "distill":
            bench_distill(args)
        elif args.workload == "copy":
            bench_copy(args)
        else:
            bench_readfloor(args)
    finally:
        if pool is not None:
            pool.close()
            pool.join()


if __name__ == "__main__":
    main()
