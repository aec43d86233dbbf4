"""GPU test of the allocation-free entry point bc_decode_step_noalloc: through the C ABI, against
bc_decode_step on an identical cache with a workspace of its own - outputs, tables and slabs must
be identical (the same kernels run) - on two calls in a row, the second on a smaller input that
takes the split-and-merge path, whose partial results live in the shared scratch array."""
import numpy as np
import pytest

from paper_2510_13797_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def _pair(wl, dev, cap=None):
    """Two runtimes with identical caches (prompt from the workload)."""
    from paper_2510_13797_amd import bc
    bc.load()
    cap = wl.capacity() if cap is None else cap
    pk, pv = zip(*[wl.prompt_kv(s) for s in range(wl.B)])
    rts = []
    for _ in range(2):
        rt = bc.Runtime(wl.B, wl.Hq, wl.Hkv, wl.d, wl.dtype, wl.scale, wl.P, wl.c, cap, dev)
        rt.cache_init(list(pk), list(pv))
        rts.append(rt)
    return rts


def _same_state(a, b):
    import torch
    na, wa, ea = a.tables()
    nb, wb, eb = b.tables()
    assert list(na) == list(nb) and list(wa) == list(wb) and ea == eb == 0
    for s in range(a.B):
        Ka, Va = a.resident(s, int(na[s]), int(wa[s]))
        Kb, Vb = b.resident(s, int(nb[s]), int(wb[s]))
        assert np.array_equal(Ka, Kb) and np.array_equal(Va, Vb), s


def test_noalloc_step_equals_the_step_with_a_workspace(dev):
    import torch
    from paper_2510_13797_amd import bc
    # first call(s): the headline shape (64 sequences, 12/2 heads, d = 128, bf16, c = 16), fused steps
    # across a window end: tickets in the scratch array, eviction by the last ticket
    wl = W.batch64(G=40)
    ref, sta = _pair(wl, dev)
    for t in range(1, 35):
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        a = ref.decode_step(k, v, q, bk, bv).clone()
        b = sta.decode_step_noalloc(k, v, q, bk, bv).clone()
        assert torch.equal(a, b), t
    _same_state(ref, sta)
    assert int(ref.tables()[0][0]) == 2          # two windows were closed on the way
    # second call: a smaller input - 8 sequences of 1500 uncompressed rows, split into chunks whose
    # partial results go through the scratch array and a merge launch
    wl2 = W.batch64(c=0, G=1500, B=8)
    ref2, sta2 = _pair(wl2, dev)
    for rt in (ref2, sta2):
        g = torch.Generator(device=dev).manual_seed(7)
        rt.k_slab.copy_(torch.randn(rt.k_slab.shape, generator=g, device=dev, dtype=torch.float32))
        rt.v_slab.copy_(torch.randn(rt.v_slab.shape, generator=g, device=dev, dtype=torch.float32))
        rt.set_tables(np.zeros(8, np.int32), np.full(8, 1200, np.int32))
    st, text = bc.bc_decode_plan_describe(sta2.shape, sta2.cache)
    assert st == 0 and "merge" in text, text
    for t in (1201, 1202):
        k, v = wl2.step_kv(t)
        q = wl2.step_q(t)
        a = ref2.decode_step(k, v, q).clone()
        b = sta2.decode_step_noalloc(k, v, q).clone()
        assert torch.equal(a, b), t
        assert not torch.equal(a, torch.zeros_like(a))
    _same_state(ref2, sta2)
    # and the first shape once more: what the smaller call left in the array does not matter
    t = 35
    k, v = wl.step_kv(t)
    q = wl.step_q(t)
    bk, bv = wl.beacon_kv(t)
    assert torch.equal(ref.decode_step(k, v, q, bk, bv), sta.decode_step_noalloc(k, v, q, bk, bv))
    _same_state(ref, sta)


def test_noalloc_step_on_the_plain_alu_path(dev):
    import torch
    # fp32 rows: the fused step on the plain-ALU kernel, one ticket per workgroup in the scratch array
    wl = W.tiny()
    ref, sta = _pair(wl, dev)
    for t in range(1, 20):
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        assert torch.equal(ref.decode_step(k, v, q, bk, bv), sta.decode_step_noalloc(k, v, q, bk, bv)), t
    _same_state(ref, sta)


def test_noalloc_step_captured_in_a_graph(dev):
    import torch
    from paper_2510_13797_amd import bc
    # the callers the entry point is for: a cycle of steps captured as a HIP graph (no allocation,
    # the counters cleared by a fill kernel, not a memset node) and replayed, with eager work and
    # synchronisations between the replays; every replay equals the eager run on a workspace
    B, cyc, ncyc = 8, 4, 4
    wl = W.Workload("noalloc_graph", 97, B, 12, 2, 128, "bf16", np.array([3, 40, 0, 17, 64, 5, 33, 1], np.int32),
                    np.full(B, cyc * ncyc, np.int32), np.array([4, 2, 0, 1, 3, 4, 2, 4], np.int32))
    ref, sta = _pair(wl, dev)
    pool = []
    for j in range(1, cyc + 1):
        k, v = wl.step_kv(j)
        bk, bv = wl.beacon_kv(j)
        pool.append({n: bc.to_device(a, "bf16", dev) for n, a in dict(k=k, v=v, q=wl.step_q(j), bk=bk, bv=bv).items()})
    outs_ref = [torch.empty_like(ref.out) for _ in range(cyc)]
    outs_sta = [torch.empty_like(sta.out) for _ in range(cyc)]
    want = []
    for _ in range(ncyc):
        for j, x in enumerate(pool):
            ref.decode_step(x["k"], x["v"], x["q"], x["bk"], x["bv"], out=outs_ref[j])
        torch.cuda.synchronize()
        want.append([o.clone() for o in outs_ref])
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for j, x in enumerate(pool):                       # first cycle eagerly (also takes the scratch address)
            sta.decode_step_noalloc(x["k"], x["v"], x["q"], x["bk"], x["bv"], out=outs_sta[j])
        st.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(outs_sta, want[0]))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            for j, x in enumerate(pool):
                sta.decode_step_noalloc(x["k"], x["v"], x["q"], x["bk"], x["bv"], out=outs_sta[j])
        for r in range(1, ncyc):
            g.replay()
            st.synchronize()
            for j in range(cyc):
                assert torch.equal(outs_sta[j], want[r][j]), (r, j)
            sta.decode_attn(pool[0]["q"], out=torch.empty_like(sta.out))      # eager work between replays
            assert sta.tables()[2] == 0
    _same_state(ref, sta)
