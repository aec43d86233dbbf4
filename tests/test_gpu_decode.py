"""GPU parity: bc_append_kv / bc_decode_attn / bc_compress_evict against the CPU oracle,
through the C ABI, on the five-config shapes (decode side).  Tolerances: max-abs-error
1e-5 for fp32 inputs, 2e-3 for bf16 inputs (fp32 accumulation); tables, error bits and
resident slab rows bit-exact."""
import numpy as np
import pytest

from oracle import attention as OA
from oracle import residency as OR
from oracle.cache import BatchCache, ERR_CAPACITY, ERR_STATE
from paper_2510_13797_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def _bc():
    from paper_2510_13797_amd import bc
    bc.load()                       # fails loudly if libbc.so is missing
    return bc


def make(wl, dev, cap=None):
    bc = _bc()
    cap = wl.capacity() if cap is None else cap
    rt = bc.Runtime(wl.B, wl.Hq, wl.Hkv, wl.d, wl.dtype, wl.scale, wl.P, wl.c, cap, dev)
    pk, pv = zip(*[wl.prompt_kv(s) for s in range(wl.B)])
    rt.cache_init(list(pk), list(pv))
    oc = BatchCache(list(pk), list(pv), wl.c, cap)
    return rt, oc


def check_tables(rt, oc, t=None):
    nb, w, err = rt.tables()
    assert list(nb) == oc.nb, ("nb", t)
    assert list(w) == oc.w, ("w", t)
    assert err == oc.err, ("err", t, err, oc.err)
    return nb, w


def check_slabs(rt, oc, seqs=None, t=None):
    nb, w, _ = rt.tables()
    for s in (range(rt.B) if seqs is None else seqs):
        K, V = rt.resident(s, int(nb[s]), int(w[s]))
        Ko, Vo = oc.resident(s)
        assert K.shape == Ko.shape, (s, t)
        assert np.array_equal(K, Ko) and np.array_equal(V, Vo), ("slab", s, t)


def check_attention(o, q, oc, wl, seqs=None, t=None):
    worst = 0.0
    for s in (range(wl.B) if seqs is None else seqs):
        K, V = oc.resident(s)
        ref = OA.decode_attention(q[s], K, V, wl.scale)
        worst = max(worst, float(np.abs(o[s].astype(np.float64) - ref).max()))
    assert worst <= TOL[wl.dtype], (t, worst)
    return worst


def rollout(wl, rt, oc, steps, attn_steps, slab_steps, table_every=1, tail_form=False,
            use_step_call=False, seq_sample=None, beacon_call=False, before_step=None):
    """Alg. 1 for `steps` decode steps; sequences whose generation is over stay resident."""
    attn_steps, slab_steps = set(attn_steps), set(slab_steps)
    worst = 0.0
    q_any = None
    for t in range(1, steps + 1):
        if before_step is not None:
            before_step(t)
        active = (wl.G >= t).astype(np.uint8)
        act = None if active.all() else active
        k, v = wl.step_kv(t)
        need_attn = t in attn_steps
        if need_attn:
            q = wl.step_q(t)
        elif use_step_call or beacon_call:
            # the step calls need a query; where the output is not compared any will do (drawing one
            # per step is most of the host time of a long rollout)
            q = q_any = wl.step_q(1) if q_any is None else q_any
        else:
            q = None
        bk, bv = wl.beacon_kv(t)
        if beacon_call:
            # token step without eviction, then the beacon's own step (bc_beacon_step): beacon row
            # at the tail, its attention, compaction - one launch each on the bf16 d=128 path
            o = rt.decode_step(k, v, q, None, None, active=act)
            oc.append(k, v, active=act)
            if need_attn:
                seqs = [s for s in (range(wl.B) if seq_sample is None else seq_sample) if active[s]]
                worst = max(worst, check_attention(o.cpu().numpy(), q, oc, wl, seqs, t))
            qb = wl.beacon_q(t) if need_attn else q
            ob = rt.beacon_step(bk, bv, qb, active=act)
            oc.append(bk, bv, active=act, beacon=True)
            due = [s for s in range(wl.B) if active[s] and oc.c[s] > 0 and oc.w[s] == oc.c[s] + 1]
            if need_attn and due:
                worst = max(worst, check_attention(ob.cpu().numpy(), qb, oc, wl, due, t))
            oc.compress_evict(active=act)
        elif use_step_call:
            o = rt.decode_step(k, v, q, bk, bv, active=act)
            oc.append(k, v, active=act)
            if need_attn:
                seqs = [s for s in (range(wl.B) if seq_sample is None else seq_sample) if active[s]]
                worst = max(worst, check_attention(o.cpu().numpy(), q, oc, wl, seqs, t))
            oc.compress_evict(bk, bv, active=act)
        else:
            rt.append_kv(k, v, active=act)
            oc.append(k, v, active=act)
            if need_attn:
                o = rt.decode_attn(q, active=act).cpu().numpy()
                seqs = [s for s in (range(wl.B) if seq_sample is None else seq_sample) if active[s]]
                worst = max(worst, check_attention(o, q, oc, wl, seqs, t))
            if tail_form:
                rt.append_kv(bk, bv, active=act, kind=1)
                oc.append(bk, bv, active=act, beacon=True)
                if need_attn:       # the beacon's own query sees prompt, beacons, window, itself
                    due = [s for s in range(wl.B) if active[s] and oc.c[s] > 0 and oc.w[s] == oc.c[s] + 1]
                    if due:
                        qb = wl.beacon_q(t)
                        dm = np.zeros(wl.B, np.uint8)
                        dm[due] = 1
                        ob = rt.decode_attn(qb, active=dm).cpu().numpy()
                        worst = max(worst, check_attention(ob, qb, oc, wl, due, t))
                rt.compress_evict(active=act)
                oc.compress_evict(active=act)
            else:
                rt.compress_evict(bk, bv, active=act)
                oc.compress_evict(bk, bv, active=act)
        if t % table_every == 0 or t in slab_steps or t == steps:
            check_tables(rt, oc, t)
        if t in slab_steps:
            check_slabs(rt, oc, seq_sample, t)
    return worst


# ---------------------------------------------------------------------------
def test_config1_tiny_every_step(dev):
    wl = W.tiny()
    rt, oc = make(wl, dev)
    steps = range(1, 257)
    worst = rollout(wl, rt, oc, 256, steps, steps)
    nb, w, _ = rt.tables()
    assert list(nb) == [16, 16] and list(w) == [0, 0]
    for s in range(wl.B):       # invariant: L = P + floor(t/c) + (t mod c)
        assert 32 + nb[s] + w[s] == OR.len_after_step(32, 16, 256)
    print("tiny worst", worst)


def test_config1_tail_form_with_beacon_query(dev):
    wl = W.tiny(seed=11)
    rt, oc = make(wl, dev)
    rollout(wl, rt, oc, 80, range(1, 81), range(1, 81), tail_form=True)


def test_config1_fused_step_call(dev):
    wl = W.tiny(seed=12)
    rt, oc = make(wl, dev)
    rollout(wl, rt, oc, 64, range(1, 65), (16, 17, 64), use_step_call=True)


@pytest.mark.parametrize("c,P,d", [(16, 256, 128), (1, 5, 128), (2, 0, 128), (3, 31, 128), (0, 40, 128),
                                   (16, 256, 64), (1, 5, 64), (3, 31, 64)])
def test_fused_step_bf16_every_step(dev, c, P, d):
    # bc_decode_step on the single-launch path (bf16, d = 128 or 64): tables, slabs, outputs each step
    wl = W.Workload("fused", 70 + c, 6, 12, 2, d, "bf16", np.full(6, P, np.int32),
                    np.array([150, 150, 90, 150, 33, 150], np.int32), np.full(6, c, np.int32))
    rt, oc = make(wl, dev)
    steps = range(1, 151)
    rollout(wl, rt, oc, 150, steps, steps, use_step_call=True)


@pytest.mark.parametrize("dtype,d,B", [("f32", 128, 6), ("f32", 64, 6), ("bf16", 128, 6), ("bf16", 64, 6),
                                       ("f32", 128, 2), ("bf16", 128, 2)])
def test_fused_step_on_the_plain_alu_kernel(dev, dtype, d, B):
    # the same single-launch step on the kernel that serves fp32 rows (and bf16 rows when the
    # plan asks for it): ragged ratios with c = 1 and no compression among them, sequences that
    # end early, the budget-free and the beacon-step forms; tables, slabs and outputs each step.
    # B = 2 with a long prompt spreads a sequence's rows over several workgroups and a merge
    # launch, each workgroup taking its own ticket.
    P = np.array([1100, 1050], np.int32) if B == 2 else np.array([40, 0, 17, 64, 5, 33], np.int32)
    c = np.array([16, 3], np.int32) if B == 2 else np.array([16, 1, 0, 3, 2, 7], np.int32)
    G = np.array([70, 70], np.int32) if B == 2 else np.array([70, 70, 50, 70, 21, 70], np.int32)
    for beacon_call in (False, True):
        wl = W.Workload("fused_alu", 90 + d + B, B, 4, 2, d, dtype, P, G, c)
        rt, oc = make(wl, dev)
        if dtype == "bf16":
            rt.cache.plan = _bc().BC_PLAN_PLAIN_ALU
        st, text = _bc().bc_decode_plan_describe(rt.shape, rt.cache)
        assert st == 0 and "decode_valu_kernel" in text, text
        if B == 2:
            assert int(text.split("chunks=")[1].split()[0]) > 1, text
        steps = range(1, 71)
        rollout(wl, rt, oc, 70, steps, steps, use_step_call=not beacon_call, beacon_call=beacon_call)


@pytest.mark.parametrize("promise", ["as built", "none", "prompt too long", "prompt too short"])
@pytest.mark.parametrize("Hkv,d", [(2, 128), (8, 128), (2, 64)])
def test_uniform_layout_promise_is_only_a_hint(dev, promise, Hkv, d):
    # equal prompt lengths and capacities: the binding states the layout and the kernel requests prompt
    # rows before it has read the tables; a promise that names another prompt length must not change
    # any result (the rows are requested again); Hkv = 8 takes the one-workgroup-per-pair kernel
    B, P, G = 40, 100, 60
    wl = W.Workload("promise", 97, B, 2 * Hkv, Hkv, d, "bf16", np.full(B, P, np.int32),
                    np.full(B, G, np.int32), np.full(B, 8, np.int32))
    cap = np.full(B, 176, np.int32)
    rt, oc = make(wl, dev, cap)
    assert rt.cache.uniform_P == P and rt.cache.uniform_cap == 176
    if promise == "none":
        rt.cache.uniform_P = rt.cache.uniform_cap = 0
    elif promise == "prompt too long":
        rt.cache.uniform_P = 160           # rows 100..159 are not all resident yet: unwritten slab rows
    elif promise == "prompt too short":
        rt.cache.uniform_P = 64
    rollout(wl, rt, oc, G, (1, 2, 8, 9, 33, 60), (8, 60), use_step_call=True)


@pytest.mark.parametrize("B,Hkv,d,P", [(12, 2, 128, 410), (40, 4, 128, 270), (12, 2, 64, 270)])
def test_second_tiles_of_the_straight_line_kernel(dev, B, Hkv, d, P):
    # short caches run on the straight-line form of the kernel, where a wave has at most two tiles:
    # 24 pairs, d = 128: two twelve-wave workgroups per pair, second tiles from row 384; 160 pairs,
    # and d = 64: eight waves, second tiles from row 256.  The rollout crosses those rows, with the
    # appended row in a first tile, in a second tile and on a tile boundary.
    G, c = 70, 8
    wl = W.Workload("twotiles", 98, B, 2 * Hkv, Hkv, d, "bf16", np.full(B, P, np.int32),
                    np.where(np.arange(B) % 3 == 2, 40, G).astype(np.int32), np.full(B, c, np.int32))
    rt, oc = make(wl, dev, np.full(B, P + G // c + c + 1, np.int32))       # one capacity: uniform layout
    st, text = _bc().bc_decode_plan_describe(rt.shape, rt.cache)
    assert st == 0 and "true>" in text, text          # the straight-line kernel serves these shapes
    rollout(wl, rt, oc, G, range(1, G + 1), (8, 40, G), use_step_call=True)
    q = wl.step_q(G + 1)
    check_attention(rt.decode_attn(q).cpu().numpy(), q, oc, wl, None, "attn")
    # the same rows on the general tile loop
    rt.cache.plan = _bc().BC_PLAN_GENERAL_LOOP
    st, text = _bc().bc_decode_plan_describe(rt.shape, rt.cache)
    assert st == 0 and "true>" not in text, text
    check_attention(rt.decode_attn(q).cpu().numpy(), q, oc, wl, None, "attn, general loop")


@pytest.mark.parametrize("Hq,Hkv,dtype,d", [(1, 1, "bf16", 128), (4, 2, "bf16", 128), (3, 1, "bf16", 128),
                                             (10, 2, "bf16", 128), (7, 1, "bf16", 128), (16, 2, "bf16", 128),
                                             (8, 1, "f32", 64), (6, 2, "bf16", 64), (5, 1, "f32", 128),
                                             (1, 1, "bf16", 64), (7, 1, "bf16", 64), (16, 2, "bf16", 64)])
def test_group_sizes_one_to_eight(dev, Hq, Hkv, dtype, d):
    # every group size g = Hq / Hkv from 1 to 8, on the MFMA kernel and on the plain-ALU kernel
    wl = W.Workload("groups", 89, 5, Hq, Hkv, d, dtype, np.array([0, 3, 31, 64, 100], np.int32),
                    np.full(5, 70, np.int32), np.array([16, 4, 0, 1, 7], np.int32))
    rt, oc = make(wl, dev)
    rollout(wl, rt, oc, 70, (1, 2, 7, 8, 16, 17, 33, 70), (16, 70), use_step_call=True)


@pytest.mark.parametrize("name,dtype,d", [("bstep", "bf16", 128), ("bstep32", "f32", 64), ("bstep64", "bf16", 64)])
def test_beacon_step_rollout(dev, name, dtype, d):
    # the beacon's own step: single launch on the bf16 paths, three launches otherwise
    c = np.array([1, 2, 4, 8, 16, 32, 0, 3], np.int32)
    wl = W.Workload(name, 85, 8, 12, 2, d, dtype,
                    np.array([0, 1, 31, 32, 33, 64, 7, 100], np.int32),
                    np.array([120, 120, 120, 77, 120, 120, 120, 50], np.int32), c)
    cap = wl.capacity()
    cap[4] = 33 + 16           # sequence 4: room for one full window but not for its beacon
    rt, oc = make(wl, dev, cap)
    steps = range(1, 121)
    rollout(wl, rt, oc, 120, steps, (1, 2, 3, 16, 17, 50, 120), beacon_call=True)
    assert oc.err & ERR_CAPACITY


def test_beacon_step_leaves_other_sequences_alone(dev):
    wl = W.Workload("bstep2", 86, 4, 12, 2, 128, "bf16", np.full(4, 40, np.int32),
                    np.full(4, 64, np.int32), np.array([4, 4, 0, 8], np.int32))
    rt, oc = make(wl, dev)
    for t in range(1, 5):                       # after 4 tokens: sequences 0, 1 are due (c = 4)
        k, v = wl.step_kv(t)
        rt.decode_step(k, v, wl.step_q(t))
        oc.append(k, v)
    bk, bv = wl.beacon_kv(4)
    qb = wl.beacon_q(4)
    rt.out.fill_(-7.0)
    o = rt.beacon_step(bk, bv, qb, active=np.array([1, 0, 1, 1], np.uint8)).cpu().numpy()
    mask = np.array([1, 0, 1, 1], np.uint8)
    oc.append(bk, bv, active=mask, beacon=True)
    check_attention(o, qb, oc, wl, [0])
    oc.compress_evict(active=mask)
    assert np.all(o[1] == -7.0) and np.all(o[2] == -7.0) and np.all(o[3] == -7.0)
    nb, w = check_tables(rt, oc)
    assert list(nb) == [1, 0, 0, 0] and list(w) == [0, 4, 4, 4]
    check_slabs(rt, oc)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64)])
def test_small_batch_rows_spread_over_workgroups(dev, dtype, d):
    # few (sequence, KV head) pairs and long sequences: the rows of a sequence are spread evenly
    # over several workgroups whose partials a second launch merges; a short sequence in the same
    # batch stays whole.  Fused steps (append + attention + eviction) against the oracle.
    B = 3
    Hq, Hkv = (12, 2) if d == 128 else (4, 1)
    wl = W.Workload("spread", 88, B, Hq, Hkv, d, dtype, np.array([1100, 2500, 300], np.int32),
                    np.full(B, 40, np.int32), np.array([0, 16, 4], np.int32))
    rt, oc = make(wl, dev)
    steps = range(1, 41)
    rollout(wl, rt, oc, 40, steps, (1, 16, 17, 40), use_step_call=True)
    q = wl.step_q(77)
    a = rt.decode_attn(q).cpu().numpy().copy()
    check_attention(a, q, oc, wl, None, 77)
    b = rt.decode_attn(q).cpu().numpy().copy()
    assert np.array_equal(a, b)                    # reproducible: fixed merge order, no atomics


def test_very_long_context_next_to_a_short_one(dev):
    # one sequence of 150,000 resident rows (64 chunks of 2,344 rows and the merge launch) beside
    # one of 40 rows that stays whole; a few fused steps, then attention, against the oracle
    wl = W.Workload("long", 89, 2, 12, 2, 128, "bf16", np.array([150000, 40], np.int32),
                    np.full(2, 6, np.int32), np.array([4, 2], np.int32))
    rt, oc = make(wl, dev)
    rollout(wl, rt, oc, 6, (1, 4, 5, 6), (6,), use_step_call=True)
    q = wl.step_q(9)
    a = rt.decode_attn(q).cpu().numpy().copy()
    check_attention(a, q, oc, wl, None, 9)


@pytest.mark.parametrize("B,Hq,Hkv,dtype,d", [(160, 12, 2, "bf16", 128), (300, 4, 1, "bf16", 128),
                                             (272, 2, 1, "f32", 64), (280, 8, 1, "bf16", 64)])
def test_longest_first_dispatch_large_ragged_batch(dev, B, Hq, Hkv, dtype, d):
    # more (sequence, KV head) pairs than compute units: bc_sort_by_length ranks the sequences by
    # resident length into the cache's dispatch order and workgroup i serves the i-th longest, in
    # bc_decode_attn and in the fused steps (B = 300: the ranking itself spans two workgroups).
    # The order is refreshed every fourth step only (a stale permutation is as good as a fresh
    # one).  Against the oracle with and without an inactive stripe, bit-equality with the plain
    # dispatch order (tuning variant 3), and a corrupt entry in the order.
    bc = _bc()
    rng = np.random.default_rng(23)
    P = rng.integers(1, 700, size=B).astype(np.int32)
    P[:4] = [1, 699, 350, 350]
    c = rng.choice([0, 2, 4, 16], size=B).astype(np.int32)
    wl = W.Workload("lpt", 87, B, Hq, Hkv, d, dtype, P, np.full(B, 40, np.int32), c)
    rt, oc = make(wl, dev)
    active = np.ones(B, np.uint8)
    active[5::7] = 0
    for t in range(1, 25):
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        act = active if t % 3 == 0 else None
        if t % 4 == 1:
            rt.sort_by_length(active=act)
        o = rt.decode_step(k, v, q, bk, bv, active=act).cpu().numpy()
        oc.append(k, v, active=act)
        seqs = [s for s in range(B) if act is None or act[s]]
        if t in (1, 2, 3, 16, 17, 24):
            check_attention(o, q, oc, wl, seqs, t)
        oc.compress_evict(bk, bv, active=act)
        check_tables(rt, oc, t)
    check_slabs(rt, oc, None, 24)
    q = wl.step_q(99)
    for act in (None, active):
        rt.out.fill_(-3.0)
        a = rt.decode_attn(q, active=act).cpu().numpy().copy()
        rt.cache.plan = bc.BC_PLAN_IGNORE_ORDER          # the same call in index order
        try:
            rt.out.fill_(-3.0)
            b = rt.decode_attn(q, active=act).cpu().numpy().copy()
        finally:
            rt.cache.plan = 0
        assert np.array_equal(a, b)
        seqs = [s for s in range(B) if act is None or act[s]]
        check_attention(a, q, oc, wl, seqs, 99)
        if act is not None:
            assert np.all(a[5::7] == -3.0)
    # the order really is the lengths sorted, longest first, inactive sequences last
    rt.sort_by_length(active=active)
    order = rt.order.cpu().numpy()
    assert sorted(order.tolist()) == list(range(B))
    L = np.array([wl.P[s] + oc.nb[s] + oc.w[s] for s in range(B)])
    key = np.where(active > 0, L + 1, 0)
    assert all(key[order[i]] >= key[order[i + 1]] for i in range(B - 1))
    # an entry that is no sequence index: state bit, its workgroups do nothing, the rest is served
    lost = int(order[3])
    rt.order[3] = B + 1000
    rt.out.fill_(-3.0)
    a = rt.decode_attn(q).cpu().numpy().copy()
    assert np.all(a[lost] == -3.0)
    check_attention(a, q, oc, wl, [s for s in range(B) if s != lost], 99)
    assert rt.tables()[2] & ERR_STATE


def test_fused_step_ragged_ratios_and_errors(dev):
    c = np.array([1, 2, 4, 8, 16, 32, 0, 3], np.int32)
    wl = W.Workload("fusedr", 80, 8, 12, 2, 128, "bf16",
                    np.array([0, 1, 31, 32, 33, 64, 7, 100], np.int32), np.full(8, 200, np.int32), c)
    cap = wl.capacity()
    cap[3] = 32 + 5            # sequence 3 runs out of slab: capacity bit, then untouched
    rt, oc = make(wl, dev, cap)
    steps = range(1, 201)
    rollout(wl, rt, oc, 200, steps, (1, 2, 3, 50, 200), use_step_call=True)
    assert oc.err == ERR_CAPACITY


@pytest.mark.parametrize("c", [16, 0])
def test_config2_batch64_full_rollout(dev, c):
    wl = W.batch64(c=c)
    rt, oc = make(wl, dev)
    rng = np.random.default_rng(5)
    sample = sorted(set([1, 2, 15, 16, 17, 31, 32, 33, 255, 256, 257, 1000, 2047, 2048, 4095, 4096])
                    | set(int(x) for x in rng.integers(1, 4097, size=48)))
    seqs = [0, 1, 31, 63] + [int(x) for x in rng.integers(0, 64, size=4)]
    worst = rollout(wl, rt, oc, 4096, sample, (16, 17, 1000, 4096), table_every=1, seq_sample=seqs,
                    use_step_call=(c > 0))
    nb, w, _ = rt.tables()
    if c > 0:
        assert int(nb[0]) == 256 and int(w[0]) == 0          # 256 + 256 + 0 = 512 rows resident
    else:
        assert int(nb[0]) == 0 and int(w[0]) == 4096
    check_slabs(rt, oc, None, 4096)
    # whole batch at the final state, fresh query
    q = wl.step_q(5000)
    o = rt.decode_attn(q).cpu().numpy()
    worst = max(worst, check_attention(o, q, oc, wl, None, 4096))
    print("batch64 c=%d worst %.3g" % (c, worst))


@pytest.mark.parametrize("mode", ["attention", "fused step in dispatch order"])
def test_config3_ragged_snapshot(dev, mode):
    wl = W.ragged256()
    T = wl.extra["T"]
    rt, oc = make(wl, dev)
    rollout(wl, rt, oc, T - 1, (), (), table_every=512)
    # snapshot at attention time of step T
    active = (wl.G >= T).astype(np.uint8)
    k, v = wl.step_kv(T)
    q = wl.step_q(T)
    if mode != "attention":
        # the way this state is timed: bc_decode_step (append + attention + eviction in one launch)
        # with the dispatch order of bc_sort_by_length attached; sequences that are over stay out
        bk, bv = wl.beacon_kv(T)
        rt.sort_by_length(active=active)
        st, text = _bc().bc_decode_plan_describe(rt.shape, rt.cache)
        assert st == 0 and "decode_lds_kernel" in text and "chunks=1" in text, text
        rt.out.fill_(-5.0)
        o = rt.decode_step(k, v, q, bk, bv, active=active).cpu().numpy()
        oc.append(k, v, active=active)
        live = [s for s in range(wl.B) if active[s]]
        worst = check_attention(o, q, oc, wl, live, T)
        assert all(np.all(o[s] == -5.0) for s in range(wl.B) if not active[s])
        oc.compress_evict(bk, bv, active=active)
        nb, w = check_tables(rt, oc, T)
        for s in live:
            assert (int(nb[s]), int(w[s])) == OR.tables_after_step(int(wl.c[s]), T)
        check_slabs(rt, oc, None, T)
        order = rt.order.cpu().numpy()
        assert sorted(order.tolist()) == list(range(wl.B))
        print("ragged fused T=%d worst %.3g" % (T, worst))
        return
    rt.append_kv(k, v, active=active)
    oc.append(k, v, active=active)
    nb, w = check_tables(rt, oc, T)
    for s in range(wl.B):       # closed form of the residency process
        t_s = min(T, int(wl.G[s]))
        if wl.G[s] >= T:
            assert (int(nb[s]), int(w[s])) == OR.tables_at_attention(int(wl.c[s]), t_s)
        else:
            assert (int(nb[s]), int(w[s])) == OR.tables_after_step(int(wl.c[s]), t_s)
    check_slabs(rt, oc, None, T)
    o = rt.decode_attn(q).cpu().numpy()          # all sequences, finished ones included
    worst = check_attention(o, q, oc, wl, None, T)
    print("ragged T=%d sumL=%d worst %.3g" % (T, sum(oc.L(s) for s in range(wl.B)), worst))


@pytest.mark.parametrize("mode", ["separate calls", "step with supplied beacon", "step and beacon step"])
def test_config4_long_peaked(dev, mode):
    # the whole 32768-token rollout, by the three separate calls, by the fused step that is handed
    # the beacon (the form the benchmark times) and by the fused step followed by the beacon
    # token's own step (bc_beacon_step)
    wl = W.long_reasoning()
    rt, oc = make(wl, dev)
    rng = np.random.default_rng(9)
    # steps whose window holds a x4 key: the 64th written row falls on a token (rows are counted
    # in write order: 512 prompt rows, then 32 tokens and one beacon per window)
    peaked = [t for t in range(1, 32769) if (512 + (t - 1) + (t - 1) // 32) % 64 == 63]
    assert len(peaked) > 400
    sample = sorted(set([1, 31, 32, 33, 63, 64, 65, 4096, 32767, 32768])
                    | set(int(x) for x in rng.integers(1, 32769, size=20))
                    | set(peaked[:2] + [peaked[len(peaked) // 2], peaked[-1], peaked[-1] + 1, peaked[-1] + 5]))
    sample = [t for t in sample if t <= 32768]
    seqs = [0, 7, 31]
    worst = rollout(wl, rt, oc, 32768, sample, (32, 33, 32768), table_every=1024, seq_sample=seqs,
                    use_step_call=(mode == "step with supplied beacon"),
                    beacon_call=(mode == "step and beacon step"))
    nb, w, _ = rt.tables()
    assert int(nb[0]) == 1024 and int(w[0]) == 0
    q = wl.step_q(40000)
    o = rt.decode_attn(q).cpu().numpy()
    worst = max(worst, check_attention(o, q, oc, wl, None, 32768))
    print("long worst %.3g" % worst)


# ---------------------------------------------------------------------------
def test_error_bits_and_inactive_rows_untouched(dev):
    import torch
    wl = W.Workload("edge", 90, 3, 4, 2, 64, "bf16", np.array([2, 0, 3], np.int32),
                    np.array([8, 8, 8], np.int32), np.array([2, 2, 0], np.int32))
    cap = np.array([2 + 1 + 2, 3, 5], np.int32)
    rt, oc = make(wl, dev, cap)
    # sequence 1 is empty: attention over it is a state error and leaves the output alone
    rt.out.fill_(123.0)
    q = wl.step_q(1)
    o = rt.decode_attn(q)
    nb, w, err = rt.tables()
    assert err == ERR_STATE
    assert torch.all(o[1] == 123.0)
    K, V = oc.resident(0)
    assert np.abs(o[0].cpu().numpy() - OA.decode_attention(q[0], K, V, wl.scale)).max() <= 2e-3
    rt.err.zero_()
    # inactive sequences: tables, slabs and outputs untouched
    k, v = wl.step_kv(1)
    rt.append_kv(k, v, active=[1, 0, 1]); oc.append(k, v, active=[1, 0, 1])
    rt.out.fill_(-7.0)
    o = rt.decode_attn(wl.step_q(2), active=[0, 0, 1])
    assert torch.all(o[0] == -7.0) and torch.all(o[1] == -7.0) and not torch.any(o[2] == -7.0)
    check_tables(rt, oc)
    # window full -> state bit; slab full -> capacity bit; sequence untouched both times
    k, v = wl.step_kv(2)
    rt.append_kv(k, v); oc.append(k, v)                 # seq0 w=2, seq1 w=1, seq2 w=2 (cap 5 reached)
    rt.append_kv(k, v, active=[1, 0, 0]); oc.append(k, v, active=[1, 0, 0])
    assert oc.err == ERR_STATE
    rt.append_kv(k, v, active=[0, 0, 1]); oc.append(k, v, active=[0, 0, 1])
    assert oc.err == ERR_STATE | ERR_CAPACITY
    check_tables(rt, oc)
    check_slabs(rt, oc)
    # partial-window compression is an opt-in extension
    bk, bv = wl.beacon_kv(2)
    rt.compress_evict(bk, bv); oc.compress_evict(bk, bv)             # seq0 only
    rt.compress_evict(bk, bv, require_full_window=False)
    oc.compress_evict(bk, bv, require_full=False)                    # seq1 (w=1)
    check_tables(rt, oc)
    check_slabs(rt, oc, [0, 2])


def test_host_side_argument_errors(dev):
    bc = _bc()
    wl = W.tiny()
    rt, _ = make(wl, dev)
    import ctypes as C
    sh = bc.bc_shape(2, 4, 3, 64, 0, 0.125)            # Hq % Hkv != 0
    assert bc.bc_decode_attn(sh, rt.cache, C.c_void_p(rt.out.data_ptr()), C.c_void_p(rt.out.data_ptr()),
                             None, C.c_void_p(rt.ws.data_ptr()), rt.ws_bytes, None) == -2
    assert bc.bc_decode_attn(rt.shape, rt.cache, None, C.c_void_p(rt.out.data_ptr()), None,
                             C.c_void_p(rt.ws.data_ptr()), rt.ws_bytes, None) == -1
    assert bc.bc_decode_attn(rt.shape, rt.cache, C.c_void_p(rt.out.data_ptr()),
                             C.c_void_p(rt.out.data_ptr()), None, C.c_void_p(rt.ws.data_ptr()), 8,
                             None) == -5
    assert bc.bc_compress_evict(rt.shape, rt.cache, None, None, None, 0, None) == -1
    assert "workspace" in bc.bc_status_str(-5)


def test_deterministic_and_split_invariant(dev):
    import torch
    bc = _bc()
    wl = W.batch64(c=0, G=1500, B=8)
    rt, oc = make(wl, dev)
    for t in range(1, 1201):
        k, v = wl.step_kv(t)
        rt.append_kv(k, v)
    q = wl.step_q(7)
    a = rt.decode_attn(q).clone()
    b = rt.decode_attn(q).clone()
    assert torch.equal(a, b)                               # fixed merge order
    rt.cache.rows_per_workgroup = 512                   # a forced chunk size, for this call only
    try:
        c = rt.decode_attn(q).clone()
    finally:
        rt.cache.rows_per_workgroup = 0
    assert float((a - c).abs().max()) < 1e-5               # independent of the split factor
    assert not torch.equal(a, torch.zeros_like(a))


# ---------------------------------------------------------------------------
# next rows: evaluation budget rule and mid-generation ratio change
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64)])
def test_budget_rule_interrupts_generation_on_device(dev, dtype, d):
    import torch
    B = 6
    c = np.array([1, 2, 4, 16, 0, 3], np.int32)
    wl = W.Workload("budget", 91, B, 12 if d == 128 else 4, 2 if d == 128 else 1, d, dtype,
                    np.array([3, 0, 17, 32, 5, 64], np.int32), np.full(B, 200, np.int32), c)
    rt, oc = make(wl, dev)
    budget = np.array([10, 12, 7, 20, 9, 15], np.int32)
    budget_rollout(wl, rt, oc, budget, 120, None, dev)


def budget_rollout(wl, rt, oc, budget, steps, attention_steps, dev, sort_every=0):
    """Steps under the evaluation cap: outputs, live flags, tables and the step at which every
    sequence ends against the oracle; attention_steps = None checks every step."""
    import torch
    B, c = wl.B, wl.c
    bud_d = torch.from_numpy(budget).to(dev)
    live_d = torch.ones(B, dtype=torch.uint8, device=dev)
    live = [1] * B
    last = [None] * B
    for t in range(1, steps + 1):
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        rt.out.fill_(77.0)
        if sort_every and t % sort_every == 1:
            rt.sort_by_length(active=live_d)
        o = rt.decode_step_budget(k, v, q, bk, bv, bud_d, live_d).cpu().numpy()
        was = list(live)
        oc.append(k, v, active=was)
        act = [s for s in range(B) if was[s]]
        if act and (attention_steps is None or t in attention_steps):
            check_attention(o, q, oc, wl, act, t)
        for s in range(B):
            if not was[s]:
                assert np.all(o[s] == 77.0), (s, t)          # finished sequences are skipped
        oc.apply_budget(budget, live)
        oc.compress_evict(bk, bv, active=was)
        assert live_d.cpu().tolist() == live, t
        check_tables(rt, oc, t)
        for s in range(B):
            if was[s] and not live[s]:
                last[s] = t
    check_slabs(rt, oc)
    for s in range(B):
        if last[s] is not None or OR.first_step_reaching(int(budget[s]), int(c[s])) <= steps:
            assert last[s] == OR.first_step_reaching(int(budget[s]), int(c[s])), (s, last[s])


def test_budget_rule_large_batch_longest_first(dev):
    # more pairs than compute units: the budget step follows a dispatch order that is refreshed
    # every fifth step from the live flags and lengths of that moment
    B = 300
    rng = np.random.default_rng(31)
    P = rng.integers(1, 400, size=B).astype(np.int32)
    c = rng.choice([0, 1, 3, 16], size=B).astype(np.int32)
    wl = W.Workload("budget_lpt", 93, B, 4, 1, 128, "bf16", P, np.full(B, 60, np.int32), c)
    rt, oc = make(wl, dev)
    budget = rng.integers(4, 30, size=B).astype(np.int32)
    budget_rollout(wl, rt, oc, budget, 36, (1, 2, 5, 17, 36), dev, sort_every=5)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64)])
def test_admission_into_finished_slots(dev, dtype, d):
    # continuous batching: the budget rule ends generations at different steps; every 10 steps
    # the finished slots take new sequences (new prompt length and ratio) and carry on
    import torch
    B = 6
    c = np.array([1, 2, 4, 16, 0, 3], np.int32)
    Hq, Hkv = (12, 2) if d == 128 else (4, 1)
    wl = W.Workload("admit", 93, B, Hq, Hkv, d, dtype, np.array([3, 0, 17, 32, 5, 64], np.int32),
                    np.full(B, 400, np.int32), c)
    cap = np.full(B, 120, np.int32)
    rt, oc = make(wl, dev, cap)
    budget = np.array([10, 12, 7, 20, 9, 15], np.int32)
    bud_d = torch.from_numpy(budget).to(dev)
    live_d = torch.ones(B, dtype=torch.uint8, device=dev)
    live = [1] * B
    rng = np.random.default_rng(17)
    admitted = 0
    for t in range(1, 161):
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        o = rt.decode_step_budget(k, v, q, bk, bv, bud_d, live_d).cpu().numpy()
        was = list(live)
        oc.append(k, v, active=was)
        act = [s for s in range(B) if was[s]]
        if act:
            check_attention(o, q, oc, wl, act, t)
        oc.apply_budget(budget, live)
        oc.compress_evict(bk, bv, active=was)
        if t % 10 == 0:
            adm = np.array([0 if x else 1 for x in live], np.uint8)
            if t == 40:
                adm[:] = 0
                adm[[s for s in range(B) if not live[s]][:1]] = 1     # one slot with too long a prompt
            newP = [int(rng.integers(1, 90)) for _ in range(B)]
            if t == 40:
                newP = [121] * B
            pk = [W.round_to_dtype(rng.standard_normal((newP[s], Hkv, d)), dtype) for s in range(B)]
            pv = [W.round_to_dtype(rng.standard_normal((newP[s], Hkv, d)), dtype) for s in range(B)]
            new_c = rng.choice([0, 1, 2, 3, 5, 8], size=B).astype(np.int32)
            rt.cache_admit(adm, pk, pv, new_c, live_d)
            oc.admit(adm, pk, pv, new_c, live)
            admitted += int(adm.sum())
        assert live_d.cpu().tolist() == live, t
        check_tables(rt, oc, t)
        assert rt.c.cpu().tolist() == oc.c and rt.P.cpu().tolist() == oc.P, t
        if t % 10 == 0 or t == 160:
            check_slabs(rt, oc, None, t)
    assert admitted >= 12 and oc.err == ERR_CAPACITY


def test_ratio_change_mid_generation(dev):
    B = 4
    wl = W.Workload("ratio", 92, B, 12, 2, 128, "bf16", np.array([8, 0, 40, 3], np.int32),
                    np.full(B, 120, np.int32), np.array([4, 16, 0, 2], np.int32))
    cap = np.full(B, 40 + 120 + 40, np.int32)
    rt, oc = make(wl, dev, cap)
    changes = {9: [2, 16, 0, 2], 17: [2, 4, 0, 2], 30: [8, 4, 0, 0], 31: [1, 1, 1, 1], 70: [0, 5, 0, 16],
               90: [3, 5, 200, 200]}
    for t in range(1, 121):
        if t in changes:
            rt.set_ratio(changes[t])
            oc.set_ratio(changes[t])
            assert rt.c.cpu().tolist() == oc.c, t
        k, v = wl.step_kv(t)
        q = wl.step_q(t)
        bk, bv = wl.beacon_kv(t)
        o = rt.decode_step(k, v, q, bk, bv).cpu().numpy()
        oc.append(k, v)
        check_attention(o, q, oc, wl, None, t)
        oc.compress_evict(bk, bv)
        check_tables(rt, oc, t)
        if t in (9, 17, 30, 31, 32, 70, 90, 120):
            check_slabs(rt, oc)
    assert oc.err == ERR_STATE          # the change at step 31 did not fit some windows


@pytest.mark.parametrize("case", range(12))
def test_randomised_small_rollouts(dev, case):
    # seeded random shapes, prompt lengths, ratios and generation lengths; the call form (separate
    # calls, tail form, fused step, fused step + beacon step) rotates with the case number
    rng = np.random.default_rng([20251013, 77, case])
    dtype, d = [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)][case % 4]
    Hq, Hkv = [(12, 2), (4, 4), (8, 1), (6, 2), (7, 1), (5, 5), (16, 2), (3, 1)][int(rng.integers(0, 8))]
    B = int(rng.integers(1, 10))
    P = rng.integers(0, 300, size=B).astype(np.int32)
    c = rng.choice([0, 1, 2, 3, 5, 8, 16], size=B).astype(np.int32)
    steps = 45
    G = rng.integers(1, steps + 1, size=B).astype(np.int32)
    G[int(rng.integers(0, B))] = steps
    for s in range(B):
        if P[s] == 0 and G[s] < 1:
            G[s] = 1
    wl = W.Workload("rand%d" % case, 200 + case, B, Hq, Hkv, d, dtype, P, G, c)
    rt, oc = make(wl, dev)
    form = case % 4
    attn = sorted(set(int(x) for x in rng.integers(1, steps + 1, size=8)) | {1, steps})
    rollout(wl, rt, oc, steps, attn, (steps // 2, steps), tail_form=(form == 1),
            use_step_call=(form == 2), beacon_call=(form == 3))


@pytest.mark.parametrize("case", range(24))
def test_randomised_rollouts_near_the_plan_boundaries(dev, case):
    # seeded random batches whose pair counts straddle the kernel choices (128 and 256 pairs) and
    # whose prompt lengths straddle the tile and capacity limits of the straight-line form (384 /
    # 768 rows) and of the twelve-wave and small-workgroup forms (1100 rows); call form, dispatch
    # order and uniform / ragged layout rotate with the seed
    rng = np.random.default_rng([424242, case])
    dtype, d = [("bf16", 128), ("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128), ("bf16", 128)][case % 6]
    Hq, Hkv = [(12, 2), (4, 4), (8, 1), (6, 2), (7, 1), (16, 2), (3, 1), (32, 8), (24, 8), (2, 2)][int(rng.integers(0, 10))]
    kind = case % 4
    if kind == 0:
        B = max(1, int(rng.integers(120, 136)) // Hkv)
    elif kind == 1:
        B = max(1, int(rng.integers(250, 264)) // Hkv)
    elif kind == 2:
        B = int(rng.integers(1, 40))
    else:
        B = max(1, int(rng.integers(300, 400)) // Hkv)
    B = min(B, 200)
    uniform = bool(rng.integers(0, 2))
    pbase = int(rng.choice([0, 31, 33, 256, 352, 383, 384, 500, 700, 760, 1060, 1090, 1500]))
    if dtype == "f32":
        pbase = min(pbase, 400)
    P = np.full(B, pbase, np.int32) if uniform else np.maximum(0, pbase + rng.integers(-40, 40, size=B)).astype(np.int32)
    c = (np.full(B, int(rng.choice([0, 1, 2, 3, 7, 16, 32])), np.int32) if uniform
         else rng.choice([0, 1, 2, 5, 16, 32], size=B).astype(np.int32))
    steps = int(rng.integers(20, 50))
    G = np.full(B, steps, np.int32) if uniform else rng.integers(1, steps + 1, size=B).astype(np.int32)
    G[int(rng.integers(0, B))] = steps
    form = int(rng.integers(0, 4))
    wl = W.Workload("bound%d" % case, 5000 + case, B, Hq, Hkv, d, dtype, P, G, c)
    rt, oc = make(wl, dev)
    sort = B * Hkv > 256 and bool(rng.integers(0, 2))
    attn = sorted(set(int(x) for x in rng.integers(1, steps + 1, size=5)) | {1, steps})
    sample = None if B <= 24 else sorted(set(int(x) for x in rng.integers(0, B, size=16)))
    rollout(wl, rt, oc, steps, attn, (steps // 2, steps), table_every=7, tail_form=(form == 1),
            use_step_call=(form == 2), beacon_call=(form == 3), seq_sample=sample,
            before_step=(lambda t: rt.sort_by_length()) if sort else None)


def test_fused_steps_under_graph_replay(dev):
    # The benchmark replays a captured cycle of fused steps.  One runtime runs five 4-step cycles
    # eagerly, a twin runs the first cycle eagerly, captures the cycle as a HIP graph and replays
    # it four times with eager calls and synchronisations in between; every step's output, the
    # tables and the slabs must be bit-equal, and the last outputs match the oracle.
    import torch
    bc = _bc()
    B, cyc, ncyc = 8, 4, 5
    wl = W.Workload("graph", 95, B, 12, 2, 128, "bf16", np.array([3, 40, 0, 17, 64, 5, 33, 1], np.int32),
                    np.full(B, cyc * ncyc, np.int32), np.array([4, 2, 0, 1, 3, 4, 2, 4], np.int32))
    rtE, oc = make(wl, dev)
    rtG, _ = make(wl, dev)
    pool = []
    for j in range(1, cyc + 1):
        k, v = wl.step_kv(j)
        bk, bv = wl.beacon_kv(j)
        host = dict(k=k, v=v, q=wl.step_q(j), bk=bk, bv=bv)
        pool.append((host, {n: bc.to_device(a, "bf16", dev) for n, a in host.items()}))
    outsE = [torch.empty_like(rtE.out) for _ in range(cyc)]
    outsG = [torch.empty_like(rtG.out) for _ in range(cyc)]

    def cycle(rt, outs):
        for j in range(cyc):
            x = pool[j][1]
            rt.decode_step(x["k"], x["v"], x["q"], x["bk"], x["bv"], out=outs[j])

    st = torch.cuda.Stream()
    ref_out = []
    for _ in range(ncyc):                                   # eager twin + oracle
        cycle(rtE, outsE)
        torch.cuda.synchronize()
        ref_out.append([o.cpu().numpy().copy() for o in outsE])
        for j in range(cyc):
            h = pool[j][0]
            oc.append(h["k"], h["v"])
            last_ref = (h["q"], [OA.decode_attention(h["q"][s], *oc.resident(s), wl.scale) for s in range(B)])
            oc.compress_evict(h["bk"], h["bv"])
    with torch.cuda.stream(st):
        cycle(rtG, outsG)                                   # first cycle eagerly
        st.synchronize()
        assert all(np.array_equal(a.cpu().numpy(), b) for a, b in zip(outsG, ref_out[0]))
        saved = (rtG.nb.clone(), rtG.w.clone())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            cycle(rtG, outsG)
        rtG.nb.copy_(saved[0]); rtG.w.copy_(saved[1])       # capture does not run; restore anyway
        for r in range(1, ncyc):
            g.replay()
            st.synchronize()
            got = [o.cpu().numpy().copy() for o in outsG]
            for j in range(cyc):
                assert np.array_equal(got[j], ref_out[r][j]), (r, j)
            # the program's own eager work between replays: an attention call and a table read
            rtG.decode_attn(pool[0][1]["q"], out=torch.empty_like(rtG.out))
            nb, w, err = rtG.tables()
            assert err == 0
    nbE, wE, _ = rtE.tables()
    nbG, wG, _ = rtG.tables()
    assert list(nbE) == list(nbG) == oc.nb and list(wE) == list(wG) == oc.w
    check_slabs(rtG, oc)
    q, ref = last_ref
    worst = max(float(np.abs(ref_out[-1][-1][s] - ref[s]).max()) for s in range(B))
    assert worst <= TOL[wl.dtype], worst
