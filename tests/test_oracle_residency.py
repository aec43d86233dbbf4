"""Pins for the residency oracle (Alg. 1, Sec. 3.1, Fig. 1): CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import residency as R
from oracle.cache import BatchCache, FlatCache, ERR_STATE, ERR_CAPACITY


def _read_golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "paper_cache_statements.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = [int(x) for x in v.split()]
    return out


def test_literal_equals_structured_brute_force():
    # every (P, c, G) with P <= 8, c <= 5, G <= 40; c = 0 is the uncompressed model
    for P, c, G in itertools.product(range(0, 9), range(0, 6), (1, 2, 7, 40)):
        a = list(R.alg1_literal(P, c, G))
        b = list(R.structured(P, c, G))
        assert a == b, (P, c, G)


def test_closed_forms_match_simulation():
    for P, c in itertools.product((0, 3, 32), (0, 1, 2, 5, 16)):
        for t, at, after in R.alg1_literal(P, c, 100):
            assert len(at) == R.len_at_attention(P, c, t)
            assert len(after) == R.len_after_step(P, c, t)
            # the invariant the benchmark spec names: P + floor(t/c) + (t mod c)
            if c > 0:
                assert len(after) == P + t // c + t % c
            nb = sum(1 for e in after if e[0] == "b")
            w = sum(1 for e in after if e[0] == "x")
            assert (nb, w) == R.tables_after_step(c, t)
            nb = sum(1 for e in at if e[0] == "b")
            w = sum(1 for e in at if e[0] == "x")
            assert (nb, w) == R.tables_at_attention(c, t)


def test_resident_ids_are_prompt_beacons_then_current_window():
    P, c = 5, 4
    for t, at, after in R.alg1_literal(P, c, 50):
        assert after[:P] == [("q", j) for j in range(P)]
        nb = t // c
        assert after[P:P + nb] == [("b", m) for m in range(1, nb + 1)]
        # window = the tokens encoded since the last beacon: x_{t - t mod c} .. x_{t-1}
        assert after[P + nb:] == [("x", i) for i in range(t - t % c, t)]
        # attention of a step always sees the token it has just encoded, last
        assert at[-1] == ("x", t - 1)


def test_no_eviction_when_c_exceeds_generation():
    for P, G in ((4, 10), (0, 31)):
        full = list(R.alg1_literal(P, 0, G))
        big = list(R.alg1_literal(P, G + 1, G))
        assert full == big
        assert len(full[-1][2]) == P + G


def test_first_window_and_guard():
    # i > 0 guard: nothing happens before c tokens are encoded; first beacon after step c
    c = 4
    steps = list(R.alg1_literal(2, c, 9))
    for t, at, after in steps:
        if t < c:
            assert not any(e[0] == "b" for e in after)
    assert steps[c - 1][2][-1] == ("b", 1)
    assert len(steps[c - 1][1]) == 2 + c          # the beacon's window held exactly c tokens
    assert len(steps[c - 1][2]) == 2 + 1


def test_paper_cache_statements(golden_dir):
    g = _read_golden(golden_dir)
    c = g["fig1_ratio"][0]
    # Fig. 1: one finished window of c tokens leaves exactly one entry
    _, _, after = list(R.alg1_literal(0, c, c))[-1]
    assert len(after) == g["fig1_entries_per_finished_window"][0]
    # growth by one entry per c generated tokens (at window boundaries)
    for c in g["ratios"]:
        for k in range(1, 6):
            assert R.len_after_step(0, c, (k + 1) * c) - R.len_after_step(0, c, k * c) \
                == g["growth_per_c_tokens"][0]
    # 1,000-entry budget: roughly c times more tokens; 32,000 vs 1,000 for c = 32
    budget = g["eval_budget_entries"][0]
    assert R.first_step_reaching(budget, 0) == budget
    for c in g["ratios"]:
        t = R.first_step_reaching(budget, c)
        assert 0.96 * budget * c <= t <= budget * c, (c, t)
    big, plain = g["ratio32_tokens_vs_uncompressed"]
    assert abs(R.first_step_reaching(budget, 32) - big) / big < 0.05
    assert R.first_step_reaching(budget, 0) == plain


# ---------------------------------------------------------------------------
# K/V-carrying simulators
# ---------------------------------------------------------------------------
def _rows(rng, n, Hkv=2, d=4):
    return rng.standard_normal((n, Hkv, d)).astype(np.float32)


@pytest.mark.parametrize("tail_form", [False, True])
def test_batchcache_equals_flat_literal(tail_form):
    rng = np.random.default_rng(7)
    B, G = 4, 37
    P = [3, 0, 5, 2]
    c = [2, 3, 0, 5]
    cap = [p + (G // cc if cc > 0 else G) + max(cc, 0) + 1 for p, cc in zip(P, c)]
    pk = [_rows(rng, p) for p in P]
    pv = [_rows(rng, p) for p in P]
    bc = BatchCache(pk, pv, c, cap)
    flats = [FlatCache(pk[s], pv[s], c[s]) for s in range(B)]
    for t in range(1, G + 1):
        k, v = _rows(rng, B), _rows(rng, B)
        bc.append(k, v)
        for s in range(B):
            flats[s].append(k[s], v[s])
        for s in range(B):   # what attention sees
            Kb, Vb = bc.resident(s)
            Kf, Vf = flats[s].resident()
            assert np.array_equal(Kb, Kf) and np.array_equal(Vb, Vf)
            assert Kb.shape[0] == R.len_at_attention(P[s], c[s], t)
        bk, bv = _rows(rng, B), _rows(rng, B)
        if tail_form:
            bc.append(bk, bv, beacon=True)
            for s in range(B):
                if c[s] > 0 and t % c[s] == 0:
                    assert bc.w[s] == c[s] + 1
            bc.compress_evict()
        else:
            bc.compress_evict(bk, bv)
        for s in range(B):
            if c[s] > 0 and t % c[s] == 0:
                flats[s].beacon_and_evict(bk[s], bv[s])
            Kb, Vb = bc.resident(s)
            Kf, Vf = flats[s].resident()
            assert np.array_equal(Kb, Kf) and np.array_equal(Vb, Vf)
            assert (bc.nb[s], bc.w[s]) == R.tables_after_step(c[s], t)
    assert bc.err == 0


def test_payload_identity():
    # rows filled with their own entry id: the slab *is* the id list of Alg. 1
    P, c, G = 3, 4, 30
    ids = {}

    def row(e):
        ids.setdefault(e, len(ids))
        return np.full((1, 1), ids[e], dtype=np.float32)

    pk = [np.stack([row(("q", j)) for j in range(P)])]
    cache = BatchCache(pk, pk, [c], [P + G // c + c + 1])
    for t, at, after in R.alg1_literal(P, c, G):
        r = row(("x", t - 1))[None]
        cache.append(r, r)
        assert [int(x) for x in cache.resident(0)[0][:, 0, 0]] == [ids[e] for e in at]
        if t % c == 0:
            b = row(("b", t // c))[None]
            cache.compress_evict(b, b)
        assert [int(x) for x in cache.resident(0)[0][:, 0, 0]] == [ids[e] for e in after]


def test_batchcache_error_rules_and_active_mask():
    rng = np.random.default_rng(3)
    pk = [_rows(rng, 2), _rows(rng, 2)]
    cache = BatchCache(pk, pk, [2, 2], [6, 3])
    k = _rows(rng, 2)
    cache.append(k, k, active=[1, 0])
    assert cache.w == [1, 0] and cache.err == 0
    cache.append(k, k)                       # seq 0 -> w 2 ; seq 1 -> w 1 (L = cap)
    assert cache.w == [2, 1]
    cache.append(k, k, active=[0, 1])        # seq 1 full slab
    assert cache.err == ERR_CAPACITY and cache.w == [2, 1]
    cache.err = 0
    cache.append(k, k, active=[1, 0])        # window full: state error, untouched
    assert cache.err == ERR_STATE and cache.w == [2, 1]
    cache.err = 0
    cache.compress_evict(k, k)               # only seq 0 has a full window
    assert cache.nb == [1, 0] and cache.w == [0, 1] and cache.err == 0
    cache.compress_evict(k, k, require_full=False)   # partial window of seq 1; seq 0 empty: skipped
    assert cache.nb == [1, 1] and cache.w == [0, 0]
    # tail form refuses to mix with the supplied form
    cache.append(k, k, active=[1, 0])
    cache.append(k, k, active=[1, 0])
    cache.append(k, k, active=[1, 0], beacon=True)
    assert cache.w[0] == 3
    cache.compress_evict(k, k)
    assert cache.err == ERR_STATE
    cache.compress_evict()
    assert cache.w[0] == 0 and cache.nb[0] == 2
