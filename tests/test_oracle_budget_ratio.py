"""Pins for the evaluation budget rule (Sec. 4, Evaluation) and the mid-generation ratio change
(named as future work in Sec. 6) in the cache oracle.  CPU only."""
import numpy as np

from oracle import residency as R
from oracle.cache import BatchCache, ERR_CAPACITY, ERR_STATE


def _rows(rng, n, Hkv=1, d=2):
    return rng.standard_normal((n, Hkv, d)).astype(np.float32)


def test_budget_interrupts_at_the_closed_form_step():
    # the step whose attention first sees `budget` generation entries is the last one
    rng = np.random.default_rng(0)
    ratios = [0, 1, 2, 4, 16]
    budget = [12] * len(ratios)
    pk = [_rows(rng, 3) for _ in ratios]
    cache = BatchCache(pk, pk, ratios, [3 + 200] * len(ratios))
    live = [1] * len(ratios)
    last_step = [None] * len(ratios)
    for t in range(1, 200):
        k = _rows(rng, len(ratios))
        cache.append(k, k, active=live)
        was = list(live)
        cache.apply_budget(budget, live)
        cache.compress_evict(k, k, active=was)
        for s in range(len(ratios)):
            if was[s] and not live[s]:
                last_step[s] = t
    for s, c in enumerate(ratios):
        assert last_step[s] == R.first_step_reaching(12, c), (c, last_step[s])
        # roughly c times more tokens under the same cap (Sec. 5; Table 3 caption)
        if c > 0:
            assert last_step[s] <= 12 * c and last_step[s] >= 12 * c - c * c
    assert cache.err == 0


def test_ratio_change_at_window_boundaries_matches_literal_lists():
    # literal form: one flat list; when the ratio in force says the window is full, append the
    # beacon and drop the entries of that window (the eviction line of Alg. 1 with the current c)
    rng = np.random.default_rng(1)
    P, G = 2, 60
    sched = {1: 4, 13: 2, 21: 5, 41: 1, 47: 0, 55: 3}      # step -> ratio taking effect before it
    pk = [_rows(rng, P)]
    cache = BatchCache(pk, pk, [4], [P + G + 8])
    flat = [("q", j) for j in range(P)]
    ids = [("q", j) for j in range(P)]
    c = 4
    w = 0
    nb = 0
    for t in range(1, G + 1):
        if t in sched and w == 0 or (t in sched and (sched[t] <= 0 or w < sched[t])):
            c = sched[t]
            cache.set_ratio([c])
        assert cache.err == 0
        k = _rows(rng, 1)
        cache.append(k, k)
        flat.append(("x", t))
        w += 1
        if c > 0 and w == c:
            nb += 1
            flat.append(("b", nb))
            flat = flat[: -c - 1] + flat[-1:]
            w = 0
        cache.compress_evict(k, k)
        assert (cache.nb[0], cache.w[0]) == (nb, w), t
        assert cache.L(0) == len(flat)
    assert nb > 5


def test_ratio_change_refused_when_window_does_not_fit():
    rng = np.random.default_rng(2)
    pk = [_rows(rng, 1), _rows(rng, 1)]
    cache = BatchCache(pk, pk, [8, 8], [40, 40])
    for _ in range(5):
        k = _rows(rng, 2)
        cache.append(k, k)
    cache.set_ratio([4, 6])            # w = 5: 4 does not fit, 6 does
    assert cache.err == ERR_STATE and cache.c == [8, 6]
    cache.err = 0
    cache.set_ratio([0, 0], active=[1, 0])      # switching compression off is always allowed
    assert cache.err == 0 and cache.c == [0, 6]


def test_admitted_slot_behaves_like_a_fresh_cache():
    # a slot taken over by a new sequence must evolve exactly like a cache created for that
    # sequence (Alg. 1 from its initialisation), whatever the slot held before
    rng = np.random.default_rng(9)
    Hkv, d = 2, 4
    mk = lambda n: rng.standard_normal((n, Hkv, d))
    pk, pv = [mk(5), mk(3)], [mk(5), mk(3)]
    old = BatchCache(pk, pv, [2, 3], [40, 40])
    for t in range(1, 8):
        old.append(mk(2), mk(2))
        old.compress_evict(mk(2), mk(2))
    nk, nv = mk(7), mk(7)
    live = [0, 1]
    old.admit([1, 0], [nk, None], [nv, None], new_c=[4, 0], live=live)
    assert live == [1, 1] and old.P[0] == 7 and old.c == [4, 3] and old.nb[0] == 0 and old.w[0] == 0
    fresh = BatchCache([nk], [nv], [4], [40])
    for t in range(1, 14):
        k, v, bk, bv = mk(2), mk(2), mk(2), mk(2)
        old.append(k, v); fresh.append(k[:1], v[:1])
        old.compress_evict(bk, bv); fresh.compress_evict(bk[:1], bv[:1])
        Ko, Vo = old.resident(0); Kf, Vf = fresh.resident(0)
        assert np.array_equal(Ko, Kf) and np.array_equal(Vo, Vf)
        assert old.L(0) == R.len_after_step(7, 4, t)
    assert old.err == 0
    # too long a prompt: capacity error, slot untouched
    before = old.resident(1)[0].copy()
    old.admit([0, 1], [None, mk(41)], [None, mk(41)])
    assert old.err == ERR_CAPACITY and np.array_equal(old.resident(1)[0], before)
