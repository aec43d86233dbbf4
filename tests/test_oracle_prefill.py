"""Pins for the training-time mask and the dense masked attention (Fig. 2,
Sec. 3.2): predicate == residency of the eviction loop, closed-form counts,
causal special case via a library routine, prefill row == decode over the
evicted cache.  CPU only."""
import itertools
import math

import numpy as np
import torch

from oracle import attention as A
from oracle import residency as R
from oracle.cache import BatchCache


def _row_of(entry, P, c):
    kind, n = entry
    if kind == "q":
        return n
    if kind == "x":                       # token x_i is the i-th response token
        return P + (n // c) * (c + 1) + n % c if c > 0 else P + n
    return P + (n - 1) * (c + 1) + c      # beacon m closes window m-1


def test_predicate_equals_residency_of_alg1():
    # Sec. 3.2: masking simulates the eviction.  The row of token x_{t-1} must see exactly
    # the entries resident when decode step t runs; the row of beacon m exactly the cache
    # at the time the beacon is encoded (prompt, earlier beacons, its full window, itself).
    for P, c, G in itertools.product((0, 1, 4), (1, 2, 3, 5), (1, 6, 23)):
        S = P + G + G // c
        for t, at, after in R.alg1_literal(P, c, G):
            r = _row_of(("x", t - 1), P, c)
            vis = {j for j in range(S) if A.visible(r, j, P, c)}
            assert vis == {_row_of(e, P, c) for e in at}, (P, c, G, t)
            assert len(vis) == A.count_visible(r, P, c)
            assert not A.is_beacon_row(r, P, c)
            if t % c == 0:
                rb = _row_of(("b", t // c), P, c)
                assert A.is_beacon_row(rb, P, c)
                vis_b = {j for j in range(S) if A.visible(rb, j, P, c)}
                assert vis_b == {_row_of(e, P, c) for e in at} | {rb}
                assert len(vis_b) == A.count_visible(rb, P, c)


def test_vectorised_row_equals_predicate_and_mask():
    for P, c, S in ((0, 2, 14), (3, 4, 31), (5, 1, 12), (4, 0, 9), (2, 16, 40)):
        m = A.visible_mask(S, P, c)
        for r in range(S):
            assert list(A.visible_row(r, P, c)) == list(np.nonzero(m[r])[0])
            assert m[r].sum() == A.count_visible(r, P, c)
        # prompt block is plain causal
        assert np.array_equal(m[:P, :P], np.tril(np.ones((P, P), dtype=bool)))


def test_fig2_structure_small_example():
    # P = 2, c = 2: rows  q0 q1 | x0 x1 b1 | x2 x3 b2 | x4
    m = A.visible_mask(9, 2, 2).astype(int)
    expect = np.array([
        [1, 0, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 1, 0, 0, 0, 0, 0, 0],   # x0: question + itself
        [1, 1, 1, 1, 0, 0, 0, 0, 0],   # x1: question + window so far
        [1, 1, 1, 1, 1, 0, 0, 0, 0],   # b1: question + its window + itself
        [1, 1, 0, 0, 1, 1, 0, 0, 0],   # x2: question + b1 + itself (x0, x1 hidden)
        [1, 1, 0, 0, 1, 1, 1, 0, 0],
        [1, 1, 0, 0, 1, 1, 1, 1, 0],   # b2
        [1, 1, 0, 0, 1, 0, 0, 1, 1],   # x4: question + b1 + b2 + itself
    ])
    assert np.array_equal(m, expect)


def test_no_compression_is_causal_attention_library():
    rng = np.random.default_rng(0)
    S, Hq, Hkv, d = 19, 4, 2, 8
    q, k, v = (rng.standard_normal((S, h, d)) for h in (Hq, Hkv, Hkv))
    for P, c in ((5, 0), (5, 64), (0, 19)):       # c >= response length: no row is hidden
        o, lse = A.masked_prefill_attention(q, k, v, P, c, 1 / math.sqrt(d))
        tq = torch.from_numpy(q).permute(1, 0, 2)
        tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
        tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
        assert np.abs(o - ref.permute(1, 0, 2).numpy()).max() < 1e-12
        s = torch.einsum("hsd,htd->hst", tq, tk) / math.sqrt(d)
        s = s.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), -math.inf)
        assert np.abs(lse - torch.logsumexp(s, dim=-1).T.numpy()).max() < 1e-12
    assert np.array_equal(A.masked_prefill_attention(q, k, v, 5, 3, 0.3, rows=[0])[0][0],
                          np.repeat(v[0], Hq // Hkv, axis=0))      # row 0: o = V_0


def test_prefill_row_equals_decode_over_evicted_cache():
    rng = np.random.default_rng(1)
    Hq, Hkv, d, P, c, G = 6, 2, 8, 3, 4, 22
    S = P + G + G // c
    q, k, v = (rng.standard_normal((S, h, d)) for h in (Hq, Hkv, Hkv))
    scale = 0.4
    o, _ = A.masked_prefill_attention(q, k, v, P, c, scale)
    cache = BatchCache([k[:P]], [v[:P]], [c], [P + G // c + c + 1])
    for t in range(1, G + 1):
        r = _row_of(("x", t - 1), P, c)
        cache.append(k[None, r], v[None, r])
        K, V = cache.resident(0)
        assert np.abs(A.decode_attention(q[r], K, V, scale) - o[r]).max() < 1e-13
        if t % c == 0:                                 # faithful form: the beacon's own query
            rb = _row_of(("b", t // c), P, c)
            cache.append(k[None, rb], v[None, rb], beacon=True)
            K, V = cache.resident(0)
            assert np.abs(A.decode_attention(q[rb], K, V, scale) - o[rb]).max() < 1e-13
            cache.compress_evict()
    assert cache.err == 0


def test_mutants_of_the_predicate_are_caught():
    # planted mistakes (here, on the CPU): each must disagree with the residency pin
    P, c, G = 2, 3, 9
    S = P + G + G // c
    good = A.visible_mask(S, P, c)

    def mask(fn):
        return np.array([[fn(r, j) for j in range(S)] for r in range(S)])

    hide_beacons = mask(lambda r, j: j <= r and (j < P or (j - P) // (c + 1) == (r - P) // (c + 1)))
    off_by_one = mask(lambda r, j: j <= r and (j < P or (j - P) % (c + 1) == c - 1
                                               or (j - P) // (c + 1) == (r - P) // (c + 1)))
    strict_diag = mask(lambda r, j: j < r and A.visible(r, j, P, c))
    for bad in (hide_beacons, off_by_one, strict_diag):
        assert not np.array_equal(bad, good)


def test_backward_matches_autograd_and_finite_differences():
    # the gradient formulas against torch autograd (fp64) on a dense masked attention written
    # with library ops, and against central finite differences of the forward oracle
    rng = np.random.default_rng(5)
    S, Hq, Hkv, d, P, c = 23, 4, 2, 6, 4, 3
    q, do = rng.standard_normal((S, Hq, d)), rng.standard_normal((S, Hq, d))
    k, v = rng.standard_normal((S, Hkv, d)), rng.standard_normal((S, Hkv, d))
    scale = 0.45
    dq, dk, dv = A.masked_prefill_attention_bwd(q, k, v, do, P, c, scale)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    mask = torch.from_numpy(A.visible_mask(S, P, c))
    kk = tk.repeat_interleave(Hq // Hkv, dim=1)
    vv = tv.repeat_interleave(Hq // Hkv, dim=1)
    s = torch.einsum("rhd,jhd->hrj", tq, kk) * scale
    a = torch.softmax(s.masked_fill(~mask, -math.inf), dim=-1)
    o = torch.einsum("hrj,jhd->rhd", a, vv)
    (o * torch.from_numpy(do)).sum().backward()
    assert np.abs(dq - tq.grad.numpy()).max() < 1e-12
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-12

    def loss(q_, k_, v_):
        return float((A.masked_prefill_attention(q_, k_, v_, P, c, scale)[0] * do).sum())
    eps = 1e-6
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in arr.shape)
            x0 = arr[idx]
            arr[idx] = x0 + eps; lp = loss(q, k, v)
            arr[idx] = x0 - eps; lm = loss(q, k, v)
            arr[idx] = x0
            assert abs((lp - lm) / (2 * eps) - grad[idx]) < 1e-6
    # hidden keys get no gradient from rows that cannot see them: a regular token of window 0
    # is seen only inside its window, so rows of later windows do not contribute
    do2 = np.zeros_like(do)
    do2[P + (c + 1) * 2:] = do[P + (c + 1) * 2:]          # upstream gradient on later windows only
    _, dk2, dv2 = A.masked_prefill_attention_bwd(q, k, v, do2, P, c, scale)
    assert np.all(dk2[P:P + c] == 0) and np.all(dv2[P:P + c] == 0)        # window-0 tokens
    assert np.abs(dv2[P + c]).max() > 0                                   # its beacon is visible


def test_gradients_at_chosen_places_equal_the_dense_form_and_autograd():
    # the per-place sums (used where S x S does not fit) against the dense oracle, every row and
    # key, ragged tail and no compression included; and against torch autograd directly
    rng = np.random.default_rng(11)
    for S, Hq, Hkv, d, P, c in ((29, 4, 2, 5, 3, 4), (17, 2, 1, 4, 0, 2), (12, 3, 3, 4, 5, 0), (20, 2, 2, 3, 2, 40)):
        q, do = rng.standard_normal((S, Hq, d)), rng.standard_normal((S, Hq, d))
        k, v = rng.standard_normal((S, Hkv, d)), rng.standard_normal((S, Hkv, d))
        dq, dk, dv = A.masked_prefill_attention_bwd(q, k, v, do, P, c, 0.37)
        everything = list(range(S))
        sq, sk, sv = A.masked_prefill_attention_bwd_at(q, k, v, do, P, c, 0.37, everything, everything)
        assert np.abs(sq - dq).max() < 1e-12 and np.abs(sk - dk).max() < 1e-12 and np.abs(sv - dv).max() < 1e-12
        # the column rule is the transpose of the row rule
        m = A.visible_mask(S, P, c)
        for j in range(S):
            assert np.array_equal(A.rows_seeing(j, S, P, c), np.nonzero(m[:, j])[0])
    S, Hq, Hkv, d, P, c = 26, 2, 1, 4, 3, 5
    q, do = rng.standard_normal((S, Hq, d)), rng.standard_normal((S, Hq, d))
    k, v = rng.standard_normal((S, Hkv, d)), rng.standard_normal((S, Hkv, d))
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    mask = torch.from_numpy(A.visible_mask(S, P, c))
    s = torch.einsum("rhd,jd->hrj", tq, tk[:, 0]) * 0.5
    a = torch.softmax(s.masked_fill(~mask, -math.inf), dim=-1)
    (torch.einsum("hrj,jd->rhd", a, tv[:, 0]) * torch.from_numpy(do)).sum().backward()
    rows, keys = [0, 4, 8, 9, 25], [1, 3, 8, 14, 20, 25]
    sq, sk, sv = A.masked_prefill_attention_bwd_at(q, k, v, do, P, c, 0.5, rows, keys)
    assert np.abs(sq - tq.grad.numpy()[rows]).max() < 1e-12
    assert np.abs(sk - tk.grad.numpy()[keys]).max() < 1e-12
    assert np.abs(sv - tv.grad.numpy()[keys]).max() < 1e-12
