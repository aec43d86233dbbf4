"""Pins for the attention oracle: closed forms, invariants, a library routine as
the no-eviction special case, brute force in pure Python.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import residency as R
from oracle.cache import BatchCache


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _brute_force(q, K, V, scale):
    """Pure-Python loops, math.exp and math.fsum: no NumPy arithmetic."""
    Hq, d = len(q), len(q[0])
    L, Hkv = len(K), len(K[0])
    g = Hq // Hkv
    out = []
    for h in range(Hq):
        kvh = h // g
        logits = [scale * math.fsum(q[h][x] * K[j][kvh][x] for x in range(d)) for j in range(L)]
        mx = max(logits)
        wts = [math.exp(l - mx) for l in logits]
        den = math.fsum(wts)
        out.append([math.fsum(wts[j] * V[j][kvh][x] for j in range(L)) / den for x in range(d)])
    return out


def test_brute_force_tiny():
    rng = np.random.default_rng(0)
    for (Hq, Hkv, d, L) in ((4, 1, 3, 5), (6, 2, 4, 7), (2, 2, 1, 1), (3, 1, 2, 9)):
        q, K, V = _rand(rng, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
        o = A.decode_attention(q, K, V, 0.37)
        ref = np.array(_brute_force(q.tolist(), K.tolist(), V.tolist(), 0.37))
        assert np.abs(o - ref).max() < 1e-13


def test_full_attention_special_case_matches_library():
    # c larger than the generated length: nothing is ever evicted, so decode attention
    # over the cache is plain softmax(QK^T/sqrt(d))V over all tokens - checked against
    # torch's scaled_dot_product_attention in fp64 (a library routine, not our formula).
    rng = np.random.default_rng(1)
    B, Hq, Hkv, d, P, G = 2, 6, 2, 16, 5, 12
    pk = [_rand(rng, P, Hkv, d) for _ in range(B)]
    pv = [_rand(rng, P, Hkv, d) for _ in range(B)]
    cache = BatchCache(pk, pv, [G + 1] * B, [P + G + 4] * B)
    for t in range(1, G + 1):
        k, v = _rand(rng, B, Hkv, d), _rand(rng, B, Hkv, d)
        cache.append(k, v)
        cache.compress_evict(k, v)          # never fires
    q = _rand(rng, B, Hq, d)
    for s in range(B):
        K, V = cache.resident(s)
        assert K.shape[0] == P + G
        o = A.decode_attention(q[s], K, V, 1 / math.sqrt(d))
        tq = torch.from_numpy(q[s])[:, None, :]                       # [Hq, 1, d]
        tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
        tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
        assert np.abs(o - ref).max() < 1e-12


def test_single_key_returns_v_exactly():
    rng = np.random.default_rng(2)
    q, K, V = _rand(rng, 4, 8), _rand(rng, 1, 2, 8), _rand(rng, 1, 2, 8)
    o = A.decode_attention(q, K, V, 0.5)
    assert np.array_equal(o[:2], np.broadcast_to(V[0, 0], (2, 8)))
    assert np.array_equal(o[2:], np.broadcast_to(V[0, 1], (2, 8)))


def test_permutation_invariance():
    rng = np.random.default_rng(3)
    q, K, V = _rand(rng, 6, 8), _rand(rng, 33, 2, 8), _rand(rng, 33, 2, 8)
    perm = rng.permutation(33)
    o1 = A.decode_attention(q, K, V, 0.3)
    o2 = A.decode_attention(q, K[perm], V[perm], 0.3)
    assert np.abs(o1 - o2).max() < 1e-13
    # ... and a transposed operand or a K/V mix-up would break it against the definition:
    assert np.abs(o1 - A.decode_attention(q, V, K, 0.3)).max() > 1e-3


def test_equal_keys_and_zero_scale_give_mean_of_v():
    rng = np.random.default_rng(4)
    q, V = _rand(rng, 4, 8), _rand(rng, 10, 1, 8)
    K = np.broadcast_to(_rand(rng, 1, 1, 8), (10, 1, 8))
    assert np.abs(A.decode_attention(q, K, V, 0.7) - V.mean(axis=0)).max() < 1e-13
    K = _rand(rng, 10, 1, 8)
    assert np.abs(A.decode_attention(q, K, V, 0.0) - V.mean(axis=0)).max() < 1e-13


def test_two_key_closed_form_pins_scale_and_sign():
    # two keys: o = sigma(scale*(q.k0 - q.k1)) v0 + (1 - sigma) v1
    q = np.array([[1.0, 2.0]])
    K = np.array([[[0.5, -1.0]], [[-0.25, 0.75]]])
    V = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    scale = 0.8
    z = scale * ((1 * 0.5 + 2 * -1.0) - (1 * -0.25 + 2 * 0.75))
    sig = 1 / (1 + math.exp(-z))
    o = A.decode_attention(q, K, V, scale)
    assert np.abs(o[0] - np.array([sig, 1 - sig])).max() < 1e-15


def test_dominated_logit_bound():
    rng = np.random.default_rng(5)
    d, L = 8, 20
    q = _rand(rng, 1, d)
    K = 0.1 * _rand(rng, L, 1, d)
    V = _rand(rng, L, 1, d)
    K[7, 0] = 30.0 * q[0] / np.dot(q[0], q[0])     # q.K_7 = 30
    s = (K[:, 0] @ q[0])
    delta = s[7] - np.delete(s, 7)
    o = A.decode_attention(q, K, V, 1.0)
    bound = 2 * np.abs(V).max() * np.exp(-delta).sum()
    assert np.abs(o[0] - V[7, 0]).max() <= bound
    assert bound < 1e-9


def test_gqa_equals_mha_with_repeated_kv_and_group_symmetry():
    rng = np.random.default_rng(6)
    Hq, Hkv, d, L = 12, 2, 8, 17
    q, K, V = _rand(rng, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    o = A.decode_attention(q, K, V, 0.35)
    g = Hq // Hkv
    Kr, Vr = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)     # consecutive heads share a KV head
    assert np.abs(o - A.decode_attention(q, Kr, Vr, 0.35)).max() < 1e-14
    # heads of one group with the same q give the same output; other groups differ
    q2 = q.copy()
    q2[0:g] = q[0]
    q2[g:2 * g] = q[0]
    o2 = A.decode_attention(q2, K, V, 0.35)
    assert np.array_equal(o2[0], o2[g - 1])
    assert np.abs(o2[0] - o2[g]).max() > 1e-3


def test_softmax_attention_agrees_with_scipy_softmax():
    from scipy.special import softmax
    rng = np.random.default_rng(8)
    q, K, V = _rand(rng, 16), _rand(rng, 40, 16), _rand(rng, 40, 16)
    ref = softmax(0.25 * K @ q) @ V
    assert np.abs(A.softmax_attention(q, K, V, 0.25) - ref).max() < 1e-13


def test_large_logits_do_not_overflow():
    q = np.array([[100.0, 0.0]])
    K = np.array([[[10.0, 0.0]], [[9.0, 0.0]]])
    V = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    o = A.decode_attention(q, K, V, 1.0)                 # logits 1000 and 900
    assert np.all(np.isfinite(o)) and abs(o[0, 0] - 1.0) < 1e-40
