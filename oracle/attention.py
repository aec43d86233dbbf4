"""Softmax attention over a given key set, and the training-time visibility rule
(oracle, test only; fp64 NumPy).

The paper changes *which* keys a query sees, never the attention itself (Sec. 2
says the model attends to the cache with the ordinary Transformer operation).  So the decode oracle
is the textbook definition over the resident entries, and the prefill oracle is
the same definition over the visible set of Fig. 2 / Sec. 3.2.

Conventions the paper leaves open (stated in the library header as well):
softmax scale is an argument (callers pass 1/sqrt(d)); grouped-query attention
maps query head h to KV head floor(h / (Hq/Hkv)).
"""
from __future__ import annotations

import numpy as np


def softmax_attention(q, K, V, scale):
    """o = sum_j softmax_j(scale * q.K_j) V_j for one query vector.

    q [d], K [L, d], V [L, d] -> [d], all fp64.  L must be >= 1.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = scale * (K @ q)
    p = np.exp(s - s.max())
    return (p @ V) / p.sum()


def decode_attention(q, K, V, scale):
    """Single-token GQA attention of one sequence over its resident entries.

    q [Hq, d]; K, V [L, Hkv, d] (entry-major) -> o [Hq, d] fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, d = q.shape
    Hkv = K.shape[1]
    assert Hq % Hkv == 0
    g = Hq // Hkv
    o = np.empty((Hq, d), dtype=np.float64)
    for h in range(Hq):
        kvh = h // g
        o[h] = softmax_attention(q[h], K[:, kvh, :], V[:, kvh, :], scale)
    return o


# ---------------------------------------------------------------------------
# Training-time mask (Fig. 2, Sec. 3.2).  Rows of one trajectory: P prompt rows,
# then response tokens with one beacon row after every c of them:
#   row = P + m*(c+1) + off,  off in [0, c):  off-th token of window m
#   row = P + m*(c+1) + c                  :  beacon closing window m
# A response row may attend to: the prompt, all previous beacons, earlier tokens
# since the most recent preceding beacon, and itself (causal diagonal).
# Prompt rows carry no beacons and use the plain causal mask.
# ---------------------------------------------------------------------------

def is_beacon_row(r: int, P: int, c: int) -> bool:
    return c > 0 and r >= P and (r - P) % (c + 1) == c


def visible(r: int, j: int, P: int, c: int) -> bool:
    """May row r attend to row j?"""
    if j > r:
        return False
    if j < P or c <= 0:
        return True                     # the question; or no compression at all
    if r < P:
        return False                    # unreachable (j >= P > r contradicts j <= r)
    if is_beacon_row(j, P, c):
        return True                     # every earlier beacon (and a beacon sees itself)
    return (j - P) // (c + 1) == (r - P) // (c + 1)   # same window, not later than r


def visible_mask(S: int, P: int, c: int) -> np.ndarray:
    """Dense [S, S] boolean mask from the predicate, one pair at a time."""
    m = np.zeros((S, S), dtype=bool)
    for r in range(S):
        for j in range(r + 1):
            m[r, j] = visible(r, j, P, c)
    return m


def visible_row(r: int, P: int, c: int) -> np.ndarray:
    """Indices j visible from row r (vectorised form of `visible`)."""
    j = np.arange(r + 1)
    if c <= 0 or r < P:
        return j
    u = j - P
    keep = (j < P) | (u % (c + 1) == c) | (u // (c + 1) == (r - P) // (c + 1))
    return j[keep]


def count_visible(r: int, P: int, c: int) -> int:
    """Closed form |vis(r)| = P + m + off + 1 for response rows."""
    if c <= 0 or r < P:
        return r + 1
    u = r - P
    return P + u // (c + 1) + u % (c + 1) + 1


def masked_prefill_attention(q, k, v, P: int, c: int, scale, rows=None):
    """Beacon-masked attention of one beacon-interleaved trajectory (forward).

    q [S, Hq, d]; k, v [S, Hkv, d]; returns (o [n, Hq, d], lse [n, Hq]) in fp64
    for the given rows (default: all S rows).  lse is the natural-log of the
    softmax denominator, log sum_j exp(scale * q.k_j), over the visible set.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    rows = range(S) if rows is None else rows
    o = np.empty((len(rows), Hq, d), dtype=np.float64)
    lse = np.empty((len(rows), Hq), dtype=np.float64)
    for n, r in enumerate(rows):
        vis = visible_row(r, P, c)
        for h in range(Hq):
            kvh = h // g
            s = scale * (k[vis, kvh, :] @ q[r, h])
            mx = s.max()
            p = np.exp(s - mx)
            den = p.sum()
            o[n, h] = (p @ v[vis, kvh, :]) / den
            lse[n, h] = mx + np.log(den)
    return o, lse


def masked_prefill_attention_bwd(q, k, v, do, P: int, c: int, scale):
    """Gradients of the beacon-masked attention of one trajectory (Sec. 3.2: training
    differentiates through the masked forward; only the student's parameters get gradients).

    With S = scale * Q K^T on the visible pairs, A = softmax(S) row-wise, O = A V and an
    upstream gradient dO:  dV = A^T dO,  dA = dO V^T,  dS = A * (dA - rowsum(dO * O)),
    dQ = scale * dS K,  dK = scale * dS^T Q; K/V gradients sum over the query heads of a group.
    q, do [S, Hq, d]; k, v [S, Hkv, d] -> (dq [S, Hq, d], dk [S, Hkv, d], dv [S, Hkv, d]) fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    mask = np.zeros((S, S), dtype=bool)
    for r in range(S):
        mask[r, visible_row(r, P, c)] = True
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(Hq):
        kvh = h // g
        s = scale * (q[:, h, :] @ k[:, kvh, :].T)
        s = np.where(mask, s, -np.inf)
        a = np.exp(s - s.max(axis=1, keepdims=True))
        a /= a.sum(axis=1, keepdims=True)
        o = a @ v[:, kvh, :]
        dv[:, kvh, :] += a.T @ do[:, h, :]
        da = do[:, h, :] @ v[:, kvh, :].T
        ds = a * (da - (do[:, h, :] * o).sum(axis=1, keepdims=True))
        dq[:, h, :] = scale * (ds @ k[:, kvh, :])
        dk[:, kvh, :] += scale * (ds.T @ q[:, h, :])
    return dq, dk, dv


def rows_seeing(j: int, S: int, P: int, c: int) -> np.ndarray:
    """Rows r of an S-row trajectory that attend to row j (the column of the mask, from the
    same rule as `visible`): the prompt and the beacons are seen by every later row, a response
    token by the later rows of its own window, the closing beacon included."""
    if j < P or c <= 0 or is_beacon_row(j, P, c):
        return np.arange(j, S)
    end = P + ((j - P) // (c + 1) + 1) * (c + 1) - 1          # the window's beacon row
    return np.arange(j, min(end, S - 1) + 1)


def masked_prefill_attention_bwd_at(q, k, v, do, P: int, c: int, scale, rows, keys):
    """The gradients of `masked_prefill_attention_bwd` at chosen places of a trajectory too long
    for its dense S x S form: dq of `rows`, dk and dv of `keys`, every entry from its own sum
    over the visible pairs (same formulas: a = softmax row, ds = a * (da - sum(do * o)),
    dq[r] = scale * sum_j ds[r, j] k[j], dk[j] = scale * sum_r ds[r, j] q[r],
    dv[j] = sum_r a[r, j] do[r], the last two also summed over the query heads of a group).
    Returns (dq [len(rows), Hq, d], dk [len(keys), Hkv, d], dv [len(keys), Hkv, d]) in fp64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv

    def row_terms(r, h):
        """(visible keys, a[r, vis], ds[r, vis]) of query row r, head h."""
        vis = visible_row(r, P, c)
        kvh = h // g
        s = scale * (k[vis, kvh, :] @ q[r, h])
        a = np.exp(s - s.max())
        a /= a.sum()
        o = a @ v[vis, kvh, :]
        da = v[vis, kvh, :] @ do[r, h]
        return vis, a, a * (da - do[r, h] @ o)

    dq = np.zeros((len(rows), Hq, d))
    for n, r in enumerate(rows):
        for h in range(Hq):
            vis, _, ds = row_terms(r, h)
            dq[n, h] = scale * (ds @ k[vis, h // g, :])
    dk = np.zeros((len(keys), Hkv, d))
    dv = np.zeros((len(keys), Hkv, d))
    for n, j in enumerate(keys):
        for r in rows_seeing(j, S, P, c):
            for h in range(Hq):
                vis, a, ds = row_terms(int(r), h)
                at = int(np.searchsorted(vis, j))
                assert vis[at] == j
                dk[n, h // g] += scale * ds[at] * q[r, h]
                dv[n, h // g] += a[at] * do[r, h]
    return dq, dk, dv
