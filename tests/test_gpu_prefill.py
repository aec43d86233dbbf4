"""GPU parity: bc_prefill_attn (beacon-masked prefill attention, forward) against the dense
masked-attention oracle, and against bc_decode_attn over the evicted cache (training-time
masking simulates the eviction).  bf16 inputs, fp32 accumulation: max-abs-error 2e-3."""
import numpy as np
import pytest

from oracle import attention as OA
from paper_2510_13797_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


# every forward test runs through both entry points: bc_prefill_attn and, when FORM says so,
# bc_prefill_attn_ws (V copied to half precision in a workspace, weights in one half-precision part)
FORM = {"workspace": False}


@pytest.fixture(params=["plain", "workspace"])
def form(request):
    """Which forward entry point _run() goes through."""
    FORM["workspace"] = request.param == "workspace"
    yield request.param
    FORM["workspace"] = False


def _run(pw, dev, want_lse=True, qkv=None):
    from paper_2510_13797_amd import bc
    bc.load()
    qkv = [pw.qkv(b) for b in range(pw.B)] if qkv is None else qkv
    off = np.zeros(pw.B + 1, np.int64)
    off[1:] = np.cumsum(pw.S)
    q = bc.to_device(np.concatenate([x[0] for x in qkv]), "bf16", dev)
    k = bc.to_device(np.concatenate([x[1] for x in qkv]), "bf16", dev)
    v = bc.to_device(np.concatenate([x[2] for x in qkv]), "bf16", dev)
    out, lse = bc.prefill_attn(q, k, v, off, pw.P, pw.c, pw.Hq, pw.Hkv, pw.d, pw.scale, want_lse,
                               workspace=FORM["workspace"])
    return qkv, off, out.cpu().numpy(), None if lse is None else lse.cpu().numpy()


def _check_rows(pw, qkv, off, out, lse, b, rows):
    q, k, v = qkv[b]
    ref, ref_lse = OA.masked_prefill_attention(q, k, v, int(pw.P[b]), int(pw.c[b]), pw.scale, rows=rows)
    got = out[off[b] + np.asarray(rows)]
    err = float(np.abs(got - ref).max())
    assert err <= TOL, (b, err)
    if lse is not None:
        lerr = float(np.abs(lse[off[b] + np.asarray(rows)] - ref_lse).max())
        assert lerr <= 1e-3, (b, lerr)
    return err


@pytest.mark.parametrize("Hq,Hkv", [(12, 2), (4, 1), (8, 8), (2, 2), (7, 1), (8, 1), (5, 1), (3, 1), (4, 2)])
def test_prefill_small_ragged_all_rows(dev, Hq, Hkv, form):
    pw = W.PrefillWorkload("pf_small", 50 + Hq, 6, Hq, Hkv, 128, "bf16",
                           np.array([0, 5, 64, 70, 33, 200], np.int32),      # prompt rows
                           np.array([150, 64, 1, 130, 97, 0], np.int32),     # response tokens
                           np.array([16, 2, 4, 0, 1, 16], np.int32))         # c (0: plain causal)
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    for b in range(pw.B):
        _check_rows(pw, qkv, off, out, lse, b, list(range(int(pw.S[b]))))


@pytest.mark.parametrize("Hq,Hkv", [(12, 2), (4, 4), (8, 1), (7, 1), (5, 1), (2, 2)])
def test_prefill_head_dimension_64_all_rows(dev, Hq, Hkv, form):
    # rows of 128 bytes: eight rows per LDS-DMA instruction, two k-steps, four output blocks, the
    # swizzle of the 8-unit rows; ragged trajectories with and without prompt, several ratios
    pw = W.PrefillWorkload("pf_d64", 64 + Hq, 4, Hq, Hkv, 64, "bf16", np.array([37, 0, 129, 64], np.int32),
                           np.array([300, 190, 75, 0], np.int32), np.array([4, 16, 0, 3], np.int32))
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    for b in range(pw.B):
        _check_rows(pw, qkv, off, out, lse, b, list(range(int(pw.S[b]))))


def test_prefill_ratios_and_long_beacon_runs(dev, form):
    # many beacons (several gathered beacon tiles) and every ratio the paper uses
    pw = W.PrefillWorkload("pf_ratios", 61, 5, 12, 2, 128, "bf16", np.array([3, 40, 128, 7, 256], np.int32),
                           np.array([700, 900, 1000, 1100, 1200], np.int32),
                           np.array([2, 4, 8, 16, 32], np.int32))
    qkv, off, out, lse = _run(pw, dev)
    rng = np.random.default_rng(0)
    for b in range(pw.B):
        S = int(pw.S[b])
        rows = sorted(set([0, 1, S - 1, S - 2, int(pw.P[b]), max(int(pw.P[b]) - 1, 0)])
                      | set(int(x) for x in rng.integers(0, S, size=150)))
        _check_rows(pw, qkv, off, out, lse, b, rows)


def test_config5_full_size(dev, form):
    pw = W.prefill_train()
    assert int(pw.S[0]) == 8688
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    rng = np.random.default_rng(1)
    # a band of consecutive rows across tile and window borders, every beacon-tile border, and
    # random rows of every trajectory
    worst = _check_rows(pw, qkv, off, out, lse, 0, list(range(0, 400)) + list(range(8300, 8688)))
    for b in range(pw.B):
        rows = sorted(set(int(x) for x in rng.integers(0, 8688, size=120)))
        worst = max(worst, _check_rows(pw, qkv, off, out, lse, b, rows))
    # every row of four (trajectory, query head) slices: first and last trajectory, heads of both
    # KV heads, first and last head of a group
    g = pw.Hq // pw.Hkv
    for b, h in ((0, 0), (0, pw.Hq - 1), (pw.B - 1, g - 1), (7, g)):
        q, k, v = qkv[b]
        kvh = h // g
        ref, ref_lse = OA.masked_prefill_attention(q[:, h:h + 1], k[:, kvh:kvh + 1], v[:, kvh:kvh + 1],
                                                   int(pw.P[b]), int(pw.c[b]), pw.scale)
        got = out[off[b]:off[b + 1], h:h + 1]
        err = float(np.abs(got - ref).max())
        lerr = float(np.abs(lse[off[b]:off[b + 1], h:h + 1] - ref_lse).max())
        assert err <= TOL and lerr <= 1e-3, (b, h, err, lerr)
        worst = max(worst, err)
    print("config5 worst", worst)


@pytest.mark.parametrize("d", [128, 64])
def test_prefill_rows_equal_decode_over_evicted_cache(dev, d, form):
    # Sec. 3.2: masking simulates eviction.  Feed the same q/k/v through the decode path
    # (append, attend, beacon append at the tail, attend with the beacon's query, evict) and
    # compare every row with the prefill output.
    from paper_2510_13797_amd import bc
    P, c, R = 37, 8, 475
    pw = W.PrefillWorkload("pf_eq", 62, 2, 12, 2, d, "bf16", np.full(2, P, np.int32),
                           np.full(2, R, np.int32), np.full(2, c, np.int32))
    qkv, off, out, _ = _run(pw, dev, want_lse=False)
    S = int(pw.S[0])
    assert S == P + R + R // c
    B = pw.B
    q = np.stack([x[0] for x in qkv]); k = np.stack([x[1] for x in qkv]); v = np.stack([x[2] for x in qkv])
    cap = np.full(B, P + R // c + c + 1, np.int32)
    rt = bc.Runtime(B, pw.Hq, pw.Hkv, pw.d, "bf16", pw.scale, pw.P, pw.c, cap, dev)
    rt.cache_init([k[b, :P] for b in range(B)], [v[b, :P] for b in range(B)])
    worst = 0.0
    row = P
    for t in range(1, R + 1):
        rt.append_kv(k[:, row], v[:, row])
        o = rt.decode_attn(q[:, row]).cpu().numpy()
        for b in range(B):
            worst = max(worst, float(np.abs(o[b] - out[off[b] + row]).max()))
        row += 1
        if t % c == 0:                                   # beacon row
            rt.append_kv(k[:, row], v[:, row], kind=bc.BC_ROW_BEACON)
            o = rt.decode_attn(q[:, row]).cpu().numpy()
            for b in range(B):
                worst = max(worst, float(np.abs(o[b] - out[off[b] + row]).max()))
            rt.compress_evict()
            row += 1
    assert row == S
    assert rt.tables()[2] == 0
    assert worst <= TOL, worst
    print("prefill vs decode worst", worst)


def test_prefill_argument_errors(dev):
    from paper_2510_13797_amd import bc
    import ctypes as C
    import torch
    x = torch.zeros(64, dtype=torch.float32, device=dev)
    p = C.c_void_p(x.data_ptr())
    sh32 = bc.bc_shape(1, 4, 1, 128, bc.BC_F32, 0.1)
    assert bc.bc_prefill_attn(sh32, p, p, p, p, p, p, 4, p, None, None) == -2      # bf16 only
    sh = bc.bc_shape(1, 4, 1, 128, bc.BC_BF16, 0.1)
    assert bc.bc_prefill_attn(sh, None, p, p, p, p, p, 4, p, None, None) == -1
    assert bc.bc_prefill_attn(sh, p, p, p, p, p, p, 0, p, None, None) == -1


# ---------------------------------------------------------------------------
# backward (next row): gradients against the dense fp64 oracle
# ---------------------------------------------------------------------------
def _run_bwd(pw, dev, half_forward=False):
    from paper_2510_13797_amd import bc
    qkv = [pw.qkv(b) for b in range(pw.B)]
    dos = [pw.dout(b) for b in range(pw.B)]
    off = np.zeros(pw.B + 1, np.int64)
    off[1:] = np.cumsum(pw.S)
    q = bc.to_device(np.concatenate([x[0] for x in qkv]), "bf16", dev)
    k = bc.to_device(np.concatenate([x[1] for x in qkv]), "bf16", dev)
    v = bc.to_device(np.concatenate([x[2] for x in qkv]), "bf16", dev)
    do = bc.to_device(np.concatenate(dos), "bf16", dev)
    # (out and lse from bc_prefill_attn, or from bc_prefill_attn_ws when the caller says so)
    out, lse = bc.prefill_attn(q, k, v, off, pw.P, pw.c, pw.Hq, pw.Hkv, pw.d, pw.scale, True, workspace=half_forward)
    dq, dk, dv = bc.prefill_attn_bwd(q, k, v, out, lse, do, off, pw.P, pw.c, pw.Hq, pw.Hkv, pw.d, pw.scale)
    return qkv, dos, off, dq.cpu().numpy(), dk.cpu().numpy(), dv.cpu().numpy()


def _check_bwd(pw, qkv, dos, off, dq, dk, dv, b):
    q, k, v = qkv[b]
    rq, rk, rv = OA.masked_prefill_attention_bwd(q, k, v, dos[b], int(pw.P[b]), int(pw.c[b]), pw.scale)
    sl = slice(int(off[b]), int(off[b + 1]))
    errs = [float(np.abs(g[sl] - r).max()) for g, r in ((dq, rq), (dk, rk), (dv, rv))]
    assert max(errs) <= TOL, (b, errs)
    return errs


@pytest.mark.parametrize("Hq,Hkv", [(12, 2), (4, 1), (8, 8), (6, 2), (7, 1), (8, 1), (5, 1)])
def test_prefill_bwd_small_ragged(dev, Hq, Hkv):
    pw = W.PrefillWorkload("pf_bwd", 55 + Hq, 6, Hq, Hkv, 128, "bf16",
                           np.array([0, 5, 64, 70, 33, 200], np.int32),
                           np.array([150, 64, 1, 130, 97, 0], np.int32),
                           np.array([16, 2, 4, 0, 1, 16], np.int32))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()   # every element written
    for b in range(pw.B):
        _check_bwd(pw, qkv, dos, off, dq, dk, dv, b)


@pytest.mark.parametrize("Hq,Hkv", [(12, 2), (4, 4), (8, 1), (7, 1), (5, 1)])
def test_prefill_bwd_head_dimension_64(dev, Hq, Hkv):
    # the gradients at d = 64: every element of dq, dk, dv of ragged trajectories (head splits of
    # the dense key blocks and the fixed-order reduction included) against the dense oracle
    pw = W.PrefillWorkload("pfb_d64", 164 + Hq, 4, Hq, Hkv, 64, "bf16", np.array([37, 0, 129, 64], np.int32),
                           np.array([300, 190, 75, 0], np.int32), np.array([4, 16, 0, 3], np.int32))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    for b in range(pw.B):
        _check_bwd(pw, qkv, dos, off, dq, dk, dv, b)


def test_prefill_bwd_many_beacons(dev):
    pw = W.PrefillWorkload("pf_bwd2", 63, 3, 12, 2, 128, "bf16", np.array([3, 128, 256], np.int32),
                           np.array([900, 1300, 1000], np.int32), np.array([2, 8, 16], np.int32))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    worst = [0, 0, 0]
    for b in range(pw.B):
        worst = [max(a, e) for a, e in zip(worst, _check_bwd(pw, qkv, dos, off, dq, dk, dv, b))]
    print("bwd worst dq/dk/dv", worst)


def test_config5_bwd_full_size(dev):
    # B = 2 trajectories of the config-5 shape (8688 rows each); the dense fp64 oracle is run
    # on the first one in full
    pw = W.prefill_train(B=2)
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    errs = _check_bwd(pw, qkv, dos, off, dq, dk, dv, 0)
    print("config5 bwd dq/dk/dv", errs)


@pytest.mark.parametrize("case", range(8))
def test_prefill_randomised_forward_and_backward(dev, case, form):
    # seeded random trajectory counts, prompt and response lengths, ratios and head layouts;
    # every row of the forward and every gradient element against the oracle
    rng = np.random.default_rng([20251013, 78, case])
    Hq, Hkv = [(12, 2), (4, 4), (8, 1), (6, 2), (7, 1), (5, 5), (16, 2), (3, 1)][case]
    B = int(rng.integers(1, 6))
    P = rng.integers(0, 150, size=B).astype(np.int32)
    R = rng.integers(0, 260, size=B).astype(np.int32)
    R[(P == 0) & (R == 0)] = 1
    c = rng.choice([0, 1, 2, 3, 7, 16, 33], size=B).astype(np.int32)
    pw = W.PrefillWorkload("pf_rand%d" % case, 300 + case, B, Hq, Hkv, 128, "bf16", P, R, c)
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    for b in range(pw.B):
        _check_rows(pw, qkv, off, out, lse, b, list(range(int(pw.S[b]))))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    for b in range(pw.B):
        _check_bwd(pw, qkv, dos, off, dq, dk, dv, b)


def test_prefill_long_trajectory(dev, form):
    # a 32k-token response (the longest generation the paper's setups allow) in one trajectory:
    # 2,048 beacons, 64 gathered beacon tiles per late query tile; sampled rows against the oracle
    pw = W.PrefillWorkload("pf_long", 64, 1, 12, 2, 128, "bf16", np.array([512], np.int32),
                           np.array([32768], np.int32), np.array([16], np.int32))
    S = int(pw.S[0])
    assert S == 512 + 32768 + 2048
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    rng = np.random.default_rng(4)
    rows = sorted(set([0, 511, 512, 528, 529, S - 1, S - 2, S - 17, S - 18])
                  | set(int(x) for x in rng.integers(0, S, size=160)))
    _check_rows(pw, qkv, off, out, lse, 0, rows)


class _PeakedKeys:
    """A PrefillWorkload whose keys have a wide range of magnitudes: every 64th key row is scaled
    by 4 and the last quarter of every trajectory by 2 (both exact in bf16), so that the softmax
    is dominated by few keys and its running reference has to move many times."""

    def __init__(self, pw):
        self._pw = pw

    def __getattr__(self, name):
        return getattr(self._pw, name)

    def qkv(self, b):
        q, k, v = self._pw.qkv(b)
        k = k.copy()
        k[63::64] *= 4.0
        k[3 * len(k) // 4:] *= 2.0
        return q, k, v


def test_prefill_peaked_keys_forward_and_backward(dev, form):
    pw = _PeakedKeys(W.PrefillWorkload("pf_peak", 65, 3, 12, 2, 128, "bf16", np.array([5, 100, 256], np.int32),
                                       np.array([600, 900, 300], np.int32), np.array([16, 4, 0], np.int32)))
    qkv, off, out, lse = _run(pw, dev)
    assert np.isfinite(out).all()
    for b in range(pw.B):
        _check_rows(pw, qkv, off, out, lse, b, list(range(int(pw.S[b]))))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    for b in range(pw.B):
        _check_bwd(pw, qkv, dos, off, dq, dk, dv, b)


def test_prefill_ratio_whose_window_index_needs_more_than_32_bits(dev, form):
    # c = 65535: rows * (c + 1) passes 2^32 inside the third window, where a multiply-high
    # estimate of offset / (c + 1) is one too large unless it is corrected (offset 131071, the
    # second beacon, is the first such place).  Forward rows and gradients around both beacons
    # and in the short third window, against the oracle's per-place sums.
    P, c = 24, 65535
    R = 2 * c + 150
    pw = W.PrefillWorkload("pf_wide_ratio", 66, 1, 2, 1, 128, "bf16", np.array([P], np.int32),
                           np.array([R], np.int32), np.array([c], np.int32))
    S = int(pw.S[0])
    assert S == P + R + 2 and (S - P) * (c + 1) > 2 ** 32
    b1, b2 = P + c, P + 2 * c + 1                      # the two beacon rows
    assert OA.is_beacon_row(b1, P, c) and OA.is_beacon_row(b2, P, c)
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev)
    _, _, out, lse = _run(pw, dev)
    assert np.isfinite(out).all() and np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    rows = [0, P - 1, P, b1 - 1, b1, b1 + 1, b2 - 2, b2 - 1, b2, b2 + 1, b2 + 2, b2 + 77, S - 2, S - 1]
    _check_rows(pw, qkv, off, out, lse, 0, rows)
    # keys whose columns are short enough to sum on the CPU: the tail of the second window, its
    # beacon, the third window
    keys = [b2 - 3, b2 - 1, b2, b2 + 1, b2 + 40, S - 1]
    q, k, v = qkv[0]
    rq, rk, rv = OA.masked_prefill_attention_bwd_at(q, k, v, dos[0], P, c, pw.scale, rows, keys)
    errs = [float(np.abs(dq[rows] - rq).max()), float(np.abs(dk[keys] - rk).max()),
            float(np.abs(dv[keys] - rv).max())]
    assert max(errs) <= TOL, errs


def test_values_beyond_half_precision_take_the_two_part_form(dev):
    # one V entry of 1e5 (finite in bf16, beyond half precision): the workspace entry point must
    # notice it on the device and compute what the plain entry point computes - bit for bit; and a
    # V whose entries all fit gives the half-precision form, which differs in the last bits but
    # stays inside the tolerance (checked by every other test of this file)
    pw = W.PrefillWorkload("pf_range", 67, 2, 12, 2, 128, "bf16", np.array([40, 7], np.int32),
                           np.array([200, 90], np.int32), np.array([16, 4], np.int32))
    qkv = [list(pw.qkv(b)) for b in range(pw.B)]
    qkv[1][2] = qkv[1][2].copy()
    qkv[1][2][50, 1, 77] = np.float32(99840.0)            # exact in bf16
    keep = FORM["workspace"]
    try:
        FORM["workspace"] = False
        _, off, plain, lse_plain = _run(pw, dev, qkv=qkv)
        FORM["workspace"] = True
        _, _, withws, lse_ws = _run(pw, dev, qkv=qkv)
    finally:
        FORM["workspace"] = keep
    assert np.array_equal(plain, withws) and np.array_equal(lse_plain, lse_ws)
    for b in range(pw.B):
        q, k, v = qkv[b]
        rows = list(range(int(pw.S[b])))
        ref, _ = OA.masked_prefill_attention(q, k, v, int(pw.P[b]), int(pw.c[b]), pw.scale, rows=rows)
        got = plain[off[b] + np.asarray(rows)]
        assert np.abs(got - ref).max() <= TOL * max(1.0, float(np.abs(ref).max()))


def test_gradients_from_the_half_form_forward(dev):
    # out and lse of the workspace form (weights in one half-precision part: out within 2e-3, but
    # some 70 times further from the oracle than the two-part form) fed to the backward: on N(0,1)
    # trajectories the gradients stay inside the same absolute bound.  The error of out enters the
    # gradients through Delta = sum(dO * out), scaled by the size of dO and K: with keys scaled
    # up as in the peaked-keys test it reaches 2.8e-3, so where gradients must meet the bound
    # whatever the data, the forward to use is bc_prefill_attn (which every other backward test takes).
    pw = W.PrefillWorkload("pf_half_bwd", 68, 3, 12, 2, 128, "bf16", np.array([37, 0, 129], np.int32),
                           np.array([300, 190, 75], np.int32), np.array([4, 16, 0], np.int32))
    qkv, dos, off, dq, dk, dv = _run_bwd(pw, dev, half_forward=True)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    for b in range(pw.B):
        _check_bwd(pw, qkv, dos, off, dq, dk, dv, b)
