"""Input generators: determinism, dtype exactness, shapes (CPU only)."""
import numpy as np
import torch

from paper_2510_13797_amd import workloads as W


def test_bf16_rounding_matches_library_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-30], np.float32)])
    ours = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = W.bf16_bits_to_f32(ours)
    assert np.array_equal(W.f32_to_bf16_bits(back), ours)
    assert np.array_equal(W.round_to_dtype(x, "bf16"), back)


def test_counter_based_and_deterministic():
    a, b = W.batch64(), W.batch64()
    k1, v1 = a.step_kv(37)
    k2, v2 = b.step_kv(37)
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert not np.array_equal(k1, a.step_kv(38)[0])
    assert not np.array_equal(a.step_q(37), W.batch64(seed=1).step_q(37))
    assert k1.shape == (64, 2, 128) and a.step_q(1).shape == (64, 12, 128)
    assert np.array_equal(W.round_to_dtype(k1, "bf16"), k1)      # already bf16-exact


def test_config_shapes():
    t = W.tiny()
    assert (t.B, t.Hq, t.Hkv, t.d, t.dtype) == (2, 4, 1, 64, "f32")
    assert list(t.capacity()) == [32 + 16 + 16 + 1] * 2
    r = W.ragged256()
    assert r.P.min() >= 64 and r.P.max() <= 512 and r.G.min() >= 1024 and r.G.max() <= 16384
    assert set(np.unique(r.c)) <= {2, 4, 8, 16, 32} and 1 <= r.extra["T"] <= 16384
    l = W.long_reasoning()
    assert list(l.capacity())[0] == 512 + 1024 + 32 + 1
    assert list(W.batch64(c=0).capacity())[0] == 256 + 4096
    p = W.prefill_train()
    assert int(p.S[0]) == 8688


def test_peaked_keys_every_64th_written_row():
    l = W.long_reasoning(G=256, B=2)
    k, _ = l.prompt_kv(0)
    big = np.abs(k).reshape(512, -1).max(axis=1)
    idx = np.nonzero(big > 8.0)[0]
    assert set(range(63, 512, 64)) <= set(idx)
    # write order: 512 prompt rows, then tokens and beacons interleaved (one beacon per 32 tokens)
    written = 512
    for t in range(1, 129):
        kt, _ = l.step_kv(t)
        peaked = np.abs(kt[0]).max() > 8.0
        if written % 64 == 63:
            assert peaked
        written += 1
        if t % 32 == 0:
            kb, _ = l.beacon_kv(t)
            if written % 64 == 63:
                assert np.abs(kb[0]).max() > 8.0
            written += 1


def test_distill_workload_rows_are_reproducible_and_well_formed():
    wl = W.DistillWorkload("t", 9, 512, 20, "bf16")
    z, tl, idx = wl.tokens([3, 7])
    z2, tl2, idx2 = wl.token(7)
    assert np.array_equal(z[1], z2) and np.array_equal(tl[1], tl2) and np.array_equal(idx[1], idx2)
    assert np.array_equal(W.round_to_dtype(z, "bf16"), z)          # exact in the logits' dtype
    assert len(set(idx[0].tolist())) == 20 and idx.min() >= 0 and idx.max() < 512
    assert np.all(np.diff(tl, axis=1) <= 0)                        # the k largest, in descending order
    assert W.distill().V == 151936 and W.distill().k == 100
