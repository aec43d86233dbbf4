"""Host-side logic of bench.py (no GPU): the one-GPU rule and the algorithmic byte / flop counts
the reported figures are built from, against the oracle's closed forms."""
import os
import subprocess
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402
from oracle import attention as OA  # noqa: E402
from oracle import residency as OR  # noqa: E402
from paper_2510_13797_amd import workloads as W  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_kv_bytes_per_step_is_the_resident_length_at_attention():
    wl = W.batch64(c=16)
    for t in (1, 15, 16, 17, 4095, 4096):
        L = OR.len_at_attention(256, 16, t)
        assert bench.kv_bytes_per_step(wl, t) == 64 * L * 2 * 128 * 2 * 2
    wl0 = W.batch64(c=0)
    assert bench.kv_bytes_per_step(wl0, 100) == 64 * (256 + 100) * 2 * 128 * 2 * 2


def test_visible_pairs_equals_the_sum_of_the_oracle_row_counts():
    for S, P, c in ((200, 17, 4), (97, 0, 16), (64, 64, 3), (50, 10, 0)):
        assert bench.visible_pairs(S, P, c) == sum(OA.count_visible(r, P, c) for r in range(S))
    pw = W.prefill_train()
    pairs = bench.visible_pairs(int(pw.S[0]), 256, 16)
    assert abs(4.0 * 128 * pairs * 12 * 16 / 1e9 - 428.0) < 0.5      # GFLOP of the forward at config 5


def test_stored_traffic_figures_are_read_from_the_profiles():
    # measured HBM-side bytes must be at least the algorithmic bytes of the same launch
    t = bench.stored_traffic()
    assert t is not None and t["bytes_per_launch"] >= t["algorithmic_bytes_per_launch"]
    pw = W.prefill_train()
    rows = int(np.sum(pw.S))
    fwd_alg = rows * pw.Hq * 128 * 2 + 2 * rows * pw.Hkv * 128 * 2 + rows * pw.Hq * 128 * 4
    assert bench.stored_value("prefill_fwd_traffic_bytes") >= fwd_alg
    assert bench.stored_value("distill_bwd_traffic_bytes") >= 2 * 4096 * 151936 * 2
    assert bench.stored_value("no_such_key") is None


def test_tables_and_rows_of_a_state_follow_the_closed_forms():
    wl = W.ragged256()
    t = np.minimum(int(wl.extra["T"]), wl.G)
    nb, w = bench.tables_at(wl, t)
    rows = bench.rows_seen(wl, t)
    for s in range(0, wl.B, 17):
        P, c, ts = int(wl.P[s]), int(wl.c[s]), int(t[s])
        assert (int(nb[s]), int(w[s])) == (ts // c, ts % c)
        assert int(rows[s]) == OR.len_at_attention(P, c, ts)
        # the state after t tokens is what the attention of step t + 1 sees, minus the new row
        assert int(wl.P[s]) + int(nb[s]) + int(w[s]) == OR.len_after_step(P, c, ts)
    wl0 = W.batch64(c=0)
    nb0, w0 = bench.tables_at(wl0, 100)
    assert nb0[0] == 0 and w0[0] == 100 and bench.rows_seen(wl0, 100)[0] == 356


def test_host_cores_is_bounded():
    assert 1 <= bench.host_cores() <= 16
