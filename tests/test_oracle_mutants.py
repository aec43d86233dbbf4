"""Planted mistakes in the oracle (CPU only): each plausible slip must be caught by at least one
of the pins in the other test files.  The mistakes are planted by monkeypatching the oracle."""
import numpy as np
import pytest

from oracle import attention as A
from oracle import cache as CA
from oracle import residency as R

import test_oracle_attention as TA
import test_oracle_prefill as TP
import test_oracle_residency as TR


def _caught(fns):
    hits = 0
    for fn in fns:
        try:
            fn()
        except (AssertionError, IndexError, ValueError):
            hits += 1
    return hits


ATTN_PINS = [TA.test_brute_force_tiny, TA.test_full_attention_special_case_matches_library,
             TA.test_single_key_returns_v_exactly, TA.test_permutation_invariance,
             TA.test_equal_keys_and_zero_scale_give_mean_of_v, TA.test_two_key_closed_form_pins_scale_and_sign,
             TA.test_gqa_equals_mha_with_repeated_kv_and_group_symmetry,
             TA.test_softmax_attention_agrees_with_scipy_softmax]


def test_all_pins_pass_unmutated():
    assert _caught(ATTN_PINS) == 0


def test_dropped_scale_is_caught(monkeypatch):
    good = A.softmax_attention
    monkeypatch.setattr(A, "softmax_attention", lambda q, K, V, scale: good(q, K, V, 1.0))
    assert _caught(ATTN_PINS) >= 2


def test_wrong_sign_is_caught(monkeypatch):
    good = A.softmax_attention
    monkeypatch.setattr(A, "softmax_attention", lambda q, K, V, scale: good(q, K, V, -scale))
    assert _caught(ATTN_PINS) >= 2


def test_unnormalised_softmax_is_caught(monkeypatch):
    def bad(q, K, V, scale):
        s = scale * (np.asarray(K, float) @ np.asarray(q, float))
        p = np.exp(s - s.max())
        return p @ np.asarray(V, float)              # forgot the denominator
    monkeypatch.setattr(A, "softmax_attention", bad)
    assert _caught(ATTN_PINS) >= 2


def test_wrong_gqa_map_is_caught(monkeypatch):
    def bad(q, K, V, scale):
        q, K, V = (np.asarray(x, float) for x in (q, K, V))
        Hq, Hkv = q.shape[0], K.shape[1]
        return np.stack([A.softmax_attention(q[h], K[:, h % Hkv], V[:, h % Hkv], scale) for h in range(Hq)])
    monkeypatch.setattr(A, "decode_attention", bad)
    assert _caught(ATTN_PINS) >= 1


def test_eviction_off_by_one_is_caught(monkeypatch):
    def bad(P, c, G):                                   # drops c - 1 entries instead of c
        kv = [("q", j) for j in range(P)]
        for i in range(1, G + 1):
            kv.append(("x", i - 1))
            at = list(kv)
            if c > 0 and i % c == 0:
                kv.append(("b", i // c))
                kv = kv[:-c] + kv[-1:]
            yield i, at, list(kv)
    monkeypatch.setattr(R, "alg1_literal", bad)
    assert _caught([TR.test_literal_equals_structured_brute_force, TR.test_closed_forms_match_simulation]) == 2


def test_compress_one_step_early_is_caught(monkeypatch):
    monkeypatch.setattr(R, "len_after_step", lambda P, c, t: P + t if c <= 0 else P + (t + 1) // c + (t + 1) % c)
    assert _caught([TR.test_closed_forms_match_simulation]) == 1


def test_batchcache_keeping_a_window_row_is_caught(monkeypatch):
    good = CA.BatchCache.compress_evict

    def bad(self, bk=None, bv=None, active=None, require_full=True):
        keep = [w[:1] for w in self.window]
        due = [self.c[s] > 0 and len(self.window[s]) == self.c[s] for s in range(self.B)]
        good(self, bk, bv, active, require_full)
        for s in range(self.B):
            if due[s] and bk is not None:
                self.window[s] = keep[s]                # a stray entry survives the eviction
    monkeypatch.setattr(CA.BatchCache, "compress_evict", bad)
    assert _caught([lambda: TR.test_batchcache_equals_flat_literal(False), TR.test_payload_identity]) == 2


def test_mask_that_hides_beacons_is_caught(monkeypatch):
    good = A.visible
    monkeypatch.setattr(A, "visible",
                        lambda r, j, P, c: good(r, j, P, c) and not (A.is_beacon_row(j, P, c) and j != r))
    assert _caught([TP.test_predicate_equals_residency_of_alg1, TP.test_fig2_structure_small_example]) == 2


def test_mask_without_the_diagonal_is_caught(monkeypatch):
    good = A.visible_row
    monkeypatch.setattr(A, "visible_row", lambda r, P, c: good(r, P, c)[:-1] if r > 0 else good(r, P, c))
    assert _caught([TP.test_vectorised_row_equals_predicate_and_mask,
                    TP.test_prefill_row_equals_decode_over_evicted_cache]) == 2


# -- distillation loss ---------------------------------------------------------------------
from oracle import distill as D          # noqa: E402
import test_oracle_distill as TD         # noqa: E402

DISTILL_PINS = [TD.test_lse_matches_library_and_kl_is_nonnegative,
                TD.test_loss_matches_torch_kl_div_on_the_same_definition,
                TD.test_zero_when_student_equals_teacher_on_full_vocabulary,
                TD.test_two_token_closed_form]


def test_distill_pins_pass_unmutated():
    assert _caught(DISTILL_PINS) == 0


def test_reversed_kl_is_caught(monkeypatch):
    good = D.topk_kl_loss

    def reversed_kl(z, tl, idx):                       # KL(student || teacher) on the stored ids
        loss, lse = good(z, tl, idx)
        z, tl = np.asarray(z, float), np.asarray(tl, float)
        out = np.empty_like(loss)
        for t in range(len(loss)):
            lps = z[t, idx[t]] - lse[t]
            lpt = tl[t] - np.log(np.exp(tl[t]).sum())
            out[t] = (np.exp(lps) * (lps - lpt)).sum()
        return out, lse
    monkeypatch.setattr(D, "topk_kl_loss", reversed_kl)
    assert _caught(DISTILL_PINS) >= 2


def test_unnormalised_teacher_and_missing_teacher_term_are_caught(monkeypatch):
    good = D.topk_kl_loss_grad
    monkeypatch.setattr(D, "topk_kl_loss_grad",
                        lambda z, tl, idx, gs: good(z, np.asarray(tl) * 0.0, idx, gs))   # teacher logits ignored
    assert _caught(DISTILL_PINS) >= 1
    monkeypatch.setattr(D, "topk_kl_loss_grad", lambda z, tl, idx, gs: good(z, tl, idx, 1.0))   # scale dropped
    assert _caught(DISTILL_PINS) >= 1
