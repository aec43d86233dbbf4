"""Token-level distillation loss (oracle, test only; fp64 NumPy).

Eq. 1 of the paper (Sec. 3.2): the loss of a trajectory is the mean over its tokens of
KL(teacher || student) over the vocabulary, and the batch loss the mean over trajectories.
App. A: only the teacher's top-100 logits per step are stored.  Reading used here (the paper does
not say how the truncated teacher enters the KL): the teacher distribution is the softmax over its
stored top-k logits (renormalised on those k tokens); the student's log-probabilities come from
its full-vocabulary log-softmax, evaluated at the same k token ids.
"""
from __future__ import annotations

import numpy as np


def topk_kl_loss(student_logits, teacher_logits, teacher_idx):
    """student_logits [T, V]; teacher_logits [T, k]; teacher_idx [T, k] (distinct per row).
    Returns (loss_per_token [T], student log-sum-exp [T]) in fp64."""
    z = np.asarray(student_logits, dtype=np.float64)
    tl = np.asarray(teacher_logits, dtype=np.float64)
    idx = np.asarray(teacher_idx)
    T = z.shape[0]
    loss = np.empty(T)
    lse = np.empty(T)
    for t in range(T):
        m = z[t].max()
        lse[t] = m + np.log(np.exp(z[t] - m).sum())
        log_ps = z[t, idx[t]] - lse[t]                       # student log-probs at the stored ids
        mt = tl[t].max()
        log_pt = tl[t] - (mt + np.log(np.exp(tl[t] - mt).sum()))   # teacher: softmax over its top-k
        loss[t] = float((np.exp(log_pt) * (log_pt - log_ps)).sum())
    return loss, lse


def topk_kl_loss_grad(student_logits, teacher_logits, teacher_idx, grad_scale):
    """d(grad_scale * sum_t loss_t) / d student_logits: softmax(student) minus the teacher
    probabilities scattered to their token ids (the teacher's probabilities sum to one)."""
    z = np.asarray(student_logits, dtype=np.float64)
    tl = np.asarray(teacher_logits, dtype=np.float64)
    idx = np.asarray(teacher_idx)
    g = np.empty_like(z)
    for t in range(z.shape[0]):
        e = np.exp(z[t] - z[t].max())
        g[t] = e / e.sum()
        et = np.exp(tl[t] - tl[t].max())
        g[t, idx[t]] -= et / et.sum()
    return grad_scale * g


def batch_loss(loss_per_token):
    """Mean over the tokens (Eq. 1 with trajectories of equal length: mean over all tokens)."""
    return float(np.mean(np.asarray(loss_per_token, dtype=np.float64)))
