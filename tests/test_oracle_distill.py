"""Pins for the top-k KL distillation loss oracle (Eq. 1, Sec. 3.2; App. A).  CPU only."""
import numpy as np
import torch
from scipy.special import logsumexp

from oracle import distill as D


def _case(rng, T=5, V=37, k=6):
    z = rng.standard_normal((T, V)) * 2
    teacher_full = z + rng.standard_normal((T, V))
    idx = np.argsort(-teacher_full, axis=1)[:, :k]
    tl = np.take_along_axis(teacher_full, idx, axis=1)
    return z, tl, idx


def test_lse_matches_library_and_kl_is_nonnegative():
    rng = np.random.default_rng(0)
    z, tl, idx = _case(rng)
    loss, lse = D.topk_kl_loss(z, tl, idx)
    assert np.abs(lse - logsumexp(z, axis=1)).max() < 1e-12
    assert np.all(loss > 0)


def test_loss_matches_torch_kl_div_on_the_same_definition():
    rng = np.random.default_rng(1)
    z, tl, idx = _case(rng, T=7, V=50, k=9)
    loss, _ = D.topk_kl_loss(z, tl, idx)
    tz = torch.tensor(z, requires_grad=True)
    log_ps = torch.log_softmax(tz, dim=1).gather(1, torch.from_numpy(idx))
    pt = torch.softmax(torch.from_numpy(tl), dim=1)
    ref = torch.nn.functional.kl_div(log_ps, pt, reduction="none").sum(dim=1)      # sum p_t (log p_t - log p_s)
    assert np.abs(loss - ref.detach().numpy()).max() < 1e-12
    gs = 0.37
    (gs * ref.sum()).backward()
    g = D.topk_kl_loss_grad(z, tl, idx, gs)
    assert np.abs(g - tz.grad.numpy()).max() < 1e-12
    assert abs(D.batch_loss(loss) - float(ref.mean())) < 1e-12


def test_zero_when_student_equals_teacher_on_full_vocabulary():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((3, 11))
    idx = np.tile(np.arange(11), (3, 1))
    loss, _ = D.topk_kl_loss(z, z.copy(), idx)
    assert np.abs(loss).max() < 1e-14
    assert np.abs(D.topk_kl_loss_grad(z, z.copy(), idx, 1.0)).max() < 1e-14
    # shifting all student logits by a constant changes nothing; so does shifting the teacher's
    z2, tl, idx2 = _case(rng)
    a, _ = D.topk_kl_loss(z2, tl, idx2)
    b, _ = D.topk_kl_loss(z2 + 3.0, tl - 5.0, idx2)
    assert np.abs(a - b).max() < 1e-12


def test_two_token_closed_form():
    # V = 2, k = 2: KL of two Bernoulli distributions
    z = np.array([[0.3, -1.1]]); tl = np.array([[2.0, 0.5]]); idx = np.array([[0, 1]])
    ps = 1 / (1 + np.exp(-(0.3 + 1.1))); pt = 1 / (1 + np.exp(-(2.0 - 0.5)))
    ref = pt * np.log(pt / ps) + (1 - pt) * np.log((1 - pt) / (1 - ps))
    assert abs(D.topk_kl_loss(z, tl, idx)[0][0] - ref) < 1e-14
