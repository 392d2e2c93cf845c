"""Pins of the head-training-loss oracle (Sec. 3.2 "Training of the draft models").  None of them re-types the
oracle's formulas: they compare with library routines that implement the textbook definitions (torch's smooth L1 and
soft-target cross entropy, torch autograd), with finite differences of the oracle's own loss, with hand numbers, and
with what a uniform law fixes; planted mistakes in a copy of the oracle are shown to fail."""
import numpy as np
import pytest
import torch

from oracle import head_loss as hl


def _case(rows=5, d=12, V=17, seed=0, spread=1.5):
    rng = np.random.default_rng(seed)
    f = rng.standard_normal((rows, d))
    fhat = f + spread * rng.standard_normal((rows, d))          # differences on both sides of the threshold 1
    W = rng.standard_normal((V, d)) * 0.7
    return f, fhat, W


def test_smooth_l1_hand_values_and_continuity():
    x = np.array([0.0, 0.5, -0.5, 1.0, -1.0, 2.0, -3.0])
    np.testing.assert_allclose(hl.smooth_l1(x), [0.0, 0.125, 0.125, 0.5, 0.5, 1.5, 2.5], rtol=0, atol=1e-15)
    e = 1e-9
    assert abs(hl.smooth_l1(np.array([1 - e]))[0] - hl.smooth_l1(np.array([1 + e]))[0]) < 1e-8


def test_hand_example_two_tokens_one_dimension():
    # d = 1, V = 2, W = [[1], [-1]]: logits (f, -f); p = sigmoid(2 f).  f = 0 -> p = (1/2, 1/2); fhat = ln 3 / 2 -> p^ = (3/4, 1/4)
    f = np.array([[0.0]]); fhat = np.array([[np.log(3.0) / 2]]); W = np.array([[1.0], [-1.0]])
    out = hl.head_loss(f, fhat, W, w_cls=0.1)
    x = np.log(3.0) / 2
    assert abs(out["L_reg"] - 0.5 * x * x) < 1e-15
    assert abs(out["L_cls"] - (-0.5 * np.log(0.75) - 0.5 * np.log(0.25))) < 1e-15
    assert abs(out["L"] - (out["L_reg"] + 0.1 * out["L_cls"])) < 1e-15
    # gradient: d/dfhat [0.5 x^2] = x ; d/dfhat CE = (p^_0 - p_0) * 1 + (p^_1 - p_1) * (-1) = 1/4 + 1/4
    g = hl.head_loss_grad(f, fhat, W, w_cls=0.1)
    assert abs(g[0, 0] - (x + 0.1 * 0.5)) < 1e-15


def test_matches_library_losses():
    f, fhat, W = _case()
    out = hl.head_loss(f, fhat, W, w_cls=0.1)
    tf, tfh, tW = (torch.tensor(a, dtype=torch.float64) for a in (f, fhat, W))
    reg = torch.nn.functional.smooth_l1_loss(tfh, tf, beta=1.0, reduction="mean")
    cls = torch.nn.functional.cross_entropy(tfh @ tW.T, torch.softmax(tf @ tW.T, dim=-1), reduction="mean")
    assert abs(out["L_reg"] - reg.item()) < 1e-13
    assert abs(out["L_cls"] - cls.item()) < 1e-12
    assert abs(out["L"] - (reg + 0.1 * cls).item()) < 1e-12


def test_cross_entropy_is_entropy_at_the_label_and_larger_elsewhere():
    f, fhat, W = _case(seed=3)
    p = torch.softmax(torch.tensor(f @ W.T), dim=-1).numpy()
    H = float((-(p * np.log(p)).sum(axis=1)).mean())
    same = hl.head_loss(f, f, W)
    assert same["L_reg"] == 0.0 and abs(same["L_cls"] - H) < 1e-12
    assert hl.head_loss(f, fhat, W)["L_cls"] > H                       # Gibbs' inequality
    np.testing.assert_allclose(hl.head_loss_grad(f, f, W), 0.0, atol=1e-16)   # a perfect head gets no gradient


def test_gradient_against_finite_differences_and_autograd():
    f, fhat, W = _case(rows=3, d=6, V=9, seed=5)
    g = hl.head_loss_grad(f, fhat, W, w_cls=0.1)
    num = np.zeros_like(g)
    h = 1e-6
    for r in range(fhat.shape[0]):
        for k in range(fhat.shape[1]):
            a = fhat.copy(); a[r, k] += h
            b = fhat.copy(); b[r, k] -= h
            num[r, k] = (hl.head_loss(f, a, W, 0.1)["L"] - hl.head_loss(f, b, W, 0.1)["L"]) / (2 * h)
    np.testing.assert_allclose(g, num, rtol=0, atol=1e-8)
    tf, tW = torch.tensor(f), torch.tensor(W)
    tfh = torch.tensor(fhat, requires_grad=True)
    L = torch.nn.functional.smooth_l1_loss(tfh, tf, beta=1.0) + 0.1 * torch.nn.functional.cross_entropy(
        tfh @ tW.T, torch.softmax(tf @ tW.T, dim=-1))
    L.backward()
    np.testing.assert_allclose(g, tfh.grad.numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("mistake", ["no_w_cls", "ce_swapped", "l1_not_smooth", "sum_not_mean", "grad_unclipped", "grad_wrong_rows"])
def test_planted_mistakes_are_caught(mistake):
    f, fhat, W = _case(seed=7)
    good = hl.head_loss(f, fhat, W, 0.1)
    good_g = hl.head_loss_grad(f, fhat, W, 0.1)
    rows, d = f.shape
    z, zh = f @ W.T, fhat @ W.T
    lp, lq = hl._log_softmax(z), hl._log_softmax(zh)
    p, q = np.exp(lp), np.exp(lq)
    if mistake == "no_w_cls":
        bad = good["L_reg"] + good["L_cls"]
        assert abs(bad - good["L"]) > 1e-3
    elif mistake == "ce_swapped":
        bad = float((-(q * lp).sum(axis=1)).mean())
        assert abs(bad - good["L_cls"]) > 1e-3
    elif mistake == "l1_not_smooth":
        bad = float(np.abs(fhat - f).mean())
        assert abs(bad - good["L_reg"]) > 1e-3
    elif mistake == "sum_not_mean":
        bad = float(hl.smooth_l1(fhat - f).sum())
        assert abs(bad - good["L_reg"]) > 1e-3
    elif mistake == "grad_unclipped":
        bad = (fhat - f) / (rows * d) + 0.1 * (q - p) @ W / rows
        assert np.abs(bad - good_g).max() > 1e-4
    else:
        bad = np.clip(fhat - f, -1, 1) / (rows * d) + 0.1 * (q - p) @ W / (rows * d)
        assert np.abs(bad - good_g).max() > 1e-4
    # and the library pins above would see each of them: the values they compare with are `good`, not `bad`
    tf, tfh, tW = (torch.tensor(a) for a in (f, fhat, W))
    ref = torch.nn.functional.smooth_l1_loss(tfh, tf, beta=1.0) + 0.1 * torch.nn.functional.cross_entropy(tfh @ tW.T, torch.softmax(tf @ tW.T, -1))
    assert abs(good["L"] - ref.item()) < 1e-12


def test_noise_is_uniform_symmetric_exact_and_reproducible():
    from scipy import stats
    n = hl.noise_unit(64, 4096, seed=11, step=3)
    assert n.dtype == np.float32 and np.all(np.abs(n) < 1.0)
    k = n.astype(np.float64) * 2.0 ** 24
    assert np.all(k == np.rint(k)) and np.all(np.abs(k) % 2 == 1)          # odd multiples of 2^-24: exact in fp32, never 0
    flat = n.ravel().astype(np.float64)
    assert stats.kstest(flat, stats.uniform(loc=-1, scale=2).cdf).pvalue > 1e-3
    assert abs(flat.mean()) < 4 * (1 / np.sqrt(3)) / np.sqrt(flat.size)
    assert abs(flat.var() - 1 / 3) < 5e-3
    # rows, steps and seeds are different streams; the same arguments give the same values
    assert abs(np.corrcoef(n[0], n[1])[0, 1]) < 0.06
    assert abs(np.corrcoef(n[0], hl.noise_unit(1, 4096, 11, 4)[0])[0, 1]) < 0.06
    assert abs(np.corrcoef(n[0], hl.noise_unit(1, 4096, 12, 3)[0])[0, 1]) < 0.06
    np.testing.assert_array_equal(n, hl.noise_unit(64, 4096, 11, 3))
    # row 65536 + r uses the sequence field: not a repeat of row r
    far = hl.noise_unit(65538, 8, 11, 3)
    assert not np.array_equal(far[65536], far[0])


def test_noisy_features_stay_within_the_amplitude_in_fp32():
    rng = np.random.default_rng(0)
    f = rng.standard_normal((8, 512)).astype(np.float32)
    g = hl.feature_noise(f, seed=1, step=0)
    assert g.dtype == np.float32
    diff = g.astype(np.float64) - f.astype(np.float64)
    assert np.all(np.abs(diff) <= 0.1 + 2.0 ** -22) and np.abs(diff).max() > 0.09
    # fl(f + fl(a n)) with a = fl32(0.1): recomputed in float64 and rounded once per operation
    a = np.float64(np.float32(0.1))
    prod = (a * hl.noise_unit(8, 512, 1, 0).astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(g, (f.astype(np.float64) + prod.astype(np.float64)).astype(np.float32))
    np.testing.assert_array_equal(hl.feature_noise(f, 1, 0, amplitude=0.0), f)
