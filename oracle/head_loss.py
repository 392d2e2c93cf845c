"""CPU oracle for the training loss of the Autoregression Head (arXiv 2401.15077, Sec. 3.2 "Training of the draft
models"): the regression loss on the predicted feature, the classification loss on the token distribution the
frozen LM head makes of it, their weighted sum, the gradient of that sum with respect to the predicted feature, and
the uniform noise the section adds to the target's features as data augmentation.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests/ may import it.  It shares no code with the HIP path.

What the section fixes (notation as there; i runs over the positions of a training batch, "rows" below):

    L_reg = SmoothL1(f, f^)                       f  = target feature of the next position (the label),
    p  = softmax(LM_Head(f)),  p^ = softmax(LM_Head(f^))      f^ = the head's prediction of it
    L_cls = CrossEntropy(p, p^)
    L     = L_reg + w_cls * L_cls                 w_cls = 0.1
    augmentation: features of the target + U(-0.1, 0.1) noise

Readings where the section is silent:
  * Smooth L1 is the usual one with threshold 1: 0.5 x^2 for |x| < 1, |x| - 0.5 otherwise, averaged over every element
    of every row (rows * d terms).
  * Cross entropy with a distribution as the target: -sum_v p_v log p^_v per row, averaged over the rows.
  * The LM head is the target's and is frozen (Fig. "pipeline": modules of the target are not trained), so the only
    gradient is the one with respect to f^:
        dL/df^ = clip(f^ - f, -1, 1) / (rows * d)  +  w_cls / rows * (p^ - p) W        (W = LM head, [V, d])
    (derivative of the smooth L1 term is the clipped difference; of the cross entropy with respect to the logits of
    f^ it is p^ - p since sum_v p_v = 1).
  * Noise: element (row r, column k) of call `step` gets a * n with n = (2 (u24 - 2^23) + 1) / 2^24, u24 the 24-bit
    integer of the build's counter-based generator (purpose id 5, sequence field r >> 16, node field r & 0xFFFF, index
    k): an odd multiple of 2^-24 in (-1, 1), symmetric about 0, exact in fp32.  The sum is formed in fp32 (one
    rounded product, one rounded sum), which is what makes the noisy features a bit-exact function of their inputs.

Everything except `feature_noise` runs in float64.
"""
from __future__ import annotations

import numpy as np

from .eagle_oracle import _u24_vec

PURPOSE_NOISE = 5
W_CLS = 0.1
NOISE_AMPLITUDE = 0.1


def smooth_l1(x: np.ndarray) -> np.ndarray:
    """Elementwise Smooth L1 of a difference x (threshold 1)."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    return np.where(a < 1.0, 0.5 * x * x, a - 0.5)


def _log_softmax(z: np.ndarray) -> np.ndarray:
    z = z - z.max(axis=-1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))


def head_loss(f: np.ndarray, fhat: np.ndarray, W_lm: np.ndarray, w_cls: float = W_CLS) -> dict:
    """f, fhat [rows, d]; W_lm [V, d] -> {"L", "L_reg", "L_cls"} (Sec. 3.2)."""
    f = np.asarray(f, dtype=np.float64)
    fhat = np.asarray(fhat, dtype=np.float64)
    W = np.asarray(W_lm, dtype=np.float64)
    L_reg = float(smooth_l1(fhat - f).mean())
    p = np.exp(_log_softmax(f @ W.T))
    logq = _log_softmax(fhat @ W.T)
    L_cls = float((-(p * logq).sum(axis=1)).mean())
    return {"L": L_reg + w_cls * L_cls, "L_reg": L_reg, "L_cls": L_cls}


def head_loss_grad(f: np.ndarray, fhat: np.ndarray, W_lm: np.ndarray, w_cls: float = W_CLS) -> np.ndarray:
    """dL/dfhat [rows, d] of `head_loss` (the LM head and the labels are constants)."""
    f = np.asarray(f, dtype=np.float64)
    fhat = np.asarray(fhat, dtype=np.float64)
    W = np.asarray(W_lm, dtype=np.float64)
    rows, d = f.shape
    g_reg = np.clip(fhat - f, -1.0, 1.0) / (rows * d)
    p = np.exp(_log_softmax(f @ W.T))
    q = np.exp(_log_softmax(fhat @ W.T))
    g_cls = (q - p) @ W / rows
    return g_reg + w_cls * g_cls


def noise_unit(rows: int, d: int, seed: int, step: int) -> np.ndarray:
    """The generator's values n in (-1, 1) for a [rows, d] block, float32 (exact)."""
    out = np.empty((rows, d), dtype=np.float32)
    for r in range(rows):
        k24 = _u24_vec(seed, PURPOSE_NOISE, step, r >> 16, r & 0xFFFF, d)
        out[r] = ((2 * (k24 - (1 << 23)) + 1).astype(np.float64) * 2.0 ** -24).astype(np.float32)
    return out


def feature_noise(f: np.ndarray, seed: int, step: int, amplitude: float = NOISE_AMPLITUDE) -> np.ndarray:
    """f + U(-amplitude, amplitude) noise, float32 arithmetic: fl(f + fl(amplitude * n))."""
    f = np.asarray(f, dtype=np.float32)
    n = noise_unit(f.shape[0], f.shape[1], seed, step)
    return (f + np.float32(amplitude) * n).astype(np.float32)
