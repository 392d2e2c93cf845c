"""CPU oracle for 4-bit weight storage (arXiv 2401.15077, Sec. 4.2: the gpt-fast case study runs the target and the
head with int4-quantised weights; Table 4 reports the tokens/s).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests/ and bench.py's cpu_baseline leg may import it.  It shares
no code with the HIP path.

The paper says nothing about the quantiser beyond "int4".  Reading taken here: weight-only, group-wise along the input dimension, symmetric:

    for every output row n and every group g of G = 128 consecutive input columns
        s[n, g]  = bf16( max_k |W[n, k]| / 7 )                      (round to nearest even; 0 if the group is all zero)
        q[n, k]  = clip( rint( W[n, k] / s[n, g] ), -8, 7 ) + 8      in {0, ..., 15}   (fp32 division, ties to even)
        W^[n, k] = s[n, g] * (q[n, k] - 8)                           (exact in fp32: an 8-bit times a 4-bit mantissa)

Activations are not quantised.  A model "with int4 weights" is the same model evaluated with W^ in place of W for
every weight MATRIX of the target's layers, the head's FC and layer, and the LM head; embedding rows, norm gains and
the FC bias keep their values.  The plain oracle (eagle_oracle.Oracle) run on `quantize_model(weights)` is therefore
the oracle of the int4 path: nothing else changes.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

GROUP = 128


def _round_bf16(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16) << np.uint64(16)
    return u.astype(np.uint32).view(np.float32)


def quantize(W: np.ndarray, group: int = GROUP):
    """W [N, K] (K a multiple of `group`) -> (codes uint8 [N, K] in 0..15, scales fp32 [N, K/group], bf16 values)."""
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    if K % group:
        raise ValueError("the input dimension must be a multiple of the group size")
    Wg = W.reshape(N, K // group, group)
    s = _round_bf16(np.max(np.abs(Wg), axis=2) / np.float32(7.0))
    safe = np.where(s > 0, s, np.float32(1.0))
    q = np.rint(Wg / safe[:, :, None])                  # fp32 division, ties to even
    q = np.clip(q, -8, 7).astype(np.int16) + 8
    return q.reshape(N, K).astype(np.uint8), s


def dequantize(q: np.ndarray, s: np.ndarray, group: int = GROUP) -> np.ndarray:
    N, K = q.shape
    w = (q.reshape(N, K // group, group).astype(np.float32) - np.float32(8.0)) * s[:, :, None]
    return w.reshape(N, K)


def is_quantized_tensor(name: str) -> bool:
    """Which tensors of a weight dictionary are stored in 4 bits: every matrix except the embedding and the router."""
    if name in ("embed", "final_norm", "head.fc_b") or name.endswith("_norm") or name.endswith(".router"):
        return False
    return True


def quantize_model(weights: Dict[str, np.ndarray], group: int = GROUP) -> Dict[str, np.ndarray]:
    """The weight dictionary of the model as the int4 path evaluates it (fp32 values W^)."""
    out = {}
    for name, w in weights.items():
        if is_quantized_tensor(name) and w.ndim >= 2:
            w2 = np.asarray(w, dtype=np.float32)
            flat = w2.reshape(-1, w2.shape[-1])
            q, s = quantize(flat, group)
            out[name] = dequantize(q, s, group).reshape(w2.shape)
        else:
            out[name] = w
    return out
