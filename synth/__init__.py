"""Seeded synthetic inputs for the EAGLE hot path: model shapes, draft-tree shapes, weights, prompts.

This module serves BOTH the CPU oracle's tests and the HIP path's tests / bench.  It contains no
arithmetic of the method (no norms, no attention, no sampling rule): only shapes and a
counter-based number generator, so that the two sides can be fed identical bits.

Value rule for every generated tensor element (integer-exact up to one fp64 multiply-add):
    h   = mix64(mix64(seed ^ (tid+1)*GOLDEN) + index)
    z   = QTABLE[h >> 48]          # 65536-point standard-normal quantile table
    val = float32(z*std + mean)    # bf16 formats then round-to-nearest-even
The C implementation (gen.c, OpenMP) is used when libsynth.so is built; the numpy implementation
below is the same rule and is the fallback (and the cross-check in tests).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field, replace
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

_qtable: Optional[np.ndarray] = None
_lib = None


def qtable() -> np.ndarray:
    """Standard-normal quantiles at (j+0.5)/65536, fp64."""
    global _qtable
    if _qtable is None:
        from scipy.special import ndtri
        _qtable = np.ascontiguousarray(ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0))
    return _qtable


def build(force: bool = False) -> str:
    """Compile gen.c into libsynth.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None and os.path.exists(_LIB_PATH):
        lib = ctypes.CDLL(_LIB_PATH)
        u64, dbl, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        for name in ("synth_normal_f32", "synth_normal_bf16", "synth_normal_bf16_as_f32"):
            getattr(lib, name).argtypes = [vp, u64, u64, u64, u64, dbl, dbl, vp]
            getattr(lib, name).restype = None
        lib.synth_tokens.argtypes = [u64, u64, u64, u64, ctypes.c_uint32, vp]
        lib.synth_tokens.restype = None
        _lib = lib
    return _lib


# ----------------------------------------------------------------------------- numpy rule
def _mix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = x + _GOLDEN
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        return x ^ (x >> np.uint64(31))


def _base(seed: int, tid: int) -> np.uint64:
    with np.errstate(over="ignore"):
        return _mix64(np.array([np.uint64(seed) ^ (np.uint64(tid + 1) * _GOLDEN)], dtype=np.uint64))[0]


def _bf16_round_bits(f32: np.ndarray) -> np.ndarray:
    u = f32.view(np.uint32).astype(np.uint64)
    u = u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    return (u >> np.uint64(16)).astype(np.uint16)


def normal_numpy(seed: int, tid: int, start: int, count: int, std: float, mean: float, fmt: str) -> np.ndarray:
    with np.errstate(over="ignore"):
        idx = _base(seed, tid) + (np.uint64(start) + np.arange(count, dtype=np.uint64))
    h = _mix64(idx)
    z = qtable()[(h >> np.uint64(48)).astype(np.int64)]
    v = (z * std + mean).astype(np.float32)
    if fmt == "f32":
        return v
    bits = _bf16_round_bits(v)
    if fmt == "bf16":
        return bits
    if fmt == "bf16_f32":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(fmt)


def normal(seed: int, tid: int, count: int, std: float, mean: float = 0.0, fmt: str = "f32",
           start: int = 0, out: Optional[np.ndarray] = None) -> np.ndarray:
    """count elements of tensor `tid` starting at element `start`.
    fmt: 'f32' | 'bf16' (raw uint16 bit patterns) | 'bf16_f32' (bf16-rounded values held as fp32)."""
    lib = _load()
    dt = np.uint16 if fmt == "bf16" else np.float32
    if out is None:
        out = np.empty(count, dtype=dt)
    assert out.dtype == dt and out.size == count and out.flags.c_contiguous
    if lib is None:
        out[...] = normal_numpy(seed, tid, start, count, std, mean, fmt).reshape(out.shape)
        return out
    fn = {"f32": lib.synth_normal_f32, "bf16": lib.synth_normal_bf16, "bf16_f32": lib.synth_normal_bf16_as_f32}[fmt]
    fn(qtable().ctypes.data, seed, tid, start, count, float(std), float(mean), out.ctypes.data)
    return out


def tokens(seed: int, tid: int, count: int, vocab: int, start: int = 0) -> np.ndarray:
    """Token ids uniform on [0, vocab)."""
    with np.errstate(over="ignore"):
        idx = _base(seed, tid) + (np.uint64(start) + np.arange(count, dtype=np.uint64))
    return ((_mix64(idx) >> np.uint64(16)) % np.uint64(vocab)).astype(np.int32)


# ----------------------------------------------------------------------------- model shapes
@dataclass(frozen=True)
class ModelShape:
    name: str
    dtype: str                 # 'fp32' | 'bf16'  (weight storage + GEMM input type)
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_experts: int = 0
    experts_per_tok: int = 0
    draft_moe: bool = False
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def twin(self, n_layers: int = 2) -> "ModelShape":
        """Reduced-depth twin: identical widths, fewer target layers."""
        return replace(self, name=f"{self.name}-L{n_layers}", n_layers=n_layers)


SHAPES: Dict[str, ModelShape] = {
    "tiny": ModelShape("tiny", "fp32", 2, 256, 4, 4, 64, 688, 1024),
    "llama2-7b": ModelShape("llama2-7b", "bf16", 32, 4096, 32, 32, 128, 11008, 32000),
    "llama2-13b": ModelShape("llama2-13b", "bf16", 40, 5120, 40, 40, 128, 13824, 32000),
    "llama2-70b": ModelShape("llama2-70b", "bf16", 80, 8192, 64, 8, 128, 28672, 32000),
    "mixtral-8x7b": ModelShape("mixtral-8x7b", "bf16", 32, 4096, 32, 8, 128, 14336, 32000,
                               n_experts=8, experts_per_tok=2, draft_moe=True),
    # small stand-ins used by CPU-side tests (not paper configs)
    "mini-gqa": ModelShape("mini-gqa", "bf16", 2, 256, 8, 2, 32, 384, 512),
    "mini-moe": ModelShape("mini-moe", "bf16", 2, 256, 8, 2, 32, 320, 512, n_experts=4, experts_per_tok=2,
                           draft_moe=True),
    # the tiny model with the LLaMA vocabulary (child selection / acceptance over 32000 entries at small cost) and with
    # a vocabulary beyond 32768 entries
    "tiny-v32k": ModelShape("tiny-v32k", "fp32", 2, 256, 4, 4, 64, 688, 32000),
    "tiny-v40k": ModelShape("tiny-v40k", "fp32", 2, 256, 4, 4, 64, 688, 40000),
}

# ----------------------------------------------------------------------------- draft trees
# A tree is given by each drafted node's "rank path": the child ranks followed from the root.
# Node 0 is the root (the last committed token); the others are numbered in BFS order.
_T26 = ["0", "1", "2", "3",
        "00", "01", "02", "10", "11", "20", "30",
        "000", "001", "002", "010", "011", "100", "200",
        "0000", "0001", "0010", "0100",
        "00000", "00001", "00010"]
_T15 = ["0", "1",
        "00", "01", "10", "11",
        "000", "001", "010", "100",
        "0000", "0001", "0010", "0100"]
_T10 = ["0", "1", "00", "01", "10", "11", "000", "001", "010", "100"]   # 10 drafted tokens in 3 draft passes
_CHAIN5 = ["0", "00", "000", "0000", "00000"]
_T8 = ["0", "1", "00", "01", "10", "000", "0000"]   # 8 nodes with the root, depth 4: four sequences fill one 32-row verify pass


def tree_from_paths(paths: List[str]) -> Tuple[np.ndarray, np.ndarray]:
    """-> (parent[int32 M], rank[int32 M]) with node 0 = root (parent -1, rank 0), BFS order."""
    order = sorted(paths, key=lambda p: (len(p), p))
    index = {"": 0}
    parent = [-1]
    rank = [0]
    for p in order:
        index[p] = len(parent)
        parent.append(index[p[:-1]])
        rank.append(int(p[-1]))
    return np.asarray(parent, np.int32), np.asarray(rank, np.int32)


def _full_binary(depth: int) -> List[str]:
    out, level = [], [""]
    for _ in range(depth):
        level = [p + c for p in level for c in "01"]
        out += level
    return out


TREES: Dict[str, Tuple[np.ndarray, np.ndarray]] = {
    "T26": tree_from_paths(_T26),
    "T15": tree_from_paths(_T15),
    "T10": tree_from_paths(_T10),
    "chain5": tree_from_paths(_CHAIN5),
    "T8": tree_from_paths(_T8),
    "root": tree_from_paths([]),             # degenerate: no drafts at all, a step is one vanilla step
    "B63": tree_from_paths(_full_binary(5)),  # full binary tree of depth 5: 63 nodes (more rows than one 32-row pass)
}


# ----------------------------------------------------------------------------- weights
_LAYER_FIELDS = ["attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "router", "gate", "up", "down"]


def _layer_specs(s: ModelShape, moe: bool) -> List[Tuple[str, Tuple[int, ...], float, float]]:
    d, hq, hk, f = s.d_model, s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim, s.d_ffn
    out = [("attn_norm", (d,), 0.02, 1.0), ("wq", (hq, d), 0.02, 0.0), ("wk", (hk, d), 0.02, 0.0),
           ("wv", (hk, d), 0.02, 0.0), ("wo", (d, hq), 0.02, 0.0), ("mlp_norm", (d,), 0.02, 1.0)]
    if moe:
        e = s.n_experts
        out += [("router", (e, d), d ** -0.5, 0.0), ("gate", (e, f, d), 0.02, 0.0),
                ("up", (e, f, d), 0.02, 0.0), ("down", (e, d, f), 0.02, 0.0)]
    else:
        out += [("gate", (f, d), 0.02, 0.0), ("up", (f, d), 0.02, 0.0), ("down", (d, f), 0.02, 0.0)]
    return out


def tensor_specs(s: ModelShape, head_recipe: str = "scaled") -> List[Tuple[str, int, Tuple[int, ...], float, float]]:
    """All tensors of target + EAGLE head: (name, tid, shape, std, mean).
    Matrices are row-major [out_features, in_features], N(0, 0.02) except the head's FC; norm gains ~ N(1, 0.02);
    FC bias ~ N(0, 0.02).  head_recipe "scaled" (default) keeps the head's features at the target's scale;
    "literal" draws every head matrix from N(0, 0.02) like the target's."""
    if head_recipe not in ("scaled", "literal"):
        raise ValueError(head_recipe)
    literal = head_recipe == "literal"
    specs = [("embed", 1, (s.vocab, s.d_model), 0.02, 0.0),
             ("lm_head", 2, (s.vocab, s.d_model), 0.02, 0.0),
             ("final_norm", 3, (s.d_model,), 0.02, 1.0),
             # std (2d)^-1/2: the FC output keeps the scale of its input, as a trained head's features keep the scale of
             # the target's; with 0.02 the head's feature norm grows 1.8-2.6x per tree level (fan-in 2d)
             ("head.fc_w", 4, (s.d_model, 2 * s.d_model), 0.02 if literal else (2 * s.d_model) ** -0.5, 0.0),
             ("head.fc_b", 5, (s.d_model,), 0.02, 0.0)]
    for li in range(s.n_layers):
        for k, (nm, shp, std, mean) in enumerate(_layer_specs(s, s.n_experts > 0)):
            specs.append((f"layers.{li}.{nm}", 1024 + li * 16 + _LAYER_FIELDS.index(nm), shp, std, mean))
    for nm, shp, std, mean in _layer_specs(s, s.n_experts > 0 and s.draft_moe):
        # the head has no final norm, so its residual branches are scaled down (output projections with gain 1/4):
        # f-hat then has the scale of the target's normalised feature, which is what a trained head regresses to
        if nm in ("wo", "down") and not literal:
            std = 0.25 * shp[-1] ** -0.5
        specs.append((f"head.layer.{nm}", 512 + _LAYER_FIELDS.index(nm), shp, std, mean))
    return specs


def is_vector(name: str) -> bool:
    return name.endswith("_norm") or name.endswith("fc_b")


def gen_tensor(s: ModelShape, seed: int, spec, fmt: str) -> np.ndarray:
    """One tensor in format fmt ('f32' | 'bf16' | 'bf16_f32').  Norm gains and the FC bias are always
    returned as fp32 arrays; under a bf16 model their VALUES are bf16-rounded."""
    name, tid, shp, std, mean = spec
    n = int(np.prod(shp))
    if is_vector(name) and fmt == "bf16":
        fmt = "bf16_f32"
    return normal(seed, tid, n, std, mean, fmt).reshape(shp)


def iter_weights(s: ModelShape, seed: int, fmt: str, head_recipe: str = "scaled") -> Iterator[Tuple[str, np.ndarray]]:
    for spec in tensor_specs(s, head_recipe):
        yield spec[0], gen_tensor(s, seed, spec, fmt)


def make_weights(s: ModelShape, seed: int, fmt: str, head_recipe: str = "scaled") -> Dict[str, np.ndarray]:
    return dict(iter_weights(s, seed, fmt, head_recipe))


def oracle_fmt(s: ModelShape) -> str:
    return "f32" if s.dtype == "fp32" else "bf16_f32"


def device_fmt(s: ModelShape) -> str:
    return "f32" if s.dtype == "fp32" else "bf16"


def prompt(seed: int, n: int, vocab: int, stream: int = 0) -> np.ndarray:
    return tokens(seed, 7000 + stream, n, vocab)


def head_param_count(s: ModelShape) -> int:
    """Matrix parameters of the Autoregression Head (FC + one decoder layer), biases/gains excluded."""
    tot = 0
    for name, _, shp, _, _ in tensor_specs(s):
        if name.startswith("head.") and not is_vector(name):
            tot += int(np.prod(shp))
    return tot
