"""Python binding of libeagle (argument marshalling only -- every step of the path runs in the HIP library).

PyTorch is used for device memory (the workspace, staging of weights) and the stream, nothing else.
The names mirror the C ABI in include/eagle.h.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeagle.so")

EAGLE_F32, EAGLE_BF16 = 0, 1
HEAD_LAYER = -1
(W_EMBED, W_LM_HEAD, W_FINAL_NORM, W_FC, W_FC_BIAS, W_ATTN_NORM, W_Q, W_K, W_V, W_O, W_MLP_NORM, W_ROUTER,
 W_GATE, W_UP, W_DOWN) = range(15)
(BUF_LOGITS, BUF_FEATURES, BUF_DRAFT_LOGITS, BUF_DRAFT_FEATURES, BUF_TREE_TOKENS, BUF_TOKENS, BUF_VANILLA_LOGITS,
 BUF_STATE, BUF_KV_ROW, BUF_GEMM_TRACE, BUF_PREFILL_FEATURES) = range(11)

_LAYER_IDS = {"attn_norm": W_ATTN_NORM, "wq": W_Q, "wk": W_K, "wv": W_V, "wo": W_O, "mlp_norm": W_MLP_NORM,
              "router": W_ROUTER, "gate": W_GATE, "up": W_UP, "down": W_DOWN}
_GLOBAL_IDS = {"embed": W_EMBED, "lm_head": W_LM_HEAD, "final_norm": W_FINAL_NORM, "head.fc_w": W_FC,
               "head.fc_b": W_FC_BIAS}

EXPORTS = ["eagle_workspace_bytes", "eagle_init", "eagle_free", "eagle_load_weight", "eagle_reset", "eagle_prefill",
           "eagle_draft_tree", "eagle_verify", "eagle_accept", "eagle_accept_static", "eagle_step", "eagle_vanilla_step", "eagle_generate",
           "eagle_set_hint", "eagle_set_page_table", "eagle_set_buffer", "eagle_force_tree", "eagle_expand_level",
           "eagle_force_accept", "eagle_get_buffer", "eagle_get_kv_row", "eagle_set_profiling", "eagle_get_profile", "eagle_get_kernel_stats", "eagle_probe_stream_read",
           "eagle_head_loss", "eagle_feature_noise", "eagle_last_error", "eagle_version"]


class EagleConfig(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("d_ffn", ctypes.c_int32), ("vocab", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("experts_per_tok", ctypes.c_int32), ("draft_moe", ctypes.c_int32), ("rms_eps", ctypes.c_float),
                ("rope_theta", ctypes.c_float), ("max_batch", ctypes.c_int32), ("max_seq", ctypes.c_int32),
                ("page_tokens", ctypes.c_int32), ("n_nodes", ctypes.c_int32),
                ("parent", ctypes.POINTER(ctypes.c_int32)), ("rank", ctypes.POINTER(ctypes.c_int32)),
                ("temperature", ctypes.c_float), ("seed", ctypes.c_uint64), ("weight_bits", ctypes.c_int32),
                ("head_loss_rows", ctypes.c_int32)]


class EagleProfile(ctypes.Structure):
    _fields_ = [("draft_ms", ctypes.c_double), ("verify_ms", ctypes.c_double), ("accept_ms", ctypes.c_double),
                ("steps", ctypes.c_int64), ("gemm_ms", ctypes.c_double), ("gemm_launches", ctypes.c_int64),
                ("gemm_weight_bytes", ctypes.c_double), ("verify_weight_bytes", ctypes.c_double),
                ("verify_kv_bytes", ctypes.c_double)]


class EagleKernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 16), ("kernel", ctypes.c_char * 48), ("ms", ctypes.c_double),
                ("launches", ctypes.c_int64), ("bytes", ctypes.c_double)]


class EagleError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libeagle error {code}: {text}")
        self.code = code


_lib = None


def load_library(need_gpu_runtime: bool = True):
    """dlopen libeagle.so.  torch is imported first so that the HIP runtime it ships is the one in the process."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(there is no fallback path)")
    if need_gpu_runtime:
        import torch  # noqa: F401  (loads libamdhip64)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    pi32 = ctypes.POINTER(ctypes.c_int32)
    lib.eagle_workspace_bytes.argtypes = [ctypes.POINTER(EagleConfig)]
    lib.eagle_workspace_bytes.restype = sz
    lib.eagle_init.argtypes = [ctypes.POINTER(EagleConfig), vp, sz, vp, ctypes.POINTER(vp)]
    lib.eagle_free.argtypes = [vp]
    lib.eagle_free.restype = None
    lib.eagle_load_weight.argtypes = [vp, i32, i32, vp]
    lib.eagle_reset.argtypes = [vp]
    lib.eagle_prefill.argtypes = [vp, i32, pi32, i32, pi32]
    lib.eagle_draft_tree.argtypes = [vp, pi32]
    lib.eagle_verify.argtypes = [vp]
    lib.eagle_accept.argtypes = [vp, pi32, pi32, pi32]
    lib.eagle_step.argtypes = [vp, pi32, pi32, pi32]
    lib.eagle_accept_static.argtypes = [vp, pi32, pi32, pi32]
    lib.eagle_vanilla_step.argtypes = [vp, pi32]
    lib.eagle_generate.argtypes = [vp, i32, pi32, i32, i32, pi32, pi32, ctypes.POINTER(ctypes.c_float)]
    lib.eagle_set_hint.argtypes = [vp, i32, pi32, i32, ctypes.c_float, ctypes.c_float, ctypes.c_uint64]
    lib.eagle_get_buffer.argtypes = [vp, i32, i32, vp, sz]
    lib.eagle_set_page_table.argtypes = [vp, pi32]
    lib.eagle_set_buffer.argtypes = [vp, i32, i32, vp, sz]
    lib.eagle_force_tree.argtypes = [vp, i32, pi32]
    lib.eagle_expand_level.argtypes = [vp, i32]
    lib.eagle_force_accept.argtypes = [vp, pi32, pi32, pi32]
    lib.eagle_get_kv_row.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
    lib.eagle_set_profiling.argtypes = [vp, i32]
    lib.eagle_get_profile.argtypes = [vp, ctypes.POINTER(EagleProfile), i32]
    lib.eagle_get_kernel_stats.argtypes = [vp, i32, ctypes.POINTER(EagleKernelStat), i32, pi32, i32]
    lib.eagle_probe_stream_read.argtypes = [vp, sz, i32, vp, ctypes.POINTER(ctypes.c_double)]
    lib.eagle_head_loss.argtypes = [vp, vp, vp, i32, ctypes.c_float, vp, ctypes.POINTER(ctypes.c_float)]
    lib.eagle_feature_noise.argtypes = [vp, vp, vp, i32, ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64]
    lib.eagle_last_error.restype = ctypes.c_char_p
    lib.eagle_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _p32(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def make_config(shape, parent, rank, *, max_batch=1, max_seq=4096, page_tokens=64, temperature=0.0, seed=0,
                kv_dtype="fp32", weight_bits=16, head_loss_rows=0):
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    rank = np.ascontiguousarray(rank, dtype=np.int32)
    cfg = EagleConfig(dtype=EAGLE_F32 if shape.dtype == "fp32" else EAGLE_BF16,
                      kv_dtype=EAGLE_F32 if kv_dtype == "fp32" else EAGLE_BF16, n_layers=shape.n_layers,
                      d_model=shape.d_model, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                      head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab, n_experts=shape.n_experts,
                      experts_per_tok=shape.experts_per_tok, draft_moe=int(shape.draft_moe), rms_eps=shape.rms_eps,
                      rope_theta=shape.rope_theta, max_batch=max_batch, max_seq=max_seq, page_tokens=page_tokens,
                      n_nodes=len(parent), parent=_p32(parent), rank=_p32(rank), temperature=temperature, seed=seed,
                      weight_bits=weight_bits, head_loss_rows=head_loss_rows)
    cfg._keep = (parent, rank)
    return cfg


def probe_stream_read(nbytes: int, iters: int = 10, device="cuda:0") -> float:
    """GB/s of a bare streaming read of `nbytes` bytes of device memory (the practical HBM ceiling)."""
    import torch
    lib = load_library()
    buf = torch.ones(nbytes // 4, dtype=torch.int32, device=device)
    gbs = ctypes.c_double()
    rc = lib.eagle_probe_stream_read(buf.data_ptr(), buf.numel() * 4, iters, torch.cuda.current_stream(buf.device).cuda_stream, ctypes.byref(gbs))
    if rc != 0:
        raise EagleError(rc, lib.eagle_last_error().decode())
    return float(gbs.value)


class Eagle:
    """One libeagle context on cuda:0 (ROCm).  Methods are the C calls, with numpy in/out."""

    def __init__(self, shape, parent, rank, *, max_batch=1, max_seq=4096, page_tokens=64, temperature=0.0, seed=0,
                 kv_dtype="fp32", weight_bits=16, head_loss_rows=0, device="cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("libeagle needs a GPU (no CPU fallback exists)")
        self.shape, self.device = shape, torch.device(device)
        self.cfg = make_config(shape, parent, rank, max_batch=max_batch, max_seq=max_seq, page_tokens=page_tokens,
                               temperature=temperature, seed=seed, kv_dtype=kv_dtype, weight_bits=weight_bits,
                               head_loss_rows=head_loss_rows)
        self.weight_bits = weight_bits
        self.M = len(parent)
        depth = [0] * self.M
        for v in range(1, self.M):
            depth[v] = depth[int(parent[v])] + 1
        self.D = max(depth)
        self.max_batch = max_batch
        need = self.lib.eagle_workspace_bytes(ctypes.byref(self.cfg))
        if need == 0:
            raise EagleError(-1, self.lib.eagle_last_error().decode())
        self.workspace_bytes = need
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.stream = torch.cuda.current_stream(self.device)
        h = ctypes.c_void_p()
        self._chk(self.lib.eagle_init(ctypes.byref(self.cfg), base, need, self.stream.cuda_stream, ctypes.byref(h)))
        self.h = h
        self.n_active = 0

    def _chk(self, rc: int) -> None:
        if rc != 0:
            raise EagleError(rc, self.lib.eagle_last_error().decode())

    def close(self) -> None:
        if getattr(self, "h", None):
            self.lib.eagle_free(self.h)
            self.h = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- training loss of the head (Sec. 3.2)
    def head_loss(self, f: np.ndarray, fhat: np.ndarray, w_cls: float = 0.1, want_grad: bool = True):
        """(L, L_reg, L_cls), dL/dfhat (numpy fp32 [rows, d] or None) for label features f and predictions fhat."""
        torch = self.torch
        tf = torch.from_numpy(np.ascontiguousarray(f, dtype=np.float32)).to(self.device)
        th = torch.from_numpy(np.ascontiguousarray(fhat, dtype=np.float32)).to(self.device)
        if tf.shape != th.shape or tf.dim() != 2 or tf.shape[1] != self.shape.d_model:
            raise ValueError("f and fhat must both be [rows, d_model]")
        tg = torch.empty_like(tf) if want_grad else None
        out = (ctypes.c_float * 3)()
        self._chk(self.lib.eagle_head_loss(self.h, tf.data_ptr(), th.data_ptr(), int(tf.shape[0]), float(w_cls),
                                           tg.data_ptr() if want_grad else None, out))
        return (float(out[0]), float(out[1]), float(out[2])), (tg.cpu().numpy() if want_grad else None)

    def head_loss_device(self, tf, th, tg, w_cls: float = 0.1):
        """The same call on tensors already on the device (fp32, contiguous, [rows, d_model]); tg may be None."""
        out = (ctypes.c_float * 3)()
        self._chk(self.lib.eagle_head_loss(self.h, tf.data_ptr(), th.data_ptr(), int(tf.shape[0]), float(w_cls),
                                           tg.data_ptr() if tg is not None else None, out))
        return float(out[0]), float(out[1]), float(out[2])

    def feature_noise(self, f: np.ndarray, seed: int, step: int, amplitude: float = 0.1) -> np.ndarray:
        torch = self.torch
        tf = torch.from_numpy(np.ascontiguousarray(f, dtype=np.float32)).to(self.device)
        self._chk(self.lib.eagle_feature_noise(self.h, tf.data_ptr(), tf.data_ptr(), int(tf.shape[0]), float(amplitude), int(seed), int(step)))
        self.torch.cuda.synchronize(self.device)
        return tf.cpu().numpy()

    # -- weights
    def load_weight(self, which: int, layer: int, host: np.ndarray) -> None:
        """Stage one host tensor on the device (torch), hand it to the library, release the staging copy."""
        torch = self.torch
        t = torch.from_numpy(np.ascontiguousarray(host))
        if t.dtype == torch.uint16:
            t = t.view(torch.int16)
        dev = t.to(self.device, non_blocking=False)
        self._chk(self.lib.eagle_load_weight(self.h, which, layer, dev.data_ptr()))
        torch.cuda.current_stream(self.device).synchronize()
        del dev

    def load_named(self, name: str, host: np.ndarray) -> None:
        if name in _GLOBAL_IDS:
            self.load_weight(_GLOBAL_IDS[name], 0, host)
            return
        parts = name.split(".")
        if parts[0] == "layers":
            self.load_weight(_LAYER_IDS[parts[2]], int(parts[1]), host)
        elif parts[0] == "head" and parts[1] == "layer":
            self.load_weight(_LAYER_IDS[parts[2]], HEAD_LAYER, host)
        else:
            raise KeyError(name)

    def load_weights(self, named) -> None:
        """named: iterable of (name, host array) in the model's dtype (fp32, or raw bf16 bits as uint16;
        norm gains and the FC bias always fp32)."""
        items = named.items() if isinstance(named, dict) else named
        for name, arr in items:
            self.load_named(name, arr)

    # -- sequences
    def reset(self) -> None:
        self._chk(self.lib.eagle_reset(self.h))
        self.n_active = 0

    def prefill(self, seq: int, prompt: Sequence[int]) -> int:
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        first = ctypes.c_int32()
        self._chk(self.lib.eagle_prefill(self.h, seq, _p32(p), len(p), ctypes.byref(first)))
        s = self.shape
        chunk = 512 if (s.dtype == "bf16" and s.d_ffn % 64 == 0 and (s.n_heads * s.head_dim) % 64 == 0) else 128
        if self.weight_bits == 4:
            chunk = 32
        self.last_prefill_rows = (len(p) - 1) % chunk + 1          # rows of the prompt's last pass
        self.n_active = max(self.n_active, seq + 1)
        return int(first.value)

    def set_hint(self, seq: int, future: Sequence[int], alpha: float, bias: float, seed: int) -> None:
        f = np.ascontiguousarray(future, dtype=np.int32)
        self._chk(self.lib.eagle_set_hint(self.h, seq, _p32(f), len(f), alpha, bias, seed))

    def draft_tree(self) -> np.ndarray:
        out = np.zeros((self.n_active, self.M), np.int32)
        self._chk(self.lib.eagle_draft_tree(self.h, _p32(out)))
        return out

    def verify(self) -> None:
        self._chk(self.lib.eagle_verify(self.h))

    def _results(self, fn):
        toks = np.zeros((self.n_active, self.D + 1), np.int32)
        lens = np.zeros(self.n_active, np.int32)
        path = np.zeros((self.n_active, self.D + 1), np.int32)
        self._chk(fn(self.h, _p32(toks), _p32(lens), _p32(path)))
        return toks, lens, path

    def accept(self):
        return self._results(self.lib.eagle_accept)

    def accept_static(self):
        return self._results(self.lib.eagle_accept_static)

    def step(self):
        return self._results(self.lib.eagle_step)

    def vanilla_step(self) -> np.ndarray:
        out = np.zeros(self.n_active, np.int32)
        self._chk(self.lib.eagle_vanilla_step(self.h, _p32(out)))
        return out

    def generate(self, prompt: Sequence[int], max_new: int):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.zeros(max_new, np.int32)
        n = ctypes.c_int32()
        tau = ctypes.c_float()
        self._chk(self.lib.eagle_generate(self.h, 0, _p32(p), len(p), max_new, _p32(out), ctypes.byref(n), ctypes.byref(tau)))
        self.n_active = 1
        return out[:n.value].copy(), float(tau.value)

    # -- injection
    @property
    def pages_per_slot(self) -> int:
        return (self.cfg.max_seq + self.cfg.page_tokens - 1) // self.cfg.page_tokens

    def set_page_table(self, table: Sequence[int]) -> None:
        t = np.ascontiguousarray(table, dtype=np.int32)
        if t.size != self.max_batch * self.pages_per_slot:
            raise ValueError("page table must hold max_batch * pages_per_slot entries")
        self._chk(self.lib.eagle_set_page_table(self.h, _p32(t)))

    def set_buffer(self, which: int, arr: np.ndarray, seq: int = 0) -> None:
        dt = np.int32 if which == BUF_TREE_TOKENS else np.float32
        a = np.ascontiguousarray(arr, dtype=dt)
        self._chk(self.lib.eagle_set_buffer(self.h, which, seq, a.ctypes.data, a.nbytes))

    def force_tree(self, seq: int, tokens: Sequence[int]) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        if t.size != self.M:
            raise ValueError("one token per tree node")
        self._chk(self.lib.eagle_force_tree(self.h, seq, _p32(t)))

    def expand_level(self, level: int) -> None:
        self._chk(self.lib.eagle_expand_level(self.h, level))

    def force_accept(self, paths, lens, bonus) -> None:
        """paths: one list of node indices per active slot (starting with 0)."""
        D1 = self.D + 1
        p = np.zeros((self.n_active, D1), np.int32)
        for s, pth in enumerate(paths):
            p[s, :len(pth)] = pth
        ln = np.ascontiguousarray(lens, dtype=np.int32)
        bo = np.ascontiguousarray(bonus, dtype=np.int32)
        self._chk(self.lib.eagle_force_accept(self.h, _p32(p), _p32(ln), _p32(bo)))

    # -- buffers
    def get_buffer(self, which: int, seq: int = 0) -> np.ndarray:
        V, d, M = self.shape.vocab, self.shape.d_model, self.M
        if which in (BUF_LOGITS, BUF_DRAFT_LOGITS):
            out = np.empty((M, V), np.float32)
        elif which in (BUF_FEATURES, BUF_DRAFT_FEATURES):
            out = np.empty((M, d), np.float32)
        elif which == BUF_TREE_TOKENS:
            out = np.empty(M, np.int32)
        elif which == BUF_VANILLA_LOGITS:
            out = np.empty(V, np.float32)
        elif which == BUF_STATE:
            out = np.empty(4, np.int32)
        elif which == BUF_TOKENS:
            n = int(self.get_buffer(BUF_STATE, seq)[0])
            out = np.empty(n, np.int32)
        elif which == BUF_GEMM_TRACE:
            out = np.zeros((1024, 8), np.uint64)
        elif which == BUF_PREFILL_FEATURES:
            rows = self.last_prefill_rows
            out = np.empty((rows, d), np.float32)
        else:
            raise ValueError(which)
        self._chk(self.lib.eagle_get_buffer(self.h, which, seq, out.ctypes.data, out.nbytes))
        return out

    def get_kv_row(self, seq: int, layer: int, pos: int):
        n = self.shape.n_kv_heads * self.shape.head_dim
        k = np.empty(n, np.float32)
        v = np.empty(n, np.float32)
        fp = ctypes.POINTER(ctypes.c_float)
        self._chk(self.lib.eagle_get_kv_row(self.h, seq, layer, pos, k.ctypes.data_as(fp), v.ctypes.data_as(fp)))
        return k, v

    def set_profiling(self, mode: int) -> None:
        self._chk(self.lib.eagle_set_profiling(self.h, mode))

    def get_profile(self, reset: bool = True) -> Dict[str, float]:
        p = EagleProfile()
        self._chk(self.lib.eagle_get_profile(self.h, ctypes.byref(p), int(reset)))
        return {f: getattr(p, f) for f, _ in p._fields_}

    def get_kernel_stats(self, phase: int, reset: bool = True):
        """Mode-2 timing per class of launch: list of dicts (name, kernel, ms, launches, bytes)."""
        arr = (EagleKernelStat * 16)()
        n = ctypes.c_int32()
        self._chk(self.lib.eagle_get_kernel_stats(self.h, phase, arr, 16, ctypes.byref(n), int(reset)))
        return [{"name": arr[i].name.decode(), "kernel": arr[i].kernel.decode(), "ms": arr[i].ms,
                 "launches": int(arr[i].launches), "bytes": arr[i].bytes} for i in range(n.value)]
