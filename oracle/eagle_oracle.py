"""CPU oracle for one EAGLE speculative-decoding step (arXiv 2401.15077).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP path and never calls it.

Plain numpy, one sequence at a time, no blocking / fusion / caching tricks: every function is the
paper's step written out.  Arithmetic runs in `dtype` (float64 for small models; float32 for the
LLaMA-sized shapes, where float64 copies of the weights would not fit the host's memory).

What follows which passage:
  * target forward, feature f = hidden state fed to the LM head, p = LM_Head(f)      -- Sec. 2 "Notations"
  * draft model: shared embedding, concat(feature, shifted-token embedding), FC 2d->d, one decoder
    layer, shared LM head, autoregression on (predicted feature, drawn token)          -- Sec. 3.1
  * tree draft: depth-m tree from m draft forwards with tree attention; greedy children are the
    top-k tokens, non-greedy children are k sampled tokens                              -- Sec. 3.1, App. A.1
  * verification: one target forward over all tree tokens with tree attention, then speculative
    sampling applied recursively at every node; accepted tokens AND their features are kept for the
    next draft phase                                                                    -- Sec. 3.3
  * multi-round speculative sampling                                                    -- App. A.2, Alg. 1
  * chain rule min(1, p/q), resample from norm(max(0, p-q))                             -- Sec. 2 "Speculative sampling"

Readings where the paper is silent or garbled:
  * decoder layer = LLaMA-style pre-norm block (RMSNorm, rotate-half RoPE, GQA, SwiGLU / top-2 MoE)
  * the feature is taken AFTER the final RMSNorm (it is what the LM head consumes); the head's output
    goes to the LM head without a further norm
  * draft row i pairs feature f[i] with token x[i+1] and uses RoPE position i
  * non-greedy children are drawn WITHOUT replacement (Gumbel-top-k == sequential renormalised draws);
    Alg. 1 is run with the renormalised q_i each t_i was actually drawn from
  * the residual line of Alg. 1 is read vector-wise: p <- norm(max(0, p - q_i))
  * accept test r < p/q is evaluated as r*q < p; ties in argmax / top-k go to the lowest token id
  * uniforms come from a counter-based integer generator (24-bit dyadic fractions, exact in fp32)
  * the paper says nothing about KV storage; a bf16 model keeps its KV cache in bf16, so with
    kv_store="bf16" every K/V row is rounded to bf16 (nearest-even) when it is written to the cache --
    a storage code both sides must produce identically -- and read back as that value

  * inverse-CDF draws carry the running sum in float64 whatever `dtype` is (a float32 running sum over
    a LLaMA-sized vocabulary is uncertain by more than many bins are wide)

PARITY UNPINNED (no value in the paper to compare with): the default tree shapes (the paper's tree
figure is not available in text form).  The layer arithmetic (attention scale, GQA map, tree mask,
RoPE, SwiGLU, MoE routing), the head over a tree, the stochastic tree builder and the acceptance rules
are pinned by tests/test_oracle_pins.py and tests/test_oracle_pins_layer.py against worked examples,
closed forms, enumeration and invariants, each with a planted mistake shown to fail.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

# ----------------------------------------------------------------------------- counter-based uniforms
_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
PURPOSE_ACCEPT, PURPOSE_FINAL, PURPOSE_GUMBEL, PURPOSE_HINT = 1, 2, 3, 4


def _mix64(x: int) -> int:
    x = (x + _GOLDEN) & _MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK
    return x ^ (x >> 31)


def u24(seed: int, purpose: int, step: int, seq: int, node: int, idx: int) -> int:
    """24-bit integer k; the uniform is k * 2^-24 (accept tests, final sample) or (k+0.5) * 2^-24 (Gumbel)."""
    a = _mix64((seed ^ (purpose * _GOLDEN)) & _MASK)
    b = _mix64((a + step) & _MASK)
    c = _mix64(b ^ ((seq << 48) | (node << 32) | idx))
    return c >> 40


def _u24_vec(seed: int, purpose: int, step: int, seq: int, node: int, n: int) -> np.ndarray:
    """u24 for idx = 0..n-1 (vectorised, same integers as u24)."""
    a = _mix64((seed ^ (purpose * _GOLDEN)) & _MASK)
    b = _mix64((a + step) & _MASK)
    x = np.uint64(b) ^ (np.uint64((seq << 48) | (node << 32)) | np.arange(n, dtype=np.uint64))
    with np.errstate(over="ignore"):
        x = x + np.uint64(_GOLDEN)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        x = x ^ (x >> np.uint64(31))
    return (x >> np.uint64(40)).astype(np.int64)


# ----------------------------------------------------------------------------- static tree
class Tree:
    """Static draft tree: node 0 = root (last committed token), BFS numbering, children ordered by rank."""

    def __init__(self, parent: Sequence[int], rank: Sequence[int]):
        self.parent = [int(p) for p in parent]
        self.rank = [int(r) for r in rank]
        self.M = len(self.parent)
        if self.M < 1 or self.parent[0] != -1:
            raise ValueError("node 0 must be the root with parent -1")
        self.depth = [0] * self.M
        self.children: List[List[int]] = [[] for _ in range(self.M)]
        for v in range(1, self.M):
            p = self.parent[v]
            if not (0 <= p < v):
                raise ValueError("parents must precede children (BFS order)")
            self.depth[v] = self.depth[p] + 1
            if self.depth[v] < self.depth[v - 1]:
                raise ValueError("nodes must be in BFS (non-decreasing depth) order")
            self.children[p].append(v)
        for v in range(self.M):
            self.children[v].sort(key=lambda c: self.rank[c])
            if [self.rank[c] for c in self.children[v]] != list(range(len(self.children[v]))):
                raise ValueError("sibling ranks must be 0..k-1")
        self.D = max(self.depth)

    def ancestors_or_self(self, v: int) -> List[int]:
        out = []
        while v >= 0:
            out.append(v)
            v = self.parent[v]
        return out[::-1]

    def level_rows(self, d: int) -> List[int]:
        """Rows of draft pass d+1 (d >= 1): depth-d nodes that have children."""
        return [v for v in range(self.M) if self.depth[v] == d and self.children[v]]


# ----------------------------------------------------------------------------- elementary pieces
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return (x / np.sqrt(ms + x.dtype.type(eps))) * g


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate-half RoPE.  x [R, heads, dh]; pos [R].  Angles are formed in fp64, then cast."""
    dh = x.shape[-1]
    half = dh // 2
    inv = np.power(np.float64(theta), -np.arange(half, dtype=np.float64) * 2.0 / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to bfloat16, returned in x's dtype (the value a bf16 cache entry holds)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16) << np.uint64(16)
    return u.astype(np.uint32).view(np.float32).astype(x.dtype)


def softmax(z: np.ndarray) -> np.ndarray:
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1 + np.exp(-x))


def topk_desc(scores: np.ndarray, k: int) -> List[int]:
    """Indices of the k largest entries, descending; equal scores -> lowest index first."""
    order = np.lexsort((np.arange(scores.size), -scores))
    return [int(i) for i in order[:k]]


def argmax_low(scores: np.ndarray) -> int:
    return int(np.argmax(scores))          # numpy returns the first (lowest-index) maximum


def top2_gap(scores: np.ndarray) -> float:
    if scores.size < 2:
        return math.inf
    two = np.partition(scores, -2)[-2:]
    return float(two[1] - two[0])


# --- Alg. 1 pieces, kept separate so tests can enumerate them
def accept_test(r: float, p_t, q_t) -> bool:
    """Accept with probability min(1, p(t)/q(t)): r < p/q evaluated without the division."""
    return bool(np.asarray(r, dtype=np.asarray(p_t).dtype) * q_t < p_t)


def residual(p: np.ndarray, q: np.ndarray) -> np.ndarray:
    """norm(max(0, p - q)), vector-wise; if nothing is left (p == q, a probability-zero branch) keep p."""
    r = np.maximum(p - q, 0)
    s = r.sum()
    if not s > 1e-20:
        return p
    return r / s


def drop_and_renorm(q: np.ndarray, t: int) -> np.ndarray:
    """Proposal for the next sibling when drawing without replacement: q with token t removed."""
    q = q.copy()
    q[t] = 0
    s = q.sum()
    return q / s if s > 0 else q


def sample_inverse_cdf(p: np.ndarray, u: float) -> int:
    """Smallest x with cumsum(p)[x] > u * sum(p).  The running sum is ALWAYS carried in fp64, whatever p's dtype: a
    vocabulary of 32000 entries has bins of ~3e-5, which an fp32 running sum (error ~1e-5) cannot resolve, so the
    draw would depend on the order of the additions instead of on p."""
    c = np.cumsum(p, dtype=np.float64)
    x = int(np.searchsorted(c, float(u) * c[-1], side="right"))
    return min(x, p.size - 1)


def multi_round(p: np.ndarray, ts: Sequence[int], qs: Sequence[np.ndarray], rs: Sequence[float]):
    """Alg. 1 up to (not including) the final draw.
    -> (index i of the accepted candidate or None, residual target distribution, trace of (p(t_i), q_i(t_i)))."""
    trace = []
    for i, (t, q, r) in enumerate(zip(ts, qs, rs)):
        trace.append((float(p[t]), float(q[t])))
        if accept_test(r, p[t], q[t]):
            return i, p, trace
        p = residual(p, q)
    return None, p, trace


# ----------------------------------------------------------------------------- the model
class Oracle:
    def __init__(self, shape, weights: Dict[str, np.ndarray], parent, rank, *, temperature: float = 0.0,
                 seed: int = 0, seq_id: int = 0, max_seq: int = 4096, dtype=np.float64, kv_store: Optional[str] = None):
        self.s = shape
        self.dt = np.dtype(dtype).type
        self.W = {k: np.asarray(v, dtype=dtype) for k, v in weights.items()}
        self.tree = Tree(parent, rank)
        self.T = float(temperature)
        if kv_store not in (None, "bf16"):
            raise ValueError("kv_store must be None (cache holds the computed values) or 'bf16'")
        self.kv_store = kv_store
        self.seed, self.seq_id, self.step = int(seed), int(seq_id), 0
        s = shape
        self.kc = [np.zeros((max_seq, s.n_kv_heads, s.head_dim), dtype) for _ in range(s.n_layers)]
        self.vc = [np.zeros((max_seq, s.n_kv_heads, s.head_dim), dtype) for _ in range(s.n_layers)]
        self.dkc = np.zeros((max_seq, s.n_kv_heads, s.head_dim), dtype)
        self.dvc = np.zeros((max_seq, s.n_kv_heads, s.head_dim), dtype)
        self.x: List[int] = []                 # committed tokens; the last one is the root, not yet in the target cache
        self.pending_f: List[np.ndarray] = []  # target features not yet consumed by the draft head
        self.hint = None                       # (future tokens by absolute index, alpha, bias, seed)
        self.forced_experts = None             # optional {(stage, layer): int array [rows, k]} for lock-step runs
        self.router_log: Dict[Tuple[str, int], np.ndarray] = {}

    # -- layer --------------------------------------------------------------------------------------
    def _lw(self, prefix: str, name: str) -> np.ndarray:
        return self.W[f"{prefix}.{name}"]

    def _mlp(self, prefix: str, x: np.ndarray, moe: bool, stage_key) -> np.ndarray:
        if not moe:
            g = x @ self._lw(prefix, "gate").T
            u = x @ self._lw(prefix, "up").T
            return (silu(g) * u) @ self._lw(prefix, "down").T
        k = self.s.experts_per_tok
        logits = x @ self._lw(prefix, "router").T                      # [R, E]
        self.router_log[stage_key] = logits
        out = np.zeros_like(x)
        for r in range(x.shape[0]):
            if self.forced_experts is not None and stage_key in self.forced_experts:
                sel = [int(e) for e in self.forced_experts[stage_key][r]]
            else:
                sel = topk_desc(logits[r], k)
            w = softmax(logits[r, sel])
            for wi, e in zip(w, sel):
                g = x[r] @ self._lw(prefix, "gate")[e].T
                u = x[r] @ self._lw(prefix, "up")[e].T
                out[r] += wi * ((silu(g) * u) @ self._lw(prefix, "down")[e].T)
        return out

    def _layer(self, prefix: str, h: np.ndarray, pos: np.ndarray, kc: np.ndarray, vc: np.ndarray,
               slots: np.ndarray, visible: np.ndarray, moe: bool, stage_key) -> np.ndarray:
        """One pre-norm decoder layer on rows h [R, d].  New K/V rows go to cache slots `slots`;
        visible[r, t] says whether row r may attend cache slot t (t < visible.shape[1])."""
        s = self.s
        R = h.shape[0]
        x = rmsnorm(h, self._lw(prefix, "attn_norm"), s.rms_eps)
        q = rope((x @ self._lw(prefix, "wq").T).reshape(R, s.n_heads, s.head_dim), pos, s.rope_theta)
        k = rope((x @ self._lw(prefix, "wk").T).reshape(R, s.n_kv_heads, s.head_dim), pos, s.rope_theta)
        v = (x @ self._lw(prefix, "wv").T).reshape(R, s.n_kv_heads, s.head_dim)
        kc[slots] = round_bf16(k) if self.kv_store == "bf16" else k
        vc[slots] = round_bf16(v) if self.kv_store == "bf16" else v
        Tn = visible.shape[1]
        group = s.n_heads // s.n_kv_heads
        scale = self.dt(1.0 / math.sqrt(s.head_dim))
        att = np.empty((R, s.n_heads, s.head_dim), dtype=h.dtype)
        for hd in range(s.n_heads):
            kv = hd // group
            sc = (q[:, hd, :] @ kc[:Tn, kv, :].T) * scale
            sc = np.where(visible, sc, -np.inf)
            att[:, hd, :] = softmax(sc) @ vc[:Tn, kv, :]
        h = h + att.reshape(R, s.n_heads * s.head_dim) @ self._lw(prefix, "wo").T
        x = rmsnorm(h, self._lw(prefix, "mlp_norm"), s.rms_eps)
        return h + self._mlp(prefix, x, moe, stage_key)

    def _target_forward(self, toks: Sequence[int], pos: np.ndarray, slots: np.ndarray, visible: np.ndarray,
                        stage: str):
        """Embedding -> all target layers -> final norm = features F; logits = LM_Head(F)."""
        h = self.W["embed"][np.asarray(toks, dtype=np.int64)]
        for li in range(self.s.n_layers):
            h = self._layer(f"layers.{li}", h, pos, self.kc[li], self.vc[li], slots, visible,
                            self.s.n_experts > 0, (stage, li))
        F = rmsnorm(h, self.W["final_norm"], self.s.rms_eps)
        return F, F @ self.W["lm_head"].T

    def _head_forward(self, feats: np.ndarray, toks: Sequence[int], pos: np.ndarray, slots: np.ndarray,
                      visible: np.ndarray, stage: str) -> np.ndarray:
        """Autoregression Head: FC(concat(feature, emb(token))) -> one decoder layer.  Returns predicted features."""
        e = self.W["embed"][np.asarray(toks, dtype=np.int64)]
        z = np.concatenate([feats, e], axis=-1) @ self.W["head.fc_w"].T
        if "head.fc_b" in self.W:
            z = z + self.W["head.fc_b"]
        return self._layer("head.layer", z, pos, self.dkc, self.dvc, slots, visible,
                           self.s.n_experts > 0 and self.s.draft_moe, (stage, -1))

    # -- token choice -------------------------------------------------------------------------------
    def _uniform(self, purpose: int, node: int, idx: int = 0) -> float:
        return u24(self.seed, purpose, self.step, self.seq_id, node, idx) * 2.0 ** -24

    def _choose(self, logits: np.ndarray, node: int) -> Tuple[int, float]:
        """Token from the target distribution at `node` (greedy: argmax).  -> (token, decision margin)."""
        if self.T == 0.0:
            return argmax_low(logits), top2_gap(logits)
        p = softmax(logits / self.dt(self.T))
        u = self._uniform(PURPOSE_FINAL, node)
        return sample_inverse_cdf(p, u), self._cdf_margin(p, u)

    @staticmethod
    def _cdf_margin(p: np.ndarray, u: float) -> float:
        """Distance of the drawn point to the nearest boundary of the drawn token's bin, relative to the bin's width."""
        c = np.cumsum(p, dtype=np.float64)
        target = float(u) * c[-1]
        x = min(int(np.searchsorted(c, target, side="right")), p.size - 1)
        lo = c[x - 1] if x > 0 else 0.0
        return float(min(target - lo, c[x] - target) / max(float(p[x]), 1e-300))

    # -- life cycle ---------------------------------------------------------------------------------
    @property
    def ctx(self) -> int:
        """Number of positions in the target KV cache (= committed tokens minus the root)."""
        return len(self.x) - 1

    def prefill(self, prompt: Sequence[int]) -> int:
        P = len(prompt)
        pos = np.arange(P)
        causal = np.tril(np.ones((P, P), dtype=bool))
        F, L = self._target_forward(prompt, pos, pos, causal, "prefill")
        self.prefill_features, self.prefill_logits = F, L
        self.step = 0                                     # the first token is draw number 0
        first, self.first_margin = self._choose(L[P - 1], 0)
        self.x = [int(t) for t in prompt] + [first]
        if P > 1:   # draft rows 0..P-2: (f[i], x[i+1])
            self._head_forward(F[:P - 1], self.x[1:P], pos[:P - 1], pos[:P - 1], causal[:P - 1, :P - 1], "dprefill")
        self.pending_f = [F[P - 1]]
        self.step = 1
        return first

    def set_hint(self, future: Sequence[int], alpha: float, bias: float, seed: int) -> None:
        """Acceptance knob of the synthetic workload: future[i] is the token the target will emit at
        absolute index i.  A draft node whose path so far follows `future` gets, at the next position pos,
        +bias on logit future[pos] when hash(seed,pos) < alpha and -bias otherwise."""
        self.hint = ([int(t) for t in future], float(alpha), float(bias), int(seed))

    def _hinted(self, logits: np.ndarray, on_path: bool, pos: int) -> Tuple[np.ndarray, Optional[int]]:
        if self.hint is None or not on_path:
            return logits, None
        fut, alpha, bias, hseed = self.hint
        if pos >= len(fut):
            return logits, None
        hit = np.float32(u24(hseed, PURPOSE_HINT, 0, self.seq_id, 0, pos) * 2.0 ** -24) < np.float32(alpha)
        out = logits.copy()
        out[fut[pos]] += self.dt(bias) if hit else -self.dt(bias)
        return out, fut[pos]

    def draft_tree(self, forced_tokens: Optional[Sequence[int]] = None) -> dict:
        """Expand the static tree with the Autoregression Head (Sec. 3.1, App. A.1).
        forced_tokens (lock-step runs): use these tokens instead of the oracle's own choices; every slot
        where they differ is reported with the oracle's score gap between the two candidates."""
        tr, n, ctx, V = self.tree, len(self.x), self.ctx, self.s.vocab
        a1 = len(self.pending_f)
        tok = [0] * tr.M
        tok[0] = self.x[-1]
        on_path = [False] * tr.M
        on_path[0] = self.hint is not None and n - 1 < len(self.hint[0]) and self.hint[0][n - 1] == tok[0]
        node_f: Dict[int, np.ndarray] = {}
        node_logits: Dict[int, np.ndarray] = {}
        node_scores: Dict[int, np.ndarray] = {}
        node_adj: Dict[int, np.ndarray] = {}
        mismatches = []

        def expand(v: int) -> None:
            kids = tr.children[v]
            logit = node_logits[v]
            pos_child = n + tr.depth[v]                     # absolute index of the children's token
            adj, hinted_tok = self._hinted(logit, on_path[v], pos_child)
            node_adj[v] = adj
            if self.T == 0.0:
                score = adj
            else:
                k24 = _u24_vec(self.seed, PURPOSE_GUMBEL, self.step, self.seq_id, v, V)
                uu = ((k24.astype(np.float64) + 0.5) * 2.0 ** -24).astype(adj.dtype)
                score = adj / self.dt(self.T) - np.log(-np.log(uu))
            node_scores[v] = score
            pick = topk_desc(score, len(kids))
            for r, c in enumerate(kids):
                t = pick[r]
                if forced_tokens is not None and int(forced_tokens[c]) != t:
                    g = int(forced_tokens[c])
                    mismatches.append((v, r, t, g, float(score[t] - score[g])))
                    t = g
                tok[c] = t
                on_path[c] = hinted_tok is not None and t == hinted_tok

        # pass 1: the pending (feature, shifted token) pairs, ending with the root pair
        p0 = ctx - a1                                        # draft rows already in the draft cache
        pos = np.arange(p0, ctx)
        vis = np.zeros((a1, ctx), dtype=bool)
        for i in range(a1):
            vis[i, :p0 + i + 1] = True
        out = self._head_forward(np.stack(self.pending_f), self.x[p0 + 1:ctx + 1], pos, pos, vis, "draft0")
        node_f[0] = out[-1]
        node_logits[0] = out[-1] @ self.W["lm_head"].T
        expand(0)
        # passes 2..D: depth-d nodes that have children; node v sits at draft slot ctx-1+v
        for d in range(1, tr.D):
            rows = tr.level_rows(d)
            if not rows:
                break
            feats = np.stack([node_f[tr.parent[v]] for v in rows])
            pos = np.full(len(rows), ctx - 1 + d)
            slots = np.asarray([ctx - 1 + v for v in rows])
            vis = np.zeros((len(rows), ctx - 1 + tr.M), dtype=bool)
            for i, v in enumerate(rows):
                vis[i, :ctx] = True                          # committed draft rows, root pair included
                for u in tr.ancestors_or_self(v)[1:]:
                    vis[i, ctx - 1 + u] = True
            out = self._head_forward(feats, [tok[v] for v in rows], pos, slots, vis, f"draft{d}")
            for i, v in enumerate(rows):
                node_f[v] = out[i]
                node_logits[v] = out[i] @ self.W["lm_head"].T
                expand(v)
        self.tok, self.node_f, self.node_logits, self.node_scores = tok, node_f, node_logits, node_scores
        self.node_adj = node_adj                             # the logits each node's children were drawn from
        return {"tokens": list(tok), "features": node_f, "logits": node_logits, "scores": node_scores,
                "mismatches": mismatches}

    def verify(self) -> Tuple[np.ndarray, np.ndarray]:
        """One target forward over all tree nodes with tree attention (Sec. 3.3)."""
        tr, ctx = self.tree, self.ctx
        pos = np.asarray([ctx + tr.depth[v] for v in range(tr.M)])
        slots = np.arange(ctx, ctx + tr.M)
        vis = np.zeros((tr.M, ctx + tr.M), dtype=bool)
        vis[:, :ctx] = True
        for v in range(tr.M):
            for u in tr.ancestors_or_self(v):
                vis[v, ctx + u] = True
        self.F, self.L = self._target_forward(self.tok, pos, slots, vis, "verify")
        return self.F, self.L

    def accept(self) -> dict:
        """Walk the tree from the root.  Greedy: follow the child whose token equals the target's argmax.
        Non-greedy: Alg. 1 at every node over its children in rank order, then one draw from what is left.
        -> path (node indices, path[0] = 0), emitted tokens (accepted drafts + one bonus), decision margin."""
        tr = self.tree
        cur, path, margin = 0, [0], math.inf
        self.trace = []                                      # ('test', node, p(t), q(t)) / ('final', node, p)
        if self.T == 0.0:
            while True:
                g = argmax_low(self.L[cur])
                margin = min(margin, top2_gap(self.L[cur]))
                nxt = [c for c in tr.children[cur] if self.tok[c] == g]
                if not nxt:
                    bonus = g
                    break
                cur = nxt[0]
                path.append(cur)
        else:
            T = self.dt(self.T)
            while True:
                p = softmax(self.L[cur] / T)
                kids = tr.children[cur]
                accepted = None
                if kids:
                    q = softmax(self.node_adj[cur] / T)
                    for c in kids:
                        t = self.tok[c]
                        r = self._uniform(PURPOSE_ACCEPT, c)
                        self.trace.append(("test", c, float(p[t]), float(q[t])))
                        lhs = np.asarray(r, dtype=p.dtype) * q[t]
                        margin = min(margin, abs(float(lhs - p[t])) / max(float(p[t]), float(lhs), 1e-30))
                        if accept_test(r, p[t], q[t]):
                            accepted = c
                            break
                        p = residual(p, q)
                        q = drop_and_renorm(q, t)
                if accepted is None:
                    self.trace.append(("final", cur, p.copy()))
                    u = self._uniform(PURPOSE_FINAL, cur)
                    bonus = sample_inverse_cdf(p, u)
                    margin = min(margin, self._cdf_margin(p, u))
                    break
                cur = accepted
                path.append(cur)
        emitted = [self.tok[v] for v in path[1:]] + [int(bonus)]
        return {"path": path, "emitted": emitted, "bonus": int(bonus), "length": len(emitted), "margin": margin}

    def commit(self, path: Sequence[int], bonus: int) -> None:
        """Keep the accepted path: its KV rows move to contiguous slots, its features feed the next draft."""
        ctx = self.ctx
        for li in range(self.s.n_layers):
            for i, v in enumerate(path):
                self.kc[li][ctx + i] = self.kc[li][ctx + v]
                self.vc[li][ctx + i] = self.vc[li][ctx + v]
        self.pending_f = [self.F[v] for v in path]
        self.x += [self.tok[v] for v in path[1:]] + [int(bonus)]
        self.step += 1

    def spec_step(self) -> dict:
        self.draft_tree()
        self.verify()
        res = self.accept()
        self.commit(res["path"], res["bonus"])
        return res

    def vanilla_step(self) -> int:
        """Plain autoregression: the target run on the root alone, one token out."""
        ctx = self.ctx
        vis = np.ones((1, ctx + 1), dtype=bool)
        F, L = self._target_forward([self.x[-1]], np.asarray([ctx]), np.asarray([ctx]), vis, "vanilla")
        self.vanilla_logits = L[0]
        t, _ = self._choose(L[0], 0)
        self.x.append(int(t))
        self.pending_f = self.pending_f + [F[0]]
        self.step += 1
        return int(t)

    def generate(self, prompt: Sequence[int], max_new: int) -> Tuple[List[int], List[int]]:
        """-> (the first max_new generated tokens, accepted length of every step)."""
        P = len(prompt)
        self.prefill(prompt)
        lens = []
        while len(self.x) - P < max_new:
            lens.append(self.spec_step()["length"])
        return self.x[P:P + max_new], lens

    def generate_vanilla(self, prompt: Sequence[int], max_new: int) -> List[int]:
        P = len(prompt)
        self.prefill(prompt)
        while len(self.x) - P < max_new:
            self.vanilla_step()
        return self.x[P:P + max_new]
