"""Pins for the parts of the CPU oracle that the whole-loop invariants cannot see (greedy == vanilla, tree == chains
and compacted == prefill hold for ANY decoder layer, and any draft is lossless):

  * SwiGLU orientation and the routed-expert weighting            -> hand-computed examples
  * softmax / SiLU                                                -> closed forms
  * attention scale 1/sqrt(dh), grouped-query head map, mask, RoPE positions on q AND k -> a worked example whose
    every number is written out with scalars
  * the head's tree mask and position ids (Sec. 3.1: tree attention in the draft phase) -> every root->leaf path of
    the draft tree re-run as an ordinary causal chain through the head
  * the head's (feature, shifted token) rows across prefill / commits -> one causal pass over the same pairs
  * non-greedy children (App. A.1 "we sample k tokens")           -> frequencies of Oracle.draft_tree's own children
    against enumerated sequential draws without replacement, at a temperature other than 1
  * temperature inside the recursive acceptance                   -> exact joint law at T = 2

Each pin is shown to be sensitive: either a planted mistake in a subclass of the oracle fails it, or the value a
plausible misreading would give is asserted to lie far from the oracle's.
"""
import math

import numpy as np
import pytest

import synth
from oracle import eagle_oracle as eo
from oracle.eagle_oracle import Oracle, Tree
from test_oracle_pins import draws_without_replacement

L3 = math.log(3.0)


def shape(**kw):
    base = dict(name="pin", dtype="fp32", n_layers=1, d_model=4, n_heads=2, n_kv_heads=1, head_dim=2, d_ffn=2, vocab=4,
                rms_eps=0.0, rope_theta=10000.0)
    base.update(kw)
    return synth.ModelShape(**base)


# ----------------------------------------------------------------------------- closed forms
def test_softmax_and_silu_closed_forms():
    np.testing.assert_allclose(eo.softmax(np.array([0.0, L3])), [0.25, 0.75], rtol=1e-15)
    np.testing.assert_allclose(eo.softmax(np.array([[1000.0, 1000.0 + L3], [-1000.0, -1000.0]])), [[0.25, 0.75], [0.5, 0.5]], rtol=1e-12)
    np.testing.assert_allclose(eo.softmax(np.array([0.0, -np.inf, 0.0])), [0.5, 0.0, 0.5])
    # silu(x) = x * sigmoid(x): sigmoid(ln 3) = 3/4, sigmoid(-ln 3) = 1/4
    np.testing.assert_allclose(eo.silu(np.array([0.0, L3, -L3])), [0.0, 0.75 * L3, -0.25 * L3], rtol=1e-15)


# ----------------------------------------------------------------------------- MLP
def test_dense_mlp_hand_example_pins_swiglu_orientation():
    """down( silu(gate x) * (up x) ) on a 2-wide example worked out by hand."""
    s = shape(d_model=2, n_heads=1, head_dim=2, d_ffn=2)
    W = {"l.gate": np.eye(2), "l.up": np.diag([2.0, 3.0]), "l.down": np.array([[1.0, 1.0], [0.0, 1.0]])}
    o = Oracle(s, W, [-1], [0], max_seq=4)
    x = np.array([[L3, -L3]])
    # gate x = (L, -L); up x = (2L, -3L); silu(gate) = (3L/4, -L/4); product = (3L^2/2, 3L^2/4); down -> (9L^2/4, 3L^2/4)
    want = np.array([[2.25 * L3 * L3, 0.75 * L3 * L3]])
    np.testing.assert_allclose(o._mlp("l", x, False, ("t", 0)), want, rtol=1e-14)
    # the misreading silu(up x) * (gate x) gives something else on this example
    g, u = x @ W["l.gate"].T, x @ W["l.up"].T
    swapped = (eo.silu(u) * g) @ W["l.down"].T
    assert np.abs(swapped - want).max() > 0.3


def test_moe_hand_example_pins_top2_and_weighting():
    """Router logits (0, ln 3, -ln 2): experts 1 and 0 are selected, weights softmax over the SELECTED logits =
    (3/4, 1/4); the third expert must not contribute and must not enter the normalisation."""
    s = shape(d_model=2, n_heads=1, head_dim=2, d_ffn=2, n_experts=3, experts_per_tok=2)
    x = np.array([[1.0, 0.0], [0.0, 1.0]])
    router = np.array([[0.0, L3], [L3, 0.0], [-math.log(2.0), -50.0]])      # row 0: (0, L3, -ln2); row 1: (L3, 0, -50)
    # expert e: gate = identity * ln 3 on the row's hot coordinate, up = c_e * identity, down = identity
    c = [2.0, 5.0, 1000.0]
    W = {"l.router": router, "l.gate": np.stack([L3 * np.eye(2)] * 3), "l.up": np.stack([ce * np.eye(2) for ce in c]),
         "l.down": np.stack([np.eye(2)] * 3)}
    o = Oracle(s, W, [-1], [0], max_seq=4)
    out = o._mlp("l", x, True, ("t", 0))
    # row 0 = e_0: expert e gives silu(L3) * c_e on coordinate 0 = (3 L3 / 4) c_e; weights: expert 1 -> 3/4, expert 0 -> 1/4
    unit = 0.75 * L3
    np.testing.assert_allclose(out[0], [unit * (0.75 * c[1] + 0.25 * c[0]), 0.0], rtol=1e-14)
    # row 1 = e_1: logits (L3, 0, -50): expert 0 -> 3/4, expert 1 -> 1/4
    np.testing.assert_allclose(out[1], [0.0, unit * (0.75 * c[0] + 0.25 * c[1])], rtol=1e-14)
    # misreadings: softmax over ALL experts without renormalising (weights 3/4.5 and 1/4.5), or unweighted sum
    assert abs(unit * (3 / 4.5 * c[1] + 1 / 4.5 * c[0]) - out[0, 0]) > 0.3
    assert abs(unit * (c[1] + c[0]) - out[0, 0]) > 1.0
    # forced experts (lock-step runs) replace the selection but not the weighting rule
    o.forced_experts = {("t", 0): np.array([[2, 0], [0, 1]])}
    out2 = o._mlp("l", x, True, ("t", 0))
    w2 = np.exp([-math.log(2.0), 0.0]); w2 /= w2.sum()
    np.testing.assert_allclose(out2[0, 0], unit * (w2[0] * c[2] + w2[1] * c[0]), rtol=1e-13)


# ----------------------------------------------------------------------------- attention
def _attention_example():
    """4 query heads on 2 KV heads, head_dim 2 (one rotate-half pair turning by `pos` radians), three new rows at
    positions 5, 6, 6 in slots 5, 6, 7 of a cache that already holds five rows; row 1 and row 2 are siblings: both
    see row 0 but not each other.  W_o = identity and the MLP is switched off, so the layer's output minus its input
    is the attention output itself."""
    s = shape(d_model=8, n_heads=4, n_kv_heads=2, head_dim=2, d_ffn=2)
    rng = np.random.default_rng(42)
    W = {"l.attn_norm": np.ones(8), "l.mlp_norm": np.ones(8), "l.wq": rng.standard_normal((8, 8)),
         "l.wk": rng.standard_normal((4, 8)), "l.wv": rng.standard_normal((4, 8)), "l.wo": np.eye(8),
         "l.gate": np.zeros((2, 8)), "l.up": np.zeros((2, 8)), "l.down": np.zeros((8, 2))}
    h = rng.choice([-1.0, 1.0], size=(3, 8))                      # rms = 1, eps = 0: the normalised rows are h itself
    kc = np.zeros((8, 2, 2)); vc = np.zeros((8, 2, 2))
    kc[:5] = rng.standard_normal((5, 2, 2)); vc[:5] = rng.standard_normal((5, 2, 2))
    pos = np.array([5, 6, 6]); slots = np.array([5, 6, 7])
    vis = np.zeros((3, 8), dtype=bool)
    vis[:, :5] = True
    vis[0, 5] = True
    vis[1, [5, 6]] = True
    vis[2, [5, 7]] = True
    vis[:, 3] = False                                             # a cached row nobody may see (mask on cached slots)
    return s, W, h, kc, vc, pos, slots, vis


def _attention_by_scalars(W, h, kc, vc, pos, slots, vis, *, scale=None, head_map=None, use_mask=True, rope_k=True):
    """The worked example with every number written out: plane rotations by `pos` radians, dot products, exponentials."""
    n_heads, n_kv, dh = 4, 2, 2
    scale = 1.0 / math.sqrt(dh) if scale is None else scale
    head_map = (lambda hd: hd // (n_heads // n_kv)) if head_map is None else head_map
    kc = kc.copy(); vc = vc.copy()

    def rot(a, b, ang):                                           # the pair (a, b) = elements (i, i + dh/2) turns by ang
        return a * math.cos(ang) - b * math.sin(ang), b * math.cos(ang) + a * math.sin(ang)

    R = h.shape[0]
    q = [[None] * n_heads for _ in range(R)]
    for r in range(R):
        for hd in range(n_heads):
            a = sum(W["l.wq"][2 * hd, j] * h[r, j] for j in range(8)); b = sum(W["l.wq"][2 * hd + 1, j] * h[r, j] for j in range(8))
            q[r][hd] = rot(a, b, float(pos[r]))                   # theta^(-0) = 1: the angle is the position itself
        for kv in range(n_kv):
            a = sum(W["l.wk"][2 * kv, j] * h[r, j] for j in range(8)); b = sum(W["l.wk"][2 * kv + 1, j] * h[r, j] for j in range(8))
            kc[slots[r], kv] = rot(a, b, float(pos[r])) if rope_k else (a, b)
            vc[slots[r], kv] = [sum(W["l.wv"][2 * kv + t, j] * h[r, j] for j in range(8)) for t in range(2)]
    out = np.zeros((R, 8))
    for r in range(R):
        for hd in range(n_heads):
            kv = head_map(hd)
            ts = [t for t in range(8) if (vis[r, t] or not use_mask)]
            sc = [(q[r][hd][0] * kc[t, kv, 0] + q[r][hd][1] * kc[t, kv, 1]) * scale for t in ts]
            mx = max(sc)
            e = [math.exp(x - mx) for x in sc]
            for t, w in zip(ts, e):
                out[r, 2 * hd] += w / sum(e) * vc[t, kv, 0]
                out[r, 2 * hd + 1] += w / sum(e) * vc[t, kv, 1]
    return out


def test_attention_worked_example_pins_scale_gqa_map_mask_and_positions():
    s, W, h, kc, vc, pos, slots, vis = _attention_example()
    o = Oracle(s, W, [-1], [0], max_seq=8)
    got = o._layer("l", h, pos, kc.copy(), vc.copy(), slots, vis, False, ("t", 0)) - h
    want = _attention_by_scalars(W, h, kc, vc, pos, slots, vis)
    np.testing.assert_allclose(got, want, atol=1e-12)
    # the example tells the plausible misreadings apart
    for wrong in (dict(scale=1.0), dict(scale=0.5), dict(head_map=lambda hd: hd % 2), dict(use_mask=False), dict(rope_k=False)):
        assert np.abs(_attention_by_scalars(W, h, kc, vc, pos, slots, vis, **wrong) - want).max() > 1e-2, wrong


def test_rope_position_enters_attention_only_as_a_difference():
    """Shifting every position (cached rows included) by the same amount leaves the layer's output unchanged: the
    reading "row i of the head uses position i" is therefore only a convention; what matters -- and what the chain
    tests below pin -- is that positions are CONSISTENT between passes."""
    s, W, h, kc, vc, pos, slots, vis = _attention_example()
    o = Oracle(s, W, [-1], [0], max_seq=8)
    # cache rows 0..4 hold keys that were rotated at positions 0..4; rebuild them at positions 3..7
    raw = kc[:5].copy()
    k0 = eo.rope(raw, np.arange(5), s.rope_theta); k3 = eo.rope(raw, np.arange(5) + 3, s.rope_theta)
    a = kc.copy(); a[:5] = k0
    b = kc.copy(); b[:5] = k3
    out_a = o._layer("l", h, pos, a, vc.copy(), slots, vis, False, ("t", 0))
    out_b = o._layer("l", h, pos + 3, b, vc.copy(), slots, vis, False, ("t", 0))
    np.testing.assert_allclose(out_a, out_b, atol=1e-12)


# ----------------------------------------------------------------------------- the head's tree passes
def _drafted(tree="T15", seed=7, temperature=0.0, steps=2, cls=Oracle):
    s = synth.SHAPES["tiny"]
    W = synth.make_weights(s, seed, "f32")
    par, rk = synth.TREES[tree]
    prompt = synth.prompt(seed, 12, s.vocab)
    future = list(prompt) + Oracle(s, W, par, rk, max_seq=128).generate_vanilla(prompt, 40)
    o = cls(s, W, par, rk, max_seq=128, temperature=temperature, seed=5)
    if temperature == 0.0:
        o.set_hint(future, 0.8, 30.0, 3)                   # several tokens accepted per step -> several pending rows
    o.prefill(prompt)
    for _ in range(steps):
        o.spec_step()
    return s, W, o


def _head_chain_mismatch(s, W, o):
    """Largest difference between the tree draft's node features and the same nodes computed as plain causal chains."""
    d = o.draft_tree()
    tr, ctx = o.tree, o.ctx
    worst = 0.0
    for leaf in [v for v in range(tr.M) if not tr.children[v]]:
        chain = tr.ancestors_or_self(leaf)[1:]               # drafted nodes root -> leaf (the root itself is pass 1's last row)
        inner = [v for v in chain if tr.children[v]]         # nodes that are rows of a level pass
        if not inner:
            continue
        p = Oracle(s, W, o.tree.parent, o.tree.rank, max_seq=128)
        p.dkc[:ctx] = o.dkc[:ctx]; p.dvc[:ctx] = o.dvc[:ctx]  # the committed head rows, root pair included
        # An ordinary causal continuation: the i-th new row sits at slot ctx + i AND has position ctx + i, sees every
        # earlier row.  Its input pairs the previous row's output feature with the node's token (Sec. 3.1).
        n = len(inner)
        feats = np.stack([d["features"][tr.parent[v]] for v in inner])
        pos = np.arange(ctx, ctx + n)
        vis = np.zeros((n, ctx + n), dtype=bool)
        for i in range(n):
            vis[i, :ctx + i + 1] = True
        out = p._head_forward(feats, [d["tokens"][v] for v in inner], pos, pos, vis, "chain")
        for i, v in enumerate(inner):
            worst = max(worst, float(np.abs(out[i] - d["features"][v]).max()))
            worst = max(worst, float(np.abs(out[i] @ W["lm_head"].T.astype(np.float64) - d["logits"][v]).max()))
    return worst


@pytest.mark.parametrize("tree", ["T15", "T26"])
def test_head_tree_draft_equals_running_each_chain(tree):
    """Sec. 3.1: tree attention lets one head pass serve every branch -- a node's predicted feature must equal what the
    plain autoregressive chain root -> node gives.  Pins the head's tree mask, its cache slots and its position ids."""
    s, W, o = _drafted(tree)
    assert len(o.pending_f) >= 2
    assert _head_chain_mismatch(s, W, o) < 1e-11


@pytest.mark.parametrize("mistake", ["pos+1", "pos=ctx+depth-2", "sees_sibling", "misses_parent"])
def test_planted_head_mask_or_position_mistakes_break_the_chain_pin(mistake):
    class Planted(Oracle):
        def _head_forward(self, feats, toks, pos, slots, visible, stage):
            if stage.startswith("draft") and stage != "draft0":
                d = int(stage[5:])
                if mistake == "pos+1":
                    pos = pos + 1
                elif mistake == "pos=ctx+depth-2":
                    pos = pos - 1
                elif mistake == "sees_sibling":
                    visible = visible.copy()
                    rows = self.tree.level_rows(d)
                    for i, v in enumerate(rows):          # let a row see the other nodes of its own level
                        for u in range(self.tree.M):
                            if self.tree.depth[u] == d and u <= v:
                                visible[i, self.ctx - 1 + u] = True
                elif mistake == "misses_parent" and d >= 2:
                    visible = visible.copy()
                    for i, v in enumerate(self.tree.level_rows(d)):
                        visible[i, self.ctx - 1 + self.tree.parent[v]] = False
            return super()._head_forward(feats, toks, pos, slots, visible, stage)

    s, W, o = _drafted("T15", cls=Planted)
    assert _head_chain_mismatch(s, W, o) > 1e-4


def test_head_rows_across_prefill_and_commits_equal_one_causal_pass():
    """The head's cache after a prefill and several commits, and the root's predicted feature, equal those of ONE causal
    head pass over all pairs (f[i], x[i+1]), i = 0..ctx-1, with f from a fresh target prefill of the committed tokens:
    pins which feature is paired with which token in the prefill rows and in the pending rows, and their positions."""
    s, W, o = _drafted("T26", seed=9, steps=4)
    d = o.draft_tree()
    ctx = o.ctx
    ref = Oracle(s, W, o.tree.parent, o.tree.rank, max_seq=128)
    ref.prefill(o.x[:-1])                                     # features f[0..ctx-1] of the committed tokens but the root
    F = ref.prefill_features
    one = Oracle(s, W, o.tree.parent, o.tree.rank, max_seq=128)
    pos = np.arange(ctx)
    out = one._head_forward(F, o.x[1:ctx + 1], pos, pos, np.tril(np.ones((ctx, ctx), dtype=bool)), "all")
    np.testing.assert_allclose(one.dkc[:ctx], o.dkc[:ctx], atol=1e-10)
    np.testing.assert_allclose(one.dvc[:ctx], o.dvc[:ctx], atol=1e-10)
    np.testing.assert_allclose(out[-1], d["features"][0], atol=1e-10)
    # a pending pass that paired f[i] with x[i] would not survive this: the cache rows written after the prefill differ
    bad = Oracle(s, W, o.tree.parent, o.tree.rank, max_seq=128)
    bad._head_forward(F, o.x[0:ctx], pos, pos, np.tril(np.ones((ctx, ctx), dtype=bool)), "all")
    assert np.abs(bad.dkc[:ctx] - o.dkc[:ctx]).max() > 1e-3


# ----------------------------------------------------------------------------- non-greedy children
def _v8_oracle(temperature, cls=Oracle):
    s = shape(name="v8", d_model=16, n_heads=2, n_kv_heads=2, head_dim=8, d_ffn=32, vocab=8, rms_eps=1e-5)
    W = synth.make_weights(s, 21, "f32")
    W["lm_head"] = W["lm_head"] * 40.0                        # a clearly non-uniform draft distribution
    par, rk = synth.tree_from_paths(["0", "1"])
    o = cls(s, W, par, rk, temperature=temperature, seed=77, max_seq=32)
    o.prefill(synth.prompt(21, 6, s.vocab))
    return s, W, o


def _child_pair_chi2(o, N=12000):
    V = o.s.vocab
    count = np.zeros((V, V))
    logits = None
    for step in range(N):
        o.step = step + 1                                     # the draw counter is the only thing that changes
        d = o.draft_tree()
        a, b = d["tokens"][1], d["tokens"][2]
        count[a, b] += 1
        logits = d["logits"][0]
    q = np.exp(logits / o.T - np.max(logits / o.T)); q /= q.sum()
    expect = np.zeros((V, V))
    for (a, b), _, pr in draws_without_replacement(q, 2):
        expect[a, b] = pr
    mask = expect * N >= 5                                    # cells with a usable expected count; the rest pooled
    chi2 = np.sum((count[mask] - N * expect[mask]) ** 2 / (N * expect[mask]))
    rest_e, rest_c = N * expect[~mask].sum(), count[~mask].sum()
    if rest_e > 0:
        chi2 += (rest_c - rest_e) ** 2 / rest_e
    assert count[np.arange(V), np.arange(V)].sum() == 0       # siblings are distinct
    return chi2, int(mask.sum()), q


def test_draft_tree_children_follow_draws_without_replacement_at_temperature_half():
    """App. A.1: non-greedy children are k sampled tokens; this build draws them without replacement from
    softmax(logits / T).  The oracle's OWN draft_tree is run 12000 times (draw counter varied) on a V = 8 model at
    T = 0.5 and the (rank 0, rank 1) frequencies are compared with the enumerated sequential-draw law."""
    s, W, o = _v8_oracle(0.5)
    chi2, cells, q = _child_pair_chi2(o)
    assert q.max() > 0.3 and cells >= 12                      # the example is not near-uniform
    assert chi2 < cells + 6 * math.sqrt(2 * cells)            # ~6 sigma of a chi-square with `cells` dof


@pytest.mark.parametrize("mistake", ["no_temperature", "temperature_inverted"])
def test_planted_sampler_mistakes_break_the_frequency_pin(mistake):
    class Planted(Oracle):
        def draft_tree(self, forced_tokens=None):
            T = self.T
            # scores = logits + G (no temperature), or logits * T + G (temperature applied the wrong way round)
            self.T = 1.0 if mistake == "no_temperature" else 1.0 / T
            try:
                return super().draft_tree(forced_tokens)
            finally:
                self.T = T

    s, W, o = _v8_oracle(0.5, cls=Planted)
    chi2, cells, _ = _child_pair_chi2(o, N=6000)
    assert chi2 > 10 * cells


def test_recursive_acceptance_keeps_the_joint_law_at_temperature_two():
    """The enumeration of the recursive acceptance at a temperature other than 1: target logits 2 log P and draft logits
    2 log Q at T = 2 must behave exactly like P and Q -- both distributions of Alg. 1 are softmax(logits / T)."""
    V = 3
    rng = np.random.default_rng(3)
    P1 = rng.dirichlet(np.ones(V)); P2 = rng.dirichlet(np.ones(V), size=V)
    Q1 = rng.dirichlet(np.ones(V))
    par, rk = synth.tree_from_paths(["0", "1"])
    T = 2.0
    o = Oracle(synth.SHAPES["tiny"], {}, par, rk, temperature=T, max_seq=4)
    law = np.zeros(V)
    for (a, b), qs, pr in draws_without_replacement(Q1, 2):
        o.tok = [0, a, b]
        o.node_adj = {0: T * np.log(Q1)}
        o.L = np.stack([T * np.log(P1), T * np.log(P2[a]), T * np.log(P2[b])])
        for script in [(True,), (False, True), (False, False)]:
            calls = {"n": 0}

            def uniform(purpose, node, idx=0, script=script, calls=calls):
                if purpose == eo.PURPOSE_FINAL:
                    return 0.0
                i = calls["n"]; calls["n"] += 1
                return 0.0 if script[i] else 1.0 - 2.0 ** -53
            o._uniform = uniform
            o.accept()
            tests = [t for t in o.trace if t[0] == "test"]
            fin = [t for t in o.trace if t[0] == "final"][0]
            prob, first = pr, None
            for (kind, node, pt, qt), want in zip(tests, script):
                acc = min(1.0, pt / qt)
                prob *= acc if want else 1.0 - acc
                if want:
                    first = o.tok[node]
            if prob == 0.0:
                continue
            if first is not None:
                law[first] += prob
            else:
                law += prob * fin[2]
    np.testing.assert_allclose(law, P1, atol=1e-12)
    # without the division by T on either side the law would be that of P^2 or Q^2 -- far from P
    assert np.abs(eo.softmax(2 * np.log(P1)) - P1).max() > 1e-2
