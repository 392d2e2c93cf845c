"""Pins for the CPU oracle: everything here compares the oracle with something that is NOT the oracle —
closed forms, brute force, exact enumeration, or an invariant the paper states.

  * Sec. 2 (speculative sampling keeps the target's distribution)  -> greedy == vanilla, enumeration of Alg. 1
  * App. A.2, Alg. 1                                               -> exact law of the output, k = 1 textbook case
  * Sec. 3.1 (m passes -> depth-m tree, > m tokens), App. A.1      -> tree builder counts
  * Sec. 3.3 (tree attention = every root->leaf chain at once)      -> tree verify vs chains
  * Sec. 4 "Training" (0.24 B / 0.37 B / 0.99 B trainable params)  -> head wiring / shapes
  * Sec. 4 "Metrics" (tau counts tokens per target forward, >= 1)   -> length bounds
"""
import itertools
import math

import os

import numpy as np
import pytest

import synth
from oracle import eagle_oracle as eo
from oracle.eagle_oracle import Oracle, Tree


def tiny(seed=1, tree="T15", **kw):
    s = synth.SHAPES["tiny"]
    W = synth.make_weights(s, seed, "f32")
    par, rk = synth.TREES[tree]
    return s, W, Oracle(s, W, par, rk, max_seq=kw.pop("max_seq", 256), **kw)


# ----------------------------------------------------------------------------- elementary pieces
def test_rmsnorm_closed_form():
    x = np.array([[3.0, 4.0, 0.0, 0.0]])
    g = np.array([1.0, 2.0, 3.0, 4.0])
    # mean square = 25/4 -> rms = 2.5
    np.testing.assert_allclose(eo.rmsnorm(x, g, 0.0), [[1.2, 3.2, 0.0, 0.0]], rtol=1e-15)
    # eps enters under the root
    np.testing.assert_allclose(eo.rmsnorm(np.array([[0.0, 0.0]]), np.ones(2), 1e-5), [[0.0, 0.0]])
    y = eo.rmsnorm(np.array([[1.0, 1.0]]), np.ones(2), 3.0)
    np.testing.assert_allclose(y, [[0.5, 0.5]], rtol=1e-15)


def test_rope_is_a_rotation_with_relative_phase():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 2, 8))
    k = rng.standard_normal((1, 2, 8))
    # position 0 is the identity, norms are preserved
    np.testing.assert_allclose(eo.rope(q, np.array([0]), 10000.0), q, atol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(eo.rope(q, np.array([37]), 10000.0)), np.linalg.norm(q), rtol=1e-13)
    # <rope(q,m), rope(k,n)> depends on m-n only
    d1 = np.sum(eo.rope(q, np.array([5]), 10000.0) * eo.rope(k, np.array([2]), 10000.0))
    d2 = np.sum(eo.rope(q, np.array([105]), 10000.0) * eo.rope(k, np.array([102]), 10000.0))
    np.testing.assert_allclose(d1, d2, rtol=1e-11)
    # pair (i, i+dh/2) turns by pos * theta^(-2i/dh): check one pair against the complex product
    x = np.zeros((1, 1, 8)); x[0, 0, 1] = 1.0                       # pair index 1: elements 1 and 5
    y = eo.rope(x, np.array([3]), 100.0)[0, 0]
    ang = 3 * 100.0 ** (-2 * 1 / 8)
    np.testing.assert_allclose([y[1], y[5]], [math.cos(ang), math.sin(ang)], rtol=1e-14)
    assert np.count_nonzero(y) == 2


def test_round_bf16_is_nearest_even_on_known_values():
    # 1 + 2^-8 lies exactly between the bf16 neighbours 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies between 1 + 2^-7 (odd) and 1 + 2^-6 (even) -> rounds up
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -0.3], dtype=np.float32)
    y = eo.round_bf16(x)
    np.testing.assert_array_equal(y[:4], np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6], np.float32))
    assert abs(y[4] + 0.3) <= 2.0 ** -10 and (y.view(np.uint32) & 0xFFFF == 0).all()
    assert np.array_equal(eo.round_bf16(synth.normal(1, 2, 64, 0.02, 0.0, "f32")), synth.normal(1, 2, 64, 0.02, 0.0, "bf16_f32"))


def test_topk_and_argmax_ties_go_to_lowest_id():
    s = np.array([1.0, 5.0, 5.0, 3.0, 5.0])
    assert eo.topk_desc(s, 4) == [1, 2, 4, 3]
    assert eo.argmax_low(s) == 1
    assert eo.top2_gap(np.array([1.0, 4.0, 2.5])) == 1.5


def test_sample_inverse_cdf_intervals():
    p = np.array([0.1, 0.0, 0.4, 0.5])
    assert eo.sample_inverse_cdf(p, 0.0) == 0
    assert eo.sample_inverse_cdf(p, 0.0999) == 0
    assert eo.sample_inverse_cdf(p, 0.1) == 2          # zero-probability token is never drawn
    assert eo.sample_inverse_cdf(p, 0.4999) == 2
    assert eo.sample_inverse_cdf(p, 0.5) == 3
    assert eo.sample_inverse_cdf(p, 1 - 2.0 ** -24) == 3


# ----------------------------------------------------------------------------- trees
def brute_ancestors(parent, v):
    out = {v}
    while parent[v] >= 0:
        v = parent[v]
        out.add(v)
    return out


@pytest.mark.parametrize("name,nodes,depth,root_k,rows", [
    ("T26", 26, 5, 4, [4, 4, 3, 2]), ("T15", 15, 4, 2, [2, 3, 3]), ("T10", 11, 3, 2, [2, 3]),
    ("chain5", 6, 5, 1, [1, 1, 1, 1])])
def test_tree_builder_counts(name, nodes, depth, root_k, rows):
    par, rk = synth.TREES[name]
    t = Tree(par, rk)
    assert t.M == nodes and t.D == depth and len(t.children[0]) == root_k
    # m draft passes <-> depth-m tree with more than m tokens (chain: exactly m)
    assert t.M - 1 >= depth
    assert [len(t.level_rows(d)) for d in range(1, t.D)] == rows
    for v in range(t.M):
        assert set(t.ancestors_or_self(v)) == brute_ancestors(list(par), v)
        assert t.ancestors_or_self(v)[0] == 0 and t.ancestors_or_self(v)[-1] == v
        assert len(t.ancestors_or_self(v)) == t.depth[v] + 1


def test_tree_rejects_bad_specs():
    with pytest.raises(ValueError):
        Tree([0, 0], [0, 0])
    with pytest.raises(ValueError):
        Tree([-1, 0, 0], [0, 0, 2])
    with pytest.raises(ValueError):
        Tree([-1, 2, 0], [0, 0, 0])


def _golden(name):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    return [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]


def test_head_parameter_counts_match_the_paper():
    # Sec. 4 "Training": trainable parameters of the head for the 7B, 13B and 70B targets (tests/golden)
    rows = _golden("head_trainable_parameters.txt")
    assert len(rows) == 3
    for shape, printed in rows:
        assert round(synth.head_param_count(synth.SHAPES[shape]) / 1e9, 2) == float(printed)


def test_tree_facts_from_the_text():
    # Sec. 3.1 / App. A.1: node counts, number of head passes and root branching stated in the text (tests/golden)
    rows = _golden("draft_tree_facts.txt")
    assert len(rows) == 3
    for name, drafted, depth, root_k in rows:
        t = Tree(*synth.TREES[name])
        assert t.D == int(depth)
        if drafted != "-":
            assert t.M - 1 == int(drafted)
        if root_k != "-":
            assert len(t.children[0]) == int(root_k)
        assert t.M - 1 >= t.D                      # m passes draft at least m tokens (more, unless a chain)


# ----------------------------------------------------------------------------- whole greedy loop
@pytest.mark.parametrize("shape,tree,kv", [("tiny", "T15", None), ("tiny", "T26", None), ("mini-gqa", "T10", "bf16"),
                                           ("mini-moe", "T15", "bf16")])
def test_greedy_speculative_equals_vanilla(shape, tree, kv):
    s = synth.SHAPES[shape]
    W = synth.make_weights(s, 3, synth.oracle_fmt(s))
    par, rk = synth.TREES[tree]
    prompt = synth.prompt(3, 32, s.vocab)
    a, lens = Oracle(s, W, par, rk, max_seq=192, kv_store=kv).generate(prompt, 64)
    b = Oracle(s, W, par, rk, max_seq=192, kv_store=kv).generate_vanilla(prompt, 64)
    assert a == b
    D = Tree(par, rk).D
    assert all(1 <= n <= D + 1 for n in lens)


def perfect_predictor_weights(s, seed):
    """A target whose next token depends on the last token only (attention and MLP outputs switched off),
    and a head that predicts the next feature exactly up to a positive factor: FC picks the embedding half."""
    W = synth.make_weights(s, seed, "f32")
    for li in range(s.n_layers):
        W[f"layers.{li}.wo"] = np.zeros_like(W[f"layers.{li}.wo"])
        W[f"layers.{li}.down"] = np.zeros_like(W[f"layers.{li}.down"])
    W["head.layer.wo"] = np.zeros_like(W["head.layer.wo"])
    W["head.layer.down"] = np.zeros_like(W["head.layer.down"])
    W["head.fc_w"] = np.concatenate([np.zeros((s.d_model, s.d_model), np.float32),
                                     np.eye(s.d_model, dtype=np.float32)], axis=1)
    W["head.fc_b"] = np.zeros(s.d_model, np.float32)
    W["final_norm"] = np.ones(s.d_model, np.float32)
    return W


def test_perfect_head_accepts_full_depth_every_step():
    """Pins the (feature, shifted token) wiring: with a head that is exact, the rank-0 spine always matches."""
    s = synth.SHAPES["tiny"]
    W = perfect_predictor_weights(s, 5)
    par, rk = synth.TREES["T15"]
    o = Oracle(s, W, par, rk, max_seq=256)
    toks, lens = o.generate(synth.prompt(5, 16, s.vocab), 60)
    assert lens == [Tree(par, rk).D + 1] * len(lens)
    assert toks == Oracle(s, W, par, rk, max_seq=256).generate_vanilla(synth.prompt(5, 16, s.vocab), 60)


def test_wrong_shift_would_be_seen_by_the_perfect_head_pin():
    """The same construction with the token half fed UNSHIFTED (a planted mistake) drops to chance."""
    s = synth.SHAPES["tiny"]
    W = perfect_predictor_weights(s, 5)
    par, rk = synth.TREES["T15"]

    class Unshifted(Oracle):
        def _head_forward(self, feats, toks, pos, slots, visible, stage):
            if stage == "draft0":                       # pair f[i] with x[i] instead of x[i+1]
                p0 = self.ctx - len(self.pending_f)
                toks = self.x[p0:self.ctx]
            return super()._head_forward(feats, toks, pos, slots, visible, stage)

    _, lens = Unshifted(s, W, par, rk, max_seq=256).generate(synth.prompt(5, 16, s.vocab), 40)
    assert np.mean(lens) < 2.0


def test_tree_verify_equals_running_each_chain():
    """Tree attention: a node's feature and logits equal those of the plain causal chain root -> node."""
    s, W, o = tiny(seed=7)
    o.prefill(synth.prompt(7, 12, s.vocab))
    o.spec_step()
    o.draft_tree()
    F, L = o.verify()
    tr = o.tree
    ctx = o.ctx
    leaves = [v for v in range(tr.M) if not tr.children[v]]
    for leaf in leaves:
        chain = tr.ancestors_or_self(leaf)
        # fresh oracle with the same committed prefix, fed the chain as ordinary causal rows
        p = Oracle(s, W, *synth.TREES["T15"], max_seq=256)
        for li in range(s.n_layers):
            p.kc[li][:ctx] = o.kc[li][:ctx]
            p.vc[li][:ctx] = o.vc[li][:ctx]
        n = len(chain)
        pos = np.arange(ctx, ctx + n)
        vis = np.zeros((n, ctx + n), dtype=bool)
        for i in range(n):
            vis[i, :ctx + i + 1] = True
        Fc, Lc = p._target_forward([o.tok[v] for v in chain], pos, pos, vis, "chain")
        np.testing.assert_allclose(Fc, F[chain], rtol=0, atol=1e-11)
        np.testing.assert_allclose(Lc, L[chain], rtol=0, atol=1e-11)


def test_compacted_cache_equals_fresh_prefill():
    """After several commits the target KV cache holds exactly what a causal pass over the committed tokens gives."""
    s, W2, _ = tiny(seed=9, tree="T26")
    par, rk = synth.TREES["T26"]
    prompt = synth.prompt(9, 10, s.vocab)
    future = list(prompt) + Oracle(s, W2, par, rk, max_seq=256).generate_vanilla(prompt, 60)
    o = Oracle(s, W2, par, rk, max_seq=256)
    o.set_hint(future, 0.8, 30.0, 5)                    # long accepted paths -> compaction really moves rows
    o.prefill(prompt)
    lens = [o.spec_step()["length"] for _ in range(6)]
    assert max(lens) > 2
    ref = Oracle(s, W2, par, rk, max_seq=256)
    ref.prefill(o.x[:-1])                                # all committed tokens but the root
    n = o.ctx
    for li in range(s.n_layers):
        np.testing.assert_allclose(o.kc[li][:n], ref.kc[li][:n], atol=1e-11)
        np.testing.assert_allclose(o.vc[li][:n], ref.vc[li][:n], atol=1e-11)
    np.testing.assert_allclose(np.stack(o.pending_f)[-1], ref.prefill_features[-1], atol=1e-11)


def test_accept_path_is_a_root_chain():
    s, W, o = tiny(seed=4, tree="T26")
    o.prefill(synth.prompt(4, 8, s.vocab))
    for _ in range(5):
        o.draft_tree(); o.verify()
        r = o.accept()
        path = r["path"]
        assert path[0] == 0 and all(o.tree.parent[path[i + 1]] == path[i] for i in range(len(path) - 1))
        assert all(path[i] >= i for i in range(len(path))) and r["length"] == len(path)
        o.commit(path, r["bonus"])


# ----------------------------------------------------------------------------- the acceptance knob
def test_hint_knob_gives_runs_of_hits():
    """With the knob, the accepted length of a step equals the run of consecutive hash hits starting at the
    step's first new position (capped at the tree depth): an exact, hash-level prediction."""
    s, W, o = tiny(seed=2)
    prompt = synth.prompt(2, 16, s.vocab)
    future = list(prompt) + Oracle(s, W, *synth.TREES["T15"], max_seq=256).generate_vanilla(prompt, 90)
    alpha, hseed = 0.7, 99
    o.set_hint(future, alpha, 30.0, hseed)
    o.prefill(prompt)
    D = o.tree.D
    lens = []
    while len(o.x) < len(prompt) + 70:
        n = len(o.x)
        run = 0
        while run < D and np.float32(eo.u24(hseed, eo.PURPOSE_HINT, 0, 0, 0, n + run) * 2.0 ** -24) < np.float32(alpha):
            run += 1
        r = o.spec_step()
        assert r["length"] == run + 1
        lens.append(r["length"])
    assert o.x[:len(prompt) + 70] == future[:len(prompt) + 70]
    assert 1.5 < np.mean(lens) < 4.5


# ----------------------------------------------------------------------------- Alg. 1
def draws_without_replacement(q, k):
    """All ordered k-tuples of distinct tokens with their probability under sequential renormalised draws,
    and the proposal distribution each element was drawn from."""
    out = []

    def rec(prefix, qs, qcur, prob):
        if len(prefix) == k:
            out.append((tuple(prefix), list(qs), prob))
            return
        for t in range(len(q)):
            if qcur[t] <= 0:
                continue
            nxt = qcur.copy(); nxt[t] = 0
            tot = nxt.sum()
            rec(prefix + [t], qs + [qcur], nxt / tot if tot > 0 else nxt, prob * qcur[t])
    rec([], [], np.asarray(q, dtype=np.float64), 1.0)
    return out


@pytest.mark.parametrize("V,k", [(3, 1), (3, 2), (4, 1), (4, 2), (4, 3), (5, 2), (5, 3)])
def test_alg1_output_law_is_the_target(V, k):
    rng = np.random.default_rng(100 * V + k)
    for trial in range(4):
        p = rng.dirichlet(np.ones(V))
        q = rng.dirichlet(np.ones(V))
        if trial == 3:
            p[0] = 0.0; p /= p.sum()                     # a token the target never emits
        law = np.zeros(V)
        for ts, qs, pdraw in draws_without_replacement(q, k):
            # the all-reject chain carries every threshold; an accept at round i ends the chain there
            _, p_left, trace = eo.multi_round(p, ts, qs, [1.0 - 2.0 ** -53] * k)
            alive = 1.0
            for i, (pt, qt) in enumerate(trace):
                acc = min(1.0, pt / qt)
                law[ts[i]] += pdraw * alive * acc
                alive *= 1.0 - acc
                if alive == 0.0:
                    break
            if alive > 0.0:
                assert len(trace) == k
                law += pdraw * alive * p_left
        np.testing.assert_allclose(law, p, atol=1e-12)


def test_alg1_control_flow_follows_the_thresholds():
    p = np.array([0.5, 0.3, 0.2]); q = np.array([0.2, 0.6, 0.2])
    # candidate 1: threshold p/q = 0.5
    assert eo.multi_round(p, [1], [q], [0.4999])[0] == 0
    i, left, _ = eo.multi_round(p, [1], [q], [0.5])
    assert i is None
    np.testing.assert_allclose(left, [1.0, 0.0, 0.0])     # max(0, p-q) = (0.3, 0, 0)
    # candidate 0: p/q > 1 -> always accepted
    assert eo.multi_round(p, [0], [q], [1 - 2.0 ** -24])[0] == 0
    # second round uses the residual target
    q2 = eo.drop_and_renorm(q, 1)
    np.testing.assert_allclose(q2, [0.5, 0.0, 0.5])
    i, left, tr = eo.multi_round(p, [1, 2], [q, q2], [0.9, 0.5])
    assert tr[1] == (0.0, 0.5) and i is None


def test_alg1_k1_is_textbook_speculative_sampling():
    rng = np.random.default_rng(5)
    p = rng.dirichlet(np.ones(6)); q = rng.dirichlet(np.ones(6))
    law = np.zeros(6)
    for t in range(6):
        _, left, tr = eo.multi_round(p, [t], [q], [1.0 - 2.0 ** -53])
        acc = min(1.0, tr[0][0] / tr[0][1])
        law[t] += q[t] * acc
        law += q[t] * (1 - acc) * left
    textbook = np.minimum(p, q) + (1 - np.minimum(p, q).sum()) * np.maximum(p - q, 0) / np.maximum(p - q, 0).sum()
    np.testing.assert_allclose(law, textbook, atol=1e-13)
    np.testing.assert_allclose(law, p, atol=1e-13)


def test_recursive_tree_acceptance_keeps_the_joint_law():
    """Tiny-vocab model given as explicit tables, depth-2 tree with 2 children per node: the joint law of the
    first two emitted tokens equals the product of the target's conditionals (exact enumeration over tree
    draws and over every accept/reject branch)."""
    V = 4
    rng = np.random.default_rng(11)
    P1 = rng.dirichlet(np.ones(V)); P2 = rng.dirichlet(np.ones(V), size=V); P3 = rng.dirichlet(np.ones(V), size=(V, V))
    Q1 = rng.dirichlet(np.ones(V)); Q2 = rng.dirichlet(np.ones(V), size=V)
    par, rk = synth.tree_from_paths(["0", "1", "00", "01", "10", "11"])
    s = synth.SHAPES["tiny"]
    o = Oracle(s, {}, par, rk, temperature=1.0, max_seq=4)
    joint = np.zeros((V, V))
    total = 0.0
    for (a, b), _, pr1 in draws_without_replacement(Q1, 2):
        for (c, d), _, pr2 in draws_without_replacement(Q2[a], 2):
            for (e, f), _, pr3 in draws_without_replacement(Q2[b], 2):
                tok = [0, a, b, c, d, e, f]
                o.tok = tok
                o.node_adj = {0: np.log(Q1), 1: np.log(Q2[a]), 2: np.log(Q2[b])}
                L = np.zeros((7, V))
                L[0] = np.log(np.maximum(P1, 1e-300))
                L[1] = np.log(P2[a]); L[2] = np.log(P2[b])
                for v, (t1, t2) in zip((3, 4, 5, 6), ((a, c), (a, d), (b, e), (b, f))):
                    L[v] = np.log(P3[t1, t2])
                o.L = L
                pdraw = pr1 * pr2 * pr3
                # explore every accept/reject script; script[i] = decision at the i-th accept test
                stack = [()]
                while stack:
                    script = stack.pop()
                    calls = {"n": 0}

                    def uniform(purpose, node, idx=0, script=script, calls=calls):
                        if purpose == eo.PURPOSE_FINAL:
                            return 0.0
                        i = calls["n"]; calls["n"] += 1
                        want_accept = script[i] if i < len(script) else True
                        return 0.0 if want_accept else 1.0 - 2.0 ** -53
                    o._uniform = uniform
                    o.accept()
                    tests = [t for t in o.trace if t[0] == "test"]
                    if len(tests) > len(script):          # a decision not yet scripted: branch on it
                        stack.append(script + (True,)); stack.append(script + (False,))
                        continue
                    prob = pdraw
                    acc_nodes = []
                    feasible = True
                    for (kind, node, pt, qt), want in zip(tests, script):
                        acc = min(1.0, pt / qt)
                        prob *= acc if want else 1.0 - acc
                        if want:
                            acc_nodes.append(node)
                        if prob == 0.0:
                            feasible = False
                            break
                    if not feasible:
                        continue
                    fin = [t for t in o.trace if t[0] == "final"][0]
                    emitted = [tok[v] for v in acc_nodes]
                    pf = fin[2]
                    total += prob
                    if len(emitted) >= 2:
                        joint[emitted[0], emitted[1]] += prob
                    elif len(emitted) == 1:
                        joint[emitted[0], :] += prob * pf
                    else:                                  # nothing accepted: bonus ~ pf, next token ~ P2[bonus]
                        joint += prob * pf[:, None] * P2
    np.testing.assert_allclose(total, 1.0, atol=1e-12)
    np.testing.assert_allclose(joint, P1[:, None] * P2, atol=1e-12)


# ----------------------------------------------------------------------------- RNG and sampler
def test_u24_vector_equals_scalar_and_is_uniform():
    v = eo._u24_vec(5, eo.PURPOSE_GUMBEL, 3, 1, 7, 257)
    assert [int(x) for x in v] == [eo.u24(5, eo.PURPOSE_GUMBEL, 3, 1, 7, i) for i in range(257)]
    big = eo._u24_vec(1, eo.PURPOSE_ACCEPT, 0, 0, 0, 1 << 18) * 2.0 ** -24
    assert big.min() >= 0 and big.max() < 1
    hist = np.histogram(big, bins=16, range=(0, 1))[0]
    chi2 = np.sum((hist - big.size / 16) ** 2 / (big.size / 16))
    assert chi2 < 45                                      # 15 dof, p ~ 1e-4


def test_gumbel_children_follow_sequential_draws_without_replacement():
    """Smoke (frequency) test of the non-greedy child sampler at V = 8, k = 2."""
    V = 8
    s = synth.SHAPES["tiny"]
    par, rk = synth.tree_from_paths(["0", "1"])
    rng = np.random.default_rng(2)
    logits = rng.standard_normal(V)
    q = np.exp(logits) / np.exp(logits).sum()
    expect = np.zeros((V, V))
    for (a, b), _, pr in draws_without_replacement(q, 2):
        expect[a, b] = pr
    count = np.zeros((V, V))
    N = 20000
    for step in range(N):
        k24 = eo._u24_vec(77, eo.PURPOSE_GUMBEL, step, 0, 0, V)
        score = logits - np.log(-np.log((k24 + 0.5) * 2.0 ** -24))
        a, b = eo.topk_desc(score, 2)
        count[a, b] += 1
    mask = expect > 0
    chi2 = np.sum((count[mask] - N * expect[mask]) ** 2 / (N * expect[mask]))
    assert chi2 < 110                                     # 55 dof, p ~ 1e-5


def test_stochastic_generation_runs_and_respects_bounds():
    s = synth.SHAPES["tiny"]
    W = synth.make_weights(s, 6, "f32")
    par, rk = synth.TREES["T15"]
    o = Oracle(s, W, par, rk, temperature=1.0, seed=123, max_seq=256)
    toks, lens = o.generate(synth.prompt(6, 16, s.vocab), 40)
    assert len(toks) == 40 and all(1 <= n <= 5 for n in lens)
    o2 = Oracle(s, W, par, rk, temperature=1.0, seed=123, max_seq=256)
    assert o2.generate(synth.prompt(6, 16, s.vocab), 40)[0] == toks      # counter-based: reproducible
