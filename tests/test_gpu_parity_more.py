"""GPU parity, second part: the configurations' true widths and modes that the first file reaches only through
stand-ins -- the Mixtral-shaped MoE twin at temperature 1, four sequences with the 26-node tree at 7B / 13B / 70B widths
(the 104-row general path), the literal N(0, 0.02) head recipe, vocabularies beyond 32768 entries, a permuted page
table -- plus kernel-level tests that feed the child-selection, acceptance and compaction kernels the ORACLE'S OWN
fp32 logits (results must then be bit-exact, no margin excuse), the oracle-driven direction of the lock-step protocol
(eagle_force_tree / eagle_force_accept), out-of-order calls, and bitwise repeatability at the shapes with the most
split-K groups and attention splits.  Everything goes through the C ABI."""
import numpy as np
import pytest

import paper_2401_15077_amd as pkg
import synth
from lockstep import Stats, _check_accept, check_prefill, lockstep_step, lockstep_step_batch
from oracle.eagle_oracle import Oracle

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def say(msg):
    print(msg, flush=True)


def vanilla_future(eng, prompts, n):
    """The engine's own greedy continuation of every prompt (the knob's hints), then a reset."""
    futs = [list(p) + [eng.prefill(b, p)] for b, p in enumerate(prompts)]
    for _ in range(n):
        tk = eng.vanilla_step()
        for b in range(len(prompts)):
            futs[b].append(int(tk[b]))
    eng.reset()
    return futs


# ----------------------------------------------------------------------------- configuration 5 at its true widths
def test_mixtral_twin_lockstep_greedy_and_temperature_one():
    """Mixtral-8x7B widths (d 4096, 32 query heads on 8 KV heads, 8 experts top-2 with expert FFN 14336, vocab 32000,
    MoE head layer), 2 target layers: lock-step against the fp32 oracle, greedy with the knob and at temperature 1.0
    (Gumbel top-k children and Alg. 1 over 32000 entries, 8-expert routing at d = 4096)."""
    s = synth.SHAPES["mixtral-8x7b"].twin(2)
    par, rk = synth.TREES["T26"]
    say("mixtral twin: generating weights")
    W = synth.make_weights(s, 13, synth.oracle_fmt(s))
    prompt = synth.prompt(13, 24, s.vocab)
    for temperature in (0.0, 1.0):
        eng = pkg.Eagle(s, par, rk, max_seq=256, temperature=temperature, seed=4242)
        eng.load_weights(synth.iter_weights(s, 13, synth.device_fmt(s)))
        orc = Oracle(s, W, par, rk, max_seq=256, temperature=temperature, seed=4242, dtype=np.float32)
        if temperature == 0.0:
            fut = vanilla_future(eng, [prompt], 30)[0]
        say(f"mixtral twin T={temperature}: prefill")
        check_prefill(eng, orc, prompt, TOL["bf16"], margin_thr=2e-2 if temperature == 0.0 else 5e-2)
        if temperature == 0.0:
            eng.set_hint(0, fut, 0.7773, 1.0e4, 5)
            orc.set_hint(fut, 0.7773, 1.0e4, 5)
        st = Stats()
        for i in range(4):
            lockstep_step(eng, orc, st, TOL["bf16"], margin_thr=2e-2, stoch_margin=5e-2)
            say(f"mixtral twin T={temperature}: step {i} len {st.lens[-1]} max|dL|={st.max_logit_err:.2e} draft {st.max_draft_logit_err:.2e}")
        assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
        assert st.excused_accepts <= 1 and st.excused_tree_slots <= 2
        if temperature == 0.0:
            assert st.tau > 1.5
        eng.close()


# ----------------------------------------------------------------------------- configurations 3 / 4: four sequences, 26-node tree
@pytest.mark.parametrize("shape_name,prompt0,steps", [("llama2-7b", 40, 3), ("llama2-13b", 36, 3), ("llama2-70b", 30, 2)])
def test_batch4_T26_general_path_lockstep(shape_name, prompt0, steps):
    """bs = 4 with the 26-node tree at real widths: 104 verify rows take the general path (4-wave GEMM, separate
    epilogue kernels, attention with four sequences side by side).  Four oracles share one weight dictionary; prompts
    have different lengths; logits and features of every slot are compared element-wise."""
    s = synth.SHAPES[shape_name].twin(2)
    par, rk = synth.TREES["T26"]
    eng = pkg.Eagle(s, par, rk, max_batch=4, max_seq=192)
    eng.load_weights(synth.iter_weights(s, 17, synth.device_fmt(s)))
    W = synth.make_weights(s, 17, synth.oracle_fmt(s))
    prompts = [synth.prompt(17, prompt0 + 9 * b, s.vocab, stream=b) for b in range(4)]
    futs = vanilla_future(eng, prompts, steps * 6 + 8)
    orcs, sts = [], []
    for b in range(4):
        orc = Oracle(s, W, par, rk, max_seq=192, seq_id=b, dtype=np.float32)
        check_prefill(eng, orc, prompts[b], TOL["bf16"], seq=b)
        eng.set_hint(b, futs[b], 0.7773, 1.0e4, 100 + b)
        orc.set_hint(futs[b], 0.7773, 1.0e4, 100 + b)
        orcs.append(orc); sts.append(Stats())
    for i in range(steps):
        lockstep_step_batch(eng, orcs, sts, TOL["bf16"])
        say(f"{s.name} bs4: step {i} lens {[st.lens[-1] for st in sts]} max|dL| {max(st.max_logit_err for st in sts):.2e}")
    for b in range(4):
        assert list(eng.get_buffer(pkg.BUF_TOKENS, b)) == orcs[b].x
        assert sts[b].max_logit_err <= TOL["bf16"] and sts[b].max_feat_err <= TOL["bf16"]
    assert sum(st.emitted for st in sts) > 4 * steps            # the knob lands: compaction moves rows on this path too
    eng.close()


# ----------------------------------------------------------------------------- the literal head recipe
@pytest.mark.parametrize("shape_name,n_layers,key", [("tiny", None, "fp32"), ("llama2-7b", 2, "bf16")])
def test_literal_head_recipe_lockstep(shape_name, n_layers, key):
    """Every head matrix drawn from N(0, 0.02) exactly like the target's (no rescaling of FC / W_o / W_down).  The head
    then feeds a growing feature back at every level and its logits grow with depth, so the draft logits are held
    to a bar RELATIVE to their magnitude (1e-3 of max|logit|, floor = the absolute bar); the verify side is the plain
    target and keeps the absolute bar."""
    s = synth.SHAPES[shape_name]
    if n_layers:
        s = s.twin(n_layers)
    par, rk = synth.TREES["T26" if key == "bf16" else "T15"]
    eng = pkg.Eagle(s, par, rk, max_seq=256)
    eng.load_weights(synth.iter_weights(s, 19, synth.device_fmt(s), head_recipe="literal"))
    orc = Oracle(s, synth.make_weights(s, 19, synth.oracle_fmt(s), head_recipe="literal"), par, rk, max_seq=256,
                 dtype=np.float32 if key == "bf16" else np.float64)
    prompt = synth.prompt(19, 40, s.vocab)
    check_prefill(eng, orc, prompt, TOL[key])
    worst_rel, worst_abs, max_logit = 0.0, 0.0, 0.0
    st = Stats()
    for step in range(4):
        toks = eng.draft_tree()[0]
        d = orc.draft_tree(forced_tokens=toks)
        dl = eng.get_buffer(pkg.BUF_DRAFT_LOGITS)
        df = eng.get_buffer(pkg.BUF_DRAFT_FEATURES)
        for v, lo in orc.node_adj.items():
            scale = max(1.0, float(np.abs(lo).max()))
            err = float(np.abs(dl[v] - lo).max())
            worst_abs = max(worst_abs, err); worst_rel = max(worst_rel, err / scale); max_logit = max(max_logit, scale)
            fscale = max(1.0, float(np.abs(orc.node_f[v]).max()))
            assert float(np.abs(df[v] - orc.node_f[v]).max()) <= max(TOL[key], 1e-3 * fscale)
            assert err <= max(TOL[key], 1e-3 * scale), f"node {v}: draft logit error {err} at magnitude {scale}"
        for (v, r, t_o, t_g, gap) in d["mismatches"]:
            assert gap < max(2e-2, 1e-3 * max_logit)
        eng.verify()
        F, L = orc.verify()
        assert float(np.abs(eng.get_buffer(pkg.BUF_LOGITS) - L).max()) <= TOL[key]
        assert float(np.abs(eng.get_buffer(pkg.BUF_FEATURES) - F).max()) <= TOL[key]
        out, lens, path = eng.accept()
        _check_accept(orc, st, out[0], int(lens[0]), path[0], 2e-2, 1e-3)
    say(f"literal head recipe {s.name}: max|draft logit| {max_logit:.1f}, worst abs err {worst_abs:.2e}, worst rel err {worst_rel:.2e}")
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    eng.close()


# ----------------------------------------------------------------------------- vocabularies beyond 32768 entries
@pytest.mark.parametrize("temperature", [0.0, 1.0])
def test_vocab_beyond_32768_lockstep(temperature):
    """40000-entry vocabulary on the tiny widths: the child-selection kernel's large-vocabulary branch (per-thread
    sorted top-k lists), greedy and Gumbel top-k."""
    s = synth.SHAPES["tiny-v40k"]
    par, rk = synth.TREES["T15"]
    eng = pkg.Eagle(s, par, rk, max_seq=160, temperature=temperature, seed=31)
    eng.load_weights(synth.iter_weights(s, 23, synth.device_fmt(s)))
    orc = Oracle(s, synth.make_weights(s, 23, synth.oracle_fmt(s)), par, rk, max_seq=160, temperature=temperature, seed=31)
    prompt = synth.prompt(23, 20, s.vocab)
    if temperature == 0.0:
        fut = list(prompt) + Oracle(s, orc.W, par, rk, max_seq=160).generate_vanilla(prompt, 50)
        orc.set_hint(fut, 0.75, 30.0, 9)
    check_prefill(eng, orc, prompt, TOL["fp32"], margin_thr=1e-4)
    if temperature == 0.0:
        eng.set_hint(0, fut, 0.75, 30.0, 9)
    st = Stats()
    for _ in range(8):
        lockstep_step(eng, orc, st, TOL["fp32"], margin_thr=1e-3, stoch_margin=1e-3)
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    assert st.excused_accepts <= 1 and st.excused_tree_slots <= 1
    if temperature == 0.0:
        assert max(st.lens) >= 3
    eng.close()


# ----------------------------------------------------------------------------- a page table that is not the default map
def test_permuted_page_table_lockstep():
    """Two sequences on a seeded random permutation of the physical pages: the indirection of every cache access
    (append, attention, compaction, row read-back) is exercised with something else than the default interleaved map;
    decoding crosses page boundaries of both slots."""
    s = synth.SHAPES["tiny"]
    par, rk = synth.TREES["T15"]
    eng = pkg.Eagle(s, par, rk, max_batch=2, max_seq=192)
    eng.load_weights(synth.iter_weights(s, 29, synth.device_fmt(s)))
    n_pages = 2 * eng.pages_per_slot
    perm = np.random.default_rng(29).permutation(n_pages).astype(np.int32)
    assert not np.array_equal(perm, np.arange(n_pages))
    eng.set_page_table(perm)
    with pytest.raises(pkg.EagleError):
        eng.set_page_table(np.zeros(n_pages, np.int32))            # not a permutation
    W = synth.make_weights(s, 29, synth.oracle_fmt(s))
    orcs, sts, futs = [], [], []
    prompts = [synth.prompt(29, 50 + 11 * b, s.vocab, stream=b) for b in range(2)]
    for b in range(2):
        futs.append(list(prompts[b]) + Oracle(s, W, par, rk, max_seq=192).generate_vanilla(prompts[b], 80))
    for b in range(2):
        orc = Oracle(s, W, par, rk, max_seq=192, seq_id=b)
        orc.set_hint(futs[b], 0.75, 30.0, 40 + b)
        check_prefill(eng, orc, prompts[b], TOL["fp32"], seq=b)
        eng.set_hint(b, futs[b], 0.75, 30.0, 40 + b)
        orcs.append(orc); sts.append(Stats())
    with pytest.raises(pkg.EagleError) as err:
        eng.set_page_table(perm)                                   # sequences are active
    assert err.value.code == -4
    while min(o.ctx for o in orcs) < 135:
        lockstep_step_batch(eng, orcs, sts, TOL["fp32"])
    for b in range(2):
        assert list(eng.get_buffer(pkg.BUF_TOKENS, b)) == orcs[b].x and sts[b].excused_accepts == 0
        for layer in range(s.n_layers):
            for pos in (0, 63, 64, 127, 128, orcs[b].ctx - 1):
                k, v = eng.get_kv_row(b, layer, pos)
                assert np.abs(k - orcs[b].kc[layer][pos].reshape(-1)).max() < 1e-4
                assert np.abs(v - orcs[b].vc[layer][pos].reshape(-1)).max() < 1e-4
    eng.close()


# ----------------------------------------------------------------------------- kernels on the oracle's own logits
@pytest.mark.parametrize("temperature", [0.0, 1.0])
def test_selection_acceptance_compaction_on_oracle_logits_are_bit_exact(temperature):
    """Child selection, acceptance and compaction fed the fp32 oracle's OWN logits at the LLaMA vocabulary (32000):
    tree tokens, accepted path, length, bonus token and the moved KV rows must be bit-exact -- no margin excuse, since
    both sides decide on the same numbers in the same precision (App. A.1; App. A.2 Alg. 1; Sec. 3.3)."""
    s = synth.SHAPES["tiny-v32k"]
    par, rk = synth.TREES["T26"]
    eng = pkg.Eagle(s, par, rk, max_seq=256, temperature=temperature, seed=2718)
    eng.load_weights(synth.iter_weights(s, 37, synth.device_fmt(s)))
    W = synth.make_weights(s, 37, synth.oracle_fmt(s))
    orc = Oracle(s, W, par, rk, max_seq=256, temperature=temperature, seed=2718, dtype=np.float32)
    prompt = synth.prompt(37, 30, s.vocab)
    if temperature == 0.0:
        fut = list(prompt) + Oracle(s, W, par, rk, max_seq=256, dtype=np.float32).generate_vanilla(prompt, 80)
        orc.set_hint(fut, 0.8, 30.0, 7)
    check_prefill(eng, orc, prompt, TOL["fp32"], margin_thr=1e-4)
    if temperature == 0.0:
        eng.set_hint(0, fut, 0.8, 30.0, 7)
    M, V, D = len(par), s.vocab, orc.tree.D
    lens = []
    for step in range(10):
        eng.draft_tree()
        d = orc.draft_tree()                                       # free-running: the oracle's own children
        raw = np.zeros((M, V), np.float32)
        for v, lg in orc.node_logits.items():
            raw[v] = lg                                            # logits before the knob: the kernel applies it itself
        eng.set_buffer(pkg.BUF_DRAFT_LOGITS, raw)
        for level in [-1] + list(range(1, D)):
            eng.expand_level(level)
        assert list(eng.get_buffer(pkg.BUF_TREE_TOKENS)) == orc.tok, f"step {step}: tree tokens differ"
        dl = eng.get_buffer(pkg.BUF_DRAFT_LOGITS)
        for v, lg in orc.node_adj.items():
            assert np.array_equal(dl[v], lg.astype(np.float32))    # the knob's adjustment, the same fp32 sum
        eng.verify()
        F, L = orc.verify()
        eng.set_buffer(pkg.BUF_LOGITS, L.astype(np.float32))
        ctx = orc.ctx
        before = {v: eng.get_kv_row(0, 1, ctx + v) for v in range(M)}
        out, ln, path = eng.accept()
        r = orc.accept()
        n = int(ln[0])
        assert [int(v) for v in path[0][:n]] == r["path"], f"step {step}: path differs (oracle margin {r['margin']})"
        assert [int(t) for t in out[0][:n]] == r["emitted"] and n == r["length"]
        for i, v in enumerate(r["path"]):
            k, vv = eng.get_kv_row(0, 1, ctx + i)
            assert np.array_equal(k, before[v][0]) and np.array_equal(vv, before[v][1])
        orc.commit(r["path"], r["bonus"])
        lens.append(n)
    say(f"kernels on oracle logits T={temperature}: accepted lengths {lens}")
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    assert max(lens) >= 3                                         # compaction really moved rows
    eng.close()


# ----------------------------------------------------------------------------- the oracle drives the engine
def test_force_tree_and_force_accept_follow_the_oracle():
    """The reverse direction of the lock-step protocol: the oracle drafts and accepts on its own, the engine is handed
    the oracle's tree (eagle_force_tree) and the oracle's path (eagle_force_accept); verify logits, the compacted
    cache and the pending features must follow."""
    s = synth.SHAPES["tiny"]
    par, rk = synth.TREES["T15"]
    eng = pkg.Eagle(s, par, rk, max_seq=160)
    eng.load_weights(synth.iter_weights(s, 41, synth.device_fmt(s)))
    W = synth.make_weights(s, 41, synth.oracle_fmt(s))
    orc = Oracle(s, W, par, rk, max_seq=160)
    prompt = synth.prompt(41, 16, s.vocab)
    fut = list(prompt) + Oracle(s, W, par, rk, max_seq=160).generate_vanilla(prompt, 60)
    orc.set_hint(fut, 0.8, 30.0, 3)                                # only the ORACLE is hinted: its tree differs from the engine's
    check_prefill(eng, orc, prompt, TOL["fp32"])
    differed = 0
    for step in range(8):
        g = list(eng.draft_tree()[0])
        orc.draft_tree()
        differed += g != orc.tok
        eng.force_tree(0, orc.tok)
        eng.verify()
        F, L = orc.verify()
        assert float(np.abs(eng.get_buffer(pkg.BUF_LOGITS) - L).max()) <= TOL["fp32"]
        r = orc.accept()
        eng.force_accept([r["path"]], [r["length"]], [r["bonus"]])
        orc.commit(r["path"], r["bonus"])
        state = eng.get_buffer(pkg.BUF_STATE)
        assert state[0] == len(orc.x) and state[1] == orc.ctx and state[2] == r["length"]
    assert differed >= 4
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    for layer in range(s.n_layers):
        for pos in range(len(prompt) - 1, orc.ctx):
            k, v = eng.get_kv_row(0, layer, pos)
            assert np.abs(k - orc.kc[layer][pos].reshape(-1)).max() < 1e-4
            assert np.abs(v - orc.vc[layer][pos].reshape(-1)).max() < 1e-4
    # a path that is not a root chain is refused and changes nothing
    eng.draft_tree(); eng.verify()
    with pytest.raises(pkg.EagleError):
        eng.force_accept([[0, 3]], [2], [1])                       # node 3 is not a child of the root in T15
    out, lens, path = eng.accept()                                 # the refused call left the verified state intact
    assert 1 <= int(lens[0]) <= orc.tree.D + 1
    eng.close()


# ----------------------------------------------------------------------------- out-of-order calls
def test_out_of_order_calls_return_estate():
    s = synth.SHAPES["tiny"]
    par, rk = synth.TREES["T15"]
    eng = pkg.Eagle(s, par, rk, max_seq=160)
    eng.load_weights(synth.iter_weights(s, 1, synth.device_fmt(s)))

    def code(fn, *a):
        with pytest.raises(pkg.EagleError) as e:
            fn(*a)
        return e.value.code

    assert code(eng.draft_tree) == -4                              # nothing prefilled
    eng.prefill(0, synth.prompt(1, 12, s.vocab))
    assert code(eng.verify) == -4                                  # verify before draft
    assert code(eng.accept) == -4                                  # accept before verify
    assert code(eng.force_tree, 0, [0] * len(par)) == -4           # no drafted tree yet
    eng.draft_tree()
    assert code(eng.accept) == -4                                  # drafted but not verified
    assert code(eng.force_accept, [[0]], [1], [0]) == -4
    eng.verify()
    out, lens, _ = eng.accept()
    eng.vanilla_step()
    assert code(eng.draft_tree) == -4                              # the head's cache is stale after a vanilla step
    assert code(eng.prefill, 1, [1, 2, 3]) == -1                   # slot beyond max_batch: EINVAL, not ESTATE
    eng.reset()
    eng.prefill(0, synth.prompt(1, 12, s.vocab))
    eng.step()                                                     # usable again after a reset
    eng.close()


# ----------------------------------------------------------------------------- bitwise repeatability, large shapes
@pytest.mark.parametrize("shape_name,tree,batch,prompt_len,steps", [
    ("llama2-13b", "T26", 1, 300, 6), ("llama2-70b", "T26", 1, 300, 4), ("llama2-7b", "T8", 4, 150, 6)])
def test_repeated_runs_are_bitwise_identical_large_shapes(shape_name, tree, batch, prompt_len, steps):
    """Split-K partials and attention split merges are read by the last work-group to arrive; a partial read before it
    landed would show as run-to-run differences.  Three runs of the same decode at the shapes with the most split-K
    groups and attention splits (13B, 70B widths; four sequences in one 32-row fast pass) must agree bit for bit;
    the comparison stops at the first differing step."""
    s = synth.SHAPES[shape_name].twin(2)
    par, rk = synth.TREES[tree]
    eng = pkg.Eagle(s, par, rk, max_batch=batch, max_seq=prompt_len + steps * 8 + 120)
    eng.load_weights(synth.iter_weights(s, 43, synth.device_fmt(s)))
    prompts = [synth.prompt(43, prompt_len + 7 * b, s.vocab, stream=b) for b in range(batch)]
    futs = vanilla_future(eng, prompts, steps * 6 + 8)
    first = None
    for rep in range(3):
        eng.reset()
        for b in range(batch):
            eng.prefill(b, prompts[b])
            eng.set_hint(b, futs[b], 0.7773, 1.0e4, 50 + b)
        logits = []
        for i in range(steps):
            eng.draft_tree()
            eng.verify()
            logits.append([eng.get_buffer(pkg.BUF_LOGITS, b).copy() for b in range(batch)])
            eng.accept()
        if first is None:
            first = logits
            continue
        for i in range(steps):
            for b in range(batch):
                assert np.array_equal(first[i][b], logits[i][b]), f"run {rep} step {i} slot {b} differs from run 0"
    eng.close()
