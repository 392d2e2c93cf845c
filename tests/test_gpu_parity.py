"""GPU parity: the HIP path against the CPU oracle on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest

import paper_2401_15077_amd as pkg
import synth
from lockstep import Stats, check_prefill, lockstep_step, lockstep_step_batch
from oracle.eagle_oracle import Oracle, u24, PURPOSE_HINT

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def make_pair(shape_name, tree, seed, *, max_seq=256, temperature=0.0, rng_seed=0, dtype=np.float64, n_layers=None,
              kv_dtype="fp32"):
    s = synth.SHAPES[shape_name]
    if n_layers is not None:
        s = s.twin(n_layers)
    par, rk = synth.TREES[tree]
    eng = pkg.Eagle(s, par, rk, max_seq=max_seq, temperature=temperature, seed=rng_seed, kv_dtype=kv_dtype)
    eng.load_weights(synth.iter_weights(s, seed, synth.device_fmt(s)))
    orc = Oracle(s, synth.make_weights(s, seed, synth.oracle_fmt(s)), par, rk, max_seq=max_seq,
                 temperature=temperature, seed=rng_seed, dtype=dtype, kv_store="bf16" if kv_dtype == "bf16" else None)
    return s, eng, orc


def test_tiny_fp32_full_run_matches_oracle_and_vanilla():
    """Config 1: tiny fp32 model, 32-token prompt, 64 new tokens, T15 tree, greedy; also vanilla greedy."""
    s, eng, orc = make_pair("tiny", "T15", seed=1)
    prompt = synth.prompt(1, 32, s.vocab)
    print("prefill", flush=True)
    check_prefill(eng, orc, prompt, TOL["fp32"])
    st = Stats()
    gen = [orc.x[-1]]
    while len(gen) < 64:
        gen += lockstep_step(eng, orc, st, TOL["fp32"])
    print(f"steps={st.steps} tau={st.tau:.2f} max|dL|={st.max_logit_err:.2e} max|dF|={st.max_feat_err:.2e} "
          f"draft {st.max_draft_logit_err:.2e}/{st.max_draft_feat_err:.2e} excused={st.excused_tree_slots}/{st.excused_accepts}", flush=True)
    assert st.excused_accepts == 0 and st.excused_tree_slots == 0
    assert list(eng.get_buffer(pkg.BUF_TOKENS))[:len(orc.x)] == orc.x
    # the paper's invariant on the GPU side: speculative greedy == vanilla greedy, token for token
    eng.reset()
    eng.prefill(0, prompt)
    van = [int(eng.get_buffer(pkg.BUF_TOKENS)[-1])]
    while len(van) < 64:
        van.append(int(eng.vanilla_step()[0]))
    assert van == gen[:64]
    out, tau = eng.generate(prompt, 64)
    assert list(out) == gen[:64] and tau >= 1.0
    eng.close()


def test_tiny_hint_knob_accept_lengths_and_compaction():
    """Acceptance knob: accepted lengths equal the runs of hash hits; the compacted KV rows equal the oracle's."""
    s, eng, orc = make_pair("tiny", "T26", seed=2)
    prompt = synth.prompt(2, 20, s.vocab)
    par, rk = synth.TREES["T26"]
    future = list(prompt) + Oracle(s, synth.make_weights(s, 2, "f32"), par, rk, max_seq=256).generate_vanilla(prompt, 80)
    alpha, hseed = 0.75, 1234
    orc.set_hint(future, alpha, 30.0, hseed)
    check_prefill(eng, orc, prompt, TOL["fp32"])
    eng.set_hint(0, future, alpha, 30.0, hseed)
    st = Stats()
    while len(orc.x) < len(prompt) + 60:
        n = len(orc.x)
        run = 0
        while run < orc.tree.D and np.float32(u24(hseed, PURPOSE_HINT, 0, 0, 0, n + run) * 2.0 ** -24) < np.float32(alpha):
            run += 1
        lockstep_step(eng, orc, st, TOL["fp32"])
        assert st.lens[-1] == run + 1
    assert max(st.lens) >= 4 and st.excused_accepts == 0
    assert orc.x[:len(prompt) + 60] == future[:len(prompt) + 60]
    for layer in range(s.n_layers):
        for pos in (0, len(prompt) - 1, len(prompt) + 7, orc.ctx - 1):
            k, v = eng.get_kv_row(0, layer, pos)
            assert np.abs(k - orc.kc[layer][pos].reshape(-1)).max() < 1e-4
            assert np.abs(v - orc.vc[layer][pos].reshape(-1)).max() < 1e-4
    state = eng.get_buffer(pkg.BUF_STATE)
    assert state[0] == len(orc.x) and state[1] == orc.ctx and state[2] == st.lens[-1]
    eng.close()


def run_twin(shape_name, tree, seed, n_layers, prompt_len, n_new, alpha, max_seq=512, dtype=np.float32):
    s, eng, orc = make_pair(shape_name, tree, seed=seed, max_seq=max_seq, dtype=dtype, n_layers=n_layers)
    prompt = synth.prompt(seed, prompt_len, s.vocab)
    print(f"{s.name}: prefill", flush=True)
    # the knob follows the GPU's own vanilla continuation (as the benchmark does)
    first = eng.prefill(0, prompt)
    future = list(prompt) + [first]
    for _ in range(n_new + 8):
        future.append(int(eng.vanilla_step()[0]))
    eng.reset()
    check_prefill(eng, orc, prompt, TOL["bf16"])
    if alpha > 0:
        eng.set_hint(0, future, alpha, 1.0e4, 77)
        orc.set_hint(future, alpha, 1.0e4, 77)
    st = Stats()
    while len(orc.x) < len(prompt) + n_new:
        lockstep_step(eng, orc, st, TOL["bf16"])
    print(f"{s.name}: steps={st.steps} tau={st.tau:.2f} max|dL|={st.max_logit_err:.2e} max|dF|={st.max_feat_err:.2e} "
          f"draft {st.max_draft_logit_err:.2e}/{st.max_draft_feat_err:.2e} excused tree/accept="
          f"{st.excused_tree_slots}/{st.excused_accepts} lens={st.lens}", flush=True)
    toks = list(eng.get_buffer(pkg.BUF_TOKENS))
    assert toks == orc.x
    eng.close()
    return st, toks, future


def test_llama7b_twin_bf16_lockstep():
    """LLaMA2-7B widths (d 4096, 32x128 heads, FFN 11008, vocab 32000), 2 target layers, bf16, T26, knob on."""
    st, toks, future = run_twin("llama2-7b", "T26", seed=2, n_layers=2, prompt_len=96, n_new=48, alpha=0.7773)
    assert toks[:96 + 48] == future[:96 + 48]          # speculative == the GPU's vanilla decoding
    assert st.tau > 2.0


def test_tiny_stochastic_lockstep():
    """Temperature 1: children drawn without replacement (Gumbel top-k), Alg. 1 at every node, counter-based draws.
    Every accept test / draw whose oracle margin is not marginal must agree bit for bit."""
    s, eng, orc = make_pair("tiny", "T15", seed=4, temperature=1.0, rng_seed=2024)
    prompt = synth.prompt(4, 24, s.vocab)
    check_prefill(eng, orc, prompt, TOL["fp32"], margin_thr=1e-4)
    st = Stats()
    while len(orc.x) < len(prompt) + 48:
        lockstep_step(eng, orc, st, TOL["fp32"], margin_thr=1e-3, stoch_margin=1e-3)
    print(f"stochastic: steps={st.steps} tau={st.tau:.2f} max|dL|={st.max_logit_err:.2e} excused tree/accept="
          f"{st.excused_tree_slots}/{st.excused_accepts} lens={st.lens}", flush=True)
    assert st.excused_accepts <= 1 and st.excused_tree_slots <= 2
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    # reproducible: the same seed gives the same tokens
    eng.reset()
    eng.prefill(0, prompt)
    n = len(orc.x) - len(prompt)
    out = [int(eng.get_buffer(pkg.BUF_TOKENS)[-1])]
    while len(out) < n:
        toks, lens, _ = eng.step()
        out += [int(t) for t in toks[0][:lens[0]]]
    assert out[:n] == orc.x[len(prompt):len(prompt) + n]
    eng.close()


def test_gqa_twin_bf16_lockstep():
    """LLaMA2-70B widths are too large for a unit test; a grouped-query model (8 query heads on 2 KV heads) with the
    bf16 path and T10 tree exercises the head -> KV-head mapping, and the tiny T26 run above the 26-node tree."""
    st, toks, future = run_twin("mini-gqa", "T10", seed=5, n_layers=2, prompt_len=40, n_new=40, alpha=0.6, max_seq=256)
    assert toks[:80] == future[:80]


def test_moe_twin_bf16_lockstep():
    """Top-2 routed experts in the target AND in the head's layer (the Mixtral-shaped configuration in small):
    4 experts, grouped-query attention, bf16 weights.  The oracle runs in fp64 so that router near-ties are not an issue."""
    st, toks, future = run_twin("mini-moe", "T15", seed=6, n_layers=2, prompt_len=40, n_new=40, alpha=0.6, max_seq=256,
                                dtype=np.float64)
    assert toks[:80] == future[:80]


def test_batch4_lockstep():
    """Four independent sequences (different prompt lengths) advance together: the head's passes put the rows of all
    slots through the same GEMMs; the 4 x 15 verify rows exceed one 32-row pass and go through the general path
    together (one 60-row pass); every slot is compared with its own oracle."""
    s = synth.SHAPES["tiny"]
    par, rk = synth.TREES["T15"]
    eng = pkg.Eagle(s, par, rk, max_batch=4, max_seq=160)
    eng.load_weights(synth.iter_weights(s, 1, synth.device_fmt(s)))
    W = synth.make_weights(s, 1, synth.oracle_fmt(s))
    orcs, sts = [], []
    for b in range(4):
        orc = Oracle(s, W, par, rk, max_seq=160, seq_id=b)
        prompt = synth.prompt(1, 12 + 5 * b, s.vocab, stream=b)
        check_prefill(eng, orc, prompt, TOL["fp32"], seq=b)
        orcs.append(orc); sts.append(Stats())
    for _ in range(12):
        lockstep_step_batch(eng, orcs, sts, TOL["fp32"])
    for b in range(4):
        assert list(eng.get_buffer(pkg.BUF_TOKENS, b)) == orcs[b].x
        assert sts[b].excused_accepts == 0 and sts[b].max_logit_err < 1e-4
    eng.close()


@pytest.mark.parametrize("shape_name,n_layers,tol_key,steps", [("tiny", None, "fp32", 12), ("llama2-7b", 2, "bf16", 6)])
def test_batch4_small_tree_one_verify_pass(shape_name, n_layers, tol_key, steps):
    """Four sequences with an 8-node tree (the smaller tree for larger batches): the 4 x 8 verify rows fill exactly one
    32-row pass, so verify runs through the fused fast-path kernels with four sequences' rows side by side."""
    s = synth.SHAPES[shape_name]
    if n_layers is not None:
        s = s.twin(n_layers)
    par, rk = synth.TREES["T8"]
    eng = pkg.Eagle(s, par, rk, max_batch=4, max_seq=160)
    eng.load_weights(synth.iter_weights(s, 5, synth.device_fmt(s)))
    W = synth.make_weights(s, 5, synth.oracle_fmt(s))
    orcs, sts = [], []
    for b in range(4):
        orc = Oracle(s, W, par, rk, max_seq=160, seq_id=b)
        prompt = synth.prompt(5, 12 + 7 * b, s.vocab, stream=b)
        check_prefill(eng, orc, prompt, TOL[tol_key], seq=b)
        orcs.append(orc); sts.append(Stats())
    for _ in range(steps):
        lockstep_step_batch(eng, orcs, sts, TOL[tol_key])
    for b in range(4):
        assert list(eng.get_buffer(pkg.BUF_TOKENS, b)) == orcs[b].x
        assert sts[b].max_logit_err <= TOL[tol_key]
        if tol_key == "fp32":
            assert sts[b].excused_accepts == 0
    eng.close()


def test_moe_stochastic_lockstep():
    """The Mixtral-shaped configuration's mode in small: MoE target and head, temperature 1, seeded draws."""
    s, eng, orc = make_pair("mini-moe", "T15", seed=8, temperature=1.0, rng_seed=77, n_layers=2, dtype=np.float64)
    prompt = synth.prompt(8, 24, s.vocab)
    # draws: a differing draw is excused only if the oracle's point lay within 5 % of a bin width of the bin's edge
    # (bf16 weights: the two sides' probabilities differ by ~1e-3 relative)
    check_prefill(eng, orc, prompt, TOL["bf16"], margin_thr=5e-2)
    st = Stats()
    for _ in range(10):
        lockstep_step(eng, orc, st, TOL["bf16"], margin_thr=1e-3, stoch_margin=5e-2)
    print(f"moe stochastic: steps={st.steps} tau={st.tau:.2f} max|dL|={st.max_logit_err:.2e} excused={st.excused_tree_slots}/{st.excused_accepts}", flush=True)
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x and st.excused_accepts <= 1
    eng.close()


def test_llama7b_full_depth_lockstep():
    """The benchmark's own configuration (LLaMA2-7B shape, all 32 layers, bf16, T26, knob) checked against the fp32
    oracle for a few steps after a short prompt (the oracle's 27 GB of fp32 weights and its prefill bound the size)."""
    st, toks, future = run_twin("llama2-7b", "T26", seed=2, n_layers=32, prompt_len=48, n_new=12, alpha=0.7773, max_seq=256)
    assert toks[:60] == future[:60]
    assert st.max_logit_err < 2e-2 and st.max_feat_err < 2e-2



@pytest.mark.parametrize("shape_name,prompt_len,steps", [("llama2-13b", 1024, 10), ("llama2-70b", 2048, 6), ("mixtral-8x7b", 1024, 6)])
def test_full_size_speculative_equals_vanilla(shape_name, prompt_len, steps):
    """Configurations 3-5 at their full depth and the benchmark's prompt lengths, where the CPU oracle cannot follow:
    the property that holds at any size (Sec. 2: the method emits exactly the target's greedy tokens) -- the tokens of
    hinted speculative decoding equal those of the engine's own vanilla decoding, accepted lengths stay within
    1..depth+1, the accepted path is a root-to-node path of the tree -- in the launch configuration bench.py times.
    (The two runs agree up to rounding only -- a tree node's key sits at another cache slot than in vanilla decoding --
    so an arg-max near-tie could part them; runs are deterministic and none occurs for these seeds and lengths.)"""
    s = synth.SHAPES[shape_name]
    par, rk = synth.TREES["T26"]
    D = 5
    n_future = (steps + 2) * (D + 1) + 8
    eng = pkg.Eagle(s, par, rk, max_seq=prompt_len + n_future + len(par) + 80)
    eng.load_weights(synth.iter_weights(s, 2, synth.device_fmt(s)))
    prompt = synth.prompt(2, prompt_len, s.vocab)
    fut = list(prompt) + [eng.prefill(0, prompt)]
    for _ in range(n_future):
        fut.append(int(eng.vanilla_step()[0]))
    eng.reset()
    assert eng.prefill(0, prompt) == fut[prompt_len]
    eng.set_hint(0, fut, 0.7773, 30.0, 20240126)
    emitted = 0
    for _ in range(steps):
        toks, lens, paths = eng.step()
        n = int(lens[0])
        assert 1 <= n <= D + 1
        pth = [int(v) for v in paths[0][:n]]
        assert pth[0] == 0 and all(par[pth[i + 1]] == pth[i] for i in range(n - 1))
        emitted += n
    got = list(eng.get_buffer(pkg.BUF_TOKENS, 0))
    assert len(got) == prompt_len + 1 + emitted
    assert got == fut[:len(got)]
    assert emitted > steps                    # the knob makes the head's proposals land: more than one token per step
    eng.close()


def test_tiny_bf16_kv_cache():
    """The optional bf16 KV cache (keys and values rounded to nearest even when written) against the oracle's model
    of it.  A cache entry whose fp32 value sits within rounding distance of a bf16 tie can round differently on the
    two sides (one bf16 ulp = 0.4 % of that entry), hence the bf16 tolerance on an fp32 model."""
    s, eng, orc = make_pair("tiny", "T15", seed=12, kv_dtype="bf16")
    prompt = synth.prompt(12, 40, s.vocab)
    check_prefill(eng, orc, prompt, TOL["bf16"])
    st = Stats()
    while len(orc.x) < len(prompt) + 40:
        lockstep_step(eng, orc, st, TOL["bf16"])
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x and st.excused_accepts <= 1
    k, v = eng.get_kv_row(0, 1, 45)                     # stored values are bf16-representable
    assert np.all((k.view(np.uint32) & 0xFFFF) == 0) and np.all((v.view(np.uint32) & 0xFFFF) == 0)
    eng.close()


def test_llama7b_twin_prompt512():
    """The benchmark's context length (512-token prompt: 4 prefill chunks, 8 KV pages, 5 KV splits in attention) at
    LLaMA2-7B widths with 2 target layers."""
    st, toks, future = run_twin("llama2-7b", "T26", seed=7, n_layers=2, prompt_len=512, n_new=16, alpha=0.7773, max_seq=640)
    assert toks[:512 + 16] == future[:512 + 16]


def test_llama13b_twin_bf16_lockstep():
    """LLaMA2-13B widths (d 5120, 40 x 128 heads, FFN 13824): K slices that are not powers of two (5 and 14)."""
    st, toks, future = run_twin("llama2-13b", "T26", seed=3, n_layers=2, prompt_len=72, n_new=24, alpha=0.7773)
    assert toks[:72 + 24] == future[:72 + 24]


def test_llama70b_twin_bf16_lockstep():
    """LLaMA2-70B widths (d 8192, 64 query heads on 8 KV heads, FFN 28672), 2 target layers: 28 K slices in the down
    projection, more work-groups than CUs in gate/up, grouped-query attention at head_dim 128."""
    st, toks, future = run_twin("llama2-70b", "T26", seed=4, n_layers=2, prompt_len=40, n_new=12, alpha=0.7773, max_seq=256)
    assert toks[:52] == future[:52]


@pytest.mark.parametrize("shape_name,n_layers", [("llama2-7b", 2), ("mini-moe", 2)])
def test_repeated_runs_are_bitwise_identical(shape_name, n_layers):
    """Every reduction on the path has a fixed order and every cross-work-group exchange is published before it is
    read, so two runs of the same decode give the same bits: verify logits compared step by step over three runs
    (hinted speculative decoding after the engine's own vanilla run), and the tokens equal the vanilla tokens."""
    s = synth.SHAPES[shape_name].twin(n_layers)
    par, rk = synth.TREES["T26" if shape_name != "mini-moe" else "T15"]
    eng = pkg.Eagle(s, par, rk, max_seq=512)
    eng.load_weights(synth.iter_weights(s, 7, synth.device_fmt(s)))
    prompt = synth.prompt(7, 130, s.vocab)
    steps = 12
    fut = list(prompt) + [eng.prefill(0, prompt)]
    for _ in range(steps * 6 + 8):
        fut.append(int(eng.vanilla_step()[0]))
    runs = []
    for rep in range(3):
        eng.reset()
        eng.prefill(0, prompt)
        eng.set_hint(0, fut, 0.7773, 30.0, 1234)
        logits = []
        for _ in range(steps):
            eng.draft_tree()
            eng.verify()
            logits.append(eng.get_buffer(pkg.BUF_LOGITS, 0).copy())
            eng.accept()
        toks = list(eng.get_buffer(pkg.BUF_TOKENS, 0))
        assert toks == fut[:len(toks)]
        runs.append(logits)
    for rep in (1, 2):
        for a, b in zip(runs[0], runs[rep]):
            assert np.array_equal(a, b)
    eng.close()


@pytest.mark.parametrize("tree,n_new", [("root", 10), ("chain5", 24), ("B63", 24)])
def test_tiny_other_trees(tree, n_new):
    """Degenerate and large trees on the tiny fp32 model: a tree of the root alone (every step is a vanilla step and
    emits exactly one token), a chain, and a 63-node full binary tree (verify rows exceed one 32-row pass: the
    128-row general path; its deepest level has 32 rows)."""
    s, eng, orc = make_pair("tiny", tree, seed=9)
    prompt = synth.prompt(9, 20, s.vocab)
    check_prefill(eng, orc, prompt, TOL["fp32"])
    st = Stats()
    while len(orc.x) < len(prompt) + n_new:
        lockstep_step(eng, orc, st, TOL["fp32"])
    assert st.excused_accepts == 0 and st.excused_tree_slots == 0
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    if tree == "root":
        assert all(n == 1 for n in st.lens)
    van = Oracle(s, synth.make_weights(s, 9, synth.oracle_fmt(s)), *synth.TREES[tree], max_seq=256).generate_vanilla(prompt, n_new)
    assert orc.x[len(prompt):len(prompt) + n_new] == van[:n_new]
    eng.close()


def test_tiny_edges_one_token_prompt_page_crossing_and_full_cache():
    """A one-token prompt; decoding across KV page boundaries (64-token pages: positions 63/64 and 127/128 are
    crossed by tree slots and by compaction); and the error when the cache cannot hold another tree."""
    s, eng, orc = make_pair("tiny", "T15", seed=11, max_seq=160)
    prompt = synth.prompt(11, 1, s.vocab)
    check_prefill(eng, orc, prompt, TOL["fp32"])
    st = Stats()
    with pytest.raises(pkg.EagleError) as err:
        while True:
            if orc.ctx + orc.tree.M + 1 > 160:
                eng.step()                      # must refuse: the tree no longer fits
                break
            lockstep_step(eng, orc, st, TOL["fp32"])
    assert err.value.code == -3                 # EAGLE_ESEQ_FULL
    assert orc.ctx > 128 and st.excused_accepts == 0
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    # KV rows on both sides of the page boundaries equal the oracle's
    for layer in range(s.n_layers):
        for pos in (0, 63, 64, 65, 127, 128, orc.ctx - 1):
            k, v = eng.get_kv_row(0, layer, pos)
            assert np.abs(k - orc.kc[layer][pos].reshape(-1)).max() < 1e-4
            assert np.abs(v - orc.vc[layer][pos].reshape(-1)).max() < 1e-4
    eng.close()
