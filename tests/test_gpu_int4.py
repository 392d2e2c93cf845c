"""GPU parity of the 4-bit weight path (Sec. 4.2: target and head with int4-quantised weights): the library quantises
the bf16 weights it is given as it loads them; the oracle is the plain oracle run on the independently quantised and
de-quantised weights (oracle/int4_weights.py).  Same lock-step protocol and the same tolerance as the bf16 path: the
codes and scales are exact on both sides, so the only difference left is the order of fp32 additions."""
import numpy as np
import pytest

import paper_2401_15077_amd as pkg
import synth
from lockstep import Stats, check_prefill, lockstep_step
from oracle.eagle_oracle import Oracle
from oracle.int4_weights import quantize_model

pytestmark = pytest.mark.gpu

TOL = 2e-2


def run_int4(shape_name, n_layers, tree, seed, prompt_len, steps, dtype):
    s = synth.SHAPES[shape_name]
    if n_layers:
        s = s.twin(n_layers)
    par, rk = synth.TREES[tree]
    eng = pkg.Eagle(s, par, rk, max_seq=prompt_len + 8 * steps + 64, weight_bits=4)
    eng.load_weights(synth.iter_weights(s, seed, synth.device_fmt(s)))
    Wq = quantize_model(synth.make_weights(s, seed, synth.oracle_fmt(s)))
    orc = Oracle(s, Wq, par, rk, max_seq=prompt_len + 8 * steps + 64, dtype=dtype)
    prompt = synth.prompt(seed, prompt_len, s.vocab)
    fut = list(prompt) + [eng.prefill(0, prompt)]
    for _ in range(6 * steps + 8):
        fut.append(int(eng.vanilla_step()[0]))
    eng.reset()
    check_prefill(eng, orc, prompt, TOL)
    eng.set_hint(0, fut, 0.7773, 1.0e4, 11)
    orc.set_hint(fut, 0.7773, 1.0e4, 11)
    st = Stats()
    for _ in range(steps):
        lockstep_step(eng, orc, st, TOL)
    print(f"int4 {s.name}: tau={st.tau:.2f} max|dL|={st.max_logit_err:.2e} max|dF|={st.max_feat_err:.2e} "
          f"draft {st.max_draft_logit_err:.2e}/{st.max_draft_feat_err:.2e} excused {st.excused_tree_slots}/{st.excused_accepts}", flush=True)
    assert list(eng.get_buffer(pkg.BUF_TOKENS)) == orc.x
    assert st.tau > 1.5 and st.excused_accepts <= 1
    eng.close()
    return st


def test_int4_small_gqa_model_lockstep():
    """d 256, 8 query heads on 2 KV heads, FFN 384, vocab 512: two groups of 128 along every K, a 70-token prompt (three
    32-row prompt passes through the fused kernels), fp64 oracle."""
    run_int4("mini-gqa", 2, "T10", 51, 70, 8, np.float64)


def test_int4_llama7b_twin_lockstep():
    """LLaMA2-7B widths (K = 4096 and 11008: 32 and 86 groups), 2 target layers, T26 tree, knob on."""
    st = run_int4("llama2-7b", 2, "T26", 52, 96, 5, np.float32)
    assert st.max_logit_err < TOL


def test_int4_llama13b_twin_lockstep():
    """LLaMA2-13B widths (K = 5120 and 13824: 40 and 108 groups -- not multiples of the 8 waves that split them)."""
    run_int4("llama2-13b", 2, "T26", 53, 40, 3, np.float32)


def test_int4_llama70b_twin_lockstep():
    """LLaMA2-70B widths (d 8192, 64 query heads on 8 KV heads, K = 28672: 224 groups; one row block per CU for O and
    down), 2 target layers."""
    run_int4("llama2-70b", 2, "T26", 54, 40, 3, np.float32)


def test_int4_rejects_what_it_cannot_run():
    s = synth.SHAPES["tiny"]                                   # fp32 model
    par, rk = synth.TREES["T15"]
    with pytest.raises(pkg.EagleError) as e:
        pkg.Eagle(s, par, rk, max_seq=128, weight_bits=4)
    assert e.value.code == -1
    with pytest.raises(pkg.EagleError):
        pkg.Eagle(synth.SHAPES["mini-gqa"], *synth.TREES["B63"], max_seq=256, weight_bits=4)      # 63 rows per pass
