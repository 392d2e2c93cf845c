"""eagle_accept_static (acceptance + commit with the kernels' scratch in the library's static device array) against
eagle_accept (scratch in the caller's workspace): same inputs, outputs bit-exact -- accepted tokens, lengths, paths --
and the same state afterwards (the next step's tree and verify logits agree bit for bit).  Two calls in a row share
the one static array: the second works on a smaller input (fewer slots, smaller vocabulary use) and must not see
anything the first left behind."""
import numpy as np
import pytest

import paper_2401_15077_amd as pkg
import synth

pytestmark = pytest.mark.gpu


def pair(shape_name, tree, batch, temperature, seed):
    s = synth.SHAPES[shape_name]
    par, rk = synth.TREES[tree]
    engs = []
    for _ in range(2):
        e = pkg.Eagle(s, par, rk, max_batch=batch, max_seq=160, temperature=temperature, seed=99)
        e.load_weights(synth.iter_weights(s, seed, synth.device_fmt(s)))
        for b in range(batch):
            e.prefill(b, synth.prompt(seed, 14 + 5 * b, s.vocab, stream=b))
        engs.append(e)
    return engs


def run_and_compare(a, b, steps):
    """a commits with eagle_accept, b with eagle_accept_static; everything observable must stay identical."""
    total = 0
    for i in range(steps):
        ta, tb = a.draft_tree(), b.draft_tree()
        assert np.array_equal(ta, tb), f"step {i}: trees differ"
        a.verify(); b.verify()
        for s in range(a.n_active):
            assert np.array_equal(a.get_buffer(pkg.BUF_LOGITS, s), b.get_buffer(pkg.BUF_LOGITS, s)), f"step {i}: verify logits differ"
        oa, la, pa = a.accept()
        ob, lb, pb = b.accept_static()
        assert np.array_equal(la, lb) and np.array_equal(oa, ob) and np.array_equal(pa, pb), f"step {i}: {la} {lb} {pa} {pb}"
        for s in range(a.n_active):
            assert np.array_equal(a.get_buffer(pkg.BUF_STATE, s), b.get_buffer(pkg.BUF_STATE, s))
        total += int(la.sum())
    for s in range(a.n_active):
        assert np.array_equal(a.get_buffer(pkg.BUF_TOKENS, s), b.get_buffer(pkg.BUF_TOKENS, s))
    return total


def test_accept_static_matches_accept_on_two_calls_in_a_row_the_second_smaller():
    # first: two sequences, temperature 1 (both probability vectors of Alg. 1 live in the static array), vocab 32000
    a, b = pair("tiny-v32k", "T15", 2, 1.0, 3)
    n1 = run_and_compare(a, b, 4)
    a.close(); b.close()
    # second, smaller: one sequence, vocab 1024, temperature 1 -- then greedy (the arg-max array overlays the same bytes)
    a, b = pair("tiny", "T15", 1, 1.0, 4)
    n2 = run_and_compare(a, b, 4)
    a.close(); b.close()
    a, b = pair("tiny", "T26", 1, 0.0, 5)
    run_and_compare(a, b, 3)
    a.close(); b.close()
    assert n1 > 8 and n2 > 4                                     # paths longer than one token were committed


def test_accept_static_rejects_sizes_beyond_the_static_array():
    s = synth.SHAPES["tiny-v40k"]
    par, rk = synth.TREES["T8"]                                  # 16 x 8 nodes = the 128 rows one pass can hold
    e = pkg.Eagle(s, par, rk, max_batch=16, max_seq=96, temperature=1.0)
    e.load_weights(synth.iter_weights(s, 1, synth.device_fmt(s)))
    for b in range(16):
        e.prefill(b, synth.prompt(1, 6, s.vocab, stream=b))
    e.draft_tree(); e.verify()
    with pytest.raises(pkg.EagleError) as err:
        e.accept_static()                                        # 2 x 16 x 40000 floats = 5.1 MB > 4 MiB
    assert err.value.code == -1 and "static" in str(err.value)
    out, lens, path = e.accept()                                 # the refused call launched nothing: the state is intact
    assert all(1 <= int(n) <= 5 for n in lens)
    e.close()
