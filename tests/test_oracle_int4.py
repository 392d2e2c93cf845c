"""Pins of the int4 weight oracle (Sec. 4.2: int4-quantised weights, gpt-fast case study): none of them re-types
the quantiser; they check it against what arithmetic fixes."""
import numpy as np
import pytest

from oracle import int4_weights as q4


def test_hand_example_codes_scales_and_values():
    # one group of 128: max |w| = 7 * 0.25 -> scale 0.25 (a bf16 value); entries on and off the grid
    w = np.zeros((1, 128), np.float32)
    w[0, :8] = [1.75, -1.75, 0.25, -0.25, 0.125, 0.375, -2.0, 0.0]     # 0.125 / 0.25 = 0.5 -> ties to even -> 0; 0.375 -> 1.5 -> 2
    w[0, 6] = -1.75
    q, s = q4.quantize(w)
    assert s.shape == (1, 1) and s[0, 0] == np.float32(0.25)
    assert list(q[0, :8]) == [8 + 7, 8 - 7, 8 + 1, 8 - 1, 8 + 0, 8 + 2, 8 - 7, 8]
    np.testing.assert_array_equal(q4.dequantize(q, s)[0, :8], np.float32([1.75, -1.75, 0.25, -0.25, 0.0, 0.5, -1.75, 0.0]))


def test_codes_in_range_and_error_within_half_a_step():
    rng = np.random.default_rng(0)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    q, s = q4.quantize(W)
    assert q.dtype == np.uint8 and q.min() >= 1 and q.max() <= 15          # -8 is never produced by max/7 scaling
    assert np.all((s.view(np.uint32) & 0xFFFF) == 0)                      # scales are bf16 values
    What = q4.dequantize(q, s)
    step = np.repeat(s, q4.GROUP, axis=1)
    # rounding error at most half a step, plus what the bf16 rounding of the scale shifts the extreme entries by
    assert np.all(np.abs(What - W) <= 0.5 * step + 7 * step * 2.0 ** -8)
    # the largest entry of every group keeps its sign and maps to +-7
    Wg = W.reshape(64, 4, 128); qg = q.reshape(64, 4, 128).astype(int) - 8
    idx = np.argmax(np.abs(Wg), axis=2)
    top = np.take_along_axis(qg, idx[:, :, None], axis=2)[:, :, 0]
    assert np.all(np.abs(top) == 7) and np.all(np.sign(top) == np.sign(np.take_along_axis(Wg, idx[:, :, None], axis=2)[:, :, 0]))


def test_values_on_the_grid_survive_exactly_and_requantising_is_idempotent():
    rng = np.random.default_rng(1)
    s = np.float32(2.0 ** -6)
    codes = rng.integers(-7, 8, size=(8, 256))
    codes[:, 0] = 7; codes[:, 128] = -7                                  # pin the maximum of every group
    W = (codes * s).astype(np.float32)
    q, sc = q4.quantize(W)
    assert np.all(sc == s) and np.array_equal(q.astype(int) - 8, codes)
    np.testing.assert_array_equal(q4.dequantize(q, sc), W)
    W2 = q4.dequantize(*q4.quantize((np.random.default_rng(2).standard_normal((16, 384)) * 0.02).astype(np.float32)))
    np.testing.assert_array_equal(q4.dequantize(*q4.quantize(W2)), W2)


def test_all_zero_group_and_bad_shapes():
    W = np.zeros((2, 256), np.float32); W[1, 130] = 0.5
    q, s = q4.quantize(W)
    assert s[0, 0] == 0 and s[0, 1] == 0 and s[1, 0] == 0 and s[1, 1] > 0
    np.testing.assert_array_equal(q4.dequantize(q, s)[0], 0)
    with pytest.raises(ValueError):
        q4.quantize(np.zeros((2, 100), np.float32))


def test_quantize_model_touches_matrices_only():
    rng = np.random.default_rng(3)
    W = {"embed": rng.standard_normal((10, 128)).astype(np.float32), "lm_head": rng.standard_normal((10, 128)).astype(np.float32),
         "final_norm": np.ones(128, np.float32), "layers.0.wq": rng.standard_normal((128, 128)).astype(np.float32),
         "layers.0.attn_norm": np.ones(128, np.float32), "head.fc_w": rng.standard_normal((128, 256)).astype(np.float32),
         "head.fc_b": rng.standard_normal(128).astype(np.float32), "layers.0.router": rng.standard_normal((4, 128)).astype(np.float32),
         "layers.0.gate": rng.standard_normal((4, 256, 128)).astype(np.float32)}
    Q = q4.quantize_model(W)
    for name in ("embed", "final_norm", "layers.0.attn_norm", "head.fc_b", "layers.0.router"):
        assert Q[name] is W[name]
    for name in ("lm_head", "layers.0.wq", "head.fc_w", "layers.0.gate"):
        assert Q[name].shape == W[name].shape and not np.array_equal(Q[name], W[name])
        assert len(np.unique(np.round(Q[name].reshape(-1, 128)[0] / np.abs(Q[name].reshape(-1, 128)[0]).max() * 7))) <= 15
