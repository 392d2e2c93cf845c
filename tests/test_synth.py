"""The seeded input generator: C and numpy implementations agree bit for bit; shapes are as stated."""
import numpy as np

import synth


def test_c_and_numpy_generators_agree():
    synth.build()
    for fmt in ("f32", "bf16", "bf16_f32"):
        a = synth.normal(11, 42, 4099, 0.02, 0.0, fmt, start=17)
        b = synth.normal_numpy(11, 42, 17, 4099, 0.02, 0.0, fmt)
        assert a.dtype == b.dtype and np.array_equal(a, b), fmt


def test_chunked_generation_is_position_addressed():
    a = synth.normal(5, 9, 1000, 0.02)
    b = np.concatenate([synth.normal(5, 9, 400, 0.02), synth.normal(5, 9, 600, 0.02, start=400)])
    assert np.array_equal(a, b)


def test_moments():
    a = synth.normal(3, 1, 1 << 20, 0.02).astype(np.float64)
    assert abs(a.mean()) < 1e-4 and abs(a.std() - 0.02) < 1e-4
    g = synth.normal(3, 2, 1 << 16, 0.02, 1.0).astype(np.float64)
    assert abs(g.mean() - 1.0) < 1e-3


def test_bf16_as_f32_is_widened_bf16():
    bits = synth.normal(8, 3, 513, 0.02, 0.0, "bf16")
    wide = synth.normal(8, 3, 513, 0.02, 0.0, "bf16_f32")
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), wide)
    full = synth.normal(8, 3, 513, 0.02, 0.0, "f32")
    assert np.max(np.abs(wide - full) / np.abs(full)) <= 2.0 ** -8


def test_prompt_range():
    p = synth.prompt(1, 4096, 1024)
    assert p.min() >= 0 and p.max() < 1024 and len(np.unique(p)) > 900
