"""The seeded input generator: determinism, value distributions of the paper-shaped workload."""
import numpy as np

from datagen import synth


def test_frames_are_a_pure_function_of_seed_stream_id():
    a = synth.frames(5, synth.STREAM_REPLAY, [3, 9, 3])
    assert a.shape == (3, 84, 84) and a.dtype == np.uint8
    assert np.array_equal(a[0], a[2]) and not np.array_equal(a[0], a[1])
    assert not np.array_equal(a[0], synth.frames(6, synth.STREAM_REPLAY, [3])[0])
    assert not np.array_equal(a[0], synth.frames(5, synth.STREAM_ACT, [3])[0])


def test_pixel_word_definition_scalar():
    # re-derive a few pixels with Python integers from the documented definition
    seed, i = 12345, 77
    f = synth.frames(seed, synth.STREAM_REPLAY, [i])[0].reshape(-1)
    a = synth.stream_key(seed, synth.STREAM_REPLAY)
    for p in (0, 1, 2, 1001, 7055):
        b = synth._mix64_int(a + i)
        w = synth._mix64_int(b + synth.GAMMA * (p // 2 + 1))
        w32 = (w >> (32 * (p % 2))) & 0xFFFFFFFF
        want = (w32 & 0xFF) if (w32 >> 8) < synth.PIX_T else 40
        assert f[p] == want


def test_distributions():
    f = synth.frames(1, synth.STREAM_REPLAY, np.arange(200))
    frac = (f != 40).mean()
    assert abs(frac - 0.05 * 255 / 256) < 0.002
    a, r, d = synth.transitions(1, np.arange(200000), 18)
    assert abs((r == -1).mean() - 0.05) < 0.003 and abs((r == 1).mean() - 0.05) < 0.003
    assert abs(d.mean() - 0.001) < 0.0004
    assert a.min() == 0 and a.max() == 17
    a2, r2, d2 = synth.transitions(1, np.arange(100000), 18, 0.1, 0.1, 0.01)
    assert abs((r2 != 0).mean() - 0.2) < 0.006 and abs(d2.mean() - 0.01) < 0.002


def test_init_params_bounds():
    p = synth.init_params(3, 6)
    assert p.dtype == np.float32 and p.size == synth.num_params(6) == 1687206
    assert np.abs(p[:8192]).max() <= 1 / 16 and np.abs(p[:8192]).max() > 0.06
