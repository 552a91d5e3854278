"""The seeded input generator is shared by the oracle's tests, the GPU tests and the benchmark; its bits are
pinned here, so that a change of the random-number library (or of the recipe) shows up as a failure of this
file and not as a silent change of every workload.  CPU only."""
import numpy as np

import workloads as wl


def _sums(t):
    return [wl.checksum(x) for x in (t.k, t.v, t.qwin, t.q)]


def test_generator_bits_are_pinned():
    assert _sums(wl.generate(wl.small())) == [537831646761, 544400921432, 66968851379, 1052754425]
    t = wl.generate(wl.config(1))
    assert _sums(t) == [8573314353636, 8570430757043, 1073256831475, 4176371207]
    assert t.cu.tolist() == [0, 1024]
    # the ragged configuration's lengths
    w4 = wl.config(4)
    assert w4.seqlens[:6].tolist() == [1000, 512, 1596, 1167, 1053, 1863] and w4.total == 83800


def test_quiet_channels_touch_the_keys_only_and_only_when_asked():
    base = wl.generate(wl.small())
    w = wl.small()
    w.quiet_fraction, w.quiet_scale = 0.6, 0.008
    t = wl.generate(w)
    assert wl.checksum(t.k) == 532793246328
    assert np.array_equal(t.v, base.v) and np.array_equal(t.q, base.q) and np.array_equal(t.qwin, base.qwin)
    # about 60 % of the channels of every head carry little magnitude
    mag = np.abs(wl.bf16_bits_to_f32(t.k)).mean(axis=1)                    # [Hkv, D]
    quiet = (mag < 0.1 * np.median(np.abs(wl.bf16_bits_to_f32(base.k)).mean(axis=1))).mean()
    assert 0.45 < quiet < 0.75


def test_bf16_rounding_is_nearest_even_and_round_trips():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40, 0.0], np.float32)
    b = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[3] == -2.5 and back[6] == 0.0
    assert back[1] == 1.0                      # 1 + 2^-8: a tie, rounds to the even neighbour 1.0
    assert back[2] == np.float32(1.015625)     # 1 + 3 * 2^-8: a tie, rounds to the even neighbour 1 + 2^-6
    assert np.array_equal(wl.f32_to_bf16_bits(back), b)
