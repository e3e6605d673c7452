"""Pins for the seed -> W generator of the oracle (Algorithm 1, step 2: rows of W i.i.d. N(0, I_d))."""
import math
import os

import numpy as np

from oracle import race_oracle as ro


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) if l[0] not in "#\n"]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        assert list(ro.philox4x32_10(v[0:4], v[4:6])) == v[6:10]


def test_box_muller_by_hand():
    # u1 = u2 = (2^31 + 0.5) / 2^32: radius sqrt(2 ln 2) to 1e-9, angle pi (+ 2 pi 2^-33)
    g0, g1 = ro._box_muller(1 << 31, 1 << 31)
    rad = math.sqrt(2 * math.log(2.0))
    assert abs(g0 + rad) < 1e-8 and abs(g1) < 1e-8
    # x1 = 2^30 - 1/2 is not representable; x1 = 2^30 gives angle pi/2 (+ tiny): cos ~ 0, sin ~ 1
    g0, g1 = ro._box_muller(1 << 31, 1 << 30)
    assert abs(g0) < 1e-8 and abs(g1 - rad) < 1e-8


def test_w_layout_seed_and_prefix_property():
    # element e = row*d + col comes from block e//4, so a shorter matrix is a prefix of a longer one
    a = ro.expand_projection(7, 2, 3, 16)
    b = ro.expand_projection(7, 4, 3, 16)
    assert a.shape == (6, 16) and np.array_equal(a, b[:6])
    assert not np.array_equal(a, ro.expand_projection(8, 2, 3, 16))
    # the high 32 bits of the seed are part of the key
    assert not np.array_equal(a, ro.expand_projection(7 + (1 << 32), 2, 3, 16))
    # values are exactly representable in fp32
    assert np.array_equal(a, a.astype(np.float32).astype(np.float64))


def test_w_is_standard_normal():
    w = ro.expand_projection(123456789, 64, 8, 128).ravel()      # 65536 samples
    n = w.size
    assert abs(w.mean()) < 4 / math.sqrt(n)
    assert abs(w.var() - 1) < 4 * math.sqrt(2 / n)
    assert abs((w ** 3).mean()) < 4 * math.sqrt(15 / n)
    assert abs((w ** 4).mean() - 3) < 4 * math.sqrt(96 / n)
    # Kolmogorov-Smirnov distance to the normal CDF
    xs = np.sort(w)
    cdf = 0.5 * (1 + np.vectorize(math.erf)(xs / math.sqrt(2)))
    ks = np.max(np.abs(cdf - (np.arange(1, n + 1) - 0.5) / n))
    assert ks < 1.95 / math.sqrt(n)
    # rows are uncorrelated
    m = w.reshape(512, 128)
    g = m @ m.T / 128
    off = g[~np.eye(512, dtype=bool)]
    assert abs(off.mean()) < 1e-3 and off.std() < 1.2 / math.sqrt(128)


def test_bf16_rounding():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.14159], dtype=np.float32)
    r = ro.round_to_bf16(x)
    # ties to even: 1 + 2^-8 -> 1 (even mantissa), 1 + 3*2^-8 -> 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.0 + 2 ** -7) and r[3] == np.float32(1.0 + 2 ** -6)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
