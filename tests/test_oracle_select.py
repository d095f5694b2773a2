"""Pins of the oracle's reuse-map selection statistic (Algorithm 2, steps 1-2): per-head mean L1
distance between adjacent layers."""
import numpy as np

from oracle import kvcar_oracle as O


def test_scalar_loops():
    rng = np.random.default_rng(0)
    T, H, dh = 5, 3, 4
    a, b = rng.normal(size=(T, H * dh)), rng.normal(size=(T, H * dh))
    want = []
    for g in range(H):
        s = 0.0
        for t in range(T):
            for k in range(dh):
                s += abs(b[t][g * dh + k] - a[t][g * dh + k])
        want.append(s / (T * dh))
    np.testing.assert_allclose(O.head_l1_distance(a, b, H, dh), want, rtol=1e-14)


def test_closed_forms():
    rng = np.random.default_rng(1)
    T, H, dh = 64, 4, 8
    a = rng.normal(size=(T, H * dh))
    assert (O.head_l1_distance(a, a, H, dh) == 0).all()                       # identical layers
    b = a.copy()
    b[:, 2 * dh:3 * dh] += 0.75                                               # one head shifted by a constant
    np.testing.assert_allclose(O.head_l1_distance(a, b, H, dh), [0, 0, 0.75, 0], atol=1e-15)
    c = rng.normal(size=(T, H * dh))
    d1, d2 = O.head_l1_distance(a, c, H, dh), O.head_l1_distance(c, a, H, dh)
    np.testing.assert_array_equal(d1, d2)                                     # symmetric
    np.testing.assert_allclose(O.head_l1_distance(3 * a, 3 * c, H, dh), 3 * d1, rtol=1e-14)   # homogeneous
    e = rng.normal(size=(T, H * dh))
    assert (O.head_l1_distance(a, e, H, dh) <= d1 + O.head_l1_distance(c, e, H, dh) + 1e-15).all()   # triangle inequality


def test_mean_of_minibatches_equals_the_whole_batch():
    """The paper averages the statistic over mini-batches: for equal-sized ones that is the statistic
    of the concatenated batch."""
    rng = np.random.default_rng(2)
    H, dh = 2, 4
    a, b = rng.normal(size=(40, H * dh)), rng.normal(size=(40, H * dh))
    parts = [O.head_l1_distance(a[i:i + 10], b[i:i + 10], H, dh) for i in range(0, 40, 10)]
    np.testing.assert_allclose(np.mean(parts, axis=0), O.head_l1_distance(a, b, H, dh), rtol=1e-14)


def test_gaussian_expectation():
    """Independent N(0, s1^2) and N(0, s2^2) entries: E|x - y| = sqrt(2 (s1^2 + s2^2) / pi)."""
    rng = np.random.default_rng(3)
    a, b = rng.normal(0, 1.0, size=(20000, 16)), rng.normal(0, 2.0, size=(20000, 16))
    got = O.head_l1_distance(a, b, 2, 8)
    np.testing.assert_allclose(got, np.sqrt(2 * 5 / np.pi), rtol=1e-2)
