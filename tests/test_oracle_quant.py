"""Pins of the oracle's int8 latent quantiser (Methodology, "Quantization", Eq. "quant") to things
other than itself: rows worked by hand (tests/golden/quant_worked_rows.txt), exact rational
arithmetic, an arithmetic progression, the half-step error bound, and invariances."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import kvcar_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_worked_rows.txt")


def golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = [c.strip() for c in line.split("|")]
        rows.append((f[0], [float(v) for v in f[1].split()], float(f[2]), int(f[3]), [int(v) for v in f[4].split()]))
    return rows


@pytest.mark.parametrize("row", golden_rows(), ids=lambda r: r[0])
def test_hand_worked_rows(row):
    _, x, scale, zp, codes = row
    c, s, z = O.quantize_rows(np.array([x]))
    assert s[0] == np.float32(scale)
    assert z[0] == zp
    assert c[0].tolist() == codes
    # last line of the equation, written out
    want = [(q - zp) / scale for q in codes]
    np.testing.assert_allclose(O.dequantize_rows(c, s, z)[0], want, rtol=0, atol=1e-15)


def rational_quantize(xs):
    """The four lines of the equation in exact rational arithmetic (Python's round() on a Fraction
    rounds half to even)."""
    xs = [Fraction(v) for v in xs]
    mn, mx = min(xs), max(xs)
    scale = Fraction(255) / (mx - mn)
    zp = -round(scale * mn) - 128
    return [max(-128, min(127, round(scale * v + zp))) for v in xs], scale, zp


def test_against_exact_rational_arithmetic():
    """Rows whose range is 255 * 2^k have a power-of-two scale, so every fp32 operation of the
    oracle is exact and must agree with rational arithmetic, ties included."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        k = int(rng.integers(-6, 4))
        step = 2.0 ** (k - 2)                                  # quarter steps: many exact ties at .5
        n = int(rng.integers(2, 40))
        lo = float(rng.integers(-300, 300)) * step * 4
        x = lo + rng.integers(0, 255 * 4 + 1, size=n) * step
        x[0], x[1] = lo, lo + 255 * 4 * step                 # range = 255 * 2^k
        want, scale, zp = rational_quantize(x.tolist())
        c, s, z = O.quantize_rows(x[None])
        assert Fraction(float(s[0])) == scale
        assert int(z[0]) == zp
        assert c[0].tolist() == want


def test_arithmetic_progression_hits_every_code():
    for lo, step in ((0.0, 1.0), (-7.5, 0.125), (3.0, 2.0 ** -10)):
        x = lo + step * np.arange(256)
        c, s, z = O.quantize_rows(x[None])
        assert c[0].tolist() == list(range(-128, 128))
        np.testing.assert_allclose(O.dequantize_rows(c, s, z)[0], x, rtol=1e-6, atol=1e-6 * abs(lo))


def test_half_step_error_bound_and_extremes():
    rng = np.random.default_rng(5)
    z = rng.normal(0, 0.3, size=(64, 128))
    z[3] *= 1e-3
    z[4] += 10.0
    c, s, zp = O.quantize_rows(z)
    z32 = z.astype(np.float32).astype(np.float64)
    err = np.abs(O.dequantize_rows(c, s, zp) - z32)
    bound = 0.5 / s.astype(np.float64)
    assert (err <= bound[:, None] * (1 + 1e-5) + 1e-7 * np.abs(z32).max(axis=1)[:, None]).all()
    # the smallest element always takes the code -128; the largest 126 or 127
    assert (c[np.arange(64), z32.argmin(axis=1)] == -128).all()
    assert (c[np.arange(64), z32.argmax(axis=1)] >= 126).all()
    assert c.min() == -128 and c.max() == 127


def test_invariance_under_dyadic_scaling_and_exact_shifts():
    rng = np.random.default_rng(9)
    x = rng.integers(-2000, 2000, size=(16, 48)).astype(np.float64) / 64.0
    c0, s0, z0 = O.quantize_rows(x)
    for k in (-5, 3):
        c, s, z = O.quantize_rows(x * 2.0 ** k)
        assert (c == c0).all() and (z == z0).all()
        np.testing.assert_array_equal(s, s0 * np.float32(2.0 ** -k))
    # a shift changes only the zero point when scale * shift is an exact even integer
    x = np.array([[0.0, 17.0, 101.0, 255.0]])
    c0, s0, z0 = O.quantize_rows(x)
    c, s, z = O.quantize_rows(x + 64.0)
    assert (c == c0).all() and s[0] == s0[0] and z[0] == z0[0] - 64


def test_int8_oracle_path_is_attention_over_dequantised_latents():
    """With latent_format='int8' the path is: encode, quantise, store codes; dequantise, decode,
    attend.  Checked against attention written out here from the stored codes."""
    rng = np.random.default_rng(11)
    hq = hkv = 2
    dh, r, L = 4, 6, 9
    d = hkv * dh
    enc = [(rng.normal(0, 0.5, (d, r)), rng.normal(0, 0.1, r))]
    dec = [(rng.normal(0, 0.5, (r, d)), rng.normal(0, 0.1, d))]
    orc = O.KVCAROracle(1, hq, hkv, dh, 1, L, "f32", latent_format="int8")
    for which in (0, 1):
        orc.set_autoencoder(0, which, O.Autoencoder([0, 1], enc, dec))
    k = rng.normal(size=(1, L, d))
    v = rng.normal(size=(1, L, d))
    orc.encode_append(0, k, v, 0)
    q = rng.normal(size=(1, hq, dh))
    got = orc.decode_attention(0, q, L)
    # written out: codes of the fp32-rounded latent rows, dequantised, decoded, softmax attention
    zk = (k[0] @ enc[0][0] + enc[0][1]).astype(np.float32)
    zv = (v[0] @ enc[0][0] + enc[0][1]).astype(np.float32)
    assert (orc.Q[(0, 0)][0] == O.quantize_rows(zk)[0]).all()
    for j in range(hq):
        kh = (O.dequantize_rows(*O.quantize_rows(zk)) @ dec[0][0] + dec[0][1])[:, j * dh:(j + 1) * dh]
        vh = (O.dequantize_rows(*O.quantize_rows(zv)) @ dec[0][0] + dec[0][1])[:, j * dh:(j + 1) * dh]
        s = kh @ q[0, j] / 2.0
        p = np.exp(s - s.max())
        np.testing.assert_allclose(got[0, j], (p / p.sum()) @ vh, rtol=1e-12, atol=1e-14)
    # quantisation error of the stored latents stays within half a step per element
    err = np.abs(orc.Z[(0, 0)][0] - zk.astype(np.float64))
    assert (err <= 0.5 / orc.Qscale[(0, 0)][0][:, None].astype(np.float64) * (1 + 1e-5) + 1e-7).all()


def test_quantized_cache_bytes():
    # TinyLlama shape, r = 128 for K and V in 22 layers: 128 + 8 bytes per row against 256 in bf16
    w = np.full((22, 2), 128)
    assert O.quantized_latent_cache_bytes(w, 8192, 256) == 22 * 2 * 136 * 8192 * 256
    assert O.latent_cache_bytes(2, w, 8192, 256) == 22 * 2 * 256 * 8192 * 256
    w[5, 0] = 0                                   # a layer-tensor that stores nothing has no row metadata either
    assert O.quantized_latent_cache_bytes(w, 1, 1) == 43 * 136
