"""Pins of the oracle's two variants of the decode step: the paper's form with the current token's
exact key / value row concatenated to the decoded cache rows ("Network Architecture", 2nd paragraph),
and ragged batches (per-sequence context lengths and append positions)."""
import math

import numpy as np
import pytest

from oracle import kvcar_oracle as O
from tests.test_oracle_pins import rand, tiny_oracle


def scalar_attention(q, krows, vrows, scale):
    """Eq. 1 for one head with Python scalars."""
    s = [scale * sum(a * b for a, b in zip(q, k)) for k in krows]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    tot = sum(e)
    return [sum(e[t] / tot * vrows[t][c] for t in range(len(vrows))) for c in range(len(vrows[0]))]


def test_exact_current_token_brute_force():
    """Cached rows are decoded, the current row is used as given: written out with scalars."""
    orc = tiny_oracle(hq=4, hkv=2, dh=3, r=4, L=6)
    D = 6
    k, v = rand(1, 5, D), rand(1, 5, D)
    orc.encode_append(0, k, v, 0)
    q, kc, vc = rand(1, 4, 3), rand(1, D), rand(1, D)
    got = orc.decode_attention(0, q, 5, k_cur=kc, v_cur=vc)
    for j in range(4):
        g = j // 2
        kh = orc.ae[(0, 0)].decode(orc.Z[(0, 0)][0, :5])[:, g * 3:(g + 1) * 3].tolist() + [kc[0, g * 3:(g + 1) * 3].tolist()]
        vh = orc.ae[(0, 1)].decode(orc.Z[(0, 1)][0, :5])[:, g * 3:(g + 1) * 3].tolist() + [vc[0, g * 3:(g + 1) * 3].tolist()]
        want = scalar_attention(q[0, j].tolist(), kh, vh, 1.0 / math.sqrt(3.0))
        np.testing.assert_allclose(got[0, j], want, rtol=1e-12, atol=1e-14)


def test_exact_current_token_with_empty_cache_returns_the_value_row():
    orc = tiny_oracle(hq=2, hkv=2, dh=2, r=3, L=4)
    q, kc, vc = rand(1, 2, 2), rand(1, 4), rand(1, 4)
    got = orc.decode_attention(0, q, 0, k_cur=kc, v_cur=vc)
    np.testing.assert_allclose(got[0].reshape(-1), vc[0], rtol=0, atol=0)


def test_lossless_autoencoder_ties_the_two_forms_together():
    """With r = D and an orthogonal encoder / transposed decoder the cache reproduces every row, so
    attending over n cached rows plus the exact current row equals the cache-only form over n + 1
    cached rows (current token appended first)."""
    hq = hkv = 2
    dh, L = 4, 7
    D = hkv * dh
    orc = O.KVCAROracle(1, hq, hkv, dh, 1, L, "f32")
    for which in (0, 1):
        qmat, _ = np.linalg.qr(rand(D, D))
        orc.set_autoencoder(0, which, O.Autoencoder(range(hkv), [(qmat, None)], [(qmat.T, None)]))
    k, v = rand(1, L, D), rand(1, L, D)
    orc.encode_append(0, k, v, 0)
    q = rand(1, hq, dh)
    cache_only = orc.decode_attention(0, q, L)
    exact = orc.decode_attention(0, q, L - 1, k_cur=k[:, L - 1], v_cur=v[:, L - 1])
    np.testing.assert_allclose(exact, cache_only, rtol=0, atol=2e-6)      # the cache holds fp32-rounded rows


def test_current_token_dominates_when_its_score_is_far_larger():
    orc = tiny_oracle(hq=2, hkv=2, dh=2, r=3, L=5)
    orc.encode_append(0, rand(1, 4, 4), rand(1, 4, 4), 0)
    q = rand(1, 2, 2)
    kc = np.concatenate([q[0, 0], q[0, 1]])[None] * 400.0
    vc = rand(1, 4)
    got = orc.decode_attention(0, q, 4, k_cur=kc, v_cur=vc)
    np.testing.assert_allclose(got[0].reshape(-1), vc[0], rtol=1e-9, atol=1e-9)


def test_ragged_lengths_equal_one_call_per_sequence():
    orc = tiny_oracle(hq=2, hkv=2, dh=2, r=3, L=9, B=3)
    k, v = rand(3, 9, 4), rand(3, 9, 4)
    orc.encode_append(0, k, v, 0)
    q = rand(3, 2, 2)
    lens = [9, 1, 5]
    got, probs = orc.decode_attention(0, q, 9, seq_lens=lens, return_probs=True)
    for b, n in enumerate(lens):
        one = O.KVCAROracle(1, 2, 2, 2, 1, 9, "f32")
        for which in (0, 1):
            one.set_autoencoder(0, which, orc.ae[(0, which)])
        one.encode_append(0, k[b:b + 1, :n], v[b:b + 1, :n], 0)
        np.testing.assert_allclose(got[b], one.decode_attention(0, q[b:b + 1], n)[0], rtol=1e-13, atol=1e-15)
        assert probs[b, :, n:].max(initial=0.0) == 0.0                       # nothing attends past a sequence's length
        np.testing.assert_allclose(probs[b].sum(axis=-1), 1.0, rtol=1e-13)


def test_ragged_append_positions_write_the_rows_a_per_sequence_append_writes():
    a = tiny_oracle(hq=2, hkv=2, dh=2, r=3, L=8, B=3)
    b = O.KVCAROracle(1, 2, 2, 2, 3, 8, "f32")
    for which in (0, 1):
        b.set_autoencoder(0, which, a.ae[(0, which)])
    k, v = rand(3, 1, 4), rand(3, 1, 4)
    pos = [0, 7, 3]
    a.encode_append(0, k, v, pos)
    for i, p0 in enumerate(pos):
        one = O.KVCAROracle(1, 2, 2, 2, 1, 8, "f32")
        for which in (0, 1):
            one.set_autoencoder(0, which, a.ae[(0, which)])
        one.encode_append(0, k[i:i + 1], v[i:i + 1], p0)
        for which in (0, 1):
            np.testing.assert_array_equal(a.Z[(0, which)][i, p0], one.Z[(0, which)][0, p0])
            others = [t for t in range(8) if t != p0]
            assert np.isnan(a.Z[(0, which)][i, others]).all()
