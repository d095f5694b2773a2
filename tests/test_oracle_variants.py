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


def test_block_diagonal_autoencoders_decompose_by_head():
    """A model whose autoencoders are block-diagonal over the KV heads is H_kv independent single-head
    models: the full-model oracle with block-diagonal dense matrices equals per-head oracles side by side
    (the mapping the per-head variant of the library relies on), also under a reuse map."""
    hkv, gq, dh, rh, L, n_layers = 3, 2, 4, 2, 6, 3
    reuse = np.zeros((n_layers, 2, hkv), dtype=bool)
    reuse[1, :, 1] = True
    reuse[2, 0, 1] = True          # chain for K, own V again in layer 2
    reuse[2, :, 2] = True
    full = O.KVCAROracle(n_layers, hkv * gq, hkv, dh, 1, L, "f32")
    heads = [O.KVCAROracle(n_layers, gq, 1, dh, 1, L, "f32") for _ in range(hkv)]
    for n in range(n_layers):
        full.set_reuse_map(n, reuse[n, 0], reuse[n, 1])
        for g in range(hkv):
            heads[g].set_reuse_map(n, reuse[n, 0, g:g + 1], reuse[n, 1, g:g + 1])
    for n in range(n_layers):
        for which in (0, 1):
            stored = [g for g in range(hkv) if not reuse[n, which, g]]
            enc = {g: (rand(dh, rh), rand(rh)) for g in range(hkv)}
            dec = {g: (rand(rh, dh), rand(dh)) for g in range(hkv)}
            for g in range(hkv):
                if g in stored:
                    heads[g].set_autoencoder(n, which, O.Autoencoder([0], [enc[g]], [dec[g]]))
                else:
                    heads[g].set_autoencoder(n, which, O.Autoencoder([], [(np.zeros((0, 0)), None)], [(np.zeros((0, 0)), None)]))
            we = np.zeros((len(stored) * dh, len(stored) * rh))
            wd = np.zeros((len(stored) * rh, len(stored) * dh))
            for i, g in enumerate(stored):
                we[i * dh:(i + 1) * dh, i * rh:(i + 1) * rh] = enc[g][0]
                wd[i * rh:(i + 1) * rh, i * dh:(i + 1) * dh] = dec[g][0]
            be = np.concatenate([enc[g][1] for g in stored]) if stored else None
            bd = np.concatenate([dec[g][1] for g in stored]) if stored else None
            full.set_autoencoder(n, which, O.Autoencoder(stored, [(we, be)], [(wd, bd)]))
    for n in range(n_layers):
        k, v = rand(1, L, hkv * dh), rand(1, L, hkv * dh)
        full.encode_append(n, k, v, 0)
        for g in range(hkv):
            heads[g].encode_append(n, k[:, :, g * dh:(g + 1) * dh], v[:, :, g * dh:(g + 1) * dh], 0)
    for n in range(n_layers):
        q = rand(1, hkv * gq, dh)
        want = full.decode_attention(n, q, L)
        got = np.concatenate([heads[g].decode_attention(n, q[:, g * gq:(g + 1) * gq], L) for g in range(hkv)], axis=1)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
