"""Pins of the oracle's prefill form: causal attention of a prompt chunk over the latent cache
(Introduction, the prefill phase; "Network Architecture", decoder at retrieval; Eq. 1 per token)."""
import math

import numpy as np
import torch

from oracle import kvcar_oracle as O
from tests.test_oracle_pins import rand, tiny_oracle


def scalar_prefill(orc, layer, q, pos0):
    """Every output element from Python scalars: decoded rows by explicit sums (linear decoder),
    scores, the causal limit, softmax and the weighted sum."""
    B, T, HQ, DH = q.shape
    group = orc.hq // orc.hkv
    out = np.zeros((B, T, HQ, DH))
    for b in range(B):
        for j in range(HQ):
            g = j // group
            rows = {}
            for which in (0, 1):
                src = O.resolve_source(orc.reuse, layer, which, g)
                ae = orc.ae[(src, which)]
                w, bias = ae.dec[0]
                col0 = ae.heads.index(g) * DH
                rows[which] = [[sum(float(orc.Z[(src, which)][b, t, c]) * float(w[c, col0 + k]) for c in range(w.shape[0])) +
                                (0.0 if bias is None else float(bias[col0 + k])) for k in range(DH)] for t in range(pos0 + T)]
            for i in range(T):
                last = pos0 + i
                s = [orc.scale * sum(float(q[b, i, j, k]) * rows[0][t][k] for k in range(DH)) for t in range(last + 1)]
                m = max(s)
                e = [math.exp(x - m) for x in s]
                tot = sum(e)
                for k in range(DH):
                    out[b, i, j, k] = sum(e[t] / tot * rows[1][t][k] for t in range(last + 1))
    return out


def test_prefill_brute_force_with_reuse_and_offset():
    reuse = [[[0, 0], [0, 0]], [[1, 0], [0, 1]]]
    orc = tiny_oracle(n_layers=2, hq=4, hkv=2, dh=3, r=4, L=9, B=2, reuse=reuse)
    D = 6
    for n in range(2):
        orc.encode_append(n, rand(2, 9, D), rand(2, 9, D), 0)
    q = rand(2, 4, 4, 3)
    for layer, pos0 in ((0, 0), (1, 5), (1, 0)):
        got = orc.prefill_attention(layer, q, pos0)
        np.testing.assert_allclose(got, scalar_prefill(orc, layer, q, pos0), rtol=1e-11, atol=1e-13)


def test_prefill_equals_library_causal_attention_on_the_decoded_rows():
    """pos0 = 0: a library scaled-dot-product attention with its causal flag on the decoded K^ / V^
    (grouped heads expanded) is the same function."""
    orc = tiny_oracle(hq=4, hkv=2, dh=8, r=5, L=12, B=2, hidden=7, act=O.ACT_GELU)
    D = 16
    orc.encode_append(0, rand(2, 12, D), rand(2, 12, D), 0)
    q = rand(2, 12, 4, 8)
    got = orc.prefill_attention(0, q, 0)
    k_hat = np.stack([orc.ae[(0, 0)].decode(orc.Z[(0, 0)][b, :12]) for b in range(2)]).reshape(2, 12, 2, 8)
    v_hat = np.stack([orc.ae[(0, 1)].decode(orc.Z[(0, 1)][b, :12]) for b in range(2)]).reshape(2, 12, 2, 8)
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)                                # [B, H_q, T, d]
    tk = torch.from_numpy(k_hat).permute(0, 2, 1, 3).repeat_interleave(2, dim=1)
    tv = torch.from_numpy(v_hat).permute(0, 2, 1, 3).repeat_interleave(2, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_prefill_is_one_decode_step_per_token():
    """Token i of the chunk is a decode step over pos0 + i + 1 cached rows."""
    orc = tiny_oracle(hq=2, hkv=1, dh=4, r=3, L=10, B=2)
    orc.encode_append(0, rand(2, 10, 4), rand(2, 10, 4), 0)
    q = rand(2, 6, 2, 4)
    got = orc.prefill_attention(0, q, 4)
    for i in range(6):
        np.testing.assert_allclose(got[:, i], orc.decode_attention(0, q[:, i], 4 + i + 1), rtol=1e-12, atol=1e-14)


def test_prefill_first_token_returns_its_own_value_row_and_later_rows_do_not_matter():
    orc = tiny_oracle(hq=2, hkv=2, dh=2, r=3, L=8)
    orc.encode_append(0, rand(1, 8, 4), rand(1, 8, 4), 0)
    q = rand(1, 5, 2, 2)
    got = orc.prefill_attention(0, q, 0)
    v0 = orc.ae[(0, 1)].decode(orc.Z[(0, 1)][0, :1])[0]
    np.testing.assert_allclose(got[0, 0].reshape(-1), v0, rtol=1e-13, atol=0)
    # causality: rows after a token's position cannot change its output
    orc.Z[(0, 0)][0, 3:] += 5.0
    orc.Z[(0, 1)][0, 3:] -= 7.0
    again = orc.prefill_attention(0, q, 0)
    np.testing.assert_array_equal(again[0, :3], got[0, :3])
    assert np.abs(again[0, 3:] - got[0, 3:]).max() > 1e-3


def test_prefill_zero_queries_give_running_means_of_the_value_rows():
    """q = 0: uniform weights over the visible rows, so output i is the mean of V^ rows 0..pos0+i."""
    orc = tiny_oracle(hq=2, hkv=1, dh=3, r=2, L=7)
    orc.encode_append(0, rand(1, 7, 3), rand(1, 7, 3), 0)
    got = orc.prefill_attention(0, np.zeros((1, 4, 2, 3)), 3)
    v_hat = orc.ae[(0, 1)].decode(orc.Z[(0, 1)][0, :7])
    for i in range(4):
        want = v_hat[:3 + i + 1].mean(axis=0)
        np.testing.assert_allclose(got[0, i, 0], want, rtol=1e-12)
        np.testing.assert_allclose(got[0, i, 1], want, rtol=1e-12)
