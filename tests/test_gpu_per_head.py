"""The per-head (block-diagonal) autoencoder variant: a model whose autoencoders are block-diagonal over the KV
heads is H_kv independent single-head models.  The oracle runs the FULL model with block-diagonal dense
matrices; the library runs one context per KV head (harness.PerHeadSessions), where a reused head reads only
its own 1/H_kv of the source layer's rows.  Both must agree element by element."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import PerHeadSessions, per_head_workloads
from tests.helpers import ABS_TOL, REL_TOL

pytestmark = pytest.mark.gpu


def block_diag(mats):
    rows, cols = sum(m.shape[0] for m in mats), sum(m.shape[1] for m in mats)
    out = np.zeros((rows, cols))
    r = c = 0
    for m in mats:
        out[r:r + m.shape[0], c:c + m.shape[1]] = m
        r, c = r + m.shape[0], c + m.shape[1]
    return out


def full_model_oracle(w, reuse, parts, with_bias):
    orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, w.batch, w.max_seq, w.dtype)
    for layer in range(w.n_layers):
        orc.set_reuse_map(layer, reuse[layer, 0], reuse[layer, 1])
    for layer in range(w.n_layers):
        for which in (0, 1):
            stored = [g for g in range(w.n_kv_heads) if not reuse[layer, which, g]]
            aes = [synth.autoencoder(parts[g][0], layer, which, parts[g][1], with_bias) for g in stored]
            cat = lambda vs: None if not with_bias else np.concatenate([v.double().numpy() for v in vs])
            if stored:
                enc = [(block_diag([a.enc[0][0].double().numpy() for a in aes]), cat([a.enc[0][1] for a in aes]))]
                dec = [(block_diag([a.dec[0][0].double().numpy() for a in aes]), cat([a.dec[0][1] for a in aes]))]
            else:
                enc, dec = [(np.zeros((0, 0)), None)], [(np.zeros((0, 0)), None)]
            orc.set_autoencoder(layer, which, O.Autoencoder(stored, enc, dec))
    return orc


@pytest.mark.parametrize("with_bias", [False, True])
def test_block_diagonal_model_equals_per_head_contexts(with_bias):
    w = synth.CONFIGS[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=1)
    reuse = synth.reuse_map(w)
    assert reuse[1:].any()
    parts = per_head_workloads(w, reuse)
    orc = full_model_oracle(w, reuse, parts, with_bias)
    ses = PerHeadSessions(w, reuse, with_bias=with_bias)
    n = w.n_cached + 1
    # the same K/V through both: head g's column block of the full-width vectors is head g's stream
    for layer in range(w.n_layers):
        k = np.concatenate([synth.kv_tokens(wg, layer, 0, 0, w.batch, 0, n).double().numpy() for wg, _ in parts], axis=2)
        v = np.concatenate([synth.kv_tokens(wg, layer, 1, 0, w.batch, 0, n).double().numpy() for wg, _ in parts], axis=2)
        orc.encode_append(layer, k, v, 0)
    ses.prefill(0, n, chunk=128)
    for layer in range(w.n_layers):
        qs = [synth.queries(wg, layer, 0, gain=20.0) for wg, _ in parts]
        want = orc.decode_attention(layer, np.concatenate([q.double().numpy() for q in qs], axis=1), n)
        got = ses.decode_attention(layer, [q.to(s.dev, s.tdt) for q, s in zip(qs, ses.sessions)], n).float().cpu().double().numpy()
        err = np.abs(got - want).max()
        assert err <= ABS_TOL[w.dtype] and err <= REL_TOL[w.dtype] * np.abs(want).max(), (layer, err)
    # what a reused head reads: the rows of ONE head of the source layer
    for g, (wg, rg) in enumerate(parts):
        for layer in range(1, w.n_layers):
            info = ses.sessions[g].ctx.describe_plan(layer, w.batch, n)
            assert info.latent_bytes == 2 * (w.latent // w.n_kv_heads) * 2 * w.batch * n
    torch.cuda.synchronize()
