"""Per-head (block-diagonal) autoencoders: every KV head has an encoder d_head -> r_h and a decoder r_h -> d_head of
its own, so a head that reuses an earlier layer's keys or values reads only its own rows of that layer.  The ORACLE
knows nothing of this: it runs the full model with dense block-diagonal matrices.  The library runs it through the
descriptor's per_head flag (one context, head-major caches, one attention launch per layer with a group per KV head),
and - the composition that existed before the flag - as one single-head context per KV head.  Both must agree with the
oracle element by element: decode steps, the in-kernel encoder of append-and-attend, prefill attention, the caches."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import PerHeadSessions, Session, per_head_workloads
from tests.helpers import ABS_TOL, REL_TOL, assert_cache_close, assert_outputs_close, elementwise_bound

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


def kv_full(parts, w, layer, which, t0, t1):
    """Head g's column block of the full-width vectors is head g's stream."""
    return np.concatenate([synth.kv_tokens(wg, layer, which, 0, w.batch, t0, t1).double().numpy() for wg, _ in parts], axis=2)


def queries_full(parts, layer, step, gain):
    return np.concatenate([synth.queries(wg, layer, step, gain=gain).double().numpy() for wg, _ in parts], axis=1)


def run_oracle_per_head(w, reuse, with_bias, gain):
    parts = per_head_workloads(w, reuse)
    orc = full_model_oracle(w, reuse, parts, with_bias)
    for n in range(w.n_layers):
        orc.encode_append(n, kv_full(parts, w, n, 0, 0, w.n_cached), kv_full(parts, w, n, 1, 0, w.n_cached), 0)
    outs = []
    for step in range(w.n_steps):
        pos = w.n_cached + step
        for n in range(w.n_layers):
            orc.encode_append(n, kv_full(parts, w, n, 0, pos, pos + 1), kv_full(parts, w, n, 1, pos, pos + 1), pos)
        outs.append({n: orc.decode_attention(n, queries_full(parts, n, step, gain), pos + 1) for n in range(w.n_layers)})
    return orc, outs


C = synth.CONFIGS
CASES = {
    # name: (workload, with_bias, session keywords, decode step in one kernel expected)
    # the long-context shape with its Bernoulli map: layers storing 0 .. 4 heads, chains of reuse
    "tinyllama-bernoulli": (C[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=2), False, {}, True),
    "tinyllama-bernoulli-bias": (C[4].scaled(n_layers=8, batch=3, n_cached=333, n_steps=2), True, {}, True),
    # keys and values reused independently of each other: a group whose keys are the layer's own and whose values are not
    "kv-independent": (C[4].scaled(n_layers=6, batch=2, n_cached=130, n_steps=2, reuse="kvbernoulli:0.4"), True, {}, True),
    # one split per sequence: the fused kernel (four and eight waves)
    "one-split-w4": (C[4].scaled(n_layers=5, batch=2, n_cached=200, n_steps=2), True, {"n_splits": 1, "wg_waves": 4}, True),
    "one-split-w8": (C[4].scaled(n_layers=5, batch=2, n_cached=200, n_steps=2), False, {"n_splits": 1, "wg_waves": 8}, True),
    # separate kernels; plain-ALU kernels; fp16 with twelve heads (two launches of groups); fp32
    "separate-kernels": (C[4].scaled(n_layers=5, batch=2, n_cached=150, n_steps=2), True, {"no_fuse": True}, False),
    "plain-alu": (C[4].scaled(n_layers=5, batch=2, n_cached=70, n_steps=2), True, {"force_generic": True}, False),
    "gpt2-f16": (C[1].scaled(n_layers=4, batch=2, n_cached=150, n_steps=2), True, {}, True),
    "f32": (C[0].scaled(n_layers=3, batch=2, n_cached=60, n_steps=2, reuse="odd:5"), True, {}, False),
}


@pytest.mark.parametrize("name", list(CASES))
def test_per_head_flag_against_the_block_diagonal_oracle(name):
    w, with_bias, skw, one_kernel = CASES[name]
    print(f"case {name}: {w} bias={with_bias} {skw}", flush=True)
    reuse = synth.reuse_map(w)
    assert reuse[1:].any()
    orc, want = run_oracle_per_head(w, reuse, with_bias, gain=20.0)
    ses = Session(w, reuse, with_bias=with_bias, poison=True, per_head=True, **skw)
    ses.prefill(0, w.n_cached, chunk=128)
    info = ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1)
    assert info.append_in_kernel == (1 if one_kernel else 0)
    assert info.n_groups == w.n_kv_heads                     # a group per KV head: each reads rows of its own
    # what a layer reads: for every head the rows of ONE head of the source layers, whatever the map
    r_h, es = w.latent // w.n_kv_heads, synth.DTYPE_BYTES[w.dtype]
    assert info.latent_bytes == 2 * r_h * es * w.n_kv_heads * w.batch * (w.n_cached + 1)
    got = []
    for step in range(w.n_steps):
        pos = w.n_cached + step
        got.append({n: ses.append_attend(n, ses.kv(n, 0, pos, pos + 1), ses.kv(n, 1, pos, pos + 1), ses.queries(n, step, gain=20.0), pos)
                    .float().cpu().double().numpy() for n in range(w.n_layers)})
    torch.cuda.synchronize()
    assert_outputs_close(w, got, want, name)
    assert_cache_close(w, ses, orc, w.n_cached + w.n_steps)
    # the two calls kvcar_append_attend stands for, on a second session: same outputs to the same tolerance
    ses2 = Session(w, reuse, with_bias=with_bias, poison=True, per_head=True, **skw)
    ses2.prefill(0, w.n_cached + w.n_steps, chunk=97)
    last = {n: ses2.decode_attention(n, ses2.queries(n, w.n_steps - 1, gain=20.0), w.n_cached + w.n_steps).float().cpu().double().numpy()
            for n in range(w.n_layers)}
    assert_outputs_close(w, [last], [want[-1]], name + " (separate calls)")
    assert_cache_close(w, ses2, orc, w.n_cached + w.n_steps)


@pytest.mark.parametrize("name", ["tinyllama-bernoulli-bias", "gpt2-f16", "f32"])
def test_per_head_prefill_attention(name):
    w, with_bias, skw, _ = CASES[name]
    reuse = synth.reuse_map(w)
    parts = per_head_workloads(w, reuse)
    orc = full_model_oracle(w, reuse, parts, with_bias)
    ses = Session(w, reuse, with_bias=with_bias, poison=True, per_head=True, **skw)
    t = min(90, w.n_cached)
    for n in range(w.n_layers):
        orc.encode_append(n, kv_full(parts, w, n, 0, 0, t), kv_full(parts, w, n, 1, 0, t), 0)
    ses.prefill(0, t, chunk=64)
    for n in range(w.n_layers):
        q = torch.cat([synth.prompt_queries(wg, n, 0, w.batch, 0, t, gain=8.0) for wg, _ in parts], dim=2)
        want = orc.prefill_attention(n, q.double().numpy(), 0)
        got = ses.prefill_attention(n, q.to(ses.dev, ses.tdt), 0).float().cpu().double().numpy()
        err = np.abs(got - want)
        assert (err <= elementwise_bound(want, w.dtype)).all() and err.max() <= REL_TOL[w.dtype] * np.abs(want).max(), (n, err.max())


@pytest.mark.parametrize("name", ["tinyllama-bernoulli-bias", "one-split-w4", "one-split-w8", "separate-kernels", "plain-alu", "gpt2-f16", "f32"])
def test_per_head_ragged_lengths_and_exact_current_row(name):
    """The extended step on per-head autoencoders: per-sequence context lengths (one sequence empty) together with the
    exact current-token row, and the same step through the entry point that uses the library's static scratch buffer."""
    w, with_bias, skw, _ = CASES[name]
    reuse = synth.reuse_map(w)
    parts = per_head_workloads(w, reuse)
    orc = full_model_oracle(w, reuse, parts, with_bias)
    ses = Session(w, reuse, with_bias=with_bias, poison=True, per_head=True, **skw)
    n = w.n_cached
    for layer in range(w.n_layers):
        orc.encode_append(layer, kv_full(parts, w, layer, 0, 0, n), kv_full(parts, w, layer, 1, 0, n), 0)
    ses.prefill(0, n, chunk=77)
    lens = np.array(([n, 0, max(1, n // 3)] * w.batch)[:w.batch])
    tl = torch.tensor(lens, dtype=torch.int32, device=ses.dev)
    ses.ensure_workspace(w.batch, n)
    for layer in range(w.n_layers):
        q = queries_full(parts, layer, 0, 20.0)
        kc, vc = kv_full(parts, w, layer, 0, n, n + 1)[:, 0], kv_full(parts, w, layer, 1, n, n + 1)[:, 0]
        want = orc.decode_attention(layer, q, n, seq_lens=lens, k_cur=kc, v_cur=vc)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(ses.dev, ses.tdt)
        out = torch.empty_like(dev(q))
        ses.ctx.decode_attention_ex(layer, dev(q), out, w.batch, n, ses.workspace, seq_lens=tl, k_cur=dev(kc), v_cur=dev(vc))
        got = out.float().cpu().double().numpy()
        err = np.abs(got - want)
        assert np.isfinite(got).all() and (err <= elementwise_bound(want, w.dtype)).all(), (layer, err.max())
        assert err.max() <= REL_TOL[w.dtype] * np.abs(want).max(), (layer, err.max())
        # the plain step on the library's static scratch buffer against the same step on the workspace: the same kernels
        a, b2 = torch.empty_like(out), torch.empty_like(out)
        ses.ctx.decode_attention(layer, dev(q), a, w.batch, n, ses.workspace)
        ses.ctx.decode_attention_static(layer, dev(q), b2, w.batch, n)
        assert torch.equal(a, b2), layer
    torch.cuda.synchronize()


@pytest.mark.parametrize("with_bias", [False, True])
def test_block_diagonal_model_equals_per_head_contexts(with_bias):
    """The composition: one single-head library context per KV head."""
    w = synth.CONFIGS[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=1)
    reuse = synth.reuse_map(w)
    assert reuse[1:].any()
    parts = per_head_workloads(w, reuse)
    orc = full_model_oracle(w, reuse, parts, with_bias)
    ses = PerHeadSessions(w, reuse, with_bias=with_bias)
    n = w.n_cached + 1
    for layer in range(w.n_layers):
        orc.encode_append(layer, kv_full(parts, w, layer, 0, 0, n), kv_full(parts, w, layer, 1, 0, n), 0)
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
