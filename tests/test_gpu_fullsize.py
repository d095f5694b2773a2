"""Parity at the full sizes of the configurations, in the launch configuration bench.py times:
the GPU runs the whole workload, the oracle recomputes sampled (layer, sequence) units one by one
from the same seeded inputs (any slice of the synthetic K/V can be regenerated on its own)."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import Session
from tests.helpers import ABS_TOL, REL_TOL, elementwise_bound, oracle_ae

pytestmark = pytest.mark.gpu


def sources(reuse, layer, which):
    return [O.resolve_source(reuse, layer, which, g) for g in range(reuse.shape[2])]


def oracle_unit(w, reuse, layer, b, n_cached, q_row, latent_format="dtype"):
    """Attention output of one (layer, sequence) at the first decode step, from scratch."""
    orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, 1, w.max_seq, w.dtype, latent_format=latent_format)
    for n in range(w.n_layers):
        orc.set_reuse_map(n, reuse[n, 0], reuse[n, 1])
    need = {layer} | set(sources(reuse, layer, 0)) | set(sources(reuse, layer, 1))
    for n in sorted(need):
        for which in (0, 1):
            orc.set_autoencoder(n, which, oracle_ae(synth.autoencoder(w, n, which, reuse)))
        k = synth.kv_tokens(w, n, 0, b, b + 1, 0, n_cached + 1).double().numpy()
        v = synth.kv_tokens(w, n, 1, b, b + 1, 0, n_cached + 1).double().numpy()
        orc.encode_append(n, k, v, 0)
    return orc.decode_attention(layer, q_row[None], n_cached + 1)[0], orc


def run_fullsize(w, layers, seqs, gain, check_cache=True, latent_format="dtype"):
    reuse = synth.reuse_map(w)
    ses = Session(w, reuse=reuse, latent_format=latent_format)
    need = set()
    for n in layers:
        need |= {n} | set(sources(reuse, n, 0)) | set(sources(reuse, n, 1))
    need = sorted(need)
    ses.prefill(0, w.n_cached, chunk=max(1, (1 << 24) // (w.batch * w.d_kv)), layers=need)
    # the decode step as bench.py runs it: kvcar_append_attend per layer (encode the step's token, append, attend); layers
    # that only supply rows to a checked layer get their token through kvcar_encode_append; sources come before their users
    outs = {}
    pos = w.n_cached
    for n in need:
        if n not in layers:
            ses.prefill(pos, pos + 1, layers=[n])
            continue
        q = synth.queries(w, n, 0, gain=gain)
        outs[n] = (q, ses.append_attend(n, ses.kv(n, 0, pos, pos + 1), ses.kv(n, 1, pos, pos + 1), q.to(ses.dev, ses.tdt), pos).float().cpu().double().numpy())
    for n in layers:
        q, out = outs[n]
        plan = ses.ctx.describe_plan(n, w.batch, w.n_cached + 1)
        print(f"layer {n}: mfma={plan.uses_mfma} groups={plan.n_groups} splits={plan.n_splits} fused={plan.fused} append_in_kernel={plan.append_in_kernel}", flush=True)
        for b in seqs:
            want, orc = oracle_unit(w, reuse, n, b, w.n_cached, q[b].double().numpy(), latent_format)
            err = np.abs(out[b] - want).max()
            ref = np.abs(want).max()
            assert err <= ABS_TOL[w.dtype], (n, b, err)
            assert err <= REL_TOL[w.dtype] * ref, (n, b, err, ref)
            if check_cache and latent_format == "int8":
                for which in (0, 1):
                    view = ses.quantized_view(n, which)
                    if view is None:
                        continue
                    codes, scale, zp = (x[b, : w.n_cached + 1].cpu().numpy() for x in view)
                    np.testing.assert_allclose(scale, orc.Qscale[(n, which)][0, : w.n_cached + 1], rtol=2e-5)
                    dz = np.abs(zp.astype(np.int64) - orc.Qzero[(n, which)][0, : w.n_cached + 1])
                    dc = np.abs(codes.astype(np.int32) - orc.Q[(n, which)][0, : w.n_cached + 1])
                    assert dz.max() <= 1 and dc.max() <= 1 and (dc > 0).mean() < 0.01
            elif check_cache:
                for which in (0, 1):
                    view = ses.cache_view(n, which)
                    if view is None:
                        continue
                    zg = view[b, : w.n_cached + 1].float().cpu().double().numpy()
                    zo = orc.Z[(n, which)][0, : w.n_cached + 1]
                    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(zo), 1e-30))) - (7 if w.dtype == "bf16" else 10))
                    assert (np.abs(zg - zo) <= 1.0001 * ulp + 2e-6 * np.abs(zo).max()).all()
    return ses


def test_long_context_tinyllama_full_size():
    """batch 256 x 8192 cached tokens, 22 layers, Bernoulli(0.3) reuse: the benchmark's workload."""
    w = synth.CONFIGS[4].scaled(n_steps=1)
    reuse = synth.reuse_map(w)
    n_src = [len(set(sources(reuse, n, 0))) for n in range(w.n_layers)]
    deepest = int(np.argmax([n - min(sources(reuse, n, 0)) for n in range(w.n_layers)]))
    layers = sorted({0, w.n_layers - 1, int(np.argmax(n_src)), deepest})
    ses = run_fullsize(w, layers, seqs=[0, 101, 255], gain=30.0)
    assert ses.ctx.describe_plan(0, w.batch, w.n_cached + 1).uses_mfma == 1


def test_long_context_tinyllama_full_size_int8():
    """The same workload with int8 latents ("Quantization"): the MFMA kernel over code bytes."""
    w = synth.CONFIGS[4].scaled(n_steps=1)
    ses = run_fullsize(w, [0, 9, w.n_layers - 1], seqs=[0, 200], gain=30.0, latent_format="int8")
    plan = ses.ctx.describe_plan(0, w.batch, w.n_cached + 1)
    assert plan.uses_mfma == 1 and plan.fused == 1


def test_tinyllama_full_size():
    w = synth.CONFIGS[2].scaled(n_steps=1)
    run_fullsize(w, layers=[0, 2, 11, 21], seqs=[0, 17, 31], gain=30.0)


def test_gpt2_fp16_full_size():
    w = synth.CONFIGS[1].scaled(n_steps=1)
    run_fullsize(w, layers=[0, 1, 6, 11], seqs=[0, 7], gain=10.0)


def test_mlp_prefill_full_size():
    """batch 16 x 4096-token prefill through the two-layer GELU encoder, then attention with the
    two-layer decoder."""
    w = synth.CONFIGS[3].scaled(n_steps=1)
    run_fullsize(w, layers=[0, 21], seqs=[0, 15], gain=8.0)


def run_prefill_fullsize(w, layers, seqs, tokens, gain):
    """kvcar_prefill_attention on the whole prompt (the shape bench.py --op prefill times); the oracle
    recomputes sampled (sequence, token) rows one by one: token i is a decode step over i + 1 rows."""
    reuse = synth.reuse_map(w)
    ses = Session(w, reuse=reuse)
    T = w.n_cached
    need = set()
    for n in layers:
        need |= {n} | set(sources(reuse, n, 0)) | set(sources(reuse, n, 1))
    need = sorted(need)
    ses.prefill(0, T, chunk=max(1, (1 << 24) // (w.batch * w.d_kv)), layers=need)
    for n in layers:
        q = synth.prompt_queries(w, n, 0, w.batch, 0, T, gain=gain)
        out = ses.prefill_attention(n, q.to(ses.dev, ses.tdt), 0).float().cpu().double().numpy()
        assert np.isfinite(out).all()
        for b in seqs:
            orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, 1, w.max_seq, w.dtype)
            for m in range(w.n_layers):
                orc.set_reuse_map(m, reuse[m, 0], reuse[m, 1])
            for m in sorted({n} | set(sources(reuse, n, 0)) | set(sources(reuse, n, 1))):
                for which in (0, 1):
                    orc.set_autoencoder(m, which, oracle_ae(synth.autoencoder(w, m, which, reuse)))
                orc.encode_append(m, synth.kv_tokens(w, m, 0, b, b + 1, 0, T).double().numpy(),
                                  synth.kv_tokens(w, m, 1, b, b + 1, 0, T).double().numpy(), 0)
            for i in tokens:
                want = orc.decode_attention(n, q[b, i].double().numpy()[None], i + 1)[0]
                err = np.abs(out[b, i] - want)
                assert (err <= elementwise_bound(want, w.dtype)).all(), (n, b, i, err.max())
                assert err.max() <= REL_TOL[w.dtype] * np.abs(want).max(), (n, b, i, err.max(), np.abs(want).max())


def test_prefill_tinyllama_full_size():
    """16 x 4096-token prompts, TinyLlama shape with a reused head per layer: first and last tokens, both sides of
    tile (64), query-block (32) and workgroup (256) boundaries."""
    w = synth.CONFIGS[2].scaled(batch=16, n_cached=4096, n_steps=0)
    run_prefill_fullsize(w, layers=[0, 11, 21], seqs=[0, 15], tokens=[0, 1, 31, 32, 63, 64, 255, 256, 2047, 2048, 4095], gain=30.0)


def test_prefill_mlp_full_size():
    """The same prompt shape through two-layer GELU decoders (the configuration named for prefill)."""
    w = synth.CONFIGS[3].scaled(n_steps=0)
    run_prefill_fullsize(w, layers=[0, 21], seqs=[3], tokens=[0, 63, 64, 1000, 4095], gain=8.0)


def test_long_context_full_size_exact_row_and_ragged_lengths():
    """The benchmark's workload through kvcar_decode_attention_ex, as `bench.py --variant exact | ragged` launches it:
    the exact current-token row merged in the fused kernel, and per-sequence context lengths in [n/2, n]; the oracle
    recomputes sampled (layer, sequence) units."""
    w = synth.CONFIGS[4].scaled(n_steps=1)
    reuse = synth.reuse_map(w)
    layers, seqs = [0, 13, w.n_layers - 1], [0, 77, 255]
    ses = Session(w, reuse=reuse)
    need = set()
    for n in layers:
        need |= {n} | set(sources(reuse, n, 0)) | set(sources(reuse, n, 1))
    ses.prefill(0, w.n_cached, chunk=max(1, (1 << 24) // (w.batch * w.d_kv)), layers=sorted(need))
    gen = torch.Generator().manual_seed(5)
    lens = torch.randint(w.n_cached // 2, w.n_cached + 1, (w.batch,), generator=gen, dtype=torch.int32)
    for n in layers:
        q = synth.queries(w, n, 0, gain=30.0)
        kc = synth.kv_tokens(w, n, 0, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
        vc = synth.kv_tokens(w, n, 1, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
        dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
        ses.ensure_workspace(w.batch, w.n_cached)
        out_exact, out_ragged = torch.empty_like(dev(q)), torch.empty_like(dev(q))
        ses.ctx.decode_attention_ex(n, dev(q), out_exact, w.batch, w.n_cached, ses.workspace, k_cur=dev(kc), v_cur=dev(vc))
        ses.ctx.decode_attention_ex(n, dev(q), out_ragged, w.batch, w.n_cached, ses.workspace, seq_lens=lens.to(ses.dev))
        assert ses.ctx.describe_plan(n, w.batch, w.n_cached).fused == 1
        out_exact, out_ragged = (o.float().cpu().double().numpy() for o in (out_exact, out_ragged))
        for b in seqs:
            _, orc = oracle_unit(w, reuse, n, b, w.n_cached - 1, q[b].double().numpy())       # caches of rows 0 .. n_cached - 1
            qb = q[b:b + 1].double().numpy()
            want = orc.decode_attention(n, qb, w.n_cached, k_cur=kc[b:b + 1].double().numpy(), v_cur=vc[b:b + 1].double().numpy())[0]
            err = np.abs(out_exact[b] - want)
            assert (err <= elementwise_bound(want, w.dtype)).all(), ("exact", n, b, err.max())
            want = orc.decode_attention(n, qb, w.n_cached, seq_lens=np.array([int(lens[b])]))[0]
            err = np.abs(out_ragged[b] - want).max()
            assert err <= ABS_TOL[w.dtype] and err <= REL_TOL[w.dtype] * np.abs(want).max(), ("ragged", n, b, err)


@pytest.mark.parametrize("fmt", ["dtype", "int8"])
def test_caches_larger_than_4_gib(fmt):
    """36 sequences with room for 2^20 tokens each: a latent cache of 9.7 GB (int8 rows: 4.8 GB of codes), so the
    rows of the later sequences lie beyond 32-bit byte and element offsets.  600 prompt tokens through the
    prompt-sized encoder, one decode-step append, then decode and prefill attention over all 36 sequences against
    the oracle (which holds the same 601 rows in arrays of their own size).  Layer 1 reads one key head and one
    value head from layer 0's caches."""
    from tests.helpers import build_oracle
    big = synth.CONFIGS[2].scaled(n_layers=2, batch=36, n_cached=600, n_steps=2 ** 20 - 600)
    small = synth.CONFIGS[2].scaled(n_layers=2, batch=36, n_cached=600, n_steps=2)
    assert big.max_seq == 2 ** 20
    reuse = np.zeros((2, 2, big.n_kv_heads), dtype=bool)
    reuse[1, 0, 0] = reuse[1, 1, 1] = True
    orc = build_oracle(small, reuse=reuse, with_bias=True, latent_format=fmt)
    ses = Session(big, reuse=reuse, with_bias=True, latent_format=fmt)
    assert ses.ctx.cache_bytes(0, 0) > 2 ** 32
    for t0, t1 in ((0, 600), (600, 601)):
        for n in range(2):
            k = synth.kv_tokens(small, n, 0, 0, 36, t0, t1)
            v = synth.kv_tokens(small, n, 1, 0, 36, t0, t1)
            orc.encode_append(n, k.double().numpy(), v.double().numpy(), t0)
            ses.encode_append(n, k.to(ses.dev, ses.tdt), v.to(ses.dev, ses.tdt), t0)
    for n in range(2):
        q = synth.queries(small, n, 0, gain=6.0)
        got = ses.decode_attention(n, q.to(ses.dev, ses.tdt), 601).float().cpu().double().numpy()
        want = orc.decode_attention(n, q.double().numpy(), 601)
        err = np.abs(got - want).max(axis=(1, 2))
        print(f"layer {n} decode: max abs err per sequence {err.max():.3e} (last sequence {err[-1]:.3e})", flush=True)
        assert np.isfinite(got).all() and err.max() <= ABS_TOL[big.dtype] and err.max() <= REL_TOL[big.dtype] * np.abs(want).max()
        qp = synth.prompt_queries(small, n, 0, 36, 0, 601, gain=6.0)
        got = ses.prefill_attention(n, qp.to(ses.dev, ses.tdt), 0).float().cpu().double().numpy()
        want = orc.prefill_attention(n, qp.double().numpy(), 0)
        err = np.abs(got - want)
        print(f"layer {n} prefill: max abs err {err.max():.3e}", flush=True)
        assert np.isfinite(got).all() and (err <= elementwise_bound(want, big.dtype)).all()


@pytest.mark.parametrize("fmt", ["dtype", "int8"])
def test_one_sequence_of_300001_tokens(fmt):
    """A single sequence far longer than the benchmark's: its token range goes to 64 splits of about 4700 tokens
    (37 wave tiles each, the last one ragged); every cached row and the attention output against the oracle."""
    from tests.helpers import assert_cache_close, assert_outputs_close, assert_quantized_cache_close, run_gpu, run_oracle
    w = synth.CONFIGS[2].scaled(n_layers=2, batch=1, n_cached=300000, n_steps=1, reuse="odd:1")
    orc, want = run_oracle(w, gain=30.0, latent_format=fmt)
    ses, got = run_gpu(w, gain=30.0, latent_format=fmt)
    if fmt == "int8":
        assert_quantized_cache_close(w, ses, orc, w.n_cached + 1)
    else:
        assert_cache_close(w, ses, orc, w.n_cached + 1)
    assert_outputs_close(w, got, want, "300001 tokens")


def test_long_context_per_head_full_size():
    """`bench.py --per-head` at full size: per-head (block-diagonal) autoencoders through the descriptor flag, one
    kvcar_append_attend per layer; the oracle recomputes sampled (layer, sequence) units with dense block-diagonal
    matrices."""
    from paper_2512_06727_amd.harness import per_head_workloads
    from tests.test_gpu_per_head import block_diag
    w = synth.CONFIGS[4].scaled(n_steps=1)
    reuse = synth.reuse_map(w)
    parts = per_head_workloads(w, reuse)
    deepest = int(np.argmax([n - min(sources(reuse, n, 0)) for n in range(w.n_layers)]))
    layers = sorted({0, w.n_layers - 1, deepest})
    need = set()
    for n in layers:
        need |= {n} | set(sources(reuse, n, 0)) | set(sources(reuse, n, 1))
    need = sorted(need)
    ses = Session(w, reuse=reuse, per_head=True)
    ses.prefill(0, w.n_cached, chunk=max(1, (1 << 24) // (w.batch * w.d_kv)), layers=need)
    pos, outs = w.n_cached, {}
    for n in need:
        if n not in layers:
            ses.prefill(pos, pos + 1, layers=[n])
            continue
        q = ses.queries(n, 0, gain=30.0)
        outs[n] = (q.float().cpu().double().numpy(), ses.append_attend(n, ses.kv(n, 0, pos, pos + 1), ses.kv(n, 1, pos, pos + 1), q, pos).float().cpu().double().numpy())
    plan = ses.ctx.describe_plan(w.n_layers - 1, w.batch, pos + 1)
    assert plan.n_groups == w.n_kv_heads and plan.fused == 1 and plan.append_in_kernel == 1 and plan.n_launches == 1

    def oracle_unit_per_head(layer, b):
        orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, 1, w.max_seq, w.dtype)
        for n in range(w.n_layers):
            orc.set_reuse_map(n, reuse[n, 0], reuse[n, 1])
        mine = {layer} | set(sources(reuse, layer, 0)) | set(sources(reuse, layer, 1))
        for n in sorted(mine):
            for which in (0, 1):
                stored = [g for g in range(w.n_kv_heads) if not reuse[n, which, g]]
                aes = [synth.autoencoder(parts[g][0], n, which, parts[g][1]) for g in stored]
                if stored:
                    enc = [(block_diag([a.enc[0][0].double().numpy() for a in aes]), None)]
                    dec = [(block_diag([a.dec[0][0].double().numpy() for a in aes]), None)]
                else:
                    enc, dec = [(np.zeros((0, 0)), None)], [(np.zeros((0, 0)), None)]
                orc.set_autoencoder(n, which, O.Autoencoder(stored, enc, dec))
            kv = lambda which: np.concatenate([synth.kv_tokens(wg, n, which, b, b + 1, 0, pos + 1).double().numpy() for wg, _ in parts], axis=2)
            orc.encode_append(n, kv(0), kv(1), 0)
        return orc

    for n in layers:
        q, out = outs[n]
        for b in (0, 131, 255):
            orc = oracle_unit_per_head(n, b)
            want = orc.decode_attention(n, q[b][None], pos + 1)[0]
            err, ref = np.abs(out[b] - want).max(), np.abs(want).max()
            assert err <= ABS_TOL[w.dtype] and err <= REL_TOL[w.dtype] * ref, (n, b, err, ref)
            for which in (0, 1):
                view = ses.cache_view(n, which)
                if view is None:
                    continue
                zg = view[b, : pos + 1].float().cpu().double().numpy()
                zo = orc.Z[(n, which)][0, : pos + 1]
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(zo), 1e-30))) - 7)
                assert (np.abs(zg - zo) <= 1.0001 * ulp + 2e-6 * np.abs(zo).max()).all(), (n, b, which)
