"""The two variants of the decode step on the GPU against the oracle: the paper's form with the
current token's exact key / value row ("Network Architecture", 2nd paragraph) and ragged batches
(per-sequence context lengths, per-sequence append positions)."""
import numpy as np
import pytest
import torch

from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import Session
from tests.helpers import ABS_TOL, REL_TOL, build_oracle, elementwise_bound, oracle_prefill

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]

C = synth.CONFIGS
CASES = {
    "c0-f32": (C[0], {}, {}),
    "c1-small-f16": (C[1].scaled(n_layers=3, batch=2, n_cached=150, n_steps=1), {}, {}),
    "c2-small-bf16": (C[2].scaled(n_layers=4, batch=5, n_cached=300, n_steps=1), {}, {}),
    "c2-small-bf16-1split": (C[2].scaled(n_layers=4, batch=5, n_cached=300, n_steps=1), {}, {"n_splits": 1}),
    "c4-small-bf16": (C[4].scaled(n_layers=5, batch=3, n_cached=260, n_steps=1), {}, {}),
    # one split: prologue, attention and epilogue in one kernel, which then also takes the exact row
    "c4-small-bf16-1split": (C[4].scaled(n_layers=8, batch=3, n_cached=260, n_steps=1), {"with_bias": True}, {"n_splits": 1}),
    "c4-small-bf16-1split-w8": (C[4].scaled(n_layers=5, batch=2, n_cached=300, n_steps=1), {}, {"n_splits": 1, "wg_waves": 8}),
    # several splits in one launch (the last workgroup merges) with eight waves per workgroup; five splits of 600 tokens
    # leave two of them without a tile
    "c4-small-bf16-3splits-w8": (C[4].scaled(n_layers=5, batch=2, n_cached=700, n_steps=1), {"with_bias": True}, {"n_splits": 3, "wg_waves": 8}),
    "c2-small-bf16-5splits-w8": (C[2].scaled(n_layers=4, batch=3, n_cached=600, n_steps=1), {}, {"n_splits": 5, "wg_waves": 8}),
    "c2-small-int8-3splits-w8": (C[2].scaled(n_layers=4, batch=3, n_cached=600, n_steps=1), {"latent_format": "int8"}, {"n_splits": 3, "wg_waves": 8}),
    "c2-small-int8-1split": (C[2].scaled(n_layers=4, batch=3, n_cached=200, n_steps=1), {"latent_format": "int8"}, {"n_splits": 1}),
    "c3-small-mlp": (C[3].scaled(n_layers=2, batch=3, n_cached=90, n_steps=1), {}, {}),
    "c2-small-int8": (C[2].scaled(n_layers=4, batch=5, n_cached=300, n_steps=1), {"latent_format": "int8"}, {}),
    "bias-f16-generic": (C[3].scaled(n_layers=2, batch=2, n_cached=40, n_steps=1, dtype="f16", act="leaky_relu", hidden=160),
                         {"with_bias": True}, {}),
}


def setup(name):
    w, okw, skw = CASES[name]
    orc = build_oracle(w, **okw)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, w.n_cached)
    ses = Session(w, poison=True, **okw, **skw)
    ses.prefill(0, w.n_cached, chunk=256)
    return w, orc, ses


# The exact current value row is N(0, 1): where it dominates, outputs are O(1) and the single rounding of
# the output to the dtype (half a unit in the last place: 2^-9 relative for bf16, 2^-12 for fp16) exceeds
# the absolute tolerance meant for the O(1e-2) outputs of the cache-only path.  Elementwise bound:
# absolute tolerance + half a unit in the last place of the reference value.


def check(w, got, want, label):
    assert np.isfinite(got).all(), label
    err = np.abs(got - want)
    bound = elementwise_bound(want, w.dtype)
    worst = (err - bound).max()
    assert worst <= 0, f"{label}: error exceeds abs tol + half an ulp by {worst:.3e}"
    assert err.max() <= REL_TOL[w.dtype] * np.abs(want).max(), f"{label}: err {err.max():.3e} vs max |ref| {np.abs(want).max():.3e}"


def test_ragged_and_exact_row_in_the_one_launch_split_kernel():
    """Several splits in one launch (the last workgroup merges): ragged context lengths - one sequence empty, one shorter
    than a split's share, so that some splits see no token at all - together with the exact current-token row."""
    w = synth.CONFIGS[2].scaled(n_layers=3, batch=4, n_cached=1500, n_steps=1)
    for fmt in ("dtype", "int8"):
        orc = build_oracle(w, latent_format=fmt)
        for n in range(w.n_layers):
            oracle_prefill(orc, w, n, 0, w.n_cached)
        ses = Session(w, poison=True, latent_format=fmt, n_splits=6)
        ses.prefill(0, w.n_cached, chunk=256)
        assert ses.ctx.describe_plan(2, w.batch, w.n_cached).fused == 2
        lens = np.array([w.n_cached, 0, 100, 777])
        tl = torch.tensor(lens, dtype=torch.int32, device=ses.dev)
        for layer in range(w.n_layers):
            q = synth.queries(w, layer, 0, gain=20.0)
            kc = synth.kv_tokens(w, layer, 0, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
            vc = synth.kv_tokens(w, layer, 1, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
            want = orc.decode_attention(layer, q.double().numpy(), w.n_cached, seq_lens=lens, k_cur=kc.double().numpy(), v_cur=vc.double().numpy())
            dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
            got = run_ex(ses, w, layer, dev(q), w.n_cached, seq_lens=tl, k_cur=dev(kc), v_cur=dev(vc))
            check(w, got, want, f"{fmt} layer {layer}")


def run_ex(ses, w, layer, q, n_ctx, **ext):
    out = torch.empty_like(q)
    ses.ensure_workspace(w.batch, max(1, n_ctx))
    ses.ctx.decode_attention_ex(layer, q, out, w.batch, n_ctx, ses.workspace, **ext)
    return out.float().cpu().double().numpy()


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("gain", [1.0, 30.0])
def test_exact_current_token(name, gain):
    w, orc, ses = setup(name)
    for layer in range(w.n_layers):
        q = synth.queries(w, layer, 0, gain=gain)
        kc = synth.kv_tokens(w, layer, 0, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
        vc = synth.kv_tokens(w, layer, 1, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
        want = orc.decode_attention(layer, q.double().numpy(), w.n_cached, k_cur=kc.double().numpy(), v_cur=vc.double().numpy())
        dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
        got = run_ex(ses, w, layer, dev(q), w.n_cached, k_cur=dev(kc), v_cur=dev(vc))
        check(w, got, want, f"{name} layer {layer}")


@pytest.mark.parametrize("name", ["c0-f32", "c2-small-bf16", "c2-small-bf16-1split", "c4-small-bf16-1split-w8", "c2-small-int8-1split", "c3-small-mlp", "c2-small-int8"])
def test_exact_current_token_with_nothing_cached(name):
    """n_ctx = 0: the output is the current value row of each head's KV head (rounded to the dtype)."""
    w, orc, ses = setup(name)
    q = synth.queries(w, 0, 0)
    kc = synth.kv_tokens(w, 0, 0, 0, w.batch, 0, 1)[:, 0]
    vc = synth.kv_tokens(w, 0, 1, 0, w.batch, 0, 1)[:, 0]
    dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
    got = run_ex(ses, w, 0, dev(q), 0, k_cur=dev(kc), v_cur=dev(vc))
    gq = w.n_q_heads // w.n_kv_heads
    want = dev(vc).float().cpu().double().numpy().reshape(w.batch, w.n_kv_heads, 1, w.d_head).repeat(gq, axis=2).reshape(w.batch, w.n_q_heads, w.d_head)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("name", list(CASES))
def test_ragged_context_lengths(name):
    w, orc, ses = setup(name)
    rng = np.random.default_rng(7)
    lens = rng.integers(1, w.n_cached + 1, size=w.batch)
    lens[0] = w.n_cached
    if w.batch > 1:
        lens[-1] = 1
    tl = torch.tensor(lens, dtype=torch.int32, device=ses.dev)
    for layer in range(w.n_layers):
        q = synth.queries(w, layer, 0, gain=20.0)
        want = orc.decode_attention(layer, q.double().numpy(), w.n_cached, seq_lens=lens)
        got = run_ex(ses, w, layer, q.to(ses.dev, ses.tdt), w.n_cached, seq_lens=tl)
        check(w, got, want, f"{name} layer {layer} lens {lens.tolist()}")


@pytest.mark.parametrize("name", ["c2-small-bf16", "c2-small-bf16-1split", "c4-small-bf16-1split", "c2-small-int8-1split", "c3-small-mlp", "c2-small-int8", "c0-f32"])
def test_ragged_lengths_with_exact_current_token_and_an_empty_sequence(name):
    w, orc, ses = setup(name)
    lens = np.array([(7 * b * b + 3) % (w.n_cached + 1) for b in range(w.batch)])
    lens[0] = 0
    tl = torch.tensor(lens, dtype=torch.int32, device=ses.dev)
    layer = w.n_layers - 1
    q = synth.queries(w, layer, 0, gain=20.0)
    kc = synth.kv_tokens(w, layer, 0, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
    vc = synth.kv_tokens(w, layer, 1, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
    want = orc.decode_attention(layer, q.double().numpy(), w.n_cached, seq_lens=lens, k_cur=kc.double().numpy(), v_cur=vc.double().numpy())
    dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
    got = run_ex(ses, w, layer, dev(q), w.n_cached, seq_lens=tl, k_cur=dev(kc), v_cur=dev(vc))
    check(w, got, want, f"{name} lens {lens.tolist()}")


@pytest.mark.parametrize("name", ["c0-f32", "c2-small-bf16", "c3-small-mlp", "c2-small-int8"])
def test_ragged_append_positions(name):
    """One new token per sequence, each at its own position: the rows written and their values
    equal the oracle's, every other row keeps what the prefill left."""
    w, okw, skw = CASES[name]
    w = w.scaled(n_cached=24, n_steps=40)
    orc = build_oracle(w, **okw)
    ses = Session(w, poison=True, **okw, **skw)
    pos = np.array([(11 * b + 5) % w.max_seq for b in range(w.batch)])
    tp = torch.tensor(pos, dtype=torch.int32, device=ses.dev)
    int8 = okw.get("latent_format") == "int8"
    for layer in range(w.n_layers):
        k = synth.kv_tokens(w, layer, 0, 0, w.batch, 100, 101)
        v = synth.kv_tokens(w, layer, 1, 0, w.batch, 100, 101)
        orc.encode_append(layer, k.double().numpy(), v.double().numpy(), pos.tolist())
        ses.ctx.encode_append_at(layer, k.to(ses.dev, ses.tdt), v.to(ses.dev, ses.tdt), w.batch, tp, 1)
    torch.cuda.synchronize()
    for layer in range(w.n_layers):
        for which in (0, 1):
            zo = orc.Z[(layer, which)]
            if zo.shape[-1] == 0:
                continue
            written = ~np.isnan(zo[..., 0])
            assert written.sum() == w.batch
            if int8:
                codes, scale, zp = (x.cpu().numpy() for x in ses.quantized_view(layer, which))
                assert (codes.view(np.uint8)[~written] == 0x7F).all()
                dc = np.abs(codes[written].astype(np.int32) - orc.Q[(layer, which)][written])
                assert dc.max() <= 1 and (dc > 0).mean() < 0.02
                np.testing.assert_allclose(scale[written], orc.Qscale[(layer, which)][written], rtol=2e-5)
            else:
                zg = ses.cache_view(layer, which).float().cpu().double().numpy()
                assert np.isnan(zg[~written]).all()
                tol = 1e-6 if w.dtype == "f32" else 2.0 ** -7 if w.dtype == "bf16" else 2.0 ** -10
                np.testing.assert_allclose(zg[written], zo[written], rtol=tol, atol=2e-6 * np.abs(zo[written]).max())


def test_single_split_exact_row_runs_in_the_fused_kernel():
    w, _, skw = CASES["c4-small-bf16-1split"]
    ses = Session(w, with_bias=True, **skw)
    assert ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached).fused == 1
