"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element.  Sizes span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from paper_2512_06727_amd import synth
from tests.helpers import (ABS_TOL, assert_cache_close, assert_outputs_close, assert_quantized_cache_close, build_oracle,
                           oracle_prefill, run_gpu, run_oracle)

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]

C = synth.CONFIGS

CASES = {
    # the small configuration exactly as specified (fp32, one layer, 128 cached tokens)
    "c0-exact": (C[0], {}),
    # GPT-2 shape, fp16, reuse in odd layers, fewer layers / sequences / tokens
    "c1-small": (C[1].scaled(n_layers=4, batch=2, n_cached=203, n_steps=2), {}),
    # TinyLlama shape, bf16, grouped-query heads, one reused KV head per layer >= 2 (chains appear)
    "c2-small": (C[2].scaled(n_layers=5, batch=3, n_cached=301, n_steps=2), {}),
    # two-layer GELU autoencoder
    "c3-small": (C[3].scaled(n_layers=2, batch=2, n_cached=77, n_steps=2), {}),
    # Bernoulli(0.3) map: layers storing 0..4 heads, mixed sources, chains
    "c4-small": (C[4].scaled(n_layers=8, batch=2, n_cached=333, n_steps=2), {}),
    # full-width latents in every layer (reuse saves no capacity; decoder columns of reused heads ignored)
    "c4-small-p2": (C[4].scaled(n_layers=6, batch=2, n_cached=150, n_steps=1, policy="P2"), {}),
    # biases everywhere and the paper's LeakyReLU between the two layers
    "leaky-bias": (C[2].scaled(n_layers=3, batch=2, n_cached=90, n_steps=1, hidden=160, act="leaky_relu", dtype="f16"),
                   {"with_bias": True}),
    # two-layer decoders on the MFMA path: LeakyReLU (the paper's activation) with biases and a reuse chain under
    # the full-width policy, and the narrower fp16 instance
    "mlp-leaky-p2": (C[3].scaled(n_layers=4, batch=2, n_cached=100, n_steps=2, act="leaky_relu", reuse="from2:1", policy="P2"),
                     {"with_bias": True}),
    "mlp-f16-narrow": (C[3].scaled(n_layers=2, batch=3, n_cached=70, n_steps=1, dtype="f16", latent=64, hidden=128), {}),
    "linear-bias-f32": (C[0].scaled(n_layers=2, batch=2, n_cached=50, n_steps=2, reuse="odd:5"), {"with_bias": True}),
    # one long sequence: the token range goes to 32 splits (more than the 16 the merge kernel requests in one go),
    # for linear and for two-layer decoders
    "c2-one-long": (C[2].scaled(n_layers=3, batch=1, n_cached=4000, n_steps=1), {}),
    "c3-one-long": (C[3].scaled(n_layers=2, batch=1, n_cached=1100, n_steps=1), {}),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("gain", [1.0, 50.0])
def test_parity(name, gain):
    w, kw = CASES[name]
    print(f"case {name} gain {gain} {w}", flush=True)
    orc, want = run_oracle(w, gain=gain, **kw)
    ses, got = run_gpu(w, gain=gain, **kw)
    assert_cache_close(w, ses, orc, w.n_cached + w.n_steps)
    assert_outputs_close(w, got, want, name)


@pytest.mark.parametrize("n_splits", [1, 2, 7])
def test_split_counts_agree_with_oracle(n_splits):
    w = C[2].scaled(n_layers=3, batch=2, n_cached=257, n_steps=1)
    _, want = run_oracle(w, gain=20.0)
    _, got = run_gpu(w, gain=20.0, n_splits=n_splits)
    assert_outputs_close(w, got, want, f"splits={n_splits}")


def test_single_token_context_and_partial_batch():
    """n_ctx = 1 (softmax over one token = that token's decoded value) and a batch
    smaller than max_batch."""
    w = C[2].scaled(n_layers=2, batch=2, n_cached=0, n_steps=2, reuse="none")
    _, want = run_oracle(w)
    _, got = run_gpu(w, max_batch=5)
    assert_outputs_close(w, got, want, "n_ctx=1")


@pytest.mark.parametrize("name", ["c1-small", "c2-small", "c4-small"])
def test_plain_alu_kernels_on_16bit_linear(name):
    """The same cases through the plain-ALU kernels (the MFMA kernels are the default)."""
    w, kw = CASES[name]
    _, want = run_oracle(w, gain=20.0, **kw)
    _, got = run_gpu(w, gain=20.0, force_generic=True, **kw)
    assert_outputs_close(w, got, want, name + "-generic")


def test_two_layer_decoder_uses_the_mfma_kernels():
    from paper_2512_06727_amd.harness import Session
    for name in ("c3-small", "mlp-leaky-p2", "mlp-f16-narrow"):
        w, kw = CASES[name]
        ses = Session(w, **{k: v for k, v in kw.items() if k == "with_bias"})
        assert ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1).uses_mfma == 1, name
    w, kw = CASES["leaky-bias"]            # hidden width 160: no resident-weight instance, plain-ALU kernels
    assert Session(w, with_bias=True).ctx.describe_plan(0, w.batch, w.n_cached + 1).uses_mfma == 0


@pytest.mark.parametrize("batch,t_new", [(16, 1), (35, 2), (1, 1), (4, 32), (43, 3)])
@pytest.mark.parametrize("variant", ["gelu-bf16", "leaky-f16-bias", "gelu-int8"])
def test_two_layer_encoder_on_a_few_tokens(batch, t_new, variant):
    """Encode calls of up to 128 tokens through a two-layer encoder: the kernel form whose waves split the hidden
    blocks (1..4 workgroups of 32 tokens, ragged), and the first sizes above it (129 tokens)."""
    from paper_2512_06727_amd.harness import Session
    kw = {"gelu-bf16": {}, "leaky-f16-bias": {"with_bias": True}, "gelu-int8": {"latent_format": "int8"}}[variant]
    over = {"leaky-f16-bias": dict(dtype="f16", act="leaky_relu")}.get(variant, {})
    w = synth.CONFIGS[3].scaled(n_layers=2, batch=batch, n_cached=t_new, n_steps=1, **over)
    from paper_2512_06727_amd import binding
    assert Session(w, **kw).ctx.describe_encode(0, batch, t_new) == binding.ENC_MFMA_TWO_LAYER
    fmt = kw.get("latent_format", "dtype")
    orc = build_oracle(w, with_bias=kw.get("with_bias", False), latent_format=fmt)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, t_new)
    ses = Session(w, poison=True, **kw)
    ses.prefill(0, t_new, chunk=t_new)
    torch.cuda.synchronize()
    if fmt == "int8":
        assert_quantized_cache_close(w, ses, orc, t_new)
    else:
        assert_cache_close(w, ses, orc, t_new)


# head widths 32, 96 and 128 in the fused kernel (its epilogue cuts the V decoder's slices into 16-byte pieces per row:
# 4, 12 and 16 pieces), with a reused head so that a group holds more than one KV head
CASES["dh32-fused"] = (C[2].scaled(n_layers=3, batch=3, n_cached=200, n_steps=1, n_q_heads=32, n_kv_heads=4, d_head=32, reuse="odd:1"), {"with_bias": True})
CASES["dh96-fused"] = (C[2].scaled(n_layers=3, batch=3, n_cached=200, n_steps=1, n_q_heads=32, n_kv_heads=4, d_head=96, latent=64, policy="P2", reuse="odd:1"), {})
CASES["dh128-fused"] = (C[2].scaled(n_layers=3, batch=3, n_cached=200, n_steps=1, n_q_heads=16, n_kv_heads=2, d_head=128, latent=64, policy="P2", reuse="odd:1",
                                    dtype="f16"), {"with_bias": True})


@pytest.mark.parametrize("name", ["c2-small", "c4-small", "c4-small-p2", "dh32-fused", "dh96-fused", "dh128-fused"])
def test_fused_single_split_kernel(name):
    """With one split the absorbed queries and the output epilogue run inside the attention kernel;
    the same cases with the three separate kernels must give the same answer as the oracle."""
    from paper_2512_06727_amd.harness import Session
    w, kw = CASES[name]
    _, want = run_oracle(w, gain=20.0, **kw)
    for no_fuse, wg_waves in ((False, 4), (False, 8), (True, 0)):       # four- and eight-wave workgroups, then unfused
        ses, got = run_gpu(w, gain=20.0, n_splits=1, no_fuse=no_fuse, wg_waves=wg_waves, **kw)
        assert ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1).fused == (0 if no_fuse else 1)
        assert_outputs_close(w, got, want, f"{name} no_fuse={no_fuse} wg_waves={wg_waves}")


@pytest.mark.parametrize("force_generic", [False, True])
def test_many_source_layers_need_several_launches(force_generic):
    """GPT-2 shape, 12 layers, KV head g reused in every layer after layer g: the last layer's heads come from
    12 different source layers (12 groups: more than one launch carries), with latent widths 384, 352, .. 32."""
    from paper_2512_06727_amd.harness import Session
    w = C[1].scaled(n_layers=12, batch=2, n_cached=100, n_steps=1)
    reuse = np.zeros((12, 2, 12), dtype=bool)
    for layer in range(12):
        reuse[layer, :, :layer] = True
    _, want = run_oracle(w, reuse=reuse, gain=10.0)
    ses, got = run_gpu(w, reuse=reuse, gain=10.0, force_generic=force_generic)
    plan = ses.ctx.describe_plan(11, w.batch, w.n_cached + 1)
    assert plan.n_groups == 12 and plan.n_launches == 2
    assert [ses.ctx.resolve_source(11, 0, g) for g in range(12)] == list(range(12))
    assert_outputs_close(w, got, want, label=f"12 sources, force_generic={force_generic}")


@pytest.mark.parametrize("gain", [1.0, 8.0])
@pytest.mark.parametrize("variant", ["gelu-bf16", "gelu-f16-narrow", "gelu-bf16-int8"])
def test_gelu_decoder_over_its_whole_range(variant, gain):
    """Two-layer GELU decoders whose pre-activations reach |x| = 8, far into both tails (the benchmark weights keep
    them below 0.1, where GELU is almost linear): first-layer weights 200 times larger, last-layer weights smaller so
    that decoded rows keep their usual size.  Decode step (the matrix-core kernel that rebuilds hidden rows per tile)
    and prefill attention (the kernel that decodes rows once) against the oracle's erf form."""
    from paper_2512_06727_amd.harness import Session
    from tests.helpers import REL_TOL, elementwise_bound
    over = {"gelu-bf16": {}, "gelu-f16-narrow": dict(dtype="f16", latent=64, hidden=128, dec_gain=(380.0, 0.35)), "gelu-bf16-int8": {}}[variant]
    fmt = "int8" if variant.endswith("int8") else "dtype"
    w = C[3].scaled(n_layers=2, batch=2, n_cached=150, n_steps=1, **{**dict(dec_gain=(200.0, 0.25), reuse="odd:1", policy="P2"), **over})
    print(f"case {variant} gain {gain} {w}", flush=True)
    orc, want = run_oracle(w, gain=gain, with_bias=True, latent_format=fmt)
    # the inputs really span the range: decoder pre-activations of the cached rows, from the oracle's latents
    for which in (0, 1):
        w1, b1 = orc.ae[(0, which)].dec[0]
        pre = orc.Z[(0, which)][:, :w.n_cached + 1] @ w1 + b1
        assert 6.0 < np.abs(pre).max() < 16.0 and (np.abs(pre) > 4.0).mean() > 0.02 and (np.abs(pre) < 1.0).mean() > 0.1, (np.abs(pre).max(), pre.std())
    ses, got = run_gpu(w, gain=gain, with_bias=True, latent_format=fmt)
    assert ses.ctx.describe_plan(1, w.batch, w.n_cached + 1).uses_mfma == 1
    assert_outputs_close(w, got, want, f"{variant} decode")
    n_rows = w.n_cached + 1
    q = synth.prompt_queries(w, 1, 0, w.batch, 0, n_rows, gain=gain)
    want_p = orc.prefill_attention(1, q.double().numpy(), 0)
    got_p = ses.prefill_attention(1, q.to(ses.dev, ses.tdt), 0).float().cpu().double().numpy()
    err = np.abs(got_p - want_p)
    assert np.isfinite(got_p).all() and (err <= elementwise_bound(want_p, w.dtype)).all(), f"{variant} prefill: max abs err {err.max():.3e}"
    assert err.max() <= REL_TOL[w.dtype] * np.abs(want_p).max()


# ---- several splits in one launch: the last workgroup of a (sequence, group) merges the partials and decodes --------
ONE_LAUNCH = {
    # TinyLlama shape, reuse chain: two groups per layer, 34 workgroup tiles per sequence
    "tinyllama": (C[2].scaled(n_layers=3, batch=2, n_cached=4300, n_steps=1), {}),
    # Bernoulli map, full-width policy, biases: groups of unequal size
    "bernoulli-p2-bias": (C[4].scaled(n_layers=5, batch=3, n_cached=1000, n_steps=1, policy="P2"), {"with_bias": True}),
    # head width 128, fp16
    "dh128-f16": (C[2].scaled(n_layers=3, batch=2, n_cached=1100, n_steps=1, n_q_heads=16, n_kv_heads=2, d_head=128, latent=64, policy="P2", reuse="odd:1",
                              dtype="f16"), {"with_bias": True}),
    "tinyllama-int8": (C[2].scaled(n_layers=3, batch=2, n_cached=4300, n_steps=1), {"latent_format": "int8"}),
}


@pytest.mark.parametrize("n_splits", [2, 7, 32])
@pytest.mark.parametrize("name", list(ONE_LAUNCH))
def test_one_launch_split_kernel(name, n_splits):
    """With several splits the attention kernel's last workgroup per (sequence, group) merges and decodes (plan.fused == 2);
    the workspace starts out as random bytes (arrival counters included).  Against the oracle, and the same with the
    partials going to the separate merge kernel (no_arrive)."""
    from paper_2512_06727_amd.harness import Session
    w, kw = ONE_LAUNCH[name]
    print(f"case {name} splits {n_splits} {w} {kw}", flush=True)
    _, want = run_oracle(w, gain=20.0, **kw)
    for no_arrive in (False, True):
        ses, got = run_gpu(w, gain=20.0, n_splits=n_splits, no_arrive=no_arrive, **kw)
        plan = ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1)
        assert plan.n_splits == min(n_splits, (w.n_cached + 1 + 127) // 128) and plan.fused == (0 if no_arrive else 2)
        assert_outputs_close(w, got, want, f"{name} splits={n_splits} no_arrive={no_arrive}")


def test_one_launch_split_kernel_repeated_on_one_workspace():
    """The same workspace serves every layer and step, with different split counts and batch sizes in turn: each
    launch must find its arrival counters at rest whatever ran before."""
    from paper_2512_06727_amd.harness import Session
    w, kw = ONE_LAUNCH["tinyllama"]
    _, want = run_oracle(w, gain=20.0)
    ses = Session(w, poison=True)
    ses.prefill(0, w.n_cached + 1, chunk=256)
    ses.ensure_workspace(w.batch, w.n_cached + 1)
    for rep, splits in enumerate([0, 5, 2, 32, 3, 0]):
        ses.ctx.set_tuning(n_splits=splits)
        ses.ensure_workspace(w.batch, w.n_cached + 1)
        for n in range(w.n_layers):
            q = synth.queries(w, n, 0, gain=20.0).to(ses.dev, ses.tdt)
            got = ses.decode_attention(n, q, w.n_cached + 1).float().cpu().double().numpy()
            assert_outputs_close(w, [{n: got}], [{n: want[0][n]}], f"repeat {rep} splits {splits} layer {n}")


def test_one_launch_split_kernel_gives_the_same_bits_every_time():
    """The splits' partials cross from one workgroup to another inside the launch (agent-scope stores and loads, an
    arrival counter): 300 launches in a row on a workspace whose contents are scrambled in between must reproduce the
    first result bit for bit (the merge order is fixed), and that result must match the oracle.  A partial read before
    it was complete, or out of a stale cache line, would show up as a differing output."""
    from paper_2512_06727_amd.harness import Session
    w = C[2].scaled(n_layers=3, batch=24, n_cached=2300, n_steps=1)
    ses = Session(w, poison=True, n_splits=6)
    ses.prefill(0, w.n_cached + 1, chunk=512)
    n_ctx = w.n_cached + 1
    plan = ses.ctx.describe_plan(2, w.batch, n_ctx)
    assert plan.fused == 2 and plan.n_splits == 6
    ses.ensure_workspace(w.batch, n_ctx)
    q = synth.queries(w, 2, 0, gain=20.0).to(ses.dev, ses.tdt)
    first = ses.decode_attention(2, q, n_ctx).clone()
    orc = build_oracle(w)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, n_ctx)
    want = orc.decode_attention(2, synth.queries(w, 2, 0, gain=20.0).double().numpy(), n_ctx)
    assert_outputs_close(w, [{2: first.float().cpu().double().numpy()}], [{2: want}], "first launch")
    out = torch.empty_like(first)
    for rep in range(300):
        if rep % 10 == 0:
            ses.workspace.random_(0, 256)           # also scrambles the arrival counters: every launch must cope with any content
        ses.ctx.decode_attention(2, q, out, w.batch, n_ctx, ses.workspace)
        if rep % 25 == 24:
            assert torch.equal(out, first), f"launch {rep} differs"
    torch.cuda.synchronize()
    assert torch.equal(out, first)
