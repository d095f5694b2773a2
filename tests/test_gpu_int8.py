"""int8 latents (Methodology, "Quantization", Eq. "quant") on the GPU against the oracle: outputs of
decode attention to the floating-point tolerance, codes / scales / zero points as integer decisions
(equal, or one apart where the encoder's rounding order moves a value across a boundary), and
bit-exact on inputs whose encoder sums are exact."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import binding, synth
from helpers import assert_outputs_close, assert_quantized_cache_close, run_gpu, run_oracle

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]

C = synth.CONFIGS
CASES = {
    "c0-f32": (C[0], {}),
    "c1-small-f16": (C[1].scaled(n_layers=4, batch=2, n_cached=150, n_steps=2), {}),
    "c2-small-bf16": (C[2].scaled(n_layers=4, batch=3, n_cached=200, n_steps=2), {}),
    "c4-small-bf16": (C[4].scaled(n_layers=5, batch=2, n_cached=300, n_steps=2), {}),
    "c3-small-mlp": (C[3].scaled(n_layers=2, batch=2, n_cached=90, n_steps=1), {}),
    "leaky-bias-f16": (C[3].scaled(n_layers=2, batch=2, n_cached=40, n_steps=1, dtype="f16", act="leaky_relu", hidden=160), {"with_bias": True}),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("gain", [1.0, 50.0])
def test_int8_parity(name, gain):
    w, kw = CASES[name]
    orc, want = run_oracle(w, gain=gain, latent_format="int8", **kw)
    ses, got = run_gpu(w, gain=gain, latent_format="int8", **kw)
    assert_outputs_close(w, got, want, label=name)
    assert_quantized_cache_close(w, ses, orc, w.n_cached + w.n_steps)


@pytest.mark.parametrize("n_splits", [1, 3, 7])
def test_int8_split_counts(n_splits):
    w, kw = CASES["c2-small-bf16"]
    orc, want = run_oracle(w, latent_format="int8", **kw)
    ses, got = run_gpu(w, latent_format="int8", n_splits=n_splits, **kw)
    assert_outputs_close(w, got, want, label=f"splits={n_splits}")


@pytest.mark.parametrize("name", ["c2-small-bf16", "c4-small-bf16"])
@pytest.mark.parametrize("gain", [1.0, 50.0])
def test_int8_mfma_kernel_is_used_and_agrees_with_plain_alu(name, gain):
    """16-bit dtypes with linear decoders of width <= 128 take the MFMA kernel over int8 rows (fused
    when one split is enough, else with the prologue / merge kernels); the plain-ALU kernels must
    give the same outputs from the same caches."""
    from paper_2512_06727_amd.harness import Session
    w, kw = CASES[name]
    assert Session(w, latent_format="int8").ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1).uses_mfma == 1
    orc, want = run_oracle(w, gain=gain, latent_format="int8", **kw)
    for session_kw in ({"n_splits": 1, "wg_waves": 4}, {"n_splits": 1, "wg_waves": 8}, {"n_splits": 1, "no_fuse": True}, {"n_splits": 4},
                       {"force_generic": True}):
        ses, got = run_gpu(w, gain=gain, latent_format="int8", **session_kw, **kw)
        assert_outputs_close(w, got, want, label=f"{name} {session_kw}")


def test_int8_two_layer_decoder_takes_the_mfma_kernel():
    """Two-layer autoencoder over int8 rows (the paper's autoencoder form with its quantisation on top): the
    matrix-core kernel dequantises while parking the tile; the plain-ALU kernels give the same outputs."""
    from paper_2512_06727_amd.harness import Session
    w, kw = CASES["c3-small-mlp"]
    assert Session(w, latent_format="int8").ctx.describe_plan(0, w.batch, w.n_cached + 1).uses_mfma == 1
    orc, want = run_oracle(w, gain=8.0, latent_format="int8", **kw)
    for session_kw in ({}, {"n_splits": 2}, {"force_generic": True}):
        ses, got = run_gpu(w, gain=8.0, latent_format="int8", **session_kw, **kw)
        assert_outputs_close(w, got, want, label=f"two-layer int8 {session_kw}")


def test_int8_cache_is_smaller_and_laid_out_as_documented():
    w = C[2].scaled(n_layers=2, batch=2, n_cached=10, n_steps=1, reuse="none")
    from paper_2512_06727_amd.harness import Session
    s16, s8 = Session(w), Session(w, latent_format="int8")
    rows = w.batch * w.max_seq
    assert s16.ctx.cache_bytes(0, 0) == rows * w.latent * 2
    assert s8.ctx.cache_bytes(0, 0) == (rows * w.latent + 255) // 256 * 256 + rows * 8
    lat = np.full((w.n_layers, 2), w.latent)
    # the accounting of the oracle, up to the padding between codes and row metadata
    total = sum(s8.ctx.cache_bytes(n, k) for n in range(w.n_layers) for k in (0, 1))
    assert 0 <= total - O.quantized_latent_cache_bytes(lat, w.max_seq, w.batch) < 256 * 2 * w.n_layers


def selection_autoencoder(width, latent, stride):
    enc = np.zeros((width, latent), np.float32)
    dec = np.zeros((latent, width), np.float32)
    for c in range(latent):
        enc[stride * c, c] = 1.0
        dec[c, stride * c] = 1.0
    return enc, dec


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_int8_bit_exact_on_exact_inputs(dtype):
    """The encoder copies input columns (every product is x*1 or x*0), inputs are small integers:
    the latent rows are identical on both sides, so codes, scales and zero points must be equal
    bit for bit, ties included (rows of range 255 * 2^k put many values on .5 boundaries)."""
    hkv, dh, hq, B, L = 2, 64, 4, 3, 70
    lat, stride = 64, 2
    dev, tdt = torch.device("cuda:0"), synth.TORCH_DTYPE[dtype]
    ctx = binding.Context(1, hq, hkv, dh, B, L, dtype, latent_format="int8")
    orc = O.KVCAROracle(1, hq, hkv, dh, B, L, dtype, latent_format="int8")
    enc, dec = selection_autoencoder(hkv * dh, lat, stride)
    caches = []
    for which in (0, 1):
        orc.set_autoencoder(0, which, O.Autoencoder(list(range(hkv)), [(enc, None)], [(dec, None)]))
        te, td = torch.from_numpy(enc).to(dev, tdt), torch.from_numpy(dec).to(dev, tdt)
        ctx.set_autoencoder(0, which, hkv * dh, 0, lat, "none", [(te, None)], [(td, None)])
        c = torch.full((ctx.cache_bytes(0, which),), 0x7F, dtype=torch.uint8, device=dev)
        ctx.bind_cache(0, which, c)
        caches.append(c)
    rng = np.random.default_rng(2)
    k = rng.integers(-60, 61, size=(B, L, hkv * dh)).astype(np.float64)
    v = rng.integers(-100, 101, size=(B, L, hkv * dh)).astype(np.float64) / 4.0
    # rows with range exactly 255 / 2: scale 2, quarter values land on .5 boundaries
    v[:, ::3, 0], v[:, ::3, stride] = -60.0, 67.5
    k[:, 5] = 7.0                       # a constant row
    k[:, 6] = 0.0                       # a zero row
    orc.encode_append(0, k, v, 0)
    ctx.encode_append(0, torch.from_numpy(k).to(dev, tdt), torch.from_numpy(v).to(dev, tdt), B, 0, L)
    torch.cuda.synchronize()
    n = B * L * lat
    off = (n + 255) // 256 * 256
    for which in (0, 1):
        raw = caches[which].cpu().numpy()
        codes = raw[:n].view(np.int8).reshape(B, L, lat)
        meta = raw[off:off + B * L * 8]
        scale = meta.view(np.float32).reshape(B, L, 2)[..., 0]
        zp = meta.view(np.int32).reshape(B, L, 2)[..., 1]
        np.testing.assert_array_equal(codes, orc.Q[(0, which)])
        np.testing.assert_array_equal(scale.view(np.uint32), orc.Qscale[(0, which)].view(np.uint32))
        np.testing.assert_array_equal(zp, orc.Qzero[(0, which)])
        assert (raw[n:off] == 0x7F).all()            # the padding between codes and metadata is not touched
    # constant rows dequantise to themselves up to the rounding of the scale, zero rows exactly
    np.testing.assert_allclose(orc.Z[(0, 0)][:, 5], 7.0, rtol=1e-7)
    np.testing.assert_array_equal(orc.Z[(0, 0)][:, 6], 0.0)


def offset_rows_case(offsets, gain, session_kw_list, n_cached=300):
    """TinyLlama-shaped bf16 model whose encoders add a constant to every latent column (keys: offsets[0], values:
    offsets[1]), so that latent rows sit far from zero and their zero points are large; every seventh token is all
    zeros, which makes its latent row constant (or zero, without an offset).  The oracle encodes and quantises; its
    codes, scales and zero points are written into the library's caches (the documented layout), so that both sides
    attend over identical int8 rows and the test isolates the attention kernels.  (Through the library's own encoder
    the rows differ slightly: fp32 sums that start from a large bias lose the low bits the oracle's fp64 sums keep.)
    Returns the workload, the oracle, its outputs and one GPU result per session setting."""
    from paper_2512_06727_amd.harness import Session
    from tests.helpers import build_oracle
    w = C[2].scaled(n_layers=2, batch=2, n_cached=n_cached, n_steps=1, reuse="odd:1", latent_offset=offsets)
    n = w.n_cached + 1
    orc = build_oracle(w, latent_format="int8")
    for layer in range(w.n_layers):
        k, v = synth.kv_tokens(w, layer, 0, 0, w.batch, 0, n), synth.kv_tokens(w, layer, 1, 0, w.batch, 0, n)
        k[:, 3::7], v[:, 3::7] = 0.0, 0.0
        orc.encode_append(layer, k.double().numpy(), v.double().numpy(), 0)
    q = [synth.queries(w, layer, 0, gain=gain) for layer in range(w.n_layers)]
    want = {layer: orc.decode_attention(layer, q[layer].double().numpy(), n) for layer in range(w.n_layers)}
    results = []
    for skw in session_kw_list:
        ses = Session(w, latent_format="int8", poison=True, **skw)
        for layer in range(w.n_layers):
            for which in (0, 1):
                view = ses.quantized_view(layer, which)
                if view is None:
                    continue
                codes, scale, zp = view
                codes[:, :n].copy_(torch.from_numpy(orc.Q[(layer, which)][:, :n]))
                scale[:, :n].copy_(torch.from_numpy(orc.Qscale[(layer, which)][:, :n]))
                zp[:, :n].copy_(torch.from_numpy(orc.Qzero[(layer, which)][:, :n]))
        got = {layer: ses.decode_attention(layer, q[layer].to(ses.dev, ses.tdt), n).float().cpu().double().numpy() for layer in range(w.n_layers)}
        torch.cuda.synchronize()
        results.append((ses, got))
    return w, orc, want, results


def assert_within(got, want, dtype, label):
    """Outputs here reach the thousands (value rows with a common offset).  Per element: the absolute tolerance, the
    rounding of the output to its dtype, and 2^-12 of the value for what precedes that rounding - the softmax weights
    enter the matrix product as fp16 numbers (relative rounding 2^-12 each), which a weighted sum of equal-signed
    rows inherits and which decides the direction of the final rounding near a midpoint."""
    from tests.helpers import REL_TOL, elementwise_bound
    assert np.isfinite(got).all(), label
    err = np.abs(got - want)
    excess = err - (elementwise_bound(want, dtype) + 2.0 ** -12 * np.abs(want))
    i = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[i] <= 0, f"{label}: |{got[i]:.6g} - {want[i]:.6g}| = {err[i]:.3e} exceeds the bound by {excess[i]:.3e}"
    assert err.max() <= REL_TOL[dtype] * np.abs(want).max(), f"{label}: max err {err.max():.3e} vs max |ref| {np.abs(want).max():.3e}"


MFMA_FORMS = [{"n_splits": 1, "wg_waves": 4}, {"n_splits": 1, "wg_waves": 8}, {"n_splits": 3}, {"n_splits": 3, "wg_waves": 8}]


@pytest.mark.parametrize("offsets,zp_decade", [((0.0, 0.0), 1e2), ((8.0, 0.0), 1e3), ((96.0, 2.0), 1e4), ((0.0, 1024.0), 1e5),
                                               ((4096.0, 4096.0), 1e6), ((24576.0, 0.0), 4e6)])
def test_int8_rows_far_from_zero_through_the_mfma_kernel(offsets, zp_decade):
    """The matrix-core kernel over int8 rows feeds codes, 1/scale and the zero point to fp16 operands and states
    |zeropoint| < 2^23: rows with zero points from 1e2 to 6e6, constant rows and zero rows, in its fused (four and
    eight waves) and split forms and on the plain-ALU kernels, against the oracle.  Value rows with a large common
    offset give outputs of that size: the bound is the tolerance plus the rounding of the output to its dtype."""
    forms = MFMA_FORMS + [{"force_generic": True}]
    w, orc, want, results = offset_rows_case(offsets, 8.0, forms)
    zmax = max(int(np.abs(orc.Qzero[(0, which)][:, :w.n_cached + 1]).max()) for which in (0, 1))
    assert zp_decade / 4 < zmax < 4 * zp_decade and zmax < 2 ** 23, zmax          # the inputs are what the case claims
    const_rows = orc.Z[(0, 0)][:, 3:w.n_cached + 1:7]
    assert (const_rows.max(axis=-1) == const_rows.min(axis=-1)).all()             # constant (or zero) latent rows are present
    for (ses, got), skw in zip(results, forms):
        assert ses.ctx.describe_plan(1, w.batch, w.n_cached + 1).uses_mfma == (0 if "force_generic" in skw else 1)
        for layer in want:
            assert_within(got[layer], want[layer], w.dtype, f"{offsets} {skw} layer {layer}")


def test_int8_rows_beyond_the_mfma_kernels_limits_take_the_plain_alu_kernels():
    """Zero points beyond 2^23 (a latent row 65536 away from zero with a range of about 2) are outside what the
    matrix-core kernel's fp16 operands hold: it saturates them, so its result is finite but not the method's.
    Callers whose latents can look like this set kvcar_tuning.force_generic: the plain-ALU kernels dequantise in fp32
    (exact up to |zeropoint| = 2^24)."""
    w, orc, want, results = offset_rows_case((65536.0, 0.0), 4.0, [{"force_generic": True}, {"n_splits": 1}], n_cached=120)
    zmax = int(np.abs(orc.Qzero[(0, 0)][:, :w.n_cached + 1]).max())
    assert 2 ** 23 < zmax < 2 ** 24, zmax
    (_, got_alu), (_, got_mfma) = results
    for layer in want:
        assert_within(got_alu[layer], want[layer], w.dtype, f"plain-ALU kernels, layer {layer}")
        assert np.isfinite(got_mfma[layer]).all()
