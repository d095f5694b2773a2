"""GPU parity of the prompt-sized encode + append (kvcar_encode_append with 8192 tokens or more per call, linear
encoders): the latent caches against the oracle's on the same seeded inputs, and bit for bit against the
library's general encoder kernel."""
import numpy as np
import pytest
import torch

from paper_2512_06727_amd import synth
from tests.helpers import assert_cache_close, assert_quantized_cache_close, build_oracle, oracle_prefill

pytestmark = pytest.mark.gpu

C = synth.CONFIGS

# 3 x 2731 = 8193 tokens per call: 64 full 128-token workgroup tiles and a tail of one token
CASES = {
    # TinyLlama shape; layer 2 stores three of four KV heads (input 192 -> latent 96), layers 0-1 all four
    "c2-bf16": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0), {}),
    "c2-f16-bias": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0, dtype="f16"), {"with_bias": True}),
    # Bernoulli(0.3) map: layers storing 1..4 heads; P2 keeps the latent at full width (64 h -> 128)
    "c4-bf16": (C[4].scaled(n_layers=8, batch=3, n_cached=2731, n_steps=0), {}),
    "c4-bf16-p2": (C[4].scaled(n_layers=6, batch=3, n_cached=2731, n_steps=0, policy="P2"), {"with_bias": True}),
    # 3 x 22000 = 66000 tokens: 516 workgroup tiles over 128 workgroups per tensor, so every wave walks four or five
    # tiles (the look-ahead slots are reused) and the last workgroup tile is ragged
    "c2-bf16-long": (C[2].scaled(n_layers=3, batch=3, n_cached=22000, n_steps=0), {}),
    "c2-int8-long": (C[2].scaled(n_layers=3, batch=3, n_cached=22000, n_steps=0), {"latent_format": "int8"}),
    # 1030 sequences of 8 tokens: fewer tokens per sequence than a wave tile has rows, so a tile's rows step through
    # several sequences (each row finds its sequence by division)
    "c2-bf16-many-short": (C[2].scaled(n_layers=2, batch=1030, n_cached=8, n_steps=0), {}),
    "c2-int8-many-short": (C[2].scaled(n_layers=2, batch=1030, n_cached=8, n_steps=0), {"latent_format": "int8"}),
    # two KV heads of width 128 (layer 2 stores one: input 128 -> latent 64), fp16 and int8 rows
    "dh128-f16": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0, n_q_heads=8, n_kv_heads=2, d_head=128, dtype="f16"), {"with_bias": True}),
    "dh128-int8": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0, n_q_heads=8, n_kv_heads=2, d_head=128), {"latent_format": "int8"}),
    # eight KV heads of width 32: layer 2 stores seven (input 224 -> latent 112, no multiple of 32: the plain-ALU kernel takes
    # that layer, the prompt-sized one layers 0 and 1)
    "dh32-bf16": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0, n_q_heads=16, n_kv_heads=8, d_head=32), {}),
    # int8 latent rows: the quantiser runs over whole rows in the same kernel
    "c2-int8": (C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=0), {"latent_format": "int8"}),
    "c4-int8-bias": (C[4].scaled(n_layers=5, batch=3, n_cached=2731, n_steps=0), {"latent_format": "int8", "with_bias": True}),
}


def filled_session(w, chunks, **kw):
    from paper_2512_06727_amd.harness import Session
    ses = Session(w, poison=True, **kw)
    for t0, t1 in chunks:
        ses.prefill(t0, t1, chunk=t1 - t0)
    torch.cuda.synchronize()
    return ses


@pytest.mark.parametrize("name", list(CASES))
def test_prompt_sized_encode_matches_oracle_and_general_kernel(name):
    w, kw = CASES[name]
    print(f"case {name} {w}", flush=True)
    fmt = kw.get("latent_format", "dtype")
    orc = build_oracle(w, with_bias=kw.get("with_bias", False), latent_format=fmt)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, w.n_cached)
    ses = filled_session(w, [(0, w.n_cached)], **kw)
    if fmt == "int8":
        assert_quantized_cache_close(w, ses, orc, w.n_cached)
    else:
        assert_cache_close(w, ses, orc, w.n_cached)
    # the general encoder kernel forms the same sums in the same order: equal bytes, poison included
    ref = filled_session(w, [(0, w.n_cached)], no_bulk_encode=True, **kw)
    for layer in range(w.n_layers):
        for which in (0, 1):
            a, b = ses.caches[layer][which], ref.caches[layer][which]
            assert (a is None) == (b is None)
            if a is not None:
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"layer {layer} tensor {which}: caches differ"


def test_prompt_sized_encode_in_two_chunks_at_an_offset():
    """Two calls of 3 x 2740 tokens: the second appends at position 2740."""
    w = C[2].scaled(n_layers=3, batch=3, n_cached=5480, n_steps=0)
    orc = build_oracle(w)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, 5480)
    ses = filled_session(w, [(0, 2740), (2740, 5480)])
    assert_cache_close(w, ses, orc, 5480)


@pytest.mark.parametrize("fmt", ["dtype", "int8"])
def test_prompt_sized_encode_at_per_sequence_positions(fmt):
    """kvcar_encode_append_at with 2731 tokens per sequence, every sequence at a position of its own."""
    from paper_2512_06727_amd.harness import Session
    w = C[2].scaled(n_layers=3, batch=3, n_cached=2731, n_steps=40)
    starts = [0, 17, 40]
    ses = Session(w, poison=True, latent_format=fmt)
    ref = Session(w, poison=True, latent_format=fmt, no_bulk_encode=True)
    pos = torch.tensor(starts, dtype=torch.int32, device=ses.dev)
    for layer in range(w.n_layers):
        k = synth.kv_tokens(w, layer, 0, 0, w.batch, 0, 2731, device=ses.dev).to(ses.tdt)
        v = synth.kv_tokens(w, layer, 1, 0, w.batch, 0, 2731, device=ses.dev).to(ses.tdt)
        for s in (ses, ref):
            s.ctx.encode_append_at(layer, k, v, w.batch, pos, 2731)
    torch.cuda.synchronize()
    orc = build_oracle(w, latent_format=fmt)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, 2731)
    for layer in range(w.n_layers):
        for which in (0, 1):
            a, b = ses.caches[layer][which], ref.caches[layer][which]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
            if fmt == "int8":
                continue
            view = ses.cache_view(layer, which).float().cpu().double().numpy()
            zo = orc.Z[(layer, which)]
            for bi, st in enumerate(starts):
                got, want = view[bi, st:st + 2731], zo[bi, :2731]
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
                assert (np.abs(got - want) <= ulp * 1.0001 + 2e-6 * np.abs(want).max()).all()
                assert np.isnan(view[bi, :st]).all() and np.isnan(view[bi, st + 2731:]).all()


@pytest.mark.parametrize("fmt", ["dtype", "int8"])
def test_prompt_sized_encode_with_different_maps_for_keys_and_values(fmt):
    """Layer 1 reuses one key head and two value heads: its K and V encoders have different widths (192 -> 96 and
    128 -> 64) and leave in a launch each; 4 x 2048 = 8192 tokens, no ragged tile."""
    w = C[2].scaled(n_layers=2, batch=4, n_cached=2048, n_steps=0, reuse="none")
    reuse = np.zeros((2, 2, w.n_kv_heads), dtype=bool)
    reuse[1, 0, 0] = True
    reuse[1, 1, 1] = reuse[1, 1, 2] = True
    orc = build_oracle(w, reuse=reuse, latent_format=fmt)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, w.n_cached)
    from paper_2512_06727_amd import binding
    from paper_2512_06727_amd.harness import Session
    ses = Session(w, reuse=reuse, poison=True, latent_format=fmt)
    assert ses.ctx.describe_encode(1, w.batch, w.n_cached) == binding.ENC_MFMA_STREAM
    ses.prefill(0, w.n_cached, chunk=w.n_cached)
    torch.cuda.synchronize()
    assert ses.caches[1][0].shape[-1] != ses.caches[1][1].shape[-1] or fmt == "int8"
    if fmt == "int8":
        assert_quantized_cache_close(w, ses, orc, w.n_cached)
    else:
        assert_cache_close(w, ses, orc, w.n_cached)
