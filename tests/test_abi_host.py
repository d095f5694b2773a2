"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and its host logic (validation, reuse resolution, sizes) behaves as documented.
No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2512_06727_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "kvcar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvcar_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert "kvcar_encode_append" in names and "kvcar_decode_attention" in names and "kvcar_set_reuse_map" in names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.SYMBOLS) == names          # the binding marshals exactly the declared calls


def make(n_layers=3, hq=8, hkv=4, dh=64, mb=2, ms=64, dtype="bf16"):
    return B.Context(n_layers, hq, hkv, dh, mb, ms, dtype)


FAKE = 0x7f0000001000          # 16-byte aligned fake device addresses: never dereferenced on the host


def desc(in_w, hid, lat, act=B.ACT_NONE, ptrs=True):
    d = B.AEDesc()
    d.in_width, d.hidden_width, d.latent_width, d.act, d.leaky_slope = in_w, hid, lat, act, 0.01
    if ptrs:
        d.enc_w1 = d.dec_w1 = FAKE
        if hid:
            d.enc_w2 = d.dec_w2 = FAKE
    return d


def test_create_validation():
    h = C.c_void_p()
    bad = B.Config(2, 7, 4, 64, 1, 8, B.BF16, 0.0)            # 7 % 4 != 0
    assert B.lib().kvcar_create(C.byref(bad), C.byref(h)) == B.ERR_SHAPE
    bad = B.Config(2, 8, 4, 64, 1, 8, 9, 0.0)
    assert B.lib().kvcar_create(C.byref(bad), C.byref(h)) == B.ERR_UNSUPPORTED
    assert B.lib().kvcar_create(None, C.byref(h)) == B.ERR_ARG
    assert B.lib().kvcar_status_string(B.ERR_REUSE) == b"KVCAR_ERR_REUSE"
    assert B.lib().kvcar_status_string(B.ERR_NOMEM) == b"KVCAR_ERR_NOMEM" and B.ERR_NOMEM == -9


def test_create_rejects_shapes_whose_offsets_do_not_fit_16_bits():
    """Query-head indices and decoder column offsets reach the kernels as 16-bit numbers."""
    h = C.c_void_p()
    for cfg in (B.Config(1, 64, 64, 512, 1, 8, B.BF16, 0.0), B.Config(1, 32768, 1, 16, 1, 8, B.BF16, 0.0)):   # 64 x 512 = 32768 columns; 32768 heads
        assert B.lib().kvcar_create(C.byref(cfg), C.byref(h)) == B.ERR_UNSUPPORTED
    assert B.lib().kvcar_create(C.byref(B.Config(1, 63, 63, 520, 1, 8, B.BF16, 0.0)), C.byref(h)) == B.OK   # 63 * 520 = 32760 columns
    B.lib().kvcar_destroy(h)


def test_reuse_resolution_matches_hand_table():
    ctx = make(n_layers=4)
    with pytest.raises(B.KVCARError) as e:
        ctx.set_reuse_map(0, [1, 0, 0, 0], [0, 0, 0, 0])
    assert e.value.status == B.ERR_REUSE
    ctx.set_reuse_map(1, [0, 1, 0, 0], [0, 0, 0, 1])
    ctx.set_reuse_map(2, [0, 1, 1, 0], [0, 0, 0, 0])
    ctx.set_reuse_map(3, [1, 1, 0, 0], [0, 0, 0, 1])
    want_k = {0: [0, 0, 0, 0], 1: [1, 0, 1, 1], 2: [2, 0, 1, 2], 3: [2, 0, 3, 3]}
    want_v = {0: [0, 0, 0, 0], 1: [1, 1, 1, 0], 2: [2, 2, 2, 2], 3: [3, 3, 3, 2]}
    for layer in range(4):
        assert [ctx.resolve_source(layer, B.K, g) for g in range(4)] == want_k[layer]
        assert [ctx.resolve_source(layer, B.V, g) for g in range(4)] == want_v[layer]


def test_autoencoder_shape_rules_and_cache_bytes():
    ctx = make()
    st = B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 0, 128)))
    assert st == B.OK
    assert ctx.cache_bytes(0, B.K) == 2 * 64 * 128 * 2                       # max_batch*max_seq*r*P
    assert B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(200, 0, 128))) == B.ERR_SHAPE
    assert B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 64, 128))) == B.ERR_SHAPE   # hidden without act
    assert B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 0, 128, B.ACT_GELU))) == B.ERR_SHAPE
    assert B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 0, 128, ptrs=False))) == B.ERR_ARG
    d = desc(256, 0, 128); d.enc_w1 = FAKE + 2
    assert B.lib().kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(d)) == B.ERR_ARG                     # misaligned
    # a layer with one reused head may cover all heads (256) or only its three stored heads (192)
    ctx.set_reuse_map(1, [0, 1, 0, 0], [0, 1, 0, 0])
    assert B.lib().kvcar_set_autoencoder(ctx._h, 1, B.K, C.byref(desc(192, 0, 96))) == B.OK
    assert ctx.cache_bytes(1, B.K) == 2 * 64 * 96 * 2
    assert B.lib().kvcar_set_autoencoder(ctx._h, 1, B.K, C.byref(desc(256, 0, 128))) == B.OK
    assert B.lib().kvcar_set_autoencoder(ctx._h, 1, B.K, C.byref(desc(128, 0, 64))) == B.ERR_SHAPE
    # changing the map drops the layer's autoencoders
    ctx.set_reuse_map(1, [0, 0, 0, 0], [0, 0, 0, 0])
    n = C.c_size_t()
    assert B.lib().kvcar_cache_bytes(ctx._h, 1, B.K, C.byref(n)) == B.ERR_STATE
    # a layer that stores nothing
    ctx.set_reuse_map(2, [1, 1, 1, 1], [1, 1, 1, 1])
    assert B.lib().kvcar_set_autoencoder(ctx._h, 2, B.K, C.byref(desc(0, 0, 0, ptrs=False))) == B.OK
    assert ctx.cache_bytes(2, B.K) == 0


def test_bind_and_capacity_errors_before_any_launch():
    ctx = make(n_layers=2)
    lib = B.lib()
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
    need = ctx.cache_bytes(0, B.K)
    assert lib.kvcar_bind_cache(ctx._h, 0, B.K, FAKE, need - 1) == B.ERR_CAPACITY
    assert lib.kvcar_bind_cache(ctx._h, 0, B.K, FAKE + 4, need) == B.ERR_ARG
    assert lib.kvcar_bind_cache(ctx._h, 0, B.K, None, need) == B.ERR_ARG
    # encode_append: state, capacity and argument errors are reported before anything is enqueued
    assert lib.kvcar_encode_append(ctx._h, 0, FAKE, FAKE, 1, 0, 1, None) == B.ERR_STATE          # caches not bound
    assert lib.kvcar_bind_cache(ctx._h, 0, B.K, FAKE, need) == B.OK
    assert lib.kvcar_bind_cache(ctx._h, 0, B.V, FAKE, need) == B.OK
    assert lib.kvcar_encode_append(ctx._h, 0, FAKE, FAKE, 3, 0, 1, None) == B.ERR_CAPACITY       # batch > max_batch
    assert lib.kvcar_encode_append(ctx._h, 0, FAKE, FAKE, 1, 60, 5, None) == B.ERR_CAPACITY      # past max_seq
    assert lib.kvcar_encode_append(ctx._h, 0, None, FAKE, 1, 0, 1, None) == B.ERR_ARG
    assert lib.kvcar_encode_append(ctx._h, 5, FAKE, FAKE, 1, 0, 1, None) == B.ERR_ARG
    assert lib.kvcar_encode_append(ctx._h, 1, FAKE, FAKE, 1, 0, 1, None) == B.ERR_STATE          # layer 1 has no autoencoder
    # decode_attention
    assert lib.kvcar_decode_attention(ctx._h, 0, FAKE, FAKE, 1, 65, FAKE, 1 << 30, None) == B.ERR_CAPACITY
    assert lib.kvcar_decode_attention(ctx._h, 0, FAKE, FAKE, 1, 0, FAKE, 1 << 30, None) == B.ERR_CAPACITY
    assert lib.kvcar_decode_attention(ctx._h, 0, FAKE, FAKE, 1, 8, FAKE, 16, None) == B.ERR_WORKSPACE
    assert lib.kvcar_decode_attention(ctx._h, 0, FAKE, None, 1, 8, FAKE, 1 << 30, None) == B.ERR_ARG
    assert lib.kvcar_decode_attention(ctx._h, 1, FAKE, FAKE, 1, 8, FAKE, 1 << 30, None) == B.ERR_STATE
    assert b"not set" in lib.kvcar_last_error(ctx._h)


def test_source_layer_must_cover_the_head():
    """Layer 1 reuses head 2 of layer 0, but layer 0's autoencoder... covers it; a layer-1
    autoencoder in the stored-heads form does not cover head 2, so layer 2 reusing head 2
    resolves past layer 1 to layer 0."""
    ctx = make(n_layers=3)
    lib = B.lib()
    ctx.set_reuse_map(1, [0, 0, 1, 0], [0, 0, 1, 0])
    ctx.set_reuse_map(2, [0, 0, 1, 0], [0, 0, 1, 0])
    assert ctx.resolve_source(2, B.K, 2) == 0
    for layer, (inw, lat) in enumerate([(256, 128), (192, 96), (192, 96)]):
        for which in (B.K, B.V):
            assert lib.kvcar_set_autoencoder(ctx._h, layer, which, C.byref(desc(inw, 0, lat))) == B.OK
            assert lib.kvcar_bind_cache(ctx._h, layer, which, FAKE, ctx.cache_bytes(layer, which)) == B.OK
    n = C.c_size_t()
    assert lib.kvcar_workspace_bytes(ctx._h, 2, 64, C.byref(n)) == B.OK and n.value > 0
    assert lib.kvcar_workspace_bytes(ctx._h, 3, 64, C.byref(n)) == B.ERR_CAPACITY


def test_workspace_grows_with_splits():
    ctx = make(n_layers=1, mb=4, ms=4096)
    lib = B.lib()
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
        assert lib.kvcar_bind_cache(ctx._h, 0, which, FAKE, ctx.cache_bytes(0, which)) == B.OK
    ctx.set_tuning(n_splits=1)
    a = ctx.workspace_bytes(4, 4096)
    ctx.set_tuning(n_splits=8)
    b = ctx.workspace_bytes(4, 4096)
    assert b > a > 0


def test_int8_latent_format_rules_and_cache_bytes():
    lib = B.lib()
    h = C.c_void_p()
    bad = B.Config(2, 8, 4, 64, 1, 8, B.BF16, 0.0, 7)                           # unknown latent format
    assert lib.kvcar_create(C.byref(bad), C.byref(h)) == B.ERR_UNSUPPORTED
    ctx = B.Context(2, 8, 4, 64, 2, 64, "bf16", latent_format="int8")
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 0, 128))) == B.OK
    rows = 2 * 64
    assert ctx.cache_bytes(0, B.K) == rows * 128 + rows * 8                    # codes (already a multiple of 256) + {scale, zeropoint} per row
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.V, C.byref(desc(256, 0, 48))) == B.OK
    assert ctx.cache_bytes(0, B.V) == (rows * 48 + 255) // 256 * 256 + rows * 8
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.V, C.byref(desc(256, 0, 24))) == B.ERR_UNSUPPORTED   # rows must be multiples of 16 bytes
    # the same width is fine with 16-bit rows (48 bytes)
    ctx16 = make()
    assert lib.kvcar_set_autoencoder(ctx16._h, 0, B.V, C.byref(desc(256, 0, 24))) == B.OK


def test_extended_step_argument_errors():
    ctx = make(n_layers=1)
    lib = B.lib()
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
        assert lib.kvcar_bind_cache(ctx._h, 0, which, FAKE, ctx.cache_bytes(0, which)) == B.OK
    ext = B.StepExt(None, FAKE, None)                                            # k_cur without v_cur
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 8, C.byref(ext), FAKE, 1 << 30, None) == B.ERR_ARG
    ext = B.StepExt(None, FAKE + 2, FAKE)                                        # misaligned
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 8, C.byref(ext), FAKE, 1 << 30, None) == B.ERR_ARG
    ext = B.StepExt(FAKE + 2, None, None)                                        # seq_lens not 4-byte aligned
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 8, C.byref(ext), FAKE, 1 << 30, None) == B.ERR_ARG
    # nothing cached yet is accepted only together with the exact current row
    ext = B.StepExt(None, None, None)
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 0, C.byref(ext), FAKE, 1 << 30, None) == B.ERR_CAPACITY
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 0, None, FAKE, 1 << 30, None) == B.ERR_CAPACITY
    ext = B.StepExt(None, FAKE, FAKE)
    assert lib.kvcar_decode_attention_ex(ctx._h, 0, FAKE, FAKE, 1, 0, C.byref(ext), FAKE, 16, None) == B.ERR_WORKSPACE   # accepted up to the workspace check
    # ragged append: positions are required
    assert lib.kvcar_encode_append_at(ctx._h, 0, FAKE, FAKE, 1, None, 1, None) == B.ERR_ARG
    assert lib.kvcar_encode_append_at(ctx._h, 0, FAKE, FAKE, 3, FAKE, 1, None) == B.ERR_CAPACITY
    assert lib.kvcar_encode_append_at(None, 0, FAKE, FAKE, 1, FAKE, 1, None) == B.ERR_ARG


def test_selection_statistic_argument_errors_and_workspace_size():
    lib = B.lib()
    n = C.c_size_t()
    assert lib.kvcar_head_l1_workspace_bytes(1000, 4, C.byref(n)) == B.OK
    assert n.value > 0 and n.value % (4 * 4) == 0                                # workgroups x heads x 4 bytes
    assert lib.kvcar_head_l1_workspace_bytes(0, 4, C.byref(n)) == B.ERR_ARG
    assert lib.kvcar_head_l1_workspace_bytes(10, 4, None) == B.ERR_ARG
    call = lib.kvcar_head_l1_distance
    assert call(None, FAKE, B.BF16, 64, 4, 64, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_ARG
    assert call(FAKE, FAKE, B.BF16, 0, 4, 64, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_ARG
    assert call(FAKE, FAKE + 8, B.BF16, 64, 4, 64, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_ARG
    assert call(FAKE, FAKE, 5, 64, 4, 64, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_UNSUPPORTED
    assert call(FAKE, FAKE, B.BF16, 64, 4, 60, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_SHAPE
    assert call(FAKE, FAKE, B.F32, 64, 4, 62, 0, FAKE, FAKE, 1 << 20, None) == B.ERR_SHAPE
    assert call(FAKE, FAKE, B.BF16, 64, 4, 64, 0, FAKE, FAKE, 4, None) == B.ERR_WORKSPACE
    assert call(FAKE, FAKE, B.BF16, 64, 2000, 64, 0, FAKE, FAKE, 1 << 30, None) == B.ERR_UNSUPPORTED


def test_prefill_workspace_size_and_argument_errors_before_any_launch():
    """Workspace of kvcar_prefill_attention = decoded keys + decoded values of the rows 0 .. n_rows - 1 in the
    model dtype; every argument, capacity, state and workspace error is reported before anything is enqueued."""
    ctx = make(n_layers=2, hq=8, hkv=4, dh=64, mb=2, ms=64, dtype="bf16")
    lib = B.lib()
    assert ctx.prefill_workspace_bytes(2, 64) == 2 * 2 * 64 * 4 * 64 * 2
    assert ctx.prefill_workspace_bytes(1, 3) == 2 * 1536            # each half is padded to 256 bytes
    n = C.c_size_t()
    assert lib.kvcar_prefill_workspace_bytes(ctx._h, 3, 8, C.byref(n)) == B.ERR_CAPACITY
    assert lib.kvcar_prefill_workspace_bytes(ctx._h, 1, 65, C.byref(n)) == B.ERR_CAPACITY
    assert lib.kvcar_prefill_workspace_bytes(ctx._h, 1, 8, None) == B.ERR_ARG
    big = 1 << 30
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_STATE        # no autoencoder yet
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_STATE        # caches not bound
    for which in (B.K, B.V):
        assert lib.kvcar_bind_cache(ctx._h, 0, which, FAKE, ctx.cache_bytes(0, which)) == B.OK
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 3, 0, 8, FAKE, big, None) == B.ERR_CAPACITY
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 60, 5, FAKE, big, None) == B.ERR_CAPACITY
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 0, 0, FAKE, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, -1, 4, FAKE, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 0, None, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE + 2, 1, 0, 8, FAKE, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 0, 8, None, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 0, FAKE, FAKE, 1, 0, 8, FAKE, ctx.prefill_workspace_bytes(1, 8) - 1, None) == B.ERR_WORKSPACE
    assert lib.kvcar_prefill_attention(ctx._h, 2, FAKE, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_ARG
    assert lib.kvcar_prefill_attention(ctx._h, 1, FAKE, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_STATE        # layer 1 has no autoencoder
    # a layer whose source does not cover a head it takes
    ctx.set_reuse_map(1, [0, 0, 1, 0], [0, 0, 0, 0])
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 1, which, C.byref(desc(256, 0, 128))) == B.OK
        assert lib.kvcar_bind_cache(ctx._h, 1, which, FAKE, ctx.cache_bytes(1, which)) == B.OK
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(desc(256, 0, 128))) == B.OK
    big_dh = make(n_layers=1, hq=2, hkv=2, dh=320, mb=1, ms=8, dtype="f32")
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(big_dh._h, 0, which, C.byref(desc(640, 0, 64))) == B.OK
        assert lib.kvcar_bind_cache(big_dh._h, 0, which, FAKE, big_dh.cache_bytes(0, which)) == B.OK
    assert lib.kvcar_prefill_attention(big_dh._h, 0, FAKE, FAKE, 1, 0, 8, FAKE, big, None) == B.ERR_UNSUPPORTED   # d_head > 256


def test_encoder_kernel_choice():
    """kvcar_describe_encode: prompt-sized calls through a linear 16-bit encoder take the streaming kernel."""
    lib = B.lib()
    ctx = make(n_layers=4, mb=16, ms=4096)
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
        assert lib.kvcar_set_autoencoder(ctx._h, 1, which, C.byref(desc(256, 256, 128, B.ACT_GELU))) == B.OK
        assert lib.kvcar_set_autoencoder(ctx._h, 2, which, C.byref(desc(256, 0, 256))) == B.OK     # latent too wide to stream
    assert ctx.describe_encode(0, 16, 1) == B.ENC_MFMA
    assert ctx.describe_encode(0, 16, 511) == B.ENC_MFMA                 # 8176 tokens
    assert ctx.describe_encode(0, 16, 512) == B.ENC_MFMA_STREAM          # 8192 tokens
    assert ctx.describe_encode(0, 16, 4096) == B.ENC_MFMA_STREAM
    assert ctx.describe_encode(1, 16, 4096) == B.ENC_MFMA_TWO_LAYER
    assert ctx.describe_encode(2, 16, 4096) == B.ENC_MFMA
    ctx.set_tuning(no_bulk_encode=True)
    assert ctx.describe_encode(0, 16, 4096) == B.ENC_MFMA
    ctx.set_tuning(force_generic=True)
    assert ctx.describe_encode(0, 16, 4096) == B.ENC_PLAIN
    ctx.set_tuning()
    k = C.c_int(-1)
    assert lib.kvcar_describe_encode(ctx._h, 3, 16, 4096, C.byref(k)) == B.ERR_STATE          # autoencoder not set
    assert lib.kvcar_describe_encode(ctx._h, 0, 17, 1, C.byref(k)) == B.ERR_CAPACITY
    assert lib.kvcar_describe_encode(ctx._h, 0, 0, 1, C.byref(k)) == B.ERR_ARG
    assert lib.kvcar_describe_encode(ctx._h, 0, 1, 1, None) == B.ERR_ARG
    # a layer that stores nothing (every head reused: its autoencoders have width zero)
    ctx.set_reuse_map(3, [1, 1, 1, 1], [1, 1, 1, 1])
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(ctx._h, 3, which, C.byref(desc(0, 0, 0, ptrs=False))) == B.OK
    assert ctx.describe_encode(3, 16, 4096) == B.ENC_NONE
    f32 = make(dtype="f32", mb=16, ms=4096)
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(f32._h, 0, which, C.byref(desc(256, 0, 128))) == B.OK
    assert f32.describe_encode(0, 16, 4096) == B.ENC_PLAIN


def test_plans_for_the_shape_sweep():
    """Host planning over the 64 shapes of the GPU shape sweep (fake device pointers, nothing launched): every shape
    is accepted, the plan's figures are consistent, and matrix-core kernels are only picked for 16-bit dtypes."""
    from paper_2512_06727_amd import synth
    from tests.test_gpu_shape_sweep import CASES
    act = {"none": B.ACT_NONE, "gelu": B.ACT_GELU, "leaky_relu": B.ACT_LEAKY_RELU}
    n_mfma = 0
    for w, kw in CASES:
        ctx = B.Context(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, w.batch, w.max_seq, w.dtype, latent_format=kw["latent_format"])
        reuse = synth.reuse_map(w)
        for layer in range(w.n_layers):
            ctx.set_reuse_map(layer, reuse[layer, 0], reuse[layer, 1])
        for layer in range(w.n_layers):
            for which in (B.K, B.V):
                stored = int((~reuse[layer, which]).sum())
                heads = stored if w.policy == "P1" else w.n_kv_heads
                lat = w.latent * stored // w.n_kv_heads if w.policy == "P1" else w.latent
                d = desc(heads * w.d_head, w.hidden if heads else 0, lat if heads else 0, act[w.act] if heads else B.ACT_NONE, ptrs=heads > 0)
                if heads and w.hidden:
                    d.enc_b1 = d.dec_b1 = FAKE
                assert B.lib().kvcar_set_autoencoder(ctx._h, layer, which, C.byref(d)) == B.OK, (w, layer, which)
                need = ctx.cache_bytes(layer, which)
                assert (need > 0) == (heads > 0)
                if need:
                    assert B.lib().kvcar_bind_cache(ctx._h, layer, which, FAKE, need) == B.OK
        n_ctx = w.n_cached + 1
        # kvcar_workspace_bytes is the largest need of any layer
        assert ctx.workspace_bytes(w.batch, n_ctx) == max(ctx.describe_plan(layer, w.batch, n_ctx).workspace_bytes for layer in range(w.n_layers))
        for layer in range(w.n_layers):
            p = ctx.describe_plan(layer, w.batch, n_ctx)
            assert 1 <= p.n_groups <= w.n_kv_heads and 1 <= p.n_splits <= 256 and p.n_launches >= 1
            assert p.workspace_bytes > 0
            assert (p.fused == 1) <= (p.n_splits == 1) and (p.fused == 2) <= (p.n_splits > 1)     # 1: single split; 2: one launch, several splits
            assert not (p.uses_mfma and w.dtype == "f32")
            n_mfma += p.uses_mfma
            kind = ctx.describe_encode(layer, w.batch, 1)
            stores = bool((~reuse[layer]).any()) if w.policy == "P1" else True
            assert (kind == B.ENC_NONE) == (not stores)
            assert not (w.dtype == "f32" and kind not in (B.ENC_NONE, B.ENC_PLAIN))
    assert n_mfma >= 40          # the sweep does reach the matrix-core kernels


def test_per_head_descriptor_rules_and_plan():
    """The per_head flag of the autoencoder descriptor (block-diagonal autoencoders; fake device pointers, nothing
    launched): what it accepts, that the cache keeps its size, that a layer is planned as one group per KV head, and that
    a head reused from an earlier layer costs that head's rows only."""
    lib = B.lib()
    ctx = make(n_layers=3, hq=32, hkv=4, dh=64, mb=8, ms=2048)

    def ph(in_w, hid, lat, act=B.ACT_NONE, flag=1):
        d = desc(in_w, hid, lat, act)
        d.per_head = flag
        return d

    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(ph(256, 0, 16))) == B.ERR_UNSUPPORTED    # 8-byte head rows
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(ph(256, 64, 128, B.ACT_GELU))) == B.ERR_UNSUPPORTED
    assert lib.kvcar_set_autoencoder(ctx._h, 0, B.K, C.byref(ph(256, 0, 128, flag=2))) == B.ERR_ARG
    ctx.set_reuse_map(1, [0, 1, 0, 0], [0, 0, 0, 1])
    ctx.set_reuse_map(2, [0, 1, 1, 0], [0, 0, 0, 0])
    assert lib.kvcar_set_autoencoder(ctx._h, 1, B.K, C.byref(ph(192, 0, 128))) == B.ERR_SHAPE         # three heads do not divide 128
    widths = {0: (4, 4), 1: (3, 3), 2: (2, 4)}            # stored heads of (K, V) per layer
    for layer, (nk, nv) in widths.items():
        for which, n in ((B.K, nk), (B.V, nv)):
            assert lib.kvcar_set_autoencoder(ctx._h, layer, which, C.byref(ph(64 * n, 0, 32 * n))) == B.OK
            need = ctx.cache_bytes(layer, which)
            assert need == 8 * 2048 * 32 * n * 2            # the head blocks together are as large as the dense rows
            assert lib.kvcar_bind_cache(ctx._h, layer, which, FAKE, need) == B.OK
    for layer in range(3):
        p = ctx.describe_plan(layer, 8, 2000)
        assert p.n_groups == 4 and p.uses_mfma == 1 and p.n_launches == 1
        assert p.latent_bytes == 4 * 2 * 32 * 2 * 8 * 2000  # 4 heads x (K + V) x 32 columns x 2 bytes, per cached token and sequence
        assert p.fused == 2 and p.append_in_kernel == 1    # 8 sequences x 4 groups: several splits, one launch
    assert ctx.describe_plan(2, 8, 2000).n_splits == 4         # 16 workgroup tiles: four per split
    assert ctx.describe_plan(2, 8, 300).n_splits == 1          # three tiles: not worth a second partial
    # int8 latents do not combine with the flag
    c8 = B.Context(2, 32, 4, 64, 2, 64, "bf16", latent_format="int8")
    assert lib.kvcar_set_autoencoder(c8._h, 0, B.K, C.byref(ph(256, 0, 128))) == B.ERR_UNSUPPORTED
    # fp32: 32-column head rows are fine, the plan takes the plain-ALU kernels
    f32 = make(n_layers=1, hq=8, hkv=4, dh=64, mb=2, ms=64, dtype="f32")
    for which in (B.K, B.V):
        assert lib.kvcar_set_autoencoder(f32._h, 0, which, C.byref(ph(256, 0, 128))) == B.OK
        assert lib.kvcar_bind_cache(f32._h, 0, which, FAKE, f32.cache_bytes(0, which)) == B.OK
    p = f32.describe_plan(0, 2, 40)
    assert p.n_groups == 4 and p.uses_mfma == 0


def test_small_launches_get_a_group_per_kv_head():
    """Host planning of the query heads per attention workgroup (fake device pointers, nothing launched): a launch that
    reads little is planned with a group per KV head - more, smaller workgroups - as long as the layer stays one launch;
    a launch that reads a lot keeps up to 32 heads per workgroup; kvcar_tuning.group_slots overrides either."""
    lib = B.lib()

    def model(hq, hkv, mb, ms, rh=32):
        ctx = make(n_layers=2, hq=hq, hkv=hkv, dh=64, mb=mb, ms=ms)
        ctx.set_reuse_map(1, [1] + [0] * (hkv - 1), [1] + [0] * (hkv - 1))
        for layer, n in ((0, hkv), (1, hkv - 1)):
            for which in (B.K, B.V):
                assert lib.kvcar_set_autoencoder(ctx._h, layer, which, C.byref(desc(64 * n, 0, rh * n))) == B.OK
                assert lib.kvcar_bind_cache(ctx._h, layer, which, FAKE, ctx.cache_bytes(layer, which)) == B.OK
        return ctx

    ctx = model(32, 4, 256, 8300)
    small, big = ctx.describe_plan(0, 32, 2049), ctx.describe_plan(0, 256, 8193)
    assert (small.n_groups, small.n_launches, small.fused) == (4, 1, 2) and small.n_splits == 2       # 4 x 32 (sequence, group) pairs: one eight-wave workgroup per compute unit
    assert (big.n_groups, big.n_splits, big.fused) == (1, 1, 1)
    assert small.latent_bytes == 4 * 2 * 128 * 2 * 32 * 2049                 # every group reads the whole rows
    assert ctx.describe_plan(1, 32, 2049).n_groups == 4                      # head 0 from layer 0, three heads of its own: 1 + 3 groups
    assert ctx.describe_plan(1, 256, 8193).n_groups == 2
    ctx.set_tuning(group_slots=32)
    assert ctx.describe_plan(0, 32, 2049).n_groups == 1
    ctx.set_tuning(group_slots=8)
    assert ctx.describe_plan(0, 256, 8193).n_groups == 4
    ctx.set_tuning(group_slots=16)
    assert ctx.describe_plan(0, 32, 2049).n_groups == 2
    t = B.Tuning()
    t.group_slots = 12
    assert lib.kvcar_set_tuning(ctx._h, C.byref(t)) == B.ERR_ARG
    # sixteen KV heads of two query heads each: a group per KV head would need two launches, so 16 heads per group
    wide = model(32, 16, 8, 600, rh=8)
    p = wide.describe_plan(0, 8, 512)
    assert p.n_groups == 2 and p.n_launches == 1
