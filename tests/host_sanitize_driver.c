/* Host-side exercise of libkvcar's C ABI for a build whose host code is compiled with -fsanitize=address,undefined
 * (tests/test_host_sanitizers.py compiles and runs it; the sanitizers abort the program on a finding).
 * Device pointers are fake, 16-byte aligned addresses that the host code never dereferences; no entry point that
 * enqueues a kernel is reached with valid arguments, so the program needs no GPU. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kvcar.h"

#define FAKE ((void *)(uintptr_t)0x7f0000001000ull)
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            fprintf(stderr, "line %d: check failed: %s\n", __LINE__, #cond); \
            exit(2);                                                         \
        }                                                                    \
    } while (0)

static kvcar_ae_desc desc(int in_w, int hid, int lat, int act, int per_head) {
    kvcar_ae_desc d;
    memset(&d, 0, sizeof d);
    d.in_width = in_w;
    d.hidden_width = hid;
    d.latent_width = lat;
    d.act = act;
    d.leaky_slope = 0.01f;
    d.per_head = per_head;
    if (in_w) {
        d.enc_w1 = d.dec_w1 = FAKE;
        if (hid) d.enc_w2 = d.dec_w2 = d.enc_b1 = d.dec_b1 = FAKE;
    }
    return d;
}

/* A model of `n_layers` layers with a reuse map that stores h(layer) heads, planned over several batch sizes and
 * context lengths (few sequences: many splits; many sequences: one). */
static void plan_model(int dtype, int latent_format, int hq, int hkv, int dh, int r_head, int hid, int per_head) {
    kvcar_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 6; cfg.n_q_heads = hq; cfg.n_kv_heads = hkv; cfg.d_head = dh;
    cfg.max_batch = 300; cfg.max_seq = 9000; cfg.dtype = dtype; cfg.latent_format = latent_format;
    kvcar_ctx *ctx = NULL;
    CHECK(kvcar_create(&cfg, &ctx) == KVCAR_OK && ctx);
    uint8_t k_map[64], v_map[64];
    for (int layer = 1; layer < cfg.n_layers; ++layer) {
        for (int g = 0; g < hkv; ++g) {
            k_map[g] = (uint8_t)((layer * 7 + g * 3) % 3 == 0);
            v_map[g] = (uint8_t)((layer * 5 + g) % 4 == 0);
        }
        CHECK(kvcar_set_reuse_map(ctx, layer, k_map, v_map) == KVCAR_OK);
    }
    for (int layer = 0; layer < cfg.n_layers; ++layer)
        for (int which = 0; which < 2; ++which) {
            int stored = 0, src = -1;
            for (int g = 0; g < hkv; ++g) {
                CHECK(kvcar_resolve_source(ctx, layer, which, g, &src) == KVCAR_OK && src >= 0 && src <= layer);
                stored += src == layer;
            }
            kvcar_ae_desc d = desc(stored * dh, stored ? hid : 0, stored * r_head, stored && hid ? KVCAR_ACT_GELU : KVCAR_ACT_NONE, stored ? per_head : 0);
            CHECK(kvcar_set_autoencoder(ctx, layer, which, &d) == KVCAR_OK);
            size_t need = 0;
            CHECK(kvcar_cache_bytes(ctx, layer, which, &need) == KVCAR_OK);
            CHECK((need > 0) == (stored > 0));
            if (need) {
                CHECK(kvcar_bind_cache(ctx, layer, which, FAKE, need - 1) == KVCAR_ERR_CAPACITY);
                CHECK(kvcar_bind_cache(ctx, layer, which, FAKE, need) == KVCAR_OK);
            }
        }
    const int batches[4] = {1, 7, 32, 300}, ctxs[4] = {1, 129, 2049, 9000};
    for (int bi = 0; bi < 4; ++bi)
        for (int ci = 0; ci < 4; ++ci) {
            size_t ws = 0, pws = 0, largest = 0;
            CHECK(kvcar_workspace_bytes(ctx, batches[bi], ctxs[ci], &ws) == KVCAR_OK);
            CHECK(kvcar_prefill_workspace_bytes(ctx, batches[bi], ctxs[ci], &pws) == KVCAR_OK && pws > 0);
            for (int layer = 0; layer < cfg.n_layers; ++layer) {
                kvcar_plan_info info;
                CHECK(kvcar_describe_plan(ctx, layer, batches[bi], ctxs[ci], &info) == KVCAR_OK);
                CHECK(info.n_groups >= 1 && info.n_splits >= 1 && info.n_launches >= 1);
                if (info.workspace_bytes > largest) largest = info.workspace_bytes;
                int kind = -1;
                CHECK(kvcar_describe_encode(ctx, layer, batches[bi], 1, &kind) == KVCAR_OK && kind >= 0);
                CHECK(kvcar_describe_encode(ctx, layer, batches[bi], 4096, &kind) == KVCAR_OK && kind >= 0);
            }
            CHECK(ws == largest);
        }
    /* tuning: every documented value, then a bad one */
    kvcar_tuning t;
    memset(&t, 0, sizeof t);
    t.n_splits = 5; t.no_fuse = 1; t.no_arrive = 1; t.tile_order = 2; t.wg_waves = 8; t.no_bulk_encode = 1; t.no_colocate = 1; t.group_slots = 16;
    CHECK(kvcar_set_tuning(ctx, &t) == KVCAR_OK);
    kvcar_plan_info info;
    CHECK(kvcar_describe_plan(ctx, 1, 7, 2049, &info) == KVCAR_OK && info.n_splits == 5 && info.fused == 0);
    t.force_generic = 1;
    CHECK(kvcar_set_tuning(ctx, &t) == KVCAR_OK);
    CHECK(kvcar_describe_plan(ctx, 1, 7, 2049, &info) == KVCAR_OK && info.uses_mfma == 0);
    t.wg_waves = 3;
    CHECK(kvcar_set_tuning(ctx, &t) == KVCAR_ERR_ARG);
    /* argument errors that must come back before any launch; the error text is kept per context */
    CHECK(kvcar_encode_append(ctx, 0, NULL, FAKE, 1, 0, 1, NULL) == KVCAR_ERR_ARG);
    CHECK(kvcar_encode_append(ctx, 0, FAKE, FAKE, 301, 0, 1, NULL) == KVCAR_ERR_CAPACITY);
    CHECK(kvcar_decode_attention(ctx, 0, FAKE, FAKE, 1, 9001, FAKE, (size_t)1 << 30, NULL) == KVCAR_ERR_CAPACITY);
    CHECK(kvcar_decode_attention(ctx, 0, FAKE, FAKE, 300, 9000, FAKE, 16, NULL) == KVCAR_ERR_WORKSPACE);
    CHECK(kvcar_append_attend(ctx, 0, FAKE, FAKE, FAKE, FAKE, 300, 9000, FAKE, (size_t)1 << 30, NULL) == KVCAR_ERR_CAPACITY);
    CHECK(kvcar_prefill_attention(ctx, 0, FAKE, FAKE, 2, 8000, 2000, FAKE, (size_t)1 << 40, NULL) == KVCAR_ERR_CAPACITY);
    CHECK(kvcar_decode_attention(ctx, 99, FAKE, FAKE, 1, 1, FAKE, 1024, NULL) == KVCAR_ERR_ARG);
    CHECK(strlen(kvcar_last_error(ctx)) > 0);
    /* a changed map invalidates the layer's autoencoders */
    memset(k_map, 0, sizeof k_map);
    memset(v_map, 0, sizeof v_map);
    CHECK(kvcar_set_reuse_map(ctx, 3, k_map, v_map) == KVCAR_OK);
    CHECK(kvcar_describe_plan(ctx, 3, 1, 10, &info) == KVCAR_ERR_STATE);
    k_map[0] = 1;
    CHECK(kvcar_set_reuse_map(ctx, 0, k_map, v_map) == KVCAR_ERR_REUSE);
    CHECK(kvcar_destroy(ctx) == KVCAR_OK);
}

int main(void) {
    CHECK(kvcar_create(NULL, NULL) == KVCAR_ERR_ARG);
    for (int code = 0; code >= -10; --code) CHECK(kvcar_status_string(code) != NULL);
    /* TinyLlama and GPT-2 shapes: dense linear, two-layer, int8 rows, per-head, fp32 */
    plan_model(KVCAR_BF16, KVCAR_LATENT_DTYPE, 32, 4, 64, 32, 0, 0);
    plan_model(KVCAR_BF16, KVCAR_LATENT_DTYPE, 32, 4, 64, 32, 256, 0);
    plan_model(KVCAR_F16, KVCAR_LATENT_INT8, 32, 4, 64, 32, 0, 0);
    plan_model(KVCAR_BF16, KVCAR_LATENT_DTYPE, 32, 4, 64, 32, 0, 1);
    plan_model(KVCAR_F16, KVCAR_LATENT_DTYPE, 12, 12, 64, 32, 0, 0);
    plan_model(KVCAR_F16, KVCAR_LATENT_DTYPE, 12, 12, 64, 32, 0, 1);
    plan_model(KVCAR_F32, KVCAR_LATENT_DTYPE, 12, 12, 64, 24, 0, 0);
    plan_model(KVCAR_F32, KVCAR_LATENT_DTYPE, 16, 2, 128, 40, 0, 1);
    puts("host sanitize driver: ok");
    return 0;
}
