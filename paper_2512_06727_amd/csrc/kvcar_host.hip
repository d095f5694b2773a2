// Host side of libkvcar: context, validation, reuse-source resolution, launch planning, C ABI.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <array>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "kvcar_internal.hpp"

using namespace kvcar;

namespace {

struct AEState {
    bool set = false;
    kvcar_ae_desc d{};
    std::vector<int> heads;        // KV heads covered, in column order
};

size_t dtype_size(int dt) { return dt == KVCAR_F32 ? 4 : 2; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// Scratch memory of kvcar_decode_attention_static (absorbed queries and split partials of one call), owned by the
// library so that the call itself allocates nothing.  Every device holds its own copy of this array; in host code
// the name below is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[KVCAR_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void* scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, looked up once per device

// Tag of one launch of the one-launch split attention: its arrival counters are valid only under this tag, so the
// counters need no initial state (see attend_body).  Never 0: that is the tag of a counter at rest.
unsigned next_epoch() {
    static std::atomic<unsigned> epoch{0x9e3779b9u};
    unsigned e = epoch.fetch_add(1u, std::memory_order_relaxed) + 1u;
    return e ? e : epoch.fetch_add(1u, std::memory_order_relaxed) + 1u;
}

// Address of the current device's copy of `scratch` (looked up on the first use on that device).
hipError_t scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct kvcar_ctx {
    kvcar_config cfg{};
    float scale = 0.f;
    std::vector<uint8_t> reuse;            // [layer][which][kv head]
    std::vector<AEState> ae;               // [layer][which]
    std::vector<void*> cache;              // [layer][which]
    std::vector<size_t> cache_bytes;
    kvcar_tuning tun{};
    int n_cu = 256;
    std::string err;
    bool profiling = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;   // events created so far
    size_t ev_used = 0;                                        // pairs recorded since the last read

    bool int8() const { return cfg.latent_format == KVCAR_LATENT_INT8; }
    size_t row_elem_bytes() const { return int8() ? 1 : dtype_size(cfg.dtype); }
    // int8 latents: byte offset of the row metadata inside a cache buffer of row width r
    size_t meta_offset(int r) const { return align_up((size_t)cfg.max_batch * cfg.max_seq * r, 256); }
    size_t cache_need(int r) const {
        if (r == 0) return 0;
        if (int8()) return meta_offset(r) + (size_t)cfg.max_batch * cfg.max_seq * sizeof(RowMeta);
        return (size_t)cfg.max_batch * cfg.max_seq * r * dtype_size(cfg.dtype);
    }
    uint8_t& reuse_at(int layer, int which, int g) { return reuse[((size_t)layer * 2 + which) * cfg.n_kv_heads + g]; }
    uint8_t reuse_at(int layer, int which, int g) const { return reuse[((size_t)layer * 2 + which) * cfg.n_kv_heads + g]; }
    AEState& ae_at(int layer, int which) { return ae[(size_t)layer * 2 + which]; }
    const AEState& ae_at(int layer, int which) const { return ae[(size_t)layer * 2 + which]; }
};

namespace {

int fail(const kvcar_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        const_cast<kvcar_ctx*>(ctx)->err = buf;
    }
    return code;
}

// Nearest layer M <= layer whose reuse bit for (which, g) is clear: the layer whose cache holds
// the head ("Network Architecture": heads of layer N reuse those of layer N-1; chains follow
// through to the layer that stores the head).
int resolve(const kvcar_ctx* ctx, int layer, int which, int g) {
    int m = layer;
    while (m > 0 && ctx->reuse_at(m, which, g)) --m;
    return m;
}

struct Plan {
    std::vector<GroupDesc> groups;
    std::vector<std::array<int, 2>> src;   // per group: the layers that supply its keys and its values
    bool mfma = false;        // an MFMA attention kernel (linear or two-layer decoder) is used
    bool mlp = false;         // ... the two-layer one
    bool i8 = false;          // ... the one over int8 latent rows (absorbed queries travel in fp32)
    bool fused = false;       // one kernel does prologue, attention and epilogue (single split, exact shapes)
    bool prologue = false;    // several splits: the attention kernel computes the absorbed queries itself
    bool arrive = false;      // ... and its last workgroup per (sequence, group) merges the splits and decodes: one launch
    bool arrive_w8 = false;   // ... with eight waves per workgroup
    int n_splits = 1;
    int qt_stride = 0;        // elements per sequence
    int part_stride = 0;      // floats per (sequence, split)
    size_t qt_bytes = 0, part_bytes = 0, arrive_bytes = 0, total_bytes = 0;
};

// Position of KV head g among the heads the autoencoder of (src, which) covers, or -1.
int head_slot(const kvcar_ctx* ctx, int src, int which, int g) {
    const AEState& a = ctx->ae_at(src, which);
    for (size_t i = 0; i < a.heads.size(); ++i)
        if (a.heads[i] == g) return (int)i;
    return -1;
}

// Width of one head's latent rows under a per-head autoencoder.
int head_latent(const AEState& a) { return a.heads.empty() ? 0 : a.d.latent_width / (int)a.heads.size(); }

// Bytes between the blocks of two consecutive heads in a head-major cache (per-head autoencoders).
size_t head_block_bytes(const kvcar_ctx* ctx, const AEState& a) {
    return (size_t)ctx->cfg.max_batch * ctx->cfg.max_seq * head_latent(a) * dtype_size(ctx->cfg.dtype);
}

// What the attention kernels need to know of the layer `src` that supplies tensor `which` to KV head g of `layer`.
// With a per-head autoencoder that is head g's own block of the cache and its own d_head-wide decoder (the kernels
// then see a single-head autoencoder whose columns start at 0); with a dense one g plays no part.
int fill_side(const kvcar_ctx* ctx, int layer, int src, int which, int g, SideDesc& sd) {
    const AEState& a = ctx->ae_at(src, which);
    if (!a.set) return fail(ctx, KVCAR_ERR_STATE, "layer %d needs the %s autoencoder of layer %d, which is not set", layer, which ? "V" : "K", src);
    void* z = ctx->cache[(size_t)src * 2 + which];
    if (a.d.latent_width > 0 && z == nullptr)
        return fail(ctx, KVCAR_ERR_STATE, "layer %d needs the %s cache of layer %d, which is not bound", layer, which ? "V" : "K", src);
    sd.act = a.d.act;
    sd.slope = a.d.leaky_slope;
    if (a.d.per_head) {
        const int i = head_slot(ctx, src, which, g);
        if (i < 0) return fail(ctx, KVCAR_ERR_REUSE, "layer %d takes head %d from a layer whose autoencoder does not cover it", layer, g);
        const int rh = head_latent(a), dh = ctx->cfg.d_head;
        const size_t es = dtype_size(ctx->cfg.dtype);
        sd.z = static_cast<const char*>(z) + (size_t)i * head_block_bytes(ctx, a);
        sd.meta = nullptr;
        sd.r = sd.c = rh;
        sd.in_width = dh;
        sd.w1 = nullptr; sd.b1 = nullptr;
        sd.wl = static_cast<const char*>(a.d.dec_w1) + (size_t)i * rh * dh * es;
        sd.bl = a.d.dec_b1 ? static_cast<const char*>(a.d.dec_b1) + (size_t)i * dh * es : nullptr;
        return KVCAR_OK;
    }
    sd.z = z;
    sd.meta = (ctx->int8() && z) ? static_cast<const char*>(z) + ctx->meta_offset(a.d.latent_width) : nullptr;
    sd.r = a.d.latent_width;
    sd.in_width = a.d.in_width;
    if (a.d.hidden_width > 0) {
        sd.w1 = a.d.dec_w1; sd.b1 = a.d.dec_b1; sd.wl = a.d.dec_w2; sd.bl = a.d.dec_b2; sd.c = a.d.hidden_width;
    } else {
        sd.w1 = nullptr; sd.b1 = nullptr; sd.wl = a.d.dec_w1; sd.bl = a.d.dec_b1; sd.c = a.d.latent_width;
    }
    return KVCAR_OK;
}

// First column of KV head g in the last decoder layer that fill_side hands to the kernels, or -1.
int head_column(const kvcar_ctx* ctx, int src, int which, int g) {
    const int i = head_slot(ctx, src, which, g);
    if (i < 0) return -1;
    return ctx->ae_at(src, which).d.per_head ? 0 : i * ctx->cfg.d_head;
}

constexpr size_t kLdsBudget = 150 * 1024;
constexpr size_t kFineGroupBytes = 320u << 20;     // bytes a launch may read with groups made as small as the maps allow

// One-launch split form: whether its workgroups run with eight waves - every workgroup with a compute unit to
// itself, and the eight waves' 256-token tiles make the longest split at most an eighth longer than 128-token tiles would
// (2049 tokens in 4 splits: 3 tiles of 256 against 5 of 128 - 16 sequences, 0.51 ms per step against 0.48).
bool eight_waves_fit(const kvcar_ctx* ctx, const Plan& plan, int batch, int n_groups, int n_ctx, int splits) {
    if (ctx->tun.wg_waves == 4) return false;
    if (ctx->tun.wg_waves == 8) return true;
    const auto longest_split = [&](int tile_tokens) { return ((n_ctx + tile_tokens - 1) / tile_tokens + splits - 1) / splits * tile_tokens; };
    return (long long)batch * n_groups * splits <= ctx->n_cu && 8 * longest_split(256) <= 9 * longest_split(128);
}

int build_plan(const kvcar_ctx* ctx, int layer, int batch, int n_ctx, Plan& plan) {
    const kvcar_config& c = ctx->cfg;
    const int gq = c.n_q_heads / c.n_kv_heads;
    // (K source, V source, head) -> KV heads; the head is part of the key only where a source has a per-head
    // autoencoder (then every KV head reads rows of its own), else -1
    std::map<std::array<int, 3>, std::vector<int>> by_src;
    for (int g = 0; g < c.n_kv_heads; ++g) {
        const int sk = resolve(ctx, layer, KVCAR_K, g), sv = resolve(ctx, layer, KVCAR_V, g);
        const bool own_rows = ctx->ae_at(sk, KVCAR_K).d.per_head || ctx->ae_at(sv, KVCAR_V).d.per_head;
        by_src[{sk, sv, own_rows ? g : -1}].push_back(g);
    }

    plan.groups.clear();
    plan.src.clear();
    // MFMA kernels: 16-bit dtype, linear decoders, latent widths that are multiples of 32
    bool mfma_ok = c.dtype != KVCAR_F32 && !ctx->tun.force_generic && attend_mfma_available() && c.d_head % 8 == 0;
    // ... or two-layer decoders of one of the shapes with a resident-weight kernel, the same for K and V
    bool mlp_ok = c.dtype != KVCAR_F32 && !ctx->tun.force_generic && c.d_head % 32 == 0 && c.d_head <= 128;
    int mlp_r = -1, mlp_c = -1, mlp_act = -1;
    float mlp_slope = 0.f;
    int r_all = 0;
    struct Base { GroupDesc gd; std::vector<int> heads; int src_k, src_v; };
    std::vector<Base> bases;
    for (auto& kv : by_src) {
        GroupDesc base{};
        const int src_k = kv.first[0], src_v = kv.first[1], g_first = kv.second.front();
        int rc = fill_side(ctx, layer, src_k, KVCAR_K, g_first, base.k);
        if (rc) return rc;
        rc = fill_side(ctx, layer, src_v, KVCAR_V, g_first, base.v);
        if (rc) return rc;
        // append-and-attend: the head's block of the layer's own per-head caches, and the head itself
        base.app_slice[0] = (short)(ctx->ae_at(src_k, KVCAR_K).d.per_head ? head_slot(ctx, src_k, KVCAR_K, g_first) : -1);
        base.app_slice[1] = (short)(ctx->ae_at(src_v, KVCAR_V).d.per_head ? head_slot(ctx, src_v, KVCAR_V, g_first) : -1);
        base.app_head = (short)g_first;
        if (base.k.c > kMaxRow || base.v.c > kMaxRow || base.k.r > kMaxRow || base.v.r > kMaxRow)
            return fail(ctx, KVCAR_ERR_UNSUPPORTED, "row width above %d", kMaxRow);
        if (base.k.w1 || base.v.w1 || base.k.r % 32 || base.v.r % 32 || base.k.r > 384 || base.v.r > 384) mfma_ok = false;
        // int8 rows: equal K and V widths up to 128 only
        if (ctx->int8() && (base.k.r != base.v.r || base.k.r > 128)) mfma_ok = false;
        for (const SideDesc* sd : {&base.k, &base.v}) {
            if (!sd->w1) { mlp_ok = false; continue; }
            if (mlp_r < 0) { mlp_r = sd->r; mlp_c = sd->c; mlp_act = sd->act; mlp_slope = sd->slope; }
            if (sd->r != mlp_r || sd->c != mlp_c || sd->act != mlp_act || sd->slope != mlp_slope) mlp_ok = false;
        }
        r_all = std::max(r_all, std::max(base.k.r, base.v.r));
        // query heads of this (K source, V source) pair, in increasing order
        std::vector<int> heads;
        for (int g : kv.second)
            for (int i = 0; i < gq; ++i) heads.push_back(g * gq + i);
        for (int j : heads) {
            const int g = j / gq;
            if (head_column(ctx, src_k, KVCAR_K, g) < 0 || head_column(ctx, src_v, KVCAR_V, g) < 0)
                return fail(ctx, KVCAR_ERR_REUSE, "layer %d takes head %d from a layer whose autoencoder does not cover it", layer, g);
        }
        bases.push_back(Base{base, heads, src_k, src_v});
    }
    if (mlp_ok) mlp_ok = ((mlp_r == 128 && mlp_c == 256) || (mlp_r == 64 && mlp_c == 128)) &&
                         (mlp_act == KVCAR_ACT_GELU || mlp_act == KVCAR_ACT_LEAKY_RELU);
    if (mlp_ok) mfma_ok = true;
    // Query heads per group on the matrix-core kernels for rows up to 128 wide.  A workgroup's fixed work - absorbed
    // queries, its partial, the merge and the V decoder - grows with the heads it serves, its share of the streaming does
    // not.  A launch that moves little (a few dozen sequences) is a chain of such fixed pieces: there every KV head gets
    // a group of its own (as few heads per workgroup as the maps allow while the layer stays one launch), although each
    // group then reads its sources' rows for itself - the copies meet in the caches.  A launch that moves a lot is bound by
    // those bytes and keeps up to 32 heads per workgroup.  Measured crossover: between 300 and 440 MB read per launch
    // (TinyLlama shape, 2048 cached tokens: 64 sequences gain a fifth with a group per KV head, 96 sequences lose a fifth).
    // Many short sequences are the other limit: once there are more (sequence, group) pairs than compute units the
    // finer groups only queue behind each other (256 sequences of 512 tokens lose a quarter), so the finer form is
    // taken only while the pairs fit the chip at one workgroup each.
    int fine_cap = 0;                                       // 0: the kernels' capacity
    if (mfma_ok && !mlp_ok && r_all <= 128) {
        if (ctx->tun.group_slots > 0) {
            fine_cap = ctx->tun.group_slots;
        } else {
            for (int cap_try : {gq, 16}) {                  // one KV head per group, else one head block
                size_t n_groups = 0, bytes = 0;             // ... and what the launch then reads
                for (auto& bh : bases) {
                    const size_t chunks = (bh.heads.size() + cap_try - 1) / cap_try;
                    n_groups += chunks;
                    bytes += chunks * (size_t)(bh.gd.k.r + bh.gd.v.r) * ctx->row_elem_bytes() * batch * n_ctx;
                }
                if (cap_try <= 32 && n_groups <= (size_t)kMaxGroups && bytes <= kFineGroupBytes &&
                    n_groups * (size_t)batch <= (size_t)ctx->n_cu) { fine_cap = cap_try; break; }
            }
        }
    }
    for (auto& bh : bases) {
        const GroupDesc& base = bh.gd;
        const std::vector<int>& heads = bh.heads;
        int cap;
        if (mfma_ok) {
            cap = (mlp_ok || r_all <= 128) ? 32 : 16;      // head blocks one wave can keep accumulators for
            if (fine_cap > 0) cap = std::min(cap, fine_cap);
        } else {
            // slot capacity of one plain-ALU workgroup: accumulators and LDS
            cap = std::min(kMaxSlots, kGenericAcc * 256 / std::max(1, base.v.c));
            while (cap > 0) {
                GroupDesc t = base; t.n_slots = cap;
                if (attend_generic_lds_bytes(t) <= kLdsBudget) break;
                --cap;
            }
            if (cap < 1) return fail(ctx, KVCAR_ERR_UNSUPPORTED, "rows too wide for the attention kernel");
        }
        for (size_t h0 = 0; h0 < heads.size(); h0 += cap) {
            GroupDesc gd = base;
            gd.n_slots = (int)std::min<size_t>(cap, heads.size() - h0);
            gd.slots_pad = (gd.n_slots + 15) / 16 * 16;
            for (int s = 0; s < gd.n_slots; ++s) {
                const int j = heads[h0 + s], g = j / gq;
                gd.q_head[s] = (short)j;
                gd.k_col[s] = (short)head_column(ctx, bh.src_k, KVCAR_K, g);
                gd.v_col[s] = (short)head_column(ctx, bh.src_v, KVCAR_V, g);
            }
            // runs of equal KV head on either side
            auto runs = [&](const short* col, short& n, short* lo, short* hi, short* c0) {
                int cnt = 0;
                for (int sl = 0; sl < gd.n_slots; ++sl) {
                    if (sl == 0 || col[sl] != col[sl - 1]) {
                        if (cnt < kMaxSeg) { lo[cnt] = (short)sl; c0[cnt] = col[sl]; }
                        ++cnt;
                    }
                    if (cnt <= kMaxSeg) hi[cnt - 1] = (short)(sl + 1);
                }
                n = (short)(cnt <= kMaxSeg ? cnt : 0);
            };
            runs(gd.k_col, gd.n_kseg, gd.kseg_lo, gd.kseg_hi, gd.kseg_col);
            runs(gd.v_col, gd.n_vseg, gd.vseg_lo, gd.vseg_hi, gd.vseg_col);
            plan.groups.push_back(gd);
            plan.src.push_back({bh.src_k, bh.src_v});
        }
    }
    plan.mfma = mfma_ok;
    plan.mlp = mlp_ok;
    plan.i8 = mfma_ok && !mlp_ok && ctx->int8();       // linear decoders over int8 rows; the two-layer kernel dequantises while parking
    int qt = 0, part = 0;
    for (auto& gd : plan.groups) {
        gd.qt_off = qt; gd.part_off = part;
        qt += gd.slots_pad * gd.k.c;
        part += gd.slots_pad * (gd.v.c + 4);
    }
    plan.qt_stride = qt;
    plan.part_stride = part;

    // whether the absorbed queries (prologue) and the output epilogue (fused) can run inside the matrix-core kernel:
    // decided over the groups, before the number of splits, which depends on it
    plan.fused = false;
    plan.prologue = false;
    plan.arrive = false;
    const bool one_launch_family = plan.mfma && !plan.mlp && !ctx->tun.no_fuse && r_all <= 128 && c.d_head % 32 == 0 && c.d_head <= 128;
    if (one_launch_family) {
        plan.fused = true;                                  // whether the epilogue can run inside
        plan.prologue = true;                               // the query side alone: also with several splits
        for (auto& gd : plan.groups) {
            if (gd.k.r != gd.v.r || gd.k.r % 32 || gd.k.r < 32 || gd.slots_pad > 32 || gd.n_kseg == 0) plan.fused = plan.prologue = false;
            if (gd.n_vseg == 0) plan.fused = false;
            int segs = 0;                                   // KV heads of the group: at most four decoder slices
            for (int sl = 0; sl < gd.n_slots; ++sl)
                if (sl == 0 || gd.v_col[sl] != gd.v_col[sl - 1]) ++segs;
            if (segs > 4 || gd.v.r * (c.d_head / 8) > 4 * 256) plan.fused = false;   // ... of at most 1024 16-byte chunks
            for (int b0 = 0; b0 < gd.n_slots; b0 += 16) {   // a 16-head block may span at most two KV heads (K side)
                int kinds = 0;
                for (int sl = b0; sl < std::min(gd.n_slots, b0 + 16); ++sl) {
                    bool seen = false;
                    for (int t = b0; t < sl; ++t) seen |= gd.k_col[t] == gd.k_col[sl];
                    if (!seen) ++kinds;
                }
                if (kinds > 2) plan.fused = plan.prologue = false;
            }
        }
    }
    const bool arrive_ok = plan.fused && plan.prologue && !ctx->tun.no_arrive;      // several splits can finish in the same launch

    // token-range splits: enough workgroups to fill the chip, never less than one tile per split
    const int n_groups = (int)plan.groups.size();
    const int tile = plan.mlp ? 32 : plan.mfma ? 128 : kGenericTile;   // tokens per workgroup iteration
    const int wg_tiles = std::max(1, (n_ctx + tile - 1) / tile);
    int splits = ctx->tun.n_splits;
    if (splits <= 0) {
        const int units = batch * n_groups;
        if (arrive_ok) {
            // The one-launch forms.  More than half a chip of (sequence, group) pairs: one long-lived workgroup each (a second
            // split costs the whole arrival tail: 36 to 63 sequences of four groups, 0.62-0.72 ms per step against 0.70-0.82).
            // Fewer: splits fill the chip, never with more workgroups than are resident at once (512: beyond, launches take
            // half as long again), and a split keeps about four workgroup tiles: with less the loop is shorter than the merge
            // of one more partial (TinyLlama at 2048 tokens, 4 sequences: 16 splits 0.49 ms per step, 5 splits 0.41; 32
            // sequences: 2 splits 0.61, 4 splits 0.58).  One workgroup per compute unit or two: whichever the measured costs
            // favour - a four-wave workgroup alone on its compute unit streams a 128-token tile in about 1.4 us, one of two
            // in about 2.2 us, and the last workgroup spends about 0.17 us per partial it merges (one sequence of 131072
            // tokens: 64 splits 48 us per launch, 128 splits 55).  Where the launch is small enough to be bound by latency
            // (the same limit as for the finer groups; measured: 270 MB yes, 335 MB no), a workgroup alone on its compute
            // unit runs with eight waves and takes about 1.1 us per 128 tokens: then half as many splits as two four-wave
            // workgroups per compute unit would take win by 3-9 % (32 sequences of 2048 tokens: 2 splits 26.0 us, 4 splits
            // of four waves 26.9; 4 of 32768: 35.9 against 39.4; 4 of 131072, 335 MB: 97 against 90).
            const int by_tiles = (wg_tiles + 3) / 4;
            const int one = std::max(1, std::min({ctx->n_cu / units, by_tiles, kArriveMaxSplits}));
            const int two = std::max(1, std::min({2 * ctx->n_cu / units, by_tiles, kArriveMaxSplits}));
            size_t launch_bytes = 0;
            for (const GroupDesc& gd : plan.groups) launch_bytes += (size_t)(gd.k.r + gd.v.r) * ctx->row_elem_bytes() * batch * n_ctx;
            const bool one_w8 = eight_waves_fit(ctx, plan, batch, n_groups, n_ctx, one) && launch_bytes <= kFineGroupBytes;
            auto cost_us = [&](int n, double tile_us) { return (wg_tiles + n - 1) / n * tile_us + 0.17 * n; };
            if (2 * units > ctx->n_cu) splits = 1;
            else splits = cost_us(two, 2.2) < cost_us(one, one_w8 ? 1.1 : 1.4) ? two : one;
        } else {
            // separate kernels: about one workgroup per compute unit for the matrix-core kernels, two for the plain ones
            splits = plan.mfma ? std::max(1, ctx->n_cu / units) : (ctx->n_cu * 2 + units - 1) / units;
        }
    }
    splits = std::max(1, std::min(splits, std::min(wg_tiles, 256)));
    plan.n_splits = splits;
    // with several splits the same prologue and epilogue run in the one-launch form whose last workgroup merges
    plan.arrive = arrive_ok && splits > 1 && splits <= kArriveMaxSplits;
    plan.arrive_w8 = plan.arrive && eight_waves_fit(ctx, plan, batch, n_groups, n_ctx, splits);
    plan.fused = plan.fused && splits == 1;
    plan.qt_bytes = align_up((size_t)batch * qt * (plan.mfma && !plan.i8 ? 2 : 4), 256);
    plan.part_bytes = align_up((size_t)batch * splits * part * sizeof(float), 256);
    // one-launch split form: an 8-byte arrival counter per (sequence, group) after the partials
    plan.arrive_bytes = plan.arrive ? (size_t)batch * plan.groups.size() * kArrivePitch * sizeof(unsigned long long) : 0;
    plan.total_bytes = plan.qt_bytes + plan.part_bytes + plan.arrive_bytes;
    return KVCAR_OK;
}

int check_layer(const kvcar_ctx* ctx, int layer) {
    if (!ctx) return KVCAR_ERR_ARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, KVCAR_ERR_ARG, "layer %d out of range", layer);
    return KVCAR_OK;
}

}  // namespace

extern "C" {

int kvcar_create(const kvcar_config* cfg, kvcar_ctx** out) try {
    if (!cfg || !out) return KVCAR_ERR_ARG;
    *out = nullptr;
    if (cfg->n_layers <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->d_head <= 0 || cfg->max_batch <= 0 ||
        cfg->max_seq <= 0 || cfg->n_q_heads % cfg->n_kv_heads != 0)
        return KVCAR_ERR_SHAPE;
    if (cfg->n_kv_heads > kMaxKvHeads) return KVCAR_ERR_UNSUPPORTED;
    // query-head indices and decoder column offsets travel to the kernels as 16-bit numbers
    if (cfg->n_q_heads > 32767 || (long long)cfg->n_kv_heads * cfg->d_head > 32767) return KVCAR_ERR_UNSUPPORTED;
    if (cfg->dtype != KVCAR_F32 && cfg->dtype != KVCAR_F16 && cfg->dtype != KVCAR_BF16) return KVCAR_ERR_UNSUPPORTED;
    if (cfg->latent_format != KVCAR_LATENT_DTYPE && cfg->latent_format != KVCAR_LATENT_INT8) return KVCAR_ERR_UNSUPPORTED;
    std::unique_ptr<kvcar_ctx> ctx(new (std::nothrow) kvcar_ctx());
    if (!ctx) return KVCAR_ERR_NOMEM;
    ctx->cfg = *cfg;
    ctx->scale = cfg->softmax_scale != 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->d_head);
    ctx->reuse.assign((size_t)cfg->n_layers * 2 * cfg->n_kv_heads, 0);
    ctx->ae.assign((size_t)cfg->n_layers * 2, AEState());
    ctx->cache.assign((size_t)cfg->n_layers * 2, nullptr);
    ctx->cache_bytes.assign((size_t)cfg->n_layers * 2, 0);
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->n_cu = prop.multiProcessorCount;
    else
        (void)hipGetLastError();   // no device here: host-side calls still work
    void* sp = nullptr;            // the static scratch buffer's address on this device, so that the first
    if (scratch_of_current_device(&sp) != hipSuccess) (void)hipGetLastError();   // ..._static call need not look it up
    *out = ctx.release();
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_destroy(kvcar_ctx* ctx) try {
    if (ctx)
        for (auto& e : ctx->ev_pool) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    delete ctx;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_set_reuse_map(kvcar_ctx* ctx, int layer, const uint8_t* k_reuse, const uint8_t* v_reuse) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!k_reuse || !v_reuse) return fail(ctx, KVCAR_ERR_ARG, "null reuse mask");
    const int h = ctx->cfg.n_kv_heads;
    if (layer == 0)
        for (int g = 0; g < h; ++g)
            if (k_reuse[g] || v_reuse[g]) return fail(ctx, KVCAR_ERR_REUSE, "layer 0 has no previous layer to reuse");
    bool changed = false;
    for (int g = 0; g < h; ++g) {
        const uint8_t kb = k_reuse[g] ? 1 : 0, vb = v_reuse[g] ? 1 : 0;
        changed |= ctx->reuse_at(layer, KVCAR_K, g) != kb || ctx->reuse_at(layer, KVCAR_V, g) != vb;
        ctx->reuse_at(layer, KVCAR_K, g) = kb;
        ctx->reuse_at(layer, KVCAR_V, g) = vb;
    }
    if (changed) {   // the stored head set changed: autoencoders of this layer must be set again
        ctx->ae_at(layer, KVCAR_K) = AEState();
        ctx->ae_at(layer, KVCAR_V) = AEState();
    }
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_resolve_source(const kvcar_ctx* ctx, int layer, int which, int kv_head, int* src_layer) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!src_layer || (which != KVCAR_K && which != KVCAR_V) || kv_head < 0 || kv_head >= ctx->cfg.n_kv_heads)
        return fail(ctx, KVCAR_ERR_ARG, "bad argument to kvcar_resolve_source");
    *src_layer = resolve(ctx, layer, which, kv_head);
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_set_autoencoder(kvcar_ctx* ctx, int layer, int which, const kvcar_ae_desc* d) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!d || (which != KVCAR_K && which != KVCAR_V)) return fail(ctx, KVCAR_ERR_ARG, "bad argument to kvcar_set_autoencoder");
    const kvcar_config& c = ctx->cfg;
    std::vector<int> stored;
    for (int g = 0; g < c.n_kv_heads; ++g)
        if (!ctx->reuse_at(layer, which, g)) stored.push_back(g);
    AEState st;
    st.d = *d;
    if (d->in_width == c.n_kv_heads * c.d_head) {
        for (int g = 0; g < c.n_kv_heads; ++g) st.heads.push_back(g);
    } else if (d->in_width == (int)stored.size() * c.d_head) {
        st.heads = stored;
    } else {
        return fail(ctx, KVCAR_ERR_SHAPE, "in_width %d is neither D_kv=%d nor stored_heads*d_head=%d", d->in_width,
                    c.n_kv_heads * c.d_head, (int)stored.size() * c.d_head);
    }
    if (d->in_width == 0) {
        if (d->latent_width != 0) return fail(ctx, KVCAR_ERR_SHAPE, "latent_width must be 0 when in_width is 0");
        st.d.per_head = 0;
    } else {
        if (d->latent_width <= 0 || d->hidden_width < 0) return fail(ctx, KVCAR_ERR_SHAPE, "non-positive widths");
        if ((d->hidden_width > 0) != (d->act != KVCAR_ACT_NONE))
            return fail(ctx, KVCAR_ERR_SHAPE, "activation requires hidden_width > 0 and vice versa");
        if (d->act != KVCAR_ACT_NONE && d->act != KVCAR_ACT_LEAKY_RELU && d->act != KVCAR_ACT_GELU)
            return fail(ctx, KVCAR_ERR_UNSUPPORTED, "unknown activation %d", d->act);
        if (d->latent_width > kMaxRow || d->hidden_width > kMaxRow)
            return fail(ctx, KVCAR_ERR_UNSUPPORTED, "widths above %d are not supported", kMaxRow);
        if ((size_t)d->latent_width * ctx->row_elem_bytes() % 16 != 0)
            return fail(ctx, KVCAR_ERR_UNSUPPORTED, "latent rows must be a multiple of 16 bytes");
        if (d->per_head != 0 && d->per_head != 1) return fail(ctx, KVCAR_ERR_ARG, "per_head must be 0 or 1");
        if (d->per_head) {
            const int n = (int)st.heads.size();
            if (d->hidden_width > 0 || ctx->int8())
                return fail(ctx, KVCAR_ERR_UNSUPPORTED, "per-head autoencoders are linear and keep latent rows in the model dtype");
            if (d->latent_width % n != 0) return fail(ctx, KVCAR_ERR_SHAPE, "latent_width %d is not a multiple of the %d covered heads", d->latent_width, n);
            if ((size_t)(d->latent_width / n) * ctx->row_elem_bytes() % 16 != 0 || (size_t)c.d_head * dtype_size(c.dtype) % 16 != 0)
                return fail(ctx, KVCAR_ERR_UNSUPPORTED, "a head's latent rows and its decoder rows must be multiples of 16 bytes");
        }
        const void* req[4] = {d->enc_w1, d->dec_w1, d->hidden_width ? d->enc_w2 : d->enc_w1, d->hidden_width ? d->dec_w2 : d->dec_w1};
        for (const void* p : req)
            if (!p) return fail(ctx, KVCAR_ERR_ARG, "null weight pointer");
        const void* all[8] = {d->enc_w1, d->enc_b1, d->enc_w2, d->enc_b2, d->dec_w1, d->dec_b1, d->dec_w2, d->dec_b2};
        for (const void* p : all)
            if (p && !aligned16(p)) return fail(ctx, KVCAR_ERR_ARG, "weight pointer not 16-byte aligned");
    }
    st.set = true;
    // a new width invalidates a bound cache that is now too small
    const size_t need = ctx->cache_need(d->latent_width);
    const bool width_changed = ctx->ae_at(layer, which).set && ctx->ae_at(layer, which).d.latent_width != d->latent_width;
    if (ctx->cache_bytes[(size_t)layer * 2 + which] < need || (ctx->int8() && width_changed)) {   // int8: the metadata offset moved
        ctx->cache[(size_t)layer * 2 + which] = nullptr;
        ctx->cache_bytes[(size_t)layer * 2 + which] = 0;
    }
    ctx->ae_at(layer, which) = st;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_cache_bytes(const kvcar_ctx* ctx, int layer, int which, size_t* bytes) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!bytes || (which != KVCAR_K && which != KVCAR_V)) return fail(ctx, KVCAR_ERR_ARG, "bad argument to kvcar_cache_bytes");
    const AEState& a = ctx->ae_at(layer, which);
    if (!a.set) return fail(ctx, KVCAR_ERR_STATE, "autoencoder of layer %d not set", layer);
    *bytes = ctx->cache_need(a.d.latent_width);
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_bind_cache(kvcar_ctx* ctx, int layer, int which, void* dev, size_t bytes) try {
    size_t need = 0;
    int rc = kvcar_cache_bytes(ctx, layer, which, &need);
    if (rc) return rc;
    if (need == 0) { ctx->cache[(size_t)layer * 2 + which] = nullptr; ctx->cache_bytes[(size_t)layer * 2 + which] = 0; return KVCAR_OK; }
    if (!dev || !aligned16(dev)) return fail(ctx, KVCAR_ERR_ARG, "cache pointer null or not 16-byte aligned");
    if (bytes < need) return fail(ctx, KVCAR_ERR_CAPACITY, "cache of %zu bytes is smaller than the %zu needed", bytes, need);
    ctx->cache[(size_t)layer * 2 + which] = dev;
    ctx->cache_bytes[(size_t)layer * 2 + which] = bytes;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_set_tuning(kvcar_ctx* ctx, const kvcar_tuning* t) try {
    if (!ctx || !t) return KVCAR_ERR_ARG;
    if (t->n_splits < 0 || t->tile_order < 0 || t->tile_order > 2 || (t->wg_waves != 0 && t->wg_waves != 4 && t->wg_waves != 8) || (t->group_slots != 0 && t->group_slots != 8 && t->group_slots != 16 && t->group_slots != 32))
        return fail(ctx, KVCAR_ERR_ARG, "bad tuning value");
    ctx->tun = *t;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_workspace_bytes(const kvcar_ctx* ctx, int batch, int n_ctx, size_t* bytes) try {
    if (!ctx || !bytes) return KVCAR_ERR_ARG;
    if (batch < 1 || batch > ctx->cfg.max_batch || n_ctx < 1 || n_ctx > ctx->cfg.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "batch %d / n_ctx %d outside [1,%d] / [1,%d]", batch, n_ctx, ctx->cfg.max_batch, ctx->cfg.max_seq);
    size_t mx = 0;
    for (int layer = 0; layer < ctx->cfg.n_layers; ++layer) {
        Plan plan;
        int rc = build_plan(ctx, layer, batch, n_ctx, plan);
        if (rc) return rc;
        mx = std::max(mx, plan.total_bytes);
    }
    *bytes = mx;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

}  // extern "C"

namespace {

// The encoder side of a call: shapes, weights and (when `bound`) the input and cache pointers.  `any` tells
// whether the layer stores anything.
// `piece`: with per-head autoencoders a call is one launch per covered head (the piece-th covered head of K beside the
// piece-th of V: each is a d_head -> r_h encoder of its own writing its own block of the cache); a side with a dense
// autoencoder belongs to piece 0.  `any` = the piece has something to encode.
int fill_encode_params(const kvcar_ctx* ctx, int layer, const void* k_new, const void* v_new, int batch, int pos0, const int32_t* positions,
                       int t_new, bool bound, EncodeParams& p, bool& any, int piece = 0) {
    const kvcar_config& c = ctx->cfg;
    p = EncodeParams{};
    p.batch = batch; p.t_new = t_new; p.pos0 = pos0; p.max_seq = c.max_seq; p.d_kv = c.n_kv_heads * c.d_head; p.d_head = c.d_head;
    p.positions = positions;
    const void* xs[2] = {k_new, v_new};
    any = false;
    for (int which = 0; which < 2; ++which) {
        const AEState& a = ctx->ae_at(layer, which);
        if (!a.set) return fail(ctx, KVCAR_ERR_STATE, "autoencoder of layer %d (%s) not set", layer, which ? "V" : "K");
        EncodeSide& s = p.s[which];
        s.x = xs[which];
        s.r = a.d.latent_width;
        if (s.r == 0) continue;
        s.z = ctx->cache[(size_t)layer * 2 + which];
        if (bound && !s.z) return fail(ctx, KVCAR_ERR_STATE, "cache of layer %d (%s) not bound", layer, which ? "V" : "K");
        if (a.d.per_head) {
            s.r = 0;
            if (piece >= (int)a.heads.size()) continue;
            const int rh = head_latent(a), dh = c.d_head;
            const size_t es = dtype_size(c.dtype);
            s.r = rh;
            if (s.z) s.z = static_cast<char*>(s.z) + (size_t)piece * head_block_bytes(ctx, a);
            s.meta = nullptr;
            s.w1 = static_cast<const char*>(a.d.enc_w1) + (size_t)piece * dh * rh * es;
            s.b1 = a.d.enc_b1 ? static_cast<const char*>(a.d.enc_b1) + (size_t)piece * rh * es : nullptr;
            s.w2 = nullptr; s.b2 = nullptr;
            s.in_width = dh; s.hidden = 0; s.act = KVCAR_ACT_NONE; s.slope = 0.f;
            s.n_heads = 1;
            s.heads[0] = (unsigned char)a.heads[piece];
            any = true;
            continue;
        }
        if (piece > 0) { s.r = 0; continue; }
        s.meta = ctx->int8() && s.z ? static_cast<char*>(s.z) + ctx->meta_offset(s.r) : nullptr;
        s.w1 = a.d.enc_w1; s.b1 = a.d.enc_b1; s.w2 = a.d.enc_w2; s.b2 = a.d.enc_b2;
        s.in_width = a.d.in_width; s.hidden = a.d.hidden_width; s.act = a.d.act; s.slope = a.d.leaky_slope;
        s.n_heads = (int)a.heads.size();
        for (size_t i = 0; i < a.heads.size(); ++i) s.heads[i] = (unsigned char)a.heads[i];
        any = true;
    }
    return KVCAR_OK;
}

// Launches an encode call of `layer` takes: one, or with per-head autoencoders one per covered head.
int encode_pieces(const kvcar_ctx* ctx, int layer) {
    int n = 1;
    for (int which = 0; which < 2; ++which) {
        const AEState& a = ctx->ae_at(layer, which);
        if (a.set && a.d.per_head) n = std::max(n, (int)a.heads.size());
    }
    return n;
}

// Which encoder kernel a call takes (the KVCAR_ENC_* values).
int encode_kernel_kind(const kvcar_ctx* ctx, const EncodeParams& p) {
    const int dtype = ctx->cfg.dtype;
    if (ctx->tun.force_generic) return KVCAR_ENC_PLAIN;
    if (encode_mlp_mfma_supported(p, dtype)) return KVCAR_ENC_MFMA_TWO_LAYER;
    if (!ctx->tun.no_bulk_encode && encode_bulk_supported(p, dtype)) return KVCAR_ENC_MFMA_STREAM;
    if (encode_mfma_supported(p, dtype)) return KVCAR_ENC_MFMA;
    return KVCAR_ENC_PLAIN;
}

int encode_impl(kvcar_ctx* ctx, int layer, const void* k_new, const void* v_new, int batch, int pos0, const int32_t* positions, int t_new,
                void* stream) {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    const kvcar_config& c = ctx->cfg;
    if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return fail(ctx, KVCAR_ERR_ARG, "k_new / v_new null or misaligned");
    if (batch < 1 || t_new < 1 || pos0 < 0) return fail(ctx, KVCAR_ERR_ARG, "batch, t_new must be >= 1 and pos0 >= 0");
    if (batch > c.max_batch || (long long)pos0 + t_new > c.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "append of %d tokens at %d for batch %d exceeds max_seq %d / max_batch %d", t_new, pos0, batch, c.max_seq, c.max_batch);
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int piece = 0; piece < encode_pieces(ctx, layer); ++piece) {
        EncodeParams p;
        bool any = false;
        rc = fill_encode_params(ctx, layer, k_new, v_new, batch, pos0, positions, t_new, true, p, any, piece);
        if (rc) return rc;
        if (!any) continue;          // nothing stored on either side
        hipError_t e;
        switch (encode_kernel_kind(ctx, p)) {
            case KVCAR_ENC_MFMA_TWO_LAYER: e = launch_encode_mlp_mfma(p, c.dtype, st); break;
            case KVCAR_ENC_MFMA_STREAM: e = launch_encode_bulk(p, c.dtype, ctx->n_cu, st); break;
            case KVCAR_ENC_MFMA: e = launch_encode_mfma(p, c.dtype, st); break;
            default: e = launch_encode_generic(p, c.dtype, st); break;
        }
        if (e != hipSuccess) return fail(ctx, KVCAR_ERR_HIP, "encode launch failed: %s", hipGetErrorString(e));
    }
    return KVCAR_OK;
}

// `library_scratch`: the workspace is the library's static buffer (sized by the caller of this function, not by the
// user) and the call must not create anything: no timing events.
// The new token of an append-and-attend call.
// The encoder launch of an append-and-attend call whose attention has a projection launch of its own: decode_impl
// enqueues it, together with that projection where both have their matrix-core forms.
struct StepEncoder {
    const EncodeParams* p;
    bool two_layer;       // the few-token form of the two-layer encoder, else the decode-step form of the linear one
};

struct NewToken {
    const void* k_new;
    const void* v_new;
};

// Whether the attention launch planned for (layer, batch, n_ctx) can encode the new token itself: a matrix-core form with
// its prologue inside (single split, or the one-launch split form; rows in the model dtype or int8 codes), linear encoders
// of the sizes the in-kernel encoder handles, contiguous token ranges per split.
bool can_append_in_kernel(const kvcar_ctx* ctx, int layer, const Plan& plan) {
    if (!(plan.fused || plan.arrive) || plan.mlp || (ctx->int8() && !plan.i8) || ctx->tun.tile_order == 2) return false;
    if (ctx->cfg.n_kv_heads > kAppendMaxHeads) return false;
    for (int which = 0; which < 2; ++which) {
        const AEState& a = ctx->ae_at(layer, which);
        if (!a.set) return false;
        if (a.d.latent_width == 0) continue;
        const int in_w = a.d.per_head ? ctx->cfg.d_head : a.d.in_width, lat = a.d.per_head ? head_latent(a) : a.d.latent_width;
        if (a.d.hidden_width != 0 || in_w > 256 || in_w % 16 || lat > 128) return false;
        if (ctx->cache[(size_t)layer * 2 + which] == nullptr) return false;
        // the row is written by a workgroup that reads it: a layer-tensor that stores rows none of the layer's own heads
        // take (a full-width autoencoder in a layer whose heads are all reused) keeps the separate encoder launch
        bool read_here = false;
        for (const auto& src : plan.src) read_here |= src[which] == layer;
        if (!read_here) return false;
        // per-head autoencoders: every covered head's block needs its writer
        if (a.d.per_head)
            for (int g : a.heads)
                if (ctx->reuse_at(layer, which, g)) return false;
    }
    return true;
}

int decode_impl(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int n_ctx, const kvcar_step_ext* ext, void* workspace,
                size_t workspace_bytes, void* stream, bool library_scratch = false, const NewToken* fresh = nullptr,
                const StepEncoder* with_encode = nullptr) {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    const kvcar_config& c = ctx->cfg;
    if (!q || !out || !aligned16(q) || !aligned16(out)) return fail(ctx, KVCAR_ERR_ARG, "q / out null or misaligned");
    const bool exact = ext && (ext->k_cur || ext->v_cur);
    if (exact && (!ext->k_cur || !ext->v_cur || !aligned16(ext->k_cur) || !aligned16(ext->v_cur)))
        return fail(ctx, KVCAR_ERR_ARG, "k_cur and v_cur must both be given, 16-byte aligned");
    if (ext && ext->seq_lens && (reinterpret_cast<uintptr_t>(ext->seq_lens) & 3u)) return fail(ctx, KVCAR_ERR_ARG, "seq_lens misaligned");
    if (batch < 1 || batch > c.max_batch || n_ctx < (exact ? 0 : 1) || n_ctx > c.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "batch %d / n_ctx %d outside [1,%d] / [%d,%d]", batch, n_ctx, c.max_batch, exact ? 0 : 1, c.max_seq);
    Plan plan;
    rc = build_plan(ctx, layer, batch, std::max(1, n_ctx), plan);
    if (rc) return rc;
    if (!workspace || !aligned16(workspace)) return fail(ctx, KVCAR_ERR_ARG, "workspace null or misaligned");
    if (workspace_bytes < plan.total_bytes)
        return library_scratch
                   ? fail(ctx, KVCAR_ERR_WORKSPACE, "this call needs %zu bytes of scratch memory, more than the %zu of the library's static buffer: "
                          "use kvcar_decode_attention with a workspace", plan.total_bytes, workspace_bytes)
                   : fail(ctx, KVCAR_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, plan.total_bytes);

    if (fresh && !can_append_in_kernel(ctx, layer, plan)) return fail(ctx, KVCAR_ERR_STATE, "internal: this plan cannot encode in the attention kernel");
    unsigned long long writer_given[2] = {0ull, 0ull};    // per side: the heads' blocks (bit 0: the dense row) that have their writer
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (size_t g0 = 0; g0 < plan.groups.size(); g0 += kMaxGroups) {
        AttendParams p{};
        p.n_groups = (int)std::min<size_t>(kMaxGroups, plan.groups.size() - g0);
        for (int i = 0; i < p.n_groups; ++i) p.g[i] = plan.groups[g0 + i];
        p.q = q; p.out = out;
        p.qt = workspace;
        p.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.qt_bytes);
        p.batch = batch; p.n_ctx = n_ctx; p.n_splits = plan.n_splits;
        p.n_q_heads = c.n_q_heads; p.d_head = c.d_head; p.max_seq = c.max_seq;
        p.qt_stride = plan.qt_stride; p.part_stride = plan.part_stride;
        p.scale_log2e = ctx->scale * kLog2e;
        p.gq = c.n_q_heads / c.n_kv_heads;
        p.seq_lens = ext ? ext->seq_lens : nullptr;
        p.k_cur = exact ? ext->k_cur : nullptr;
        p.v_cur = exact ? ext->v_cur : nullptr;
        p.tile_order = ctx->tun.tile_order == 2 ? 1 : 0;
        // groups that stream the same rows: keep the groups of a (split, sequence) on one XCD - where the launch is small
        // enough for an L2 to hold what they share for as long as it takes them to get there; large launches are faster in
        // launch order (long context, independent key and value maps: 463 us against 538 per launch)
        size_t launch_bytes = 0;
        for (int i = 0; i < p.n_groups; ++i) launch_bytes += (size_t)(p.g[i].k.r + p.g[i].v.r) * ctx->row_elem_bytes() * batch * std::max(1, n_ctx);
        const bool may_colocate = !ctx->tun.no_colocate && launch_bytes <= kFineGroupBytes;
        for (int i = 0; i < p.n_groups && may_colocate && !p.colocate; ++i)
            for (int k = 0; k < i; ++k)
                if (p.g[i].k.z == p.g[k].k.z || p.g[i].v.z == p.g[k].v.z) p.colocate = 1;
        if (fresh) {
            p.append = 1;
            const void* xs[2] = {fresh->k_new, fresh->v_new};
            for (int which = 0; which < 2; ++which) {
                const AEState& a = ctx->ae_at(layer, which);
                AppendSide& e = p.enc[which];
                e.x = xs[which];
                e.z = ctx->cache[(size_t)layer * 2 + which];
                e.meta = ctx->int8() && e.z ? static_cast<char*>(e.z) + ctx->meta_offset(a.d.latent_width) : nullptr;
                e.w = a.d.enc_w1; e.b = a.d.enc_b1;
                e.in_width = a.d.in_width; e.r = a.d.latent_width;
                e.head_block = 0;
                if (a.d.per_head && e.r > 0) {       // every group encodes its own head: d_head -> r_h, into the head's block
                    e.in_width = c.d_head; e.r = head_latent(a);
                    e.head_block = (long long)head_block_bytes(ctx, a);
                }
                for (size_t i = 0; i < a.heads.size() && i < (size_t)kAppendMaxHeads; ++i) e.heads[i] = (unsigned char)a.heads[i];
                if (e.r == 0) continue;
                for (int i = 0; i < p.n_groups; ++i) {
                    if (plan.src[g0 + i][which] != layer) continue;  // rows of another layer
                    p.g[i].append |= (short)(1 << which);
                    // one group writes the row to the cache: per side, or per head's block
                    const int unit = a.d.per_head ? p.g[i].app_slice[which] : 0;
                    if (!(writer_given[which] >> unit & 1ull)) { p.g[i].append |= (short)(4 << which); writer_given[which] |= 1ull << unit; }
                }
            }
        }
        // fused: 1 = four waves per workgroup; 2 = eight, when the launch has no more workgroups than compute units
        const bool w8 = ctx->tun.wg_waves == 8 || (ctx->tun.wg_waves == 0 && batch * p.n_groups <= ctx->n_cu);
        if (plan.arrive) {
            p.arrive = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + plan.qt_bytes + plan.part_bytes) + g0 * kArrivePitch;
            p.arrive_stride = (int)plan.groups.size();
            p.epoch = next_epoch();
        }
        const bool one_launch = plan.fused || plan.arrive;
        // the one-launch split form likewise: 4 = four waves, 5 = eight
        p.fused = plan.fused ? (w8 ? 2 : 1) : plan.arrive ? (plan.arrive_w8 ? 5 : 4) : plan.prologue ? 3 : 0;
        const bool proj = plan.mfma && proj_mfma_supported(p, c.dtype);
        hipError_t e = hipSuccess;
        // append-and-attend (with_encode): the step's encoder launch and the projection of the absorbed queries are
        // independent: where both are the matrix-core forms they share one launch, else the encoder goes first
        const bool own_qtilde = !plan.fused && !plan.prologue;
        const bool together = with_encode && g0 == 0 && own_qtilde && proj && !plan.i8;
        if (with_encode && g0 == 0 && !together)
            e = with_encode->two_layer ? launch_encode_mlp_mfma(*with_encode->p, c.dtype, st) : launch_encode_mfma(*with_encode->p, c.dtype, st);
        if (e == hipSuccess && together) {
            int qx, qy, qz;
            qtilde_mfma_grid(p, qx, qy, qz);
            e = with_encode->two_layer ? launch_encode_mlp_step_qtilde(*with_encode->p, p, qx, qy, qz, c.dtype, st)
                                       : launch_encode_step_qtilde(*with_encode->p, p, qx, qy, qz, c.dtype, st);
        } else if (e == hipSuccess && own_qtilde) {
            e = proj && !plan.i8 ? launch_qtilde_mfma(p, c.dtype, st) : launch_qtilde(p, c.dtype, !plan.mfma || plan.i8, st);
        }
        std::pair<hipEvent_t, hipEvent_t>* ev = nullptr;
        if (e == hipSuccess && ctx->profiling && !library_scratch) {
            if (ctx->ev_used == ctx->ev_pool.size()) {
                hipEvent_t a, b2;
                e = hipEventCreate(&a);
                if (e == hipSuccess) e = hipEventCreate(&b2);
                if (e == hipSuccess) ctx->ev_pool.emplace_back(a, b2);
            }
            if (e == hipSuccess) { ev = &ctx->ev_pool[ctx->ev_used++]; e = hipEventRecord(ev->first, st); }
        }
        if (e == hipSuccess)
            e = plan.mlp ? launch_attend_mlp_mfma(p, c.dtype, st)
                         : plan.i8 ? launch_attend_i8_mfma(p, c.dtype, st)
                         : plan.mfma ? launch_attend_mfma(p, c.dtype, st) : launch_attend_generic(p, c.dtype, st);
        if (e == hipSuccess && ev) e = hipEventRecord(ev->second, st);
        if (e == hipSuccess && !one_launch) e = proj ? launch_combine_mfma(p, c.dtype, st) : launch_combine(p, c.dtype, st);
        if (e != hipSuccess) return fail(ctx, KVCAR_ERR_HIP, "attention launch failed: %s", hipGetErrorString(e));
    }
    return KVCAR_OK;
}

// Sources to decode for prefill attention of `layer`: one entry per (source layer, K or V), listing the KV heads that take it.
int build_recon(const kvcar_ctx* ctx, int layer, std::vector<ReconEntry>& entries) {
    const kvcar_config& c = ctx->cfg;
    entries.clear();
    for (int which = 0; which < 2; ++which) {
        std::map<std::pair<int, int>, std::vector<int>> by_src;     // (source, head where the source's autoencoder is per-head, else -1)
        for (int g = 0; g < c.n_kv_heads; ++g) {
            const int src = resolve(ctx, layer, which, g);
            by_src[{src, ctx->ae_at(src, which).d.per_head ? g : -1}].push_back(g);
        }
        for (auto& kvp : by_src) {
            const std::pair<const int, std::vector<int>> kv{kvp.first.first, kvp.second};
            SideDesc sd{};
            int rc = fill_side(ctx, layer, kv.first, which, kv.second.front(), sd);
            if (rc) return rc;
            if (sd.c > kMaxRow || sd.r > kMaxRow) return fail(ctx, KVCAR_ERR_UNSUPPORTED, "row width above %d", kMaxRow);
            for (size_t h0 = 0; h0 < kv.second.size(); h0 += kMaxReconHeads) {
                ReconEntry e{};
                e.d = sd;
                e.which = which;
                e.n_heads = (int)std::min<size_t>(kMaxReconHeads, kv.second.size() - h0);
                for (int i = 0; i < e.n_heads; ++i) {
                    const int g = kv.second[h0 + i];
                    const int col = head_column(ctx, kv.first, which, g);
                    if (col < 0) return fail(ctx, KVCAR_ERR_REUSE, "layer %d takes head %d from a layer whose autoencoder does not cover it", layer, g);
                    e.head[i] = (short)g;
                    e.col[i] = (short)col;
                }
                entries.push_back(e);
            }
        }
    }
    return KVCAR_OK;
}

size_t prefill_need(const kvcar_ctx* ctx, int batch, int n_rows) {
    const kvcar_config& c = ctx->cfg;
    return 2 * align_up((size_t)batch * n_rows * c.n_kv_heads * c.d_head * dtype_size(c.dtype), 256);
}

int prefill_impl(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int pos0, int t_new, void* workspace, size_t workspace_bytes,
                 void* stream) {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    const kvcar_config& c = ctx->cfg;
    if (!q || !out || !aligned16(q) || !aligned16(out)) return fail(ctx, KVCAR_ERR_ARG, "q / out null or misaligned");
    if (batch < 1 || t_new < 1 || pos0 < 0) return fail(ctx, KVCAR_ERR_ARG, "batch, t_new must be >= 1 and pos0 >= 0");
    if (batch > c.max_batch || (long long)pos0 + t_new > c.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "chunk of %d tokens at %d for batch %d exceeds max_seq %d / max_batch %d", t_new, pos0, batch, c.max_seq, c.max_batch);
    if (c.d_head > 256) return fail(ctx, KVCAR_ERR_UNSUPPORTED, "prefill attention handles d_head up to 256");
    const int n_rows = pos0 + t_new;
    std::vector<ReconEntry> entries;
    rc = build_recon(ctx, layer, entries);
    if (rc) return rc;
    const size_t need = prefill_need(ctx, batch, n_rows);
    if (!workspace || !aligned16(workspace)) return fail(ctx, KVCAR_ERR_ARG, "workspace null or misaligned");
    if (workspace_bytes < need) return fail(ctx, KVCAR_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);

    hipStream_t st = static_cast<hipStream_t>(stream);
    void* khat = workspace;
    void* vhat = static_cast<char*>(workspace) + need / 2;
    hipError_t e = hipSuccess;
    for (size_t e0 = 0; e0 < entries.size() && e == hipSuccess; e0 += kMaxReconEntries) {
        ReconParams rp{};
        rp.n_entries = (int)std::min<size_t>(kMaxReconEntries, entries.size() - e0);
        for (int i = 0; i < rp.n_entries; ++i) rp.e[i] = entries[e0 + i];
        rp.khat = khat; rp.vhat = vhat;
        rp.batch = batch; rp.n_rows = n_rows; rp.max_seq = c.max_seq; rp.n_kv_heads = c.n_kv_heads; rp.d_head = c.d_head;
        rp.k_scale = ctx->scale * kLog2e;
        e = (!ctx->tun.force_generic && recon_mfma_supported(rp, c.dtype)) ? launch_recon_mfma(rp, c.dtype, st) : launch_recon_generic(rp, c.dtype, st);
    }
    PrefillParams pp{};
    pp.q = q; pp.out = out; pp.khat = khat; pp.vhat = vhat;
    pp.batch = batch; pp.t_new = t_new; pp.pos0 = pos0; pp.n_rows = n_rows;
    pp.n_q_heads = c.n_q_heads; pp.n_kv_heads = c.n_kv_heads; pp.d_head = c.d_head;
    std::pair<hipEvent_t, hipEvent_t>* ev = nullptr;
    if (e == hipSuccess && ctx->profiling) {
        if (ctx->ev_used == ctx->ev_pool.size()) {
            hipEvent_t a, b2;
            e = hipEventCreate(&a);
            if (e == hipSuccess) e = hipEventCreate(&b2);
            if (e == hipSuccess) ctx->ev_pool.emplace_back(a, b2);
        }
        if (e == hipSuccess) { ev = &ctx->ev_pool[ctx->ev_used++]; e = hipEventRecord(ev->first, st); }
    }
    if (e == hipSuccess)
        e = (!ctx->tun.force_generic && prefill_mfma_supported(pp, c.dtype)) ? launch_prefill_mfma(pp, c.dtype, ctx->n_cu, st)
                                                                              : launch_prefill_generic(pp, c.dtype, st);
    if (e == hipSuccess && ev) e = hipEventRecord(ev->second, st);
    if (e != hipSuccess) return fail(ctx, KVCAR_ERR_HIP, "prefill launch failed: %s", hipGetErrorString(e));
    return KVCAR_OK;
}

}  // namespace

extern "C" {

int kvcar_encode_append(kvcar_ctx* ctx, int layer, const void* k_new, const void* v_new, int batch, int pos0, int t_new, void* stream) try {
    return encode_impl(ctx, layer, k_new, v_new, batch, pos0, nullptr, t_new, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_encode_append_at(kvcar_ctx* ctx, int layer, const void* k_new, const void* v_new, int batch, const int32_t* positions, int t_new,
                           void* stream) try {
    if (!ctx) return KVCAR_ERR_ARG;
    if (!positions || (reinterpret_cast<uintptr_t>(positions) & 3u)) return fail(ctx, KVCAR_ERR_ARG, "positions null or misaligned");
    return encode_impl(ctx, layer, k_new, v_new, batch, 0, positions, t_new, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_decode_attention(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int n_ctx, void* workspace,
                           size_t workspace_bytes, void* stream) try {
    return decode_impl(ctx, layer, q, out, batch, n_ctx, nullptr, workspace, workspace_bytes, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_decode_attention_ex(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int n_ctx, const kvcar_step_ext* ext,
                              void* workspace, size_t workspace_bytes, void* stream) try {
    return decode_impl(ctx, layer, q, out, batch, n_ctx, ext, workspace, workspace_bytes, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_decode_attention_static(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int n_ctx, void* stream) try {
    if (!ctx) return KVCAR_ERR_ARG;
    void* sp = nullptr;
    const hipError_t e = scratch_of_current_device(&sp);
    if (e != hipSuccess) return fail(ctx, KVCAR_ERR_HIP, "the static scratch buffer's device address is not available: %s", hipGetErrorString(e));
    return decode_impl(ctx, layer, q, out, batch, n_ctx, nullptr, sp, KVCAR_STATIC_SCRATCH_BYTES, stream, true);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_append_attend(kvcar_ctx* ctx, int layer, const void* k_new, const void* v_new, const void* q, void* out, int batch, int pos,
                        void* workspace, size_t workspace_bytes, void* stream) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    const kvcar_config& c = ctx->cfg;
    if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return fail(ctx, KVCAR_ERR_ARG, "k_new / v_new null or misaligned");
    if (batch < 1 || pos < 0) return fail(ctx, KVCAR_ERR_ARG, "batch must be >= 1 and pos >= 0");
    if (batch > c.max_batch || (long long)pos + 1 > c.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "append at %d for batch %d exceeds max_seq %d / max_batch %d", pos, batch, c.max_seq, c.max_batch);
    Plan plan;
    rc = build_plan(ctx, layer, batch, pos + 1, plan);
    if (rc) return rc;
    if (can_append_in_kernel(ctx, layer, plan)) {
        // every stored side of the layer must be read by the layer itself (its own heads are), or nobody would write the row
        const NewToken fresh{k_new, v_new};
        return decode_impl(ctx, layer, q, out, batch, pos + 1, nullptr, workspace, workspace_bytes, stream, false, &fresh);
    }
    // two launches: what the second would refuse is refused before the first appends anything
    if (!q || !out || !aligned16(q) || !aligned16(out)) return fail(ctx, KVCAR_ERR_ARG, "q / out null or misaligned");
    if (!workspace || !aligned16(workspace)) return fail(ctx, KVCAR_ERR_ARG, "workspace null or misaligned");
    if (workspace_bytes < plan.total_bytes) return fail(ctx, KVCAR_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, plan.total_bytes);
    // where the attention needs a projection launch of its own for the absorbed queries and the encoder is the decode-step
    // form of the linear matrix-core encoder, the two share a launch; decode_impl reports whether it took the encoder in
    if (plan.mfma && !plan.i8 && !plan.fused && !plan.prologue && encode_pieces(ctx, layer) == 1 && !ctx->int8()) {
        EncodeParams ep;
        bool any = false;
        rc = fill_encode_params(ctx, layer, k_new, v_new, batch, pos, nullptr, 1, true, ep, any);
        if (rc) return rc;
        const int kind = any ? encode_kernel_kind(ctx, ep) : KVCAR_ENC_NONE;
        const bool linear = kind == KVCAR_ENC_MFMA && encode_step_qtilde_supported(ep, c.dtype);
        const bool two_layer = kind == KVCAR_ENC_MFMA_TWO_LAYER && encode_mlp_step_qtilde_supported(ep, c.dtype);
        if (linear || two_layer) {
            const StepEncoder enc{&ep, two_layer};
            return decode_impl(ctx, layer, q, out, batch, pos + 1, nullptr, workspace, workspace_bytes, stream, false, nullptr, &enc);
        }
    }
    rc = encode_impl(ctx, layer, k_new, v_new, batch, pos, nullptr, 1, stream);
    if (rc) return rc;
    return decode_impl(ctx, layer, q, out, batch, pos + 1, nullptr, workspace, workspace_bytes, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_prefill_workspace_bytes(const kvcar_ctx* ctx, int batch, int n_rows, size_t* bytes) try {
    if (!ctx || !bytes) return KVCAR_ERR_ARG;
    if (batch < 1 || batch > ctx->cfg.max_batch || n_rows < 1 || n_rows > ctx->cfg.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "batch %d / n_rows %d outside [1,%d] / [1,%d]", batch, n_rows, ctx->cfg.max_batch, ctx->cfg.max_seq);
    *bytes = prefill_need(ctx, batch, n_rows);
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_prefill_attention(kvcar_ctx* ctx, int layer, const void* q, void* out, int batch, int pos0, int t_new, void* workspace,
                            size_t workspace_bytes, void* stream) try {
    return prefill_impl(ctx, layer, q, out, batch, pos0, t_new, workspace, workspace_bytes, stream);
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_describe_plan(const kvcar_ctx* ctx, int layer, int batch, int n_ctx, kvcar_plan_info* out) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!out) return fail(ctx, KVCAR_ERR_ARG, "null output");
    if (batch < 1 || batch > ctx->cfg.max_batch || n_ctx < 1 || n_ctx > ctx->cfg.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "batch %d / n_ctx %d outside [1,%d] / [1,%d]", batch, n_ctx, ctx->cfg.max_batch, ctx->cfg.max_seq);
    Plan plan;
    rc = build_plan(ctx, layer, batch, n_ctx, plan);
    if (rc) return rc;
    out->uses_mfma = plan.mfma ? 1 : 0;
    out->n_groups = (int)plan.groups.size();
    out->n_splits = plan.n_splits;
    out->n_launches = (int)((plan.groups.size() + kMaxGroups - 1) / kMaxGroups);
    out->fused = plan.fused ? 1 : plan.arrive ? 2 : 0;
    out->workspace_bytes = plan.total_bytes;
    size_t lat = 0;
    for (auto& g : plan.groups) lat += (size_t)(g.k.r + g.v.r);
    out->latent_bytes = lat * ctx->row_elem_bytes() * batch * n_ctx;
    if (ctx->int8()) out->latent_bytes += plan.groups.size() * 2 * sizeof(RowMeta) * (size_t)batch * n_ctx;
    out->append_in_kernel = can_append_in_kernel(ctx, layer, plan) ? 1 : 0;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_describe_encode(const kvcar_ctx* ctx, int layer, int batch, int t_new, int* kernel) try {
    int rc = check_layer(ctx, layer);
    if (rc) return rc;
    if (!kernel) return fail(ctx, KVCAR_ERR_ARG, "null output");
    if (batch < 1 || t_new < 1) return fail(ctx, KVCAR_ERR_ARG, "batch, t_new must be >= 1");
    if (batch > ctx->cfg.max_batch || t_new > ctx->cfg.max_seq)
        return fail(ctx, KVCAR_ERR_CAPACITY, "batch %d / t_new %d exceed max_batch %d / max_seq %d", batch, t_new, ctx->cfg.max_batch, ctx->cfg.max_seq);
    EncodeParams p;
    bool any = false;
    rc = fill_encode_params(ctx, layer, nullptr, nullptr, batch, 0, nullptr, t_new, false, p, any);
    if (rc) return rc;
    *kernel = any ? encode_kernel_kind(ctx, p) : KVCAR_ENC_NONE;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_profile_enable(kvcar_ctx* ctx, int enable) try {
    if (!ctx) return KVCAR_ERR_ARG;
    ctx->profiling = enable != 0;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_profile_read(kvcar_ctx* ctx, double* attend_ms, long* n_launches) try {
    if (!ctx || !attend_ms || !n_launches) return KVCAR_ERR_ARG;
    double total = 0.0;
    for (size_t i = 0; i < ctx->ev_used; ++i) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ctx->ev_pool[i].second);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev_pool[i].first, ctx->ev_pool[i].second);
        if (e != hipSuccess) return fail(ctx, KVCAR_ERR_HIP, "event read failed: %s", hipGetErrorString(e));
        total += ms;
    }
    *attend_ms = total;
    *n_launches = (long)ctx->ev_used;
    ctx->ev_used = 0;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

static int device_cu_count() {
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    return n_cu;
}

int kvcar_head_l1_workspace_bytes(size_t n_tokens, int n_kv_heads, size_t* bytes) try {
    if (!bytes || n_tokens == 0 || n_kv_heads < 1) return KVCAR_ERR_ARG;
    *bytes = (size_t)kvcar::head_l1_workgroups(n_tokens, device_cu_count()) * n_kv_heads * sizeof(float);
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_head_l1_distance(const void* x_prev, const void* x_cur, int dtype, size_t n_tokens, int n_kv_heads, int d_head, int accumulate,
                           float* dist, void* workspace, size_t workspace_bytes, void* stream) try {
    if (!x_prev || !x_cur || !dist || !workspace || n_tokens == 0 || n_kv_heads < 1 || d_head < 1) return KVCAR_ERR_ARG;
    if (!aligned16(x_prev) || !aligned16(x_cur) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(dist) & 3u)) return KVCAR_ERR_ARG;
    if (dtype != KVCAR_F32 && dtype != KVCAR_F16 && dtype != KVCAR_BF16) return KVCAR_ERR_UNSUPPORTED;
    if (n_kv_heads > 1024) return KVCAR_ERR_UNSUPPORTED;
    const int el = dtype == KVCAR_F32 ? 4 : 8;                 // elements per 16-byte chunk
    if (d_head % el) return KVCAR_ERR_SHAPE;                   // a chunk must lie inside one head
    const int n_wg = kvcar::head_l1_workgroups(n_tokens, device_cu_count());
    if (workspace_bytes < (size_t)n_wg * n_kv_heads * sizeof(float)) return KVCAR_ERR_WORKSPACE;
    hipError_t e = kvcar::launch_head_l1(x_prev, x_cur, dtype, n_tokens, n_kv_heads, d_head, accumulate, dist, static_cast<float*>(workspace), n_wg,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KVCAR_OK : KVCAR_ERR_HIP;
} catch (...) { return KVCAR_ERR_NOMEM; }

int kvcar_probe_read_bandwidth(const void* dev_buf, size_t bytes, int repeats, void* stream, double* gb_per_s) try {
    if (!dev_buf || !gb_per_s || bytes < 16 || bytes % 16 || repeats < 1 || (reinterpret_cast<uintptr_t>(dev_buf) & 15)) return KVCAR_ERR_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return KVCAR_ERR_HIP;
    if (n_cu <= 0) n_cu = 256;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return KVCAR_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return KVCAR_ERR_HIP; }
    // the best of a few launch shapes (workgroups per compute unit x lanes per workgroup)
    static const int shapes[][2] = {{4, 256}, {8, 256}, {16, 256}, {32, 256}, {4, 512}, {8, 512}, {16, 512}};
    double best = 0.0;
    hipError_t e = hipSuccess;
    for (const auto& sh : shapes) {
        const int n_blocks = sh[0] * n_cu;
        e = kvcar::launch_stream_read(dev_buf, bytes, n_blocks, sh[1], nullptr, st);          // untimed first pass
        if (e == hipSuccess) e = hipEventRecord(e0, st);
        for (int i = 0; i < repeats && e == hipSuccess; ++i) e = kvcar::launch_stream_read(dev_buf, bytes, n_blocks, sh[1], nullptr, st);
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) break;
        if (ms > 0.f) best = std::max(best, (double)bytes * repeats / (ms * 1e-3) / 1e9);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess || best <= 0.0) return KVCAR_ERR_HIP;
    *gb_per_s = best;
    return KVCAR_OK;
} catch (...) { return KVCAR_ERR_NOMEM; }

const char* kvcar_status_string(int s) {
    switch (s) {
        case KVCAR_OK: return "KVCAR_OK";
        case KVCAR_ERR_ARG: return "KVCAR_ERR_ARG";
        case KVCAR_ERR_SHAPE: return "KVCAR_ERR_SHAPE";
        case KVCAR_ERR_CAPACITY: return "KVCAR_ERR_CAPACITY";
        case KVCAR_ERR_REUSE: return "KVCAR_ERR_REUSE";
        case KVCAR_ERR_UNSUPPORTED: return "KVCAR_ERR_UNSUPPORTED";
        case KVCAR_ERR_STATE: return "KVCAR_ERR_STATE";
        case KVCAR_ERR_HIP: return "KVCAR_ERR_HIP";
        case KVCAR_ERR_WORKSPACE: return "KVCAR_ERR_WORKSPACE";
        case KVCAR_ERR_NOMEM: return "KVCAR_ERR_NOMEM";
        default: return "KVCAR_ERR_UNKNOWN";
    }
}

const char* kvcar_last_error(const kvcar_ctx* ctx) { return ctx ? ctx->err.c_str() : ""; }

}  // extern "C"
