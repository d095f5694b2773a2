// MFMA attention over the latent cache for gfx950 (16-bit dtypes, linear decoders).
//
// One workgroup = 4 independent wavefronts serving ALL query heads of a group for one sequence and
// one token split: the autoencoder latent mixes heads, so every head needs the whole latent row and
// the row is read from HBM once for all of them.  Per 32-token tile a wave
//   1. streams the K and V latent rows with fully coalesced 128-bit loads (next tile prefetched in
//      registers), parks them in its private LDS region (padded rows, no bank conflicts),
//   2. S^T[token, head] = Z_K . Qt^T      v_mfma_f32_16x16x32 (A = latent rows from LDS, B = absorbed
//                                          queries resident in registers)
//   3. online softmax in base 2: the MFMA result layout gives a lane 8 tokens of ONE head, so the
//      max / sum reductions are in-lane plus two cross-lane steps
//   4. O^T[latent col, head] += Z_V^T . P^T  with P^T taken straight from the softmax registers
//      (the S^T result layout IS the B-operand layout) and Z_V^T read from LDS with the gfx950
//      transposing load ds_read_b64_tr_b16.
// No barrier is needed in the loop; the four waves merge their (m, l, O) once at the end and write
// one partial per (sequence, split, group).  Attention itself is Eq. 1 of the paper; the decoder is
// applied to the query before (prologue kernel) and to the weighted latent sum after (combine
// kernel), which equals decoding every cached row first ("Network Architecture", 2nd paragraph).
//
// The loop body is compiled once per exact shape (latent width R for both K and V, 16-head blocks)
// so that every LDS address is lane base + immediate and no width test survives in the loop; a
// workgroup picks its instance from its group's widths.  Other width mixes take an instance with
// run-time widths.
#pragma once

#include <type_traits>

#include "kvcar_device.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct Mma;
template <> struct Mma<BF16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        bf16x2_t v = {(__bf16)lo, (__bf16)hi};          // round to nearest even
        return __builtin_bit_cast(unsigned, v);
    }
    static __device__ __forceinline__ float unpack_lo(unsigned w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float unpack_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
    static __device__ __forceinline__ uint16_t to16(float v) { return f32_to_bf16_bits(v); }
};
template <> struct Mma<F16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
        f16x2_t v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(unsigned, v);
    }
    static __device__ __forceinline__ float unpack_lo(unsigned w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu)); }
    static __device__ __forceinline__ float unpack_hi(unsigned w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
    static __device__ __forceinline__ uint16_t to16(float v) { _Float16 h = (_Float16)v; return __builtin_bit_cast(uint16_t, h); }
};

// The (latent width, 16-head blocks) pairs the loop is compiled for with every size a constant.  The kernels' switches
// and the host's test of whether a launch may use them (exact_shape) are both generated from this one list, so a
// launch that passes the host's test always finds its instance.
#define KVCAR_EXACT_SHAPES(X) X(128, 2) X(128, 1) X(96, 2) X(96, 1) X(64, 2) X(64, 1) X(32, 2) X(32, 1)
inline bool exact_shape(int r, int nhb) {
#define X(R, N) if (r == R && nhb == N) return true;
    KVCAR_EXACT_SHAPES(X)
#undef X
    return false;
}

constexpr int kWaveTile = 32;     // tokens per wave per iteration
constexpr int kWaves = 4;

// One-launch split form, last workgroup: where in LDS the table of the splits' (m, l) pairs [split][slot] and the table
// of the splits' scaling factors [split][slot] live while the partials are merged - past the first kilobyte (the
// arrival flag, the per-slot weights), inside what every launch of these kernels is given (the staging regions of a
// 128-wide latent, 71680 bytes); the merged sums and the decoder slices overwrite them afterwards.
constexpr int kArriveMlTab = 1024;
constexpr int kArriveFTab = kArriveMlTab + kArriveMaxSplits * 32 * 8;
static_assert(kArriveFTab + kArriveMaxSplits * 32 * 4 <= 71680, "the merge tables must fit the staging regions");

#ifndef KVCAR_APPEND_IN_KERNEL
#define KVCAR_APPEND_IN_KERNEL 1
#endif

#ifndef KVCAR_NT_LOADS
#define KVCAR_NT_LOADS 1
#endif

__device__ __forceinline__ u32x4_t ld_global_16(const char* p) {
#if KVCAR_NT_LOADS
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
#else
    return *reinterpret_cast<const u32x4_t*>(p);
#endif
}

// Shapes of one loop instance.  Exact: everything is a compile-time constant.
template <int R, int NHB_> struct DimsExact {
    static constexpr int RMAX = R, NHB = NHB_;
    static constexpr bool kExact = true;
    static constexpr int rk = R, rv = R, nhb = NHB_;
    __device__ DimsExact(int, int, int) {}
};
template <int RMAX_, int NHB_> struct DimsAny {
    static constexpr int RMAX = RMAX_, NHB = NHB_;
    static constexpr bool kExact = false;
    int rk, rv, nhb;
    __device__ DimsAny(int rk_, int rv_, int nhb_) : rk(rk_), rv(rv_), nhb(nhb_) {}
};

template <int RMAX> struct Geo {
    static constexpr bool kPrefetch = RMAX <= 128;            // next tile's K and V rows held in registers
    static constexpr int kRegionK = kWaveTile * (2 * RMAX + 16);
    static constexpr int kRegionV = kWaveTile * (2 * RMAX + 32);
    static constexpr int kWaveLds = kPrefetch ? kRegionK + kRegionV : kRegionV;   // wide rows: K, V take turns
};

// This lane's share of a [kWaveTile x r] tile whose rows are contiguous in memory: 16-byte chunk
// f = i*64 + lane.  Full tiles need no test; on the ragged last tile chunks of rows >= n_valid read 0.
template <int NL>
__device__ __forceinline__ void load_tile(u32x4_t (&st)[NL], const char* tile, int n_loads, int valid_chunks, bool full, int lane) {
    if (full) {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (i < n_loads) st[i] = ld_global_16(tile + lane * 16 + i * 1024);
    } else {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (i < n_loads) {
                const int f = i * 64 + lane;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (f < valid_chunks) v = ld_global_16(tile + f * 16);
                st[i] = v;
            }
    }
}

// Park the tile in LDS: chunk f -> row f / cpr, chunk-in-row f % cpr, padded row stride.
template <int NL>
__device__ __forceinline__ void park_tile(const u32x4_t (&st)[NL], char* region, int n_loads, int cpr, int stride, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
        if (i < n_loads) {
            const unsigned f = i * 64 + lane;
            const unsigned row = f / (unsigned)cpr;
            const unsigned ch = f - row * cpr;
            *reinterpret_cast<u32x4_t*>(region + row * stride + ch * 16) = st[i];
        }
}

// The kernel reads its argument block through the kernel-argument segment pointer (constant address
// space): run-time indexed reads of the by-value argument would otherwise make the compiler copy the
// whole block into per-lane scratch memory.  The block is the kernel's only explicit argument, so it
// sits at offset 0 of the segment.
typedef const __attribute__((address_space(4))) AttendParams* KArgs;
typedef const __attribute__((address_space(4))) GroupDesc* KGroup;
typedef const __attribute__((address_space(4))) short* KShorts;

// Entry `base + idx` of a small table that lives in the kernel arguments, for a lane-dependent idx in
// [0, 16): done with 16 uniform reads and selects, because indexing the argument block with a
// lane-dependent index would make the compiler copy the whole block to scratch memory.
__device__ __forceinline__ int lane_lookup16(KShorts table, int base, int limit, int idx, int otherwise) {
    int r = otherwise;
#pragma unroll
    for (int s = 0; s < 16; ++s)
        if (base + s < limit && idx == s) r = table[base + s];
    return r;
}

// int8 latents ("Quantization", Eq. "quant"): a row is r codes plus {scale, zeropoint}.  A code byte
// c is turned into the fp16 number 1024 + (c + 128) by one byte permute (0x64 in the high byte makes
// the mantissa count in units of one), so the products below run on v_mfma_f32_16x16x32_f16 whatever
// the model dtype is; the constant 1152 and the zero point are taken out afterwards:
//   x^_tc = (u_tc - off_t) / scale_t,   u_tc = 1152 + code_tc,  off_t = 1152 + zeropoint_t
//   score = (1/scale_t) (sum_c qt_c u_tc - off_t sum_c qt_c)
//   sum_t p_t x^_tc = sum_t P_t u_tc - sum_t P_t off_t,   P_t = p_t / scale_t
// where sum_t P_t off_t comes out of the same MFMA from three extra columns of the V tile (off_t
// split as 4096 h2 + 64 h1 + h0, each exact in fp16), which sit in the padding of the LDS rows.
constexpr float kI8Offset = 1152.f;       // 1024 (fp16 exponent trick) + 128 (codes are signed)
constexpr float kI8PScale = 256.f;        // keeps P_t = p_t / scale_t in fp16's normal range

// 16 code bytes -> 16 fp16 numbers 1024 + (code + 128), as two 16-byte halves
__device__ __forceinline__ void i8_chunk_to_f16(const u32x4_t c, u32x4_t& lo, u32x4_t& hi) {
    unsigned h[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned x = c[i] ^ 0x80808080u;
        // selector bytes 0..3 pick bytes of the second operand, 4..7 of the first
        h[2 * i] = __builtin_amdgcn_perm(0x64646464u, x, 0x04010400u);
        h[2 * i + 1] = __builtin_amdgcn_perm(0x64646464u, x, 0x04030402u);
    }
    lo = u32x4_t{h[0], h[1], h[2], h[3]};
    hi = u32x4_t{h[4], h[5], h[6], h[7]};
}

// Park an int8 tile: 16-byte chunk f holds 16 codes of row f / cpr8 -> 32 bytes of fp16 in the padded row.
// A lane's two 16-byte stores lie 32 bytes from its neighbours': eight consecutive lanes, which share the 128 bytes of
// LDS banks, would cover only every other 16-byte bank group, twice.  So in the upper half of a 256-byte row (fp16
// chunks 8 and up) the two chunks of a pair swap places: lanes 0-3 of a row then write bank groups 0, 2, 4, 6 and lanes
// 4-7 write 1, 3, 5, 7 in the same instruction.  Readers undo the swap (kI8SwapFrom).
constexpr int kI8SwapFrom = 8;       // first 16-byte chunk of a parked int8 row that sits in its pair's other slot
template <int NL>
__device__ __forceinline__ void park_tile_i8(const u32x4_t (&st)[NL], char* region, int n_loads, int cpr8, int stride, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
        if (i < n_loads) {
            const unsigned f = i * 64 + lane;
            const unsigned row = f / (unsigned)cpr8;
            const unsigned ch = f - row * cpr8;
            const unsigned sw = 2 * ch >= (unsigned)kI8SwapFrom ? 16u : 0u;
            u32x4_t lo, hi;
            i8_chunk_to_f16(st[i], lo, hi);
            *reinterpret_cast<u32x4_t*>(region + row * stride + ch * 32 + sw) = lo;
            *reinterpret_cast<u32x4_t*>(region + row * stride + ch * 32 + (16u ^ sw)) = hi;
        }
}

// Two floats to / from global memory as one 8-byte access at agent scope: such accesses go past the per-XCD L2 caches,
// so that workgroups on different XCDs can exchange them inside one launch (ordinary stores would sit in the writer's
// L2, ordinary loads could hit a stale line in the reader's).  p must be 8-byte aligned.
__device__ __forceinline__ void st_agent2(float* p, float a, float b) {
    const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same for 8 and 16 bytes through buffer accesses whose cache policy carries the agent-scope bit (the bit the
// compiler puts on agent-scope atomic loads and stores).  `base` must be 16-byte aligned; offsets are in bytes from
// it; accesses at or beyond `bytes` touch nothing and loads there return zeros.
struct AgentBuf {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ AgentBuf(const void* base, unsigned bytes)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000)) {}      // raw buffer, 32-bit elements
    static constexpr int kAgentScope = 16;          // cache-policy bit sc1
    static constexpr unsigned kNowhere = 0xffffff00u;      // an offset beyond any buffer
    __device__ __forceinline__ void store(unsigned byte_off, f32x4_t v) const {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), rsrc, (int)byte_off, 0, kAgentScope);
    }
    __device__ __forceinline__ f32x4_t load(unsigned byte_off) const {
        return __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, kAgentScope));
    }
    __device__ __forceinline__ u32x2_t load8(unsigned byte_off) const {
        return __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)byte_off, 0, kAgentScope);
    }
};

// kFused (single split, exact shapes only): the absorbed queries are computed in the prologue and the
// last decoder layer of V is applied in the epilogue, so the whole decode attention of a layer is this
// one kernel and neither the absorbed queries nor the partials travel through memory.
// kPrologue without kFused (several splits): every split's workgroup computes the absorbed queries itself
// (a few microseconds, in parallel) instead of a prologue kernel running first; partials go to memory.
// kArrive (several splits, one launch; with kPrologue, without kFused): every workgroup writes its partial past the
// per-XCD L2 caches (agent-scope stores), waits for those stores and counts itself in at the (sequence, group)'s
// arrival counter; the workgroup that finds all others already counted reads the partials back (agent-scope
// loads), merges them and runs the same epilogue as the fused form.  Nobody waits for anybody: every workgroup exits
// after its own work, so the grid drains whatever the scheduling order.
// The counter lives in the caller's workspace, whose contents are arbitrary: it is a {tag, count} pair that means
// something only while its tag equals the launch's epoch.  Every workgroup looks at it when it starts and, if the tag
// is another, tries once to replace what it saw by {epoch, 0} (compare-and-swap: if that fails, somebody else has set it
// up, or has even counted itself in already); a workgroup arrives only after its own attempt, so the counter is set up
// by then and arriving is one atomic add.  The last workgroup leaves {0, 0}, so a replay of a captured launch (same
// epoch) starts over.
// Which (split, sequence, group) a workgroup takes: (blockIdx.x, blockIdx.y, blockIdx.z), unless groups of the launch
// read the same latent rows (small launches give every KV head a group of its own).  Workgroups are dealt round-robin
// over the chip's eight XCDs in launch order (x fastest, z slowest), which would scatter the groups of one (split,
// sequence) over the XCDs whenever splits x batch is not a multiple of eight; each XCD has an L2 of its own, so the
// repeated reads would then miss.  With `colocate` the workgroup whose place in the launch order is L takes unit
// ((L / 8) / G) * 8 + L % 8 (units = (split, sequence) pairs, split fastest) and group (L / 8) % G: all G groups of a unit
// sit on XCD L % 8.  The last units, which do not fill a round of eight, keep an order of their own.
struct WgCoords {
    int split, b, z;
};
__device__ __forceinline__ WgCoords wg_coords(KArgs p) {
    if (!p->colocate) return WgCoords{(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z};
    const unsigned n_sp = (unsigned)p->n_splits, G = (unsigned)p->n_groups;
    const unsigned L = blockIdx.x + n_sp * (blockIdx.y + (unsigned)p->batch * blockIdx.z);
    const unsigned U = n_sp * (unsigned)p->batch, U8 = U & ~7u, N8 = U8 * G;
    unsigned u, z;
    if (L < N8) {
        const unsigned k = L >> 3;
        z = k % G;
        u = (k / G) * 8 + (L & 7u);
    } else {
        const unsigned i = L - N8, rest = U - U8;
        z = i / rest;
        u = U8 + i % rest;
    }
    return WgCoords{(int)(u % n_sp), (int)(u / n_sp), (int)z};
}

template <typename E, typename D, bool kFused, bool kI8 = false, int NW = kWaves, bool kPrologue = kFused, bool kArrive = false>
__device__ __forceinline__ void attend_body(KArgs p, KGroup g, const WgCoords& wc, char* lds_raw, size_t wave_lds) {
    static_assert(!kArrive || (kPrologue && !kFused && D::kExact && (NW == kWaves || NW == 2 * kWaves)), "the arrival form is a split form of the exact shapes");
    constexpr int RMAX = D::RMAX, NHB = D::NHB;
    using G = Geo<RMAX>;
    using ML = typename std::conditional<kI8, F16, E>::type;    // element type of the products in the loop
    static_assert(!kI8 || (D::kExact && G::kPrefetch), "int8 latents: exact shapes up to 128 only");
    constexpr int KS = RMAX / 32;      // k-steps of the score product
    constexpr int MB = RMAX / 16;      // 16-column blocks of the latent accumulator
    constexpr int NL = kI8 ? RMAX / 32 : RMAX / 16;      // 128-bit loads per lane per tile
    constexpr int EB = kI8 ? 1 : 2;    // bytes per cached latent element

    const D d(g->k.r, g->v.r, g->slots_pad >> 4);
    const int split = wc.split, b = wc.b;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;

    const int rk = d.rk, rv = d.rv, nhb = d.nhb;
    const int ksteps = rk >> 5, mblocks = rv >> 4;
    const int nlk = kI8 ? rk >> 5 : rk >> 4, nlv = kI8 ? rv >> 5 : rv >> 4;     // loads per lane per tile
    const int cprk = kI8 ? rk >> 4 : rk >> 3, cprv = kI8 ? rv >> 4 : rv >> 3;   // 16-byte chunks per cached row
    const int stride_k = 2 * rk + 16, stride_v = 2 * rv + 32;

    char* my_lds = lds_raw + wave * wave_lds;
    char* lds_k = my_lds;
    char* lds_v = G::kPrefetch ? my_lds + kWaveTile * stride_k : my_lds;

    // Workgroup tiles (4 wave tiles = 128 tokens each) of this split.  tile_order 0: a contiguous
    // token range per split; 1: tiles dealt round-robin over the splits, so that workgroups running
    // at the same time read neighbouring addresses.
    // context length of this sequence (ragged batches pass one per sequence)
    const int n_ctx = p->seq_lens ? min(p->seq_lens[b], p->n_ctx) : p->n_ctx;
    const int wg_tiles = (n_ctx + kWaveTile * NW - 1) / (kWaveTile * NW);
    int j0, j1, jstep;
    if (p->tile_order == 0) {
        const int per_split = (wg_tiles + p->n_splits - 1) / p->n_splits;
        j0 = split * per_split;
        j1 = min(wg_tiles, j0 + per_split);
        jstep = 1;
    } else {
        j0 = split; j1 = wg_tiles; jstep = p->n_splits;
    }

    const char* zk = static_cast<const char*>(g->k.z) + (size_t)b * p->max_seq * rk * EB;
    const char* zv = static_cast<const char*>(g->v.z) + (size_t)b * p->max_seq * rv * EB;
    // int8: {scale, zeropoint} of this sequence's rows; lanes 0..31 take the K rows of a tile, 32..63 the V rows
    const RowMeta* mrow = nullptr;
    float* mlds = nullptr;               // per wave: ak[32] (1/scale_K), bk[32] (off_K/scale_K), av[32] (256/scale_V)
    if constexpr (kI8) {
        mrow = static_cast<const RowMeta*>(lane < 32 ? g->k.meta : g->v.meta) + (size_t)b * p->max_seq;
        mlds = reinterpret_cast<float*>(my_lds + kWaveTile * stride_k + kWaveTile * stride_v);
    }

    // kPrefetch: both tiles of the next iteration are in flight while this one computes.  Otherwise (wide
    // rows) a tile is loaded right before it is parked and K, V take turns.  PF = iterations of look-ahead;
    // two was measured slower for int8 rows (the second set of staging registers spills).
    constexpr int PF = 1;
    struct Stage {
        u32x4_t k[NL];
        u32x4_t v[G::kPrefetch ? NL : 1];
        u32x2_t m;
    };
    Stage stage[PF];
    auto issue = [&](Stage& sg, int j) {
        const int t0 = (j * NW + wave) * kWaveTile;
        const int nv = max(0, min(kWaveTile, n_ctx - t0));
        load_tile<NL>(sg.k, zk + (size_t)t0 * rk * EB, nlk, nv * cprk, nv == kWaveTile, lane);
        if constexpr (G::kPrefetch) load_tile<NL>(sg.v, zv + (size_t)t0 * rv * EB, nlv, nv * cprv, nv == kWaveTile, lane);
        if constexpr (kI8) {
            const int tok = t0 + (lane & 31);
            sg.m = u32x2_t{0x3f800000u, 0u};                      // rows past the context: scale 1, zero point 0
            if (tok < n_ctx) sg.m = *reinterpret_cast<const u32x2_t*>(mrow + tok);
        }
    };
    if constexpr (G::kPrefetch) {                  // first tiles in flight while the queries are prepared
#pragma unroll
        for (int pf = 0; pf < PF; ++pf)
            if (j0 + pf * jstep < j1) issue(stage[pf], j0 + pf * jstep);
    }

    // arrival form: what the (sequence, group)'s counter holds now (used after the prologue, so the load flies meanwhile)
    unsigned long long* counter = nullptr;
    unsigned long long seen = 0;
    if constexpr (kArrive) {
        counter = p->arrive + ((size_t)b * p->arrive_stride + wc.z) * kArrivePitch;
        if (threadIdx.x == 0) seen = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- append-and-attend: the new token's latent rows ("Network Architecture", 1st paragraph: the encoder after K/V
    // generation), computed by the workgroup that holds the context's last tile instead of by an encoder launch
    // before this one.  z = x[columns of the stored heads] . W_enc + b in fp32, rounded once to the cache dtype; the
    // row is written to the layer's cache (by one group per side) and kept in LDS, from where it replaces the last row
    // of the tile as parked - the copy of that row loaded from memory may predate the write.
    const char* znew = nullptr;
    bool patch_k = false, patch_v = false;
    auto encode_new_token = [&]() {
        // runs between the prologue's exchange barrier and the reads of the query operands: few registers are live then,
        // and the waves' staging regions (the first tiles are still in flight, in registers) serve as scratch
        // eight waves: the first four take the keys, the other four the values; four waves: every thread works on both
        // sides, phase by phase, so that the two sides' memory round trips overlap (three barriers either way)
        constexpr int S = NW >= 8 ? 1 : 2;
        float* xs_all = reinterpret_cast<float*>(lds_raw);   // [2 sides][in_width <= 256]
        float* ps_all = xs_all + 512;                        // [2 sides][4 waves][128]
        uint16_t* zn = reinterpret_cast<uint16_t*>(lds_raw + NW * wave_lds + 2 * 4 * 64 * 16);      // [2 sides][128], past the exchange area: kept through the loop
        char* zi8 = lds_raw + kWaveTile * (stride_k + stride_v) + 384;                              // int8 rows: see below
        const int dh = p->d_head, d_kv = (p->n_q_heads / p->gq) * dh;
        const int tid = threadIdx.x & 255, w4 = wave & 3;
        // one side's encoder (read with constant indices: the argument block must not be indexed by a run-time value)
        struct Side {
            bool on, v_side;
            int inw, r, b_off;
            long long head_block;
            const void* ex;
            const char* ew;
            const void* eb;
            char* ez;
        };
        auto side_of = [&](int side) {
            Side e;
            e.v_side = side == 1;
            e.on = ((g->append >> side) & 1) != 0;
            e.inw = e.v_side ? p->enc[1].in_width : p->enc[0].in_width;
            e.r = e.v_side ? p->enc[1].r : p->enc[0].r;
            e.ex = e.v_side ? p->enc[1].x : p->enc[0].x;
            e.ew = static_cast<const char*>(e.v_side ? p->enc[1].w : p->enc[0].w);
            e.eb = e.v_side ? p->enc[1].b : p->enc[0].b;
            e.ez = static_cast<char*>(e.v_side ? p->enc[1].z : p->enc[0].z);
            // per-head autoencoders: this group's head has an encoder, a bias and a block of the cache of its own
            e.head_block = e.v_side ? p->enc[1].head_block : p->enc[0].head_block;
            const int slice = e.head_block ? (int)(e.v_side ? g->app_slice[1] : g->app_slice[0]) : 0;
            e.ew += (size_t)slice * e.inw * e.r * 2;
            e.ez += (size_t)slice * e.head_block;
            e.b_off = slice * e.r;
            return e;
        };
        Side sd[S];
#pragma unroll
        for (int si = 0; si < S; ++si) sd[si] = side_of(S == 1 ? (int)(threadIdx.x >> 8) : si);
        // ---- the token's vectors into LDS, as fp32
#pragma unroll
        for (int si = 0; si < S; ++si) {
            const Side& e = sd[si];
            if (e.on && tid < e.inw) {
                // column tid of the encoder input = component tid % dh of the (tid / dh)-th stored head
                const int k = tid / dh;
                int head = 0;
#pragma unroll
                for (int i = 0; i < kAppendMaxHeads; ++i) head = i == k ? (int)(e.v_side ? p->enc[1].heads[i] : p->enc[0].heads[i]) : head;
                if (e.head_block) head = g->app_head;
                xs_all[(e.v_side ? 256 : 0) + tid] = Elem<E>::load(e.ex, (size_t)b * d_kv + head * dh + (tid - k * dh));
            }
        }
        __syncthreads();
        // ---- thread = (row group rg of 16, column group cg of 16): rows rg * in_width / 16 .., columns 8 cg .. 8 cg + 7;
        // its 16-byte loads of the matrix (of both sides, with four waves) are in flight eight rows at a time
        {
            const int rg = tid >> 4, c = 8 * (tid & 15);
            float a[S][8];
            int rows[S];
            bool live[S];
            const char* w[S];
            int rows_max = 0;
#pragma unroll
            for (int si = 0; si < S; ++si) {
#pragma unroll
                for (int e = 0; e < 8; ++e) a[si][e] = 0.f;
                rows[si] = sd[si].inw >> 4;
                live[si] = sd[si].on && c < sd[si].r;
                w[si] = sd[si].ew + ((size_t)rg * rows[si] * sd[si].r + c) * 2;
                rows_max = live[si] && rows[si] > rows_max ? rows[si] : rows_max;
            }
            for (int i0 = 0; i0 < rows_max; i0 += 8) {
                u32x4_t wv[S][8];
#pragma unroll
                for (int si = 0; si < S; ++si)
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        wv[si][u] = live[si] && i0 + u < rows[si] ? *reinterpret_cast<const u32x4_t*>(w[si] + (size_t)(i0 + u) * sd[si].r * 2) : u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
                for (int si = 0; si < S; ++si) {
                    const float* xs = xs_all + (sd[si].v_side ? 256 : 0);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float x = live[si] && i0 + u < rows[si] ? xs[rg * rows[si] + i0 + u] : 0.f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            a[si][2 * e] = fmaf(x, Mma<E>::unpack_lo(wv[si][u][e]), a[si][2 * e]);
                            a[si][2 * e + 1] = fmaf(x, Mma<E>::unpack_hi(wv[si][u][e]), a[si][2 * e + 1]);
                        }
                    }
                }
            }
            // the four row groups of a wave (lane / 16) meet by two cross-lane steps, the four waves through LDS
#pragma unroll
            for (int si = 0; si < S; ++si) {
                if (!sd[si].on) continue;                    // the same for the whole workgroup
                float* ps = ps_all + (sd[si].v_side ? 512 : 0);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    a[si][e] += __shfl_xor(a[si][e], 16);
                    a[si][e] += __shfl_xor(a[si][e], 32);
                }
                if (lane < 16 && live[si]) {
                    *reinterpret_cast<f32x4_t*>(ps + w4 * 128 + c) = f32x4_t{a[si][0], a[si][1], a[si][2], a[si][3]};
                    *reinterpret_cast<f32x4_t*>(ps + w4 * 128 + c + 4) = f32x4_t{a[si][4], a[si][5], a[si][6], a[si][7]};
                }
            }
        }
        __syncthreads();
        // ---- the waves' sums in wave order, the bias, one rounding to the cache dtype; into LDS and (one group) to the cache
        if constexpr (!kI8) {
#pragma unroll
            for (int si = 0; si < S; ++si) {
                const Side& e = sd[si];
                if (e.on && tid < e.r) {
                    const float* ps = ps_all + (e.v_side ? 512 : 0);
                    const float z = ((ps[tid] + ps[128 + tid]) + (ps[256 + tid] + ps[384 + tid])) + (e.eb ? Elem<E>::load(e.eb, e.b_off + tid) : 0.f);
                    const uint16_t z16 = Mma<E>::to16(z);
                    zn[(e.v_side ? 128 : 0) + tid] = z16;
                    if ((g->append >> (e.v_side ? 3 : 2)) & 1)
                        reinterpret_cast<uint16_t*>(e.ez)[((size_t)b * p->max_seq + (n_ctx - 1)) * e.r + tid] = z16;
                }
            }
            __syncthreads();
        } else {
            // int8 rows ("Quantization", Eq. "quant"): the row's minimum and maximum first (the first two waves of a side
            // hold its r <= 128 entries: butterfly inside a wave, the two waves meet in LDS), then scale, zero point and
            // codes with the encoders' arithmetic; codes and {scale, zero point} go to LDS and (one group) to the cache
            float* mm = ps_all + 1024;                        // [2 sides][2 waves][min, max]
            float zf[S];
#pragma unroll
            for (int si = 0; si < S; ++si) {
                const Side& e = sd[si];
                const float* ps = ps_all + (e.v_side ? 512 : 0);
                const bool mine = e.on && tid < e.r;
                zf[si] = mine ? ((ps[tid] + ps[128 + tid]) + (ps[256 + tid] + ps[384 + tid])) + (e.eb ? Elem<E>::load(e.eb, e.b_off + tid) : 0.f) : 0.f;
                float mn = mine ? zf[si] : INFINITY, mx = mine ? zf[si] : -INFINITY;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    mn = fminf(mn, __shfl_xor(mn, off));
                    mx = fmaxf(mx, __shfl_xor(mx, off));
                }
                if (e.on && w4 < 2 && lane == 0) { mm[(e.v_side ? 4 : 0) + 2 * w4] = mn; mm[(e.v_side ? 4 : 0) + 2 * w4 + 1] = mx; }
            }
            __syncthreads();
            // kept through the loop in the 128 spare bytes after each wave's per-row terms (its last 512 bytes hold 96
            // floats): the key codes with wave 0, the value codes with wave 1, the two {scale, zero point} with wave 2
            signed char* zn8 = reinterpret_cast<signed char*>(zi8);              // side s: [128] codes at s * wave_lds
            u32x2_t* znm = reinterpret_cast<u32x2_t*>(zi8 + 2 * wave_lds);        // [2 sides] {scale, zero point}
#pragma unroll
            for (int si = 0; si < S; ++si) {
                const Side& e = sd[si];
                if (e.on && tid < e.r) {
                    const float* m4 = mm + (e.v_side ? 4 : 0);
                    const QuantParams qp = quant_params(fminf(m4[0], m4[2]), fmaxf(m4[1], m4[3]));
                    const signed char code = quant_code(zf[si], qp);
                    const RowMeta meta = quant_meta(qp);
                    zn8[(e.v_side ? wave_lds : 0) + tid] = code;
                    if (tid == 0) znm[e.v_side ? 1 : 0] = u32x2_t{__float_as_uint(meta.scale), (unsigned)meta.zeropoint};
                    if ((g->append >> (e.v_side ? 3 : 2)) & 1) {
                        const size_t row = (size_t)b * p->max_seq + (n_ctx - 1);
                        reinterpret_cast<signed char*>(e.ez)[row * e.r + tid] = code;
                        if (tid == 0) static_cast<RowMeta*>(e.v_side ? p->enc[1].meta : p->enc[0].meta)[row] = meta;
                    }
                }
            }
            __syncthreads();
        }
        znew = kI8 ? zi8 : reinterpret_cast<const char*>(zn);
        patch_k = (g->append & 1) != 0;
        patch_v = (g->append & 2) != 0;
    };
    bool encode_here = false;
    if constexpr (kPrologue && KVCAR_APPEND_IN_KERNEL) encode_here = p->append && (g->append & 3) && j0 < j1 && j1 == wg_tiles;     // the same for the whole workgroup

    // absorbed queries of this sequence and group, resident as MFMA B operands
    u32x4_t qb[NHB][KS];
    if constexpr (kPrologue) {
        // Qt^T[c, head] = scale*log2e * sum_k Wl_K[c, col(head)+k] q[head, k], by MFMA straight from global
        // memory: A = rows of the decoder matrix, B = the queries of one KV head's heads (other heads of
        // the 16-block masked to zero; a block spans at most two KV heads: two passes).  Row rho of result
        // tile (s, hh) is latent index 32s + 8(rho/4) + 4hh + rho%4, so that the result registers of tiles
        // (s,0) and (s,1) are exactly the B operand of score k-step s.  Wave w computes k-step s = w for
        // all heads (its loads are independent and fly together) and the waves swap through LDS.
        const int dh = p->d_head;
        const char* wl = static_cast<const char*>(g->k.wl);
        u32x4_t* qlds = reinterpret_cast<u32x4_t*>(lds_raw + NW * wave_lds);      // [NHB][KS][64], past the staging regions
        if (wave < KS) {
            const int s2 = wave;
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) {
                const int my_slot = nb * 16 + l16;
                const bool live = my_slot < g->n_slots;
                const int my_col = live ? (int)g->k_col[my_slot] : -1;
                const int my_head = live ? (int)g->q_head[my_slot] : 0;
                const char* qrow = static_cast<const char*>(p->q) + ((size_t)b * p->n_q_heads + my_head) * dh * 2;
                // the (at most two) KV heads of this 16-head block, from the host's table of runs
                int col_a = -1, col_b = -1;
#pragma unroll
                for (int sg = 0; sg < kMaxSeg; ++sg)
                    if (sg < g->n_kseg && g->kseg_lo[sg] < nb * 16 + 16 && g->kseg_hi[sg] > nb * 16) {
                        if (col_a < 0) col_a = g->kseg_col[sg];
                        else col_b = g->kseg_col[sg];
                    }
                f32x4_t t[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
                // two 32-wide steps of the head dimension per round: all loads of a round are issued before its
                // products, so a head dimension of 64 costs one memory latency
                for (int k0 = 0; k0 < dh; k0 += 64) {
                    u32x4_t bq[2][2], aw[2][2][2];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int k = k0 + 32 * u;
                        const bool on = k < dh;
                        const u32x4_t qv = (on && my_col >= 0) ? *reinterpret_cast<const u32x4_t*>(qrow + (k + 8 * lg) * 2) : u32x4_t{0u, 0u, 0u, 0u};
                        bq[u][0] = my_col == col_a ? qv : u32x4_t{0u, 0u, 0u, 0u};
                        bq[u][1] = my_col == col_b ? qv : u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
                        for (int sg = 0; sg < 2; ++sg)
#pragma unroll
                            for (int hh = 0; hh < 2; ++hh) {
                                const int c = 32 * s2 + 8 * (l16 >> 2) + 4 * hh + (l16 & 3);
                                const int col = sg == 0 ? col_a : col_b;
                                aw[u][sg][hh] = u32x4_t{0u, 0u, 0u, 0u};
                                if (on && col >= 0) aw[u][sg][hh] = *reinterpret_cast<const u32x4_t*>(wl + ((size_t)c * g->k.in_width + col + k + 8 * lg) * 2);
                            }
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int sg = 0; sg < 2; ++sg)
#pragma unroll
                            for (int hh = 0; hh < 2; ++hh) t[hh] = Mma<E>::mfma(aw[u][sg][hh], bq[u][sg], t[hh]);
                }
                const float sc = p->scale_log2e;
                qlds[(nb * KS + s2) * 64 + lane] =
                    u32x4_t{Mma<ML>::pack2(t[0][0] * sc, t[0][1] * sc), Mma<ML>::pack2(t[0][2] * sc, t[0][3] * sc),
                            Mma<ML>::pack2(t[1][0] * sc, t[1][1] * sc), Mma<ML>::pack2(t[1][2] * sc, t[1][3] * sc)};
            }
        }
        __syncthreads();
        if constexpr (KVCAR_APPEND_IN_KERNEL) {
            if (encode_here) encode_new_token();
        }
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int s2 = 0; s2 < KS; ++s2) qb[nb][s2] = qlds[(nb * KS + s2) * 64 + lane];
    } else if constexpr (kI8) {
        // the prologue kernel leaves the absorbed queries in fp32; they enter the products as fp16
        const float* qt = static_cast<const float*>(p->qt) + (size_t)b * p->qt_stride + g->qt_off;
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const float* src = qt + (size_t)(nb * 16 + l16) * rk + 8 * (4 * s + lg);
                const f32x4_t x0 = *reinterpret_cast<const f32x4_t*>(src), x1 = *reinterpret_cast<const f32x4_t*>(src + 4);
                qb[nb][s] = u32x4_t{Mma<F16>::pack2(x0[0], x0[1]), Mma<F16>::pack2(x0[2], x0[3]), Mma<F16>::pack2(x1[0], x1[1]), Mma<F16>::pack2(x1[2], x1[3])};
            }
    } else {
        const char* qt = static_cast<const char*>(p->qt) + ((size_t)b * p->qt_stride + g->qt_off) * 2;
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (nb < nhb && s < ksteps) v = *reinterpret_cast<const u32x4_t*>(qt + ((size_t)(nb * 16 + l16) * rk + 8 * (4 * s + lg)) * 2);
                qb[nb][s] = v;
            }
    }
    if constexpr (kArrive) {
        const unsigned long long fresh = (unsigned long long)p->epoch << 32;
        if (threadIdx.x == 0 && (unsigned)(seen >> 32) != p->epoch)
            __hip_atomic_compare_exchange_strong(counter, &seen, fresh, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // int8: Qsum[nb] = sum over the latent index of this lane's head's absorbed query, as rounded to fp16
    float qsum[NHB];
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) qsum[nb] = 0.f;
    if constexpr (kI8) {
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            float a = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) a += Mma<F16>::unpack_lo(qb[nb][s][e]) + Mma<F16>::unpack_hi(qb[nb][s][e]);
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            qsum[nb] = a;
        }
    }

    f32x4_t acc[NHB][MB];
    f32x4_t accx[NHB];                 // int8: rows 0..2 accumulate sum_t P_t (h2, h1, h0)_t
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        accx[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    float m_run[NHB], l_run[NHB];
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) { m_run[nb] = -INFINITY; l_run[nb] = 0.f; }


    auto tile = [&](Stage& sg, int j) -> bool {
        const int t0 = (j * NW + wave) * kWaveTile;
        const int nv = min(kWaveTile, n_ctx - t0);
        if (nv <= 0) return false;   // wave tile past the context: only in the last workgroup tile, the last one visited

        if constexpr (!G::kPrefetch) issue(sg, j);
        if constexpr (kI8) {
            park_tile_i8<NL>(sg.k, lds_k, nlk, cprk, stride_k, lane);
            park_tile_i8<NL>(sg.v, lds_v, nlv, cprv, stride_v, lane);
            if constexpr (KVCAR_APPEND_IN_KERNEL) {
                if (znew != nullptr && n_ctx - 1 >= t0 && n_ctx - 1 < t0 + kWaveTile) {      // append-and-attend: the row encoded above
                    const int rown = n_ctx - 1 - t0;
                    const u32x2_t* znm = reinterpret_cast<const u32x2_t*>(znew + 2 * wave_lds);
#pragma unroll
                    for (int side = 0; side < 2; ++side) {
                        if (!(side == 0 ? patch_k : patch_v)) continue;
                        char* region = side == 0 ? lds_k : lds_v;
                        const int stride = side == 0 ? stride_k : stride_v, cpr8 = side == 0 ? cprk : cprv;
                        if (lane < cpr8) {                       // 16 codes per lane, parked as park_tile_i8 parks them
                            u32x4_t lo, hi;
                            i8_chunk_to_f16(*reinterpret_cast<const u32x4_t*>(znew + side * wave_lds + lane * 16), lo, hi);
                            const unsigned sw = 2 * lane >= kI8SwapFrom ? 16u : 0u;
                            *reinterpret_cast<u32x4_t*>(region + rown * stride + lane * 32 + sw) = lo;
                            *reinterpret_cast<u32x4_t*>(region + rown * stride + lane * 32 + (16u ^ sw)) = hi;
                        }
                        if (lane == side * 32 + rown) sg.m = znm[side];       // the lane that holds this row's scale and zero point
                    }
                }
            }
            const float inv = __builtin_amdgcn_rcpf(__uint_as_float(sg.m[0]));
            const float off = kI8Offset + (float)(int)sg.m[1];
            if (lane < 32) {
                mlds[lane] = inv;
                mlds[32 + lane] = inv * off;
            } else {
                mlds[32 + lane] = fminf(inv * kI8PScale, 60000.f);
                // off = 4096 h2 + 64 h1 + h0 with |h1|, |h0| <= 32 and h2 exact in fp16 up to 2048
                const float h2 = fminf(fmaxf(rintf(off * (1.f / 4096.f)), -2048.f), 2048.f);
                const float r1 = off - 4096.f * h2;
                const float h1 = rintf(r1 * (1.f / 64.f));
                const float h0 = r1 - 64.f * h1;
                *reinterpret_cast<u32x2_t*>(lds_v + (lane - 32) * stride_v + 2 * rv) = u32x2_t{Mma<F16>::pack2(h2, h1), Mma<F16>::pack2(h0, 0.f)};
            }
            if (j + PF * jstep < j1) issue(sg, j + PF * jstep);
        } else {
        park_tile<NL>(sg.k, lds_k, nlk, cprk, stride_k, lane);
        if constexpr (G::kPrefetch) {
            park_tile<NL>(sg.v, lds_v, nlv, cprv, stride_v, lane);
            if (j + PF * jstep < j1) issue(sg, j + PF * jstep);
            if (znew != nullptr && n_ctx - 1 >= t0 && n_ctx - 1 < t0 + kWaveTile) {      // append-and-attend: the row encoded above
                const int rown = n_ctx - 1 - t0;
                if (patch_k && lane < cprk) *reinterpret_cast<u32x4_t*>(lds_k + rown * stride_k + lane * 16) = *reinterpret_cast<const u32x4_t*>(znew + lane * 16);
                if (patch_v && lane < cprv) *reinterpret_cast<u32x4_t*>(lds_v + rown * stride_v + lane * 16) = *reinterpret_cast<const u32x4_t*>(znew + 256 + lane * 16);
            }
        }
        }

        // ---- scores: S^T[token, head] ------------------------------------------------------
        f32x4_t sT[2][NHB];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) sT[a][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        const char* krow = lds_k + l16 * stride_k + lg * 16;
        const char* krow_sw = lds_k + l16 * stride_k + (lg ^ 1) * 16;       // int8 rows: chunks whose pair is swapped
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s < ksteps) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const char* kr = kI8 && 4 * s >= kI8SwapFrom ? krow_sw : krow;
                    const u32x4_t ka = *reinterpret_cast<const u32x4_t*>(kr + a * 16 * stride_k + s * 64);
#pragma unroll
                    for (int nb = 0; nb < NHB; ++nb)
                        if (nb < nhb) sT[a][nb] = Mma<ML>::mfma(ka, qb[nb][s], sT[a][nb]);
                }
            }
        }
        if constexpr (!G::kPrefetch) {
            // K and V share the staging registers and the LDS region: V rows replace K rows
            // (LDS operations of one wave complete in order, so the score reads are done)
            load_tile<NL>(sg.k, zv + (size_t)t0 * rv * 2, nlv, nv * cprv, nv == kWaveTile, lane);
            park_tile<NL>(sg.k, lds_v, nlv, cprv, stride_v, lane);
        }
        f32x4_t av4[2];                   // int8: 256 / scale_V of this lane's eight tokens
        if constexpr (kI8) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const f32x4_t ak4 = *reinterpret_cast<const f32x4_t*>(mlds + 16 * a + 4 * lg);
                const f32x4_t bk4 = *reinterpret_cast<const f32x4_t*>(mlds + 32 + 16 * a + 4 * lg);
                av4[a] = *reinterpret_cast<const f32x4_t*>(mlds + 64 + 16 * a + 4 * lg);
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) sT[a][nb][v] = fmaf(ak4[v], sT[a][nb][v], -bk4[v] * qsum[nb]);
            }
        }
        if (nv < kWaveTile) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (16 * a + 4 * lg + v >= nv) sT[a][nb][v] = -INFINITY;
        }

        // ---- online softmax (base 2) and P^T as B operand -------------------------------------
        u32x4_t pb[NHB];
        float alpha[NHB];
        bool rescale = false;
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            float mx = fmaxf(fmaxf(fmaxf(sT[0][nb][0], sT[0][nb][1]), fmaxf(sT[0][nb][2], sT[0][nb][3])),
                             fmaxf(fmaxf(sT[1][nb][0], sT[1][nb][1]), fmaxf(sT[1][nb][2], sT[1][nb][3])));
            // The four lanes of a head share its running maximum.  They exchange their tile maxima only when some lane
            // of the wave holds a score above its running maximum: after the first tiles the maxima have settled and
            // the two cross-lane steps, the exponential of the correction and the rescaling are skipped.
            alpha[nb] = 1.f;
            if (__builtin_amdgcn_ballot_w64(mx > m_run[nb]) != 0) {
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[nb], mx);
                alpha[nb] = __builtin_amdgcn_exp2f(m_run[nb] - m_new);     // m_run = -inf on the first tile gives 0
                rescale |= m_new != m_run[nb];
                m_run[nb] = m_new;
                l_run[nb] *= alpha[nb];
            }
            const float m_new = m_run[nb];
            float e[8];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                e[v] = __builtin_amdgcn_exp2f(sT[0][nb][v] - m_new);
                e[4 + v] = __builtin_amdgcn_exp2f(sT[1][nb][v] - m_new);
            }
            l_run[nb] += ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
            if constexpr (kI8) {
#pragma unroll
                for (int v = 0; v < 4; ++v) { e[v] *= av4[0][v]; e[4 + v] *= av4[1][v]; }
            }
            pb[nb] = u32x4_t{Mma<ML>::pack2(e[0], e[1]), Mma<ML>::pack2(e[2], e[3]), Mma<ML>::pack2(e[4], e[5]), Mma<ML>::pack2(e[6], e[7])};
        }
        // the running maxima settle after a few tiles; rescale the accumulators only when one moved
        if (__builtin_amdgcn_ballot_w64(rescale) != 0) {
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    if (nb < nhb && mb < mblocks) acc[nb][mb] *= alpha[nb];
            if constexpr (kI8) {
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb) accx[nb] *= alpha[nb];
            }
        }

        // ---- O^T[latent col, head] += Z_V^T . P^T --------------------------------------------
        // 16 lanes of a block supply the addresses of a 4-token x 16-column patch; the transposing
        // load hands lane i its column i for the 4 tokens
        const char* vrow = lds_v + (4 * lg + (l16 >> 2)) * stride_v + (l16 & 3) * 8;
        const char* vrow_sw = lds_v + (4 * lg + (l16 >> 2)) * stride_v + (((l16 & 3) * 8) ^ 16);      // int8 rows: the other slot of the pair
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (mb < mblocks) {
                const char* vr = kI8 && 2 * mb >= kI8SwapFrom ? vrow_sw : vrow;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vr + mb * 32));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vr + mb * 32 + 16 * stride_v));
                const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
                const u32x4_t va = {lo2[0], lo2[1], hi2[0], hi2[1]};
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb)
                    if (nb < nhb) acc[nb][mb] = Mma<ML>::mfma(va, pb[nb], acc[nb][mb]);
            }
        }
        if constexpr (kI8) {             // the three off_t columns in the padding of the V rows
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vrow + MB * 32));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vrow + MB * 32 + 16 * stride_v));
            const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
            const u32x4_t va = {lo2[0], lo2[1], hi2[0], hi2[1]};
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) accx[nb] = Mma<ML>::mfma(va, pb[nb], accx[nb]);
        }
        return true;
    };
    for (int j = j0; j < j1; j += PF * jstep) {
        bool more = true;
#pragma unroll
        for (int pf = 0; pf < PF; ++pf)
            if (more && j + pf * jstep < j1) more = tile(stage[pf], j + pf * jstep);
        if (!more) break;
    }
    if constexpr (kI8) {
        // sum_t P_t x^_t = (sum_t P_t u_t - sum_t P_t off_t) / 256; the second sum sits in rows 0..2 of accx,
        // i.e. in the lanes of quarter 0, column = head
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            const float corr = __shfl(4096.f * accx[nb][0] + 64.f * accx[nb][1] + accx[nb][2], l16);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = (acc[nb][mb] - corr) * (1.f / kI8PScale);
        }
    }

    // ---- merge the four waves and write one partial --------------------------------------------
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        l_run[nb] += __shfl_xor(l_run[nb], 16);
        l_run[nb] += __shfl_xor(l_run[nb], 32);
    }
    // Fused kernel: a wave parks its accumulators (unscaled) and its running (m, l) in its own staging region as soon as
    // it leaves the loop, without waiting for the others: one barrier instead of three before the sums can be merged.
    constexpr size_t kAccBytes = (size_t)NHB * MB * 1024;          // a wave's accumulators: [NHB][MB][64] x 16 bytes
    static_assert(!kFused || kAccBytes + NHB * 128 <= G::kWaveLds, "accumulators and (m, l) must fit the wave's own staging region");
    if constexpr (!kFused) __syncthreads();            // every wave is done with its staging region
    // m of (wave w, head slot nb*16 + l): red[w * red_stride + nb*16 + l]; l of the same: red[red_l + w * red_stride + nb*16 + l]
    float* red = kFused ? reinterpret_cast<float*>(lds_raw + kAccBytes) : reinterpret_cast<float*>(lds_raw);
    const int red_stride = kFused ? (int)(wave_lds >> 2) : NHB * 16;
    const int red_l = kFused ? NHB * 16 : NW * NHB * 16;
    float* accs = reinterpret_cast<float*>(lds_raw) + 2 * NW * NHB * 16;   // not fused: [wave][NHB][MB][64][4]
    if (lane < 16) {
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            red[wave * red_stride + nb * 16 + lane] = m_run[nb];
            red[red_l + wave * red_stride + nb * 16 + lane] = l_run[nb];
        }
    }
    if constexpr (kFused) {
        float* mine = reinterpret_cast<float*>(lds_raw + wave * wave_lds);     // [NHB][MB][64][4]
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) *reinterpret_cast<f32x4_t*>(mine + ((size_t)(nb * MB + mb) * 64 + lane) * 4) = acc[nb][mb];
    }
    __syncthreads();
    float m_all[NHB], l_all[NHB], f_own[NHB];
    float f_wave[kFused ? NW : 1][NHB];                // fused: every wave's factor 2^(m_w - M) for this lane's head slot
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, red[w * red_stride + nb * 16 + l16]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = red[w * red_stride + nb * 16 + l16];
            L += mw == -INFINITY ? 0.f : red[red_l + w * red_stride + nb * 16 + l16] * exp2f(mw - M);
        }
        f_own[nb] = m_run[nb] == -INFINITY ? 0.f : exp2f(m_run[nb] - M);
        if constexpr (kFused) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float mw = red[w * red_stride + nb * 16 + l16];
                f_wave[w][nb] = mw == -INFINITY ? 0.f : exp2f(mw - M);
            }
        }
        m_all[nb] = M;
        l_all[nb] = L;
    }
    // Arrival form, last workgroup.  The splits' partials are read as what they are in memory, runs of consecutive bytes:
    // 16-byte chunk i of a partial's latent sums (i = t, t + 256, ..: head slot i / (rv / 4), columns 4 (i % (rv / 4)) ..)
    // goes to thread t, so a wave's load covers whole cache lines (loads that leave the chip's caches are paid per line
    // touched: a layout that follows the accumulator's lanes takes three times as long).  kAB splits per memory round trip:
    // more do not help, the merge then runs at what one compute unit reads (about 50 GB/s).
    constexpr int NS = NHB * 16;                          // head slots of a partial
    constexpr int kRowChunks = kArrive ? RMAX / 4 : 1;    // 16-byte chunks of a slot's latent sums (exact shapes: rv = RMAX)
    constexpr int kJ = kArrive ? (NS * kRowChunks + 64 * NW - 1) / (64 * NW) : 1;      // chunks per thread
    constexpr int kAB = kArrive ? (16 / kJ < 4 ? 4 : 16 / kJ) : 1;      // as many as registers allow without spilling
    f32x4_t batch_x[kAB][kJ];
    int mslot[kJ], mcol[kJ];
    unsigned moff[kJ];                                    // byte offset of the chunk in a partial, kNowhere: none
#pragma unroll
    for (int j = 0; j < kJ; ++j) {
        const int i = j * (64 * NW) + (int)threadIdx.x;
        mslot[j] = i / kRowChunks;
        mcol[j] = 4 * (i % kRowChunks);
        moff[j] = mslot[j] < g->n_slots ? (unsigned)((mslot[j] * (rv + 4) + 4 + mcol[j]) * 4) : AgentBuf::kNowhere;
    }
    auto arrive_issue = [&](const AgentBuf& buf, int s0, int n_sp, unsigned split_bytes) {
#pragma unroll
        for (int u = 0; u < kAB; ++u)
#pragma unroll
            for (int j = 0; j < kJ; ++j)
                batch_x[u][j] = buf.load(s0 + u < n_sp && moff[j] != AgentBuf::kNowhere ? (unsigned)(s0 + u) * split_bytes + moff[j] : AgentBuf::kNowhere);
    };
    if constexpr (!kFused) {
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            if (mb < mblocks && nb < nhb)
                *reinterpret_cast<f32x4_t*>(accs + ((size_t)((wave * NHB + nb) * MB + mb) * 64 + lane) * 4) = acc[nb][mb] * f_own[nb];
    __syncthreads();
    float* part = p->part + ((size_t)b * p->n_splits + split) * p->part_stride + g->part_off;
    const int pstride = rv + 4;
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        if (nb >= nhb) continue;
        const int slot = nb * 16 + l16;
        if (wave == 0 && lane < 16) {
            if constexpr (kArrive) st_agent2(part + (size_t)slot * pstride, m_all[nb], l_all[nb]);
            else { part[(size_t)slot * pstride] = m_all[nb]; part[(size_t)slot * pstride + 1] = l_all[nb]; }
        }
        // 16-column blocks are shared out over the four waves
        for (int mb = wave; mb < mblocks; mb += NW) {
            f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < NW; ++w) s += *reinterpret_cast<const f32x4_t*>(accs + ((size_t)((w * NHB + nb) * MB + mb) * 64 + lane) * 4);
            if constexpr (kArrive) AgentBuf(part, (unsigned)(NHB * 16 * pstride * 4)).store((unsigned)((slot * pstride + 4 + 16 * mb + 4 * lg) * 4), s);
            else *reinterpret_cast<f32x4_t*>(part + (size_t)slot * pstride + 4 + 16 * mb + 4 * lg) = s;
        }
    }
    }
    if constexpr (kArrive) {
        // this workgroup's partial has left the chip's caches before it counts itself in
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        unsigned* flag = reinterpret_cast<unsigned*>(lds_raw);
        if (threadIdx.x == 0) *flag = (unsigned)__hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*flag + 1u != (unsigned)p->n_splits) return;          // the same for every thread of the workgroup
        if (threadIdx.x == 0) __hip_atomic_store(counter, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Last to arrive: every split's partial is complete in memory.  All loads of a batch are issued before anything
        // waits (a loop that loads, waits and adds per split pays a memory round trip per split).  The first batch of
        // latent sums is requested here already, ahead of the (m, l) pairs that scale them.
        const float* pall = p->part + (size_t)b * p->n_splits * p->part_stride + g->part_off;
        const int pstride = rv + 4;
        const int n_sp = p->n_splits;
        const unsigned split_bytes = (unsigned)p->part_stride * 4u;
        const AgentBuf pbuf(pall, (unsigned)(n_sp - 1) * split_bytes + (unsigned)(NS * pstride * 4));
        arrive_issue(pbuf, 0, n_sp, split_bytes);
        // the (m, l) pairs of every split and head slot: one load each, shared out over the workgroup, into a table in LDS
        constexpr int kMl = kArriveMaxSplits * NS / (64 * NW);
        u32x2_t ml[kMl];
#pragma unroll
        for (int k = 0; k < kMl; ++k) {
            const int e = k * (64 * NW) + (int)threadIdx.x, sp = e / NS, slot = e % NS;
            ml[k] = pbuf.load8(sp < n_sp && slot < g->n_slots ? (unsigned)sp * split_bytes + (unsigned)(slot * pstride * 4) : AgentBuf::kNowhere);
        }
        u32x2_t* ml_tab = reinterpret_cast<u32x2_t*>(lds_raw + kArriveMlTab);          // [split][slot]
#pragma unroll
        for (int k = 0; k < kMl; ++k) {
            const int e = k * (64 * NW) + (int)threadIdx.x, sp = e / NS, slot = e % NS;
            if (sp < n_sp) ml_tab[e] = slot < g->n_slots ? ml[k] : u32x2_t{__float_as_uint(-INFINITY), 0u};
        }
        __syncthreads();
        // two passes over the table, the maximum and then the sum: neither carries more than one operation from a split to
        // the next (the running form, which rescales the sum at every split, takes 80 ns per split)
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) { m_all[nb] = -INFINITY; l_all[nb] = 0.f; }
#pragma unroll 8
        for (int sp = 0; sp < n_sp; ++sp)
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) m_all[nb] = fmaxf(m_all[nb], __uint_as_float(ml_tab[sp * NS + nb * 16 + l16][0]));
#pragma unroll 8
        for (int sp = 0; sp < n_sp; ++sp)
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) {
                const u32x2_t e = ml_tab[sp * NS + nb * 16 + l16];
                const float ms = __uint_as_float(e[0]), ls = __uint_as_float(e[1]);
                l_all[nb] += ms == -INFINITY ? 0.f : ls * exp2f(ms - m_all[nb]);
            }
    }
    if constexpr (kFused || kArrive) {
        // ---- the current token's exact row, if given ("Network Architecture", 2nd paragraph: the decoded cache
        // rows are concatenated with the exact key / value of the current token): one more softmax term per head,
        // s = scale q . (k_cur - b_K) (the cached scores were formed without the K decoder's bias, which cancels
        // among them), so that  out = (L (o W + b) + 2^(s-M') v_cur) / (L + 2^(s-M')),  M' = max(M, s).
        // Per lane (head slot nb*16 + l16): inv_l = what the accumulators are divided by, w_bias and w_cur the
        // weights of the V decoder's bias and of v_cur.
        const bool exact_row = p->k_cur != nullptr;
        float inv_l[NHB], w_bias[NHB], w_cur[NHB];
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            inv_l[nb] = l_all[nb] > 0.f ? 1.f / l_all[nb] : 0.f;     // an empty context leaves the bias
            w_bias[nb] = 1.f;
            w_cur[nb] = 0.f;
        }
        if (exact_row) {
            const int dh = p->d_head, dq = dh >> 2;                 // each quarter of the lanes takes a quarter of the dot product
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) {
                const int slot = nb * 16 + l16;
                const int head = lane_lookup16(g->q_head, nb * 16, g->n_slots, l16, 0);
                const int kcol = lane_lookup16(g->k_col, nb * 16, g->n_slots, l16, 0);
                const size_t qo = ((size_t)b * p->n_q_heads + head) * dh + lg * dq;
                const size_t ko = ((size_t)b * (p->n_q_heads / p->gq) + head / p->gq) * dh + lg * dq;
                float d = 0.f;
                for (int k = 0; k < dq; ++k)
                    d = fmaf(Elem<E>::load(p->q, qo + k), Elem<E>::load(p->k_cur, ko + k) - (g->k.bl ? Elem<E>::load(g->k.bl, kcol + lg * dq + k) : 0.f), d);
                d += __shfl_xor(d, 16);
                d += __shfl_xor(d, 32);
                const float s_cur = slot < g->n_slots ? d * p->scale_log2e : -INFINITY;
                const float M = m_all[nb], M2 = fmaxf(M, s_cur);
                const float w_cache = M == -INFINITY ? 0.f : exp2f(M - M2);
                const float pc = s_cur == -INFINITY ? 0.f : exp2f(s_cur - M2);
                const float L2 = l_all[nb] * w_cache + pc;
                const float inv = L2 > 0.f ? 1.f / L2 : 0.f;
                inv_l[nb] = w_cache * inv;
                w_bias[nb] = l_all[nb] * w_cache * inv;
                w_cur[nb] = pc * inv;
            }
        }
        // ---- epilogue: out[head, :] = (O[head, :] / L) . Wl_V[:, col(head) ..] + bias -------------------
        // The slices [rv, d_head] of the decoder matrix (one per KV head of the group, at most four) are
        // fetched into registers now, so that their latency hides under the merge of the waves.  Per KV head:
        // slice -> LDS, transposing loads as B operand, latent sums as hi + lo 16-bit A operands; wave w owns
        // output column blocks w, w + NW, ..
        constexpr int kCpt = 1024 / (64 * NW);                // 16-byte chunks per thread and decoder slice
        const int dh = p->d_head;
        const int ostride = rv + 4;
        float* olat = reinterpret_cast<float*>(lds_raw) + 2 * NW * NHB * 16;
        char* wst = reinterpret_cast<char*>(olat + (size_t)NHB * 16 * ostride);
        const int stride_w = 2 * dh + 32;
        const int cpr = dh >> 3;
        const char* wlv = static_cast<const char*>(g->v.wl);
        int seg_lo[kMaxSeg], seg_hi[kMaxSeg], seg_col[kMaxSeg];
        const int nseg = g->n_vseg;
#pragma unroll
        for (int sg = 0; sg < kMaxSeg; ++sg) { seg_lo[sg] = g->vseg_lo[sg]; seg_hi[sg] = g->vseg_hi[sg]; seg_col[sg] = g->vseg_col[sg]; }
        // query heads of this lane's four result rows in every head block: read now (the group tables sit in the
        // kernel-argument segment, a memory round trip away) rather than inside the loop over the KV heads
        int heads_of[NHB][4];
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) heads_of[nb][v] = nb * 16 + 4 * lg + v < g->n_slots ? (int)g->q_head[nb * 16 + 4 * lg + v] : 0;
        // chunk f of a slice is (row f / cpr, 16-byte piece f % cpr): the same for every KV head, so worked out once, and
        // with a multiplication instead of a division per chunk ((f * inv) >> 16 is exact for f < 8192 when a row has 4, 8,
        // 12 or 16 pieces, i.e. for every head width this kernel takes)
        const unsigned inv_cpr = (65536u + cpr - 1) / cpr;
        int wrow[kCpt], wch[kCpt];
#pragma unroll
        for (int i = 0; i < kCpt; ++i) {
            const unsigned f = i * (64 * NW) + threadIdx.x;
            wrow[i] = (int)((f * inv_cpr) >> 16);
            wch[i] = (int)f - wrow[i] * cpr;
        }
        u32x4_t wreg[kMaxSeg][kCpt];
#pragma unroll
        for (int sg = 0; sg < kMaxSeg; ++sg)
#pragma unroll
            for (int i = 0; i < kCpt; ++i) {
                const int f = i * (64 * NW) + threadIdx.x;
                if (sg < nseg && f < rv * cpr)
                    wreg[sg][i] = *reinterpret_cast<const u32x4_t*>(wlv + ((size_t)wrow[i] * g->v.in_width + seg_col[sg]) * 2 + wch[i] * 16);
            }
        // Merge of the waves' normalised latent sums: every wave parks its scaled accumulators, then each thread
        // adds the waves' copies of its share in wave order (a fixed order: deterministic) and writes the result
        // as olat[slot][rv + 4], which overlays the parked copies once every thread has read its inputs.
        constexpr int kItems = NHB * MB * 64;                  // float4 items of the merged sums
        constexpr int kPerThread = (kItems + 64 * NW - 1) / (64 * NW);
        f32x4_t merged[kArrive ? 1 : kPerThread];
        f32x4_t msum[kJ];                                      // arrival form: the merged sums of this thread's chunks
        if constexpr (kArrive) {
            // Merge of the splits' partials, in split order (deterministic).  What a split's sums are scaled by,
            // 2^(m_split - M) / L per head slot, goes through a second table in LDS: the thread that holds a chunk is not
            // the thread whose lanes hold that slot's M and L.
            const int n_sp = p->n_splits;
            const u32x2_t* ml_tab = reinterpret_cast<const u32x2_t*>(lds_raw + kArriveMlTab);
            float* f_tab = reinterpret_cast<float*>(lds_raw + kArriveFTab);            // [split][slot]
            for (int sp = 4 * wave + lg; sp < n_sp; sp += 4 * NW)
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb) {
                    const float ms = __uint_as_float(ml_tab[sp * NS + nb * 16 + l16][0]);
                    f_tab[sp * NS + nb * 16 + l16] = ms == -INFINITY ? 0.f : exp2f(ms - m_all[nb]) * inv_l[nb];
                }
            __syncthreads();
            const float* pall = p->part + (size_t)b * p->n_splits * p->part_stride + g->part_off;
            const unsigned split_bytes = (unsigned)p->part_stride * 4u;
            const AgentBuf pbuf(pall, (unsigned)(n_sp - 1) * split_bytes + (unsigned)(NS * ostride * 4));
#pragma unroll
            for (int j = 0; j < kJ; ++j) msum[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            for (int s0 = 0; s0 < n_sp; s0 += kAB) {
                if (s0 > 0) arrive_issue(pbuf, s0, n_sp, split_bytes);
#pragma unroll
                for (int u = 0; u < kAB; ++u)
#pragma unroll
                    for (int j = 0; j < kJ; ++j) {
                        const float f = s0 + u < n_sp && mslot[j] < NS ? f_tab[(s0 + u) * NS + mslot[j]] : 0.f;
                        msum[j] += batch_x[u][j] * f;
                    }
            }
        } else {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            // item = (head block nb, column block mb, lane): its lane is this thread's lane, so the factors above apply
            const int item = i * (64 * NW) + threadIdx.x;
            f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
            if (item < kItems) {
                const int nb_i = (item >> 6) / MB;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    float sc = f_wave[w][0] * inv_l[0];
#pragma unroll
                    for (int n2 = 1; n2 < NHB; ++n2) sc = nb_i == n2 ? f_wave[w][n2] * inv_l[n2] : sc;
                    sum += *reinterpret_cast<const f32x4_t*>(lds_raw + w * wave_lds + (size_t)item * 16) * sc;
                }
            }
            merged[i] = sum;
        }
        }
        __syncthreads();
        red = reinterpret_cast<float*>(lds_raw);               // from here on: per-slot weights, merged sums, decoder slices
        if (exact_row && wave == 0 && lane < 16) {             // per-slot weights for the store
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) {
                red[nb * 16 + lane] = w_bias[nb];
                red[NHB * 16 + nb * 16 + lane] = w_cur[nb];
            }
        }
        if constexpr (kArrive) {
#pragma unroll
            for (int j = 0; j < kJ; ++j)
                if (mslot[j] < NS) *reinterpret_cast<f32x4_t*>(olat + (size_t)mslot[j] * ostride + mcol[j]) = msum[j];
        } else {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int item = i * (64 * NW) + threadIdx.x;
            if (item < kItems) {
                const int ln = item & 63, blk = item >> 6, mb = blk % MB, nb = blk / MB;
                *reinterpret_cast<f32x4_t*>(olat + (size_t)(nb * 16 + (ln & 15)) * ostride + 16 * mb + 4 * (ln >> 4)) = merged[i];
            }
        }
        }
        __syncthreads();
        uint16_t* out = static_cast<uint16_t*>(p->out);
#pragma unroll
        for (int sg = 0; sg < kMaxSeg; ++sg) {
            if (sg >= nseg) break;
#pragma unroll
            for (int i = 0; i < kCpt; ++i) {
                const int f = i * (64 * NW) + threadIdx.x;
                if (f < rv * cpr) *reinterpret_cast<u32x4_t*>(wst + wrow[i] * stride_w + wch[i] * 16) = wreg[sg][i];
            }
            __syncthreads();
            const int col = seg_col[sg];
            for (int nb = seg_lo[sg] >> 4; nb <= (seg_hi[sg] - 1) >> 4; ++nb) {
                int heads4[4];                          // query heads of this lane's four result rows
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    heads4[v] = heads_of[0][v];
#pragma unroll
                    for (int n2 = 1; n2 < NHB; ++n2) heads4[v] = nb == n2 ? heads_of[n2][v] : heads4[v];
                }
                for (int nbo = wave; nbo < (dh >> 4); nbo += NW) {
                    f32x4_t o = {0.f, 0.f, 0.f, 0.f};
                    for (int k0 = 0; k0 < rv; k0 += 32) {
                        const float* arow = olat + (size_t)(nb * 16 + l16) * ostride + k0 + 8 * lg;
                        const f32x4_t x0 = *reinterpret_cast<const f32x4_t*>(arow);
                        const f32x4_t x1 = *reinterpret_cast<const f32x4_t*>(arow + 4);
                        const float xv[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
                        unsigned hi[4], lo[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            hi[e] = Mma<E>::pack2(xv[2 * e], xv[2 * e + 1]);
                            lo[e] = Mma<E>::pack2(xv[2 * e] - Mma<E>::unpack_lo(hi[e]), xv[2 * e + 1] - Mma<E>::unpack_hi(hi[e]));
                        }
                        const char* wrow = wst + (k0 + 8 * lg + (l16 >> 2)) * stride_w + (l16 & 3) * 8 + nbo * 32;
                        const s16x4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow));
                        const s16x4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + 4 * stride_w));
                        const u32x2_t a0 = __builtin_bit_cast(u32x2_t, t0), a1 = __builtin_bit_cast(u32x2_t, t1);
                        const u32x4_t bw = {a0[0], a0[1], a1[0], a1[1]};
                        o = Mma<E>::mfma(u32x4_t{hi[0], hi[1], hi[2], hi[3]}, bw, o);
                        o = Mma<E>::mfma(u32x4_t{lo[0], lo[1], lo[2], lo[3]}, bw, o);
                    }
                    const int kcol = nbo * 16 + l16;
                    const float bias = g->v.bl ? Elem<E>::load(g->v.bl, col + kcol) : 0.f;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int slot = nb * 16 + 4 * lg + v;
                        if (slot >= seg_lo[sg] && slot < seg_hi[sg]) {
                            float y = o[v] + bias;
                            if (exact_row)
                                y = o[v] + red[slot] * bias +
                                    red[NHB * 16 + slot] * Elem<E>::load(p->v_cur, ((size_t)b * (p->n_q_heads / p->gq) + heads4[v] / p->gq) * dh + kcol);
                            out[((size_t)b * p->n_q_heads + heads4[v]) * dh + kcol] = Mma<E>::to16(y);
                        }
                    }
                }
            }
            __syncthreads();                             // the slice buffer is rewritten for the next KV head
        }
    }
}

constexpr size_t mfma_lds_bytes(int rmax, int nhb) {
    size_t stage = (size_t)kWaves * (rmax <= 128 ? kWaveTile * (2 * rmax + 16) + kWaveTile * (2 * rmax + 32) : kWaveTile * (2 * rmax + 32));
    size_t merge = (size_t)(2 * kWaves * nhb * 16 + kWaves * nhb * (rmax / 16) * 64 * 4) * sizeof(float);
    return stage > merge ? stage : merge;
}

}  // namespace kvcar
