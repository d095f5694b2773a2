// MFMA attention over the latent cache for TWO-LAYER decoders (gfx950, 16-bit dtypes).
//
// The decoder of the paper is FC -> activation -> FC ("Network Architecture", 2nd paragraph).  Its last
// layer is linear and is absorbed into the query and the output exactly as for a linear decoder, so the
// kernel attends over the hidden rows h_t = act(z_t W1 + b1), which it rebuilds from the latent rows on
// the fly, per tile, never writing them to memory:
//
//   H_K^T[c, t] = W1K^T . Z_K^T     (MFMA)  -> +b1, act -> is the A operand of   S^T[t, head] = H_K . Qt^T
//   H_V [t, c]  = Z_V . W1V         (MFMA)  -> +b1, act -> is the A operand of   O^T[c, head] += H_V^T . P^T
//
// (the result layout of each first product is the operand layout the second one needs, so the hidden
// activations never leave registers).  All products use v_mfma_f32_32x32x16 (on this chip it sustains
// twice the flop rate of the 16x16x32 form, and this kernel is bound by matrix + vector issue): tokens,
// heads and hidden columns are handled in blocks of 32.  The waves of a workgroup (eight, or four for the narrow shape) share a 32-token tile and split the
// hidden width: each keeps its share of W1K and W1V resident in registers as MFMA operands.  Scores
// are a contraction over the whole hidden width, so the per-wave partial scores are summed through LDS
// (each wave adds a share of the entries over the waves, the waves then trade the sums); every wave then
// runs the same online softmax and accumulates its share of O^T.
#include "kvcar_device.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct MMma;
template <> struct MMma<BF16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        bf16x2_t v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(unsigned, v);
    }
};
template <> struct MMma<F16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
        f16x2_t v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(unsigned, v);
    }
};

constexpr int kMlpTile = 32;      // tokens per workgroup iteration

// 32x32 result layout: register v of lane (l32, h) holds row 8*(v/4) + 4*h + v%4 of column l32.  As an
// operand of the next product, k-step s (16 of the 32 rows) is registers 8s..8s+7 of the lane.
template <typename E, int ACT>
__device__ __forceinline__ void act_pack(const f32x16_t& t, float slope, u32x4_t (&out)[2]) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        unsigned w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = MMma<E>::pack2(fast_act<ACT>(t[8 * s + 2 * e], slope), fast_act<ACT>(t[8 * s + 2 * e + 1], slope));
        out[s] = u32x4_t{w[0], w[1], w[2], w[3]};
    }
}

// kI8: the cache holds int8 codes with a scale and a zero point per row ("Quantization", Eq. "quant").  The
// rows are dequantised, x^ = (code - zeropoint) / scale, on their way from the staging registers into LDS and
// rounded there to the model dtype - the precision a 16-bit model holds the dequantised tensor in before
// the decoder - so everything after the park is the 16-bit path.
template <typename E, int R, int C, int ACT, bool kI8, int NW>
__global__ __launch_bounds__(64 * NW, 1) void attend_mlp_mfma_kernel(AttendParams p) {
    constexpr int NT = 64 * NW;        // threads
    constexpr int CW = C / NW;         // hidden columns per wave
    constexpr int MB = CW / 32;        // 32-column blocks per wave
    constexpr int KS = R / 16;         // k-steps over the latent width
    constexpr int STRIDE = 2 * R + 16; // LDS row stride of a latent tile
    constexpr int EB = kI8 ? 1 : 2;    // bytes per cached latent element
    constexpr int CPR = R * EB / 16;   // 16-byte chunks per cached row
    constexpr int NLD = (kMlpTile * CPR) / NT > 0 ? (kMlpTile * CPR) / NT : 1;         // 16-byte chunks per thread per tile
    static_assert(CW % 32 == 0 && R % 16 == 0, "shape");

    extern __shared__ __attribute__((aligned(16))) char lds[];
    // two buffers of a K tile + a V tile (the next tile is parked at the end of the current one), then the score exchange
    float* sbuf = reinterpret_cast<float*>(lds + 4 * kMlpTile * STRIDE);    // partial scores [wave][4 chunks][64 lanes][4]
    float* stot = sbuf + NW * 64 * 16;                                      // their sums [4 chunks][64 lanes][4]

    const GroupDesc& g = p.g[blockIdx.z];
    const int split = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int l16 = lane & 15;
    const int cw0 = wave * CW;
    const float slope = g.k.slope;

    // ---- resident operands ----------------------------------------------------------------------
    // W1K^T as A operand (row = hidden column, k = 8 consecutive latent indices) and W1V as B operand
    // (column = hidden column, same k): both are "8 consecutive rows of one column" of the row-major
    // [R, C] matrix.  The matrix goes through LDS once (coalesced 16-byte loads) and the transposing load
    // hands every lane its column: 16 lanes supply a 4-row x 16-column patch, lane i gets column i.
    u32x4_t wk[MB][KS], wv[MB][KS];
    {
        constexpr int WSTRIDE = 2 * C + 32;
        typedef __attribute__((ext_vector_type(4))) short s16x4_t;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const char* w1 = static_cast<const char*>(which == 0 ? g.k.w1 : g.v.w1);
            __syncthreads();
            for (int f = tid; f < R * (C / 8); f += NT) {
                const int row = f / (C / 8), ch = f % (C / 8);
                *reinterpret_cast<u32x4_t*>(lds + row * WSTRIDE + ch * 16) = *reinterpret_cast<const u32x4_t*>(w1 + (size_t)f * 16);
            }
            __syncthreads();
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const char* src = lds + (16 * ks + 8 * h + (l16 >> 2)) * WSTRIDE + (cw0 + 32 * mb + 16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
                    const s16x4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(src));
                    const s16x4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(src + 4 * WSTRIDE));
                    const u32x2_t a0 = __builtin_bit_cast(u32x2_t, t0), a1 = __builtin_bit_cast(u32x2_t, t1);
                    const u32x4_t v = {a0[0], a0[1], a1[0], a1[1]};
                    if (which == 0) wk[mb][ks] = v; else wv[mb][ks] = v;
                }
        }
        __syncthreads();          // the staging area becomes the tile and score buffers
    }
    // first-layer biases in the two result layouts (rows of H_K^T, column of H_V)
    float bk[MB][16], bv[MB][16];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float bcol = g.v.b1 ? Elem<E>::load(g.v.b1, cw0 + 32 * mb + l32) : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            bk[mb][v] = g.k.b1 ? Elem<E>::load(g.k.b1, cw0 + 32 * mb + 8 * (v >> 2) + 4 * h + (v & 3)) : 0.f;
            bv[mb][v] = bcol;
        }
    }
    // absorbed queries of this wave's hidden slice as B operand (column = head l32; padding heads are
    // zero rows of qt): k-slots of lane half h in k-step s of block mb are the hidden columns
    // 16s + 4h + j and 16s + 8 + 4h + j, which is what the H_K^T result layout delivers
    u32x4_t qb[MB][2];
    {
        const char* qt = static_cast<const char*>(p.qt) + ((size_t)b * p.qt_stride + g.qt_off) * 2;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (l32 < g.slots_pad) {
                    const char* row = qt + ((size_t)l32 * C + cw0 + 32 * mb + 16 * s + 4 * h) * 2;
                    const u32x2_t x0 = *reinterpret_cast<const u32x2_t*>(row);
                    const u32x2_t x1 = *reinterpret_cast<const u32x2_t*>(row + 16);
                    v = u32x4_t{x0[0], x0[1], x1[0], x1[1]};
                }
                qb[mb][s] = v;
            }
    }

    f32x16_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int n_ctx = p.seq_lens ? min(p.seq_lens[b], p.n_ctx) : p.n_ctx;      // ragged batches: one length per sequence
    const int tiles = (n_ctx + kMlpTile - 1) / kMlpTile;
    const int per_split = (tiles + p.n_splits - 1) / p.n_splits;
    const int j0 = split * per_split;
    const int j1 = min(tiles, j0 + per_split);
    const char* zk = static_cast<const char*>(g.k.z) + (size_t)b * p.max_seq * R * EB;
    const char* zv = static_cast<const char*>(g.v.z) + (size_t)b * p.max_seq * R * EB;
    const RowMeta* mk = static_cast<const RowMeta*>(g.k.meta) + (size_t)b * p.max_seq;     // int8 rows only
    const RowMeta* mv = static_cast<const RowMeta*>(g.v.meta) + (size_t)b * p.max_seq;

    // tile chunks of this thread: chunk f = i*256 + tid of the contiguous [32, R] tile
    u32x4_t stk[NLD], stv[NLD];
    u32x2_t smk[NLD], smv[NLD];        // int8: {scale, zeropoint} of the row each chunk belongs to
    auto issue = [&](int j) {
        const int t0 = j * kMlpTile;
        const int valid = max(0, min(kMlpTile, n_ctx - t0)) * CPR;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = i * NT + tid;
            u32x4_t a = {0u, 0u, 0u, 0u}, c2 = {0u, 0u, 0u, 0u};
            smk[i] = smv[i] = u32x2_t{0x3f800000u, 0u};
            if (f < valid) {
                a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(zk + (size_t)t0 * R * EB + (size_t)f * 16));
                c2 = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(zv + (size_t)t0 * R * EB + (size_t)f * 16));
                if constexpr (kI8) {
                    smk[i] = *reinterpret_cast<const u32x2_t*>(mk + t0 + f / CPR);
                    smv[i] = *reinterpret_cast<const u32x2_t*>(mv + t0 + f / CPR);
                }
            }
            stk[i] = a; stv[i] = c2;
        }
    };
    // 16 codes -> 16 dequantised values in the model dtype (two 16-byte halves)
    auto dequant = [&](const u32x4_t c, const u32x2_t m, u32x4_t& lo, u32x4_t& hi) {
        const float inv = 1.f / __uint_as_float(m[0]);
        const float sub = (128.f + (float)(int)m[1]) * inv;         // codes are read as unsigned bytes code + 128
        unsigned w[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned x = c[i] ^ 0x80808080u;
            const float f0 = fmaf((float)(x & 0xffu), inv, -sub), f1 = fmaf((float)((x >> 8) & 0xffu), inv, -sub);
            const float f2 = fmaf((float)((x >> 16) & 0xffu), inv, -sub), f3 = fmaf((float)(x >> 24), inv, -sub);
            w[2 * i] = MMma<E>::pack2(f0, f1);
            w[2 * i + 1] = MMma<E>::pack2(f2, f3);
        }
        lo = u32x4_t{w[0], w[1], w[2], w[3]};
        hi = u32x4_t{w[4], w[5], w[6], w[7]};
    };
    auto park = [&](int buf) {
        char* tile_k = lds + buf * 2 * kMlpTile * STRIDE;
        char* tile_v = tile_k + kMlpTile * STRIDE;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = i * NT + tid;
            if (f < kMlpTile * CPR) {
                const int row = f / CPR, ch = f % CPR;
                if constexpr (kI8) {
                    u32x4_t lo, hi;
                    dequant(stk[i], smk[i], lo, hi);
                    *reinterpret_cast<u32x4_t*>(tile_k + row * STRIDE + ch * 32) = lo;
                    *reinterpret_cast<u32x4_t*>(tile_k + row * STRIDE + ch * 32 + 16) = hi;
                    dequant(stv[i], smv[i], lo, hi);
                    *reinterpret_cast<u32x4_t*>(tile_v + row * STRIDE + ch * 32) = lo;
                    *reinterpret_cast<u32x4_t*>(tile_v + row * STRIDE + ch * 32 + 16) = hi;
                } else {
                    *reinterpret_cast<u32x4_t*>(tile_k + row * STRIDE + ch * 16) = stk[i];
                    *reinterpret_cast<u32x4_t*>(tile_v + row * STRIDE + ch * 16) = stv[i];
                }
            }
        }
    };
    if (j0 < j1) {
        issue(j0);
        park(0);
        if (j0 + 1 < j1) issue(j0 + 1);
    }
    __syncthreads();

    for (int j = j0; j < j1; ++j) {
        const int nv = min(kMlpTile, n_ctx - j * kMlpTile);
        const char* tile_k = lds + ((j - j0) & 1) * 2 * kMlpTile * STRIDE;
        const char* tile_v = tile_k + kMlpTile * STRIDE;

        // ---- H_K^T for this wave's hidden slice, then partial scores ------------------------------
        // One wave per SIMD: matrix and vector instructions only overlap if they alternate in program
        // order, so the MFMA chain of the next block is placed under the activations of the previous one.
        f32x16_t sT;
#pragma unroll
        for (int v = 0; v < 16; ++v) sT[v] = 0.f;
        {
            u32x4_t zb[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) zb[ks] = *reinterpret_cast<const u32x4_t*>(tile_k + l32 * STRIDE + (2 * ks + h) * 16);
            f32x16_t hk[MB];
            // the products start from the first-layer bias: no addition per hidden value afterwards
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) hk[mb][v] = bk[mb][v];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) hk[0] = MMma<E>::mfma(wk[0][ks], zb[ks], hk[0]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (mb + 1 < MB) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) hk[mb + 1] = MMma<E>::mfma(wk[mb + 1][ks], zb[ks], hk[mb + 1]);
                }
                u32x4_t ha[2];
                act_pack<E, ACT>(hk[mb], slope, ha);       // lane: token l32, hidden rows of block mb
                if (mb + 1 < MB) {
#pragma unroll
                    for (int i = 0; i < KS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x002, 24, 0);    // then vector work
                    }
                }
#pragma unroll
                for (int s = 0; s < 2; ++s) sT = MMma<E>::mfma(ha[s], qb[mb][s], sT);
            }
        }
        // ---- sum the partial scores of the waves, in wave order.  Every wave needs all 16 sums of its lanes; a wave
        // adds 16 / NW of them over the waves and the waves trade the sums (each adding all of them itself costs
        // NW * 16 additions and LDS words per lane and tile) ---------------------------------------------------------
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<f32x4_t*>(sbuf + ((size_t)(wave * 4 + q) * 64 + lane) * 4) = f32x4_t{sT[4 * q], sT[4 * q + 1], sT[4 * q + 2], sT[4 * q + 3]};
        __syncthreads();
        {
            constexpr int EPW = 16 / NW;                       // entries per wave: 2 (eight waves) or 4 (four)
            const int e0 = wave * EPW;                         // entries e0 .. e0 + EPW - 1 = part of chunk e0 / 4
            float t[EPW];
#pragma unroll
            for (int e = 0; e < EPW; ++e) t[e] = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float* src = sbuf + ((size_t)(w * 4 + (e0 >> 2)) * 64 + lane) * 4 + (e0 & 3);
                if constexpr (EPW == 2) {
                    const f32x2_t x = *reinterpret_cast<const f32x2_t*>(src);
                    t[0] += x[0]; t[1] += x[1];
                } else {
                    const f32x4_t x = *reinterpret_cast<const f32x4_t*>(src);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] += x[e];
                }
            }
            float* dst = stot + ((size_t)(e0 >> 2) * 64 + lane) * 4 + (e0 & 3);
            if constexpr (EPW == 2) *reinterpret_cast<f32x2_t*>(dst) = f32x2_t{t[0], t[1]};
            else *reinterpret_cast<f32x4_t*>(dst) = f32x4_t{t[0], t[1], t[2], t[3]};
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4_t s4 = *reinterpret_cast<const f32x4_t*>(stot + ((size_t)q * 64 + lane) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) sT[4 * q + e] = s4[e];
        }
        if (nv < kMlpTile) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + 4 * h + (v & 3) >= nv) sT[v] = -INFINITY;
        }

        // ---- online softmax (identical in every wave); lane holds head l32, 16 of the 32 tokens ------
        u32x4_t pb[2];
        {
            float mx = sT[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sT[v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            const bool rescale = m_new != m_run;
            m_run = m_new;
            float e[16], sum = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) { e[v] = __builtin_amdgcn_exp2f(sT[v] - m_new); sum += e[v]; }
            l_run = l_run * alpha + sum;
#pragma unroll
            for (int s = 0; s < 2; ++s)
                pb[s] = u32x4_t{MMma<E>::pack2(e[8 * s], e[8 * s + 1]), MMma<E>::pack2(e[8 * s + 2], e[8 * s + 3]),
                                MMma<E>::pack2(e[8 * s + 4], e[8 * s + 5]), MMma<E>::pack2(e[8 * s + 6], e[8 * s + 7])};
            if (__builtin_amdgcn_ballot_w64(rescale) != 0) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb] *= alpha;
            }
        }

        // ---- H_V for this wave's hidden slice, then O^T += H_V^T . P^T ------------------------------
        {
            u32x4_t za[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) za[ks] = *reinterpret_cast<const u32x4_t*>(tile_v + l32 * STRIDE + (2 * ks + h) * 16);
            f32x16_t hv[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) hv[mb][v] = bv[mb][v];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) hv[0] = MMma<E>::mfma(za[ks], wv[0][ks], hv[0]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (mb + 1 < MB) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) hv[mb + 1] = MMma<E>::mfma(za[ks], wv[mb + 1][ks], hv[mb + 1]);
                }
                u32x4_t va[2];
                act_pack<E, ACT>(hv[mb], slope, va);       // lane: hidden column l32 of block mb, 16 tokens
                if (mb + 1 < MB) {
#pragma unroll
                    for (int i = 0; i < KS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 24, 0);
                    }
                }
#pragma unroll
                for (int s = 0; s < 2; ++s) acc[mb] = MMma<E>::mfma(va[s], pb[s], acc[mb]);
            }
        }
        // the next tile goes into the other buffer (its loads were issued one tile ago; that buffer was last read
        // one tile ago, before the previous end-of-tile barrier)
        if (j + 1 < j1) {
            park(((j - j0) & 1) ^ 1);
            if (j + 2 < j1) issue(j + 2);
        }
        __syncthreads();          // the score buffer is rewritten by the next iteration, which reads the tile just parked
    }

    // ---- partial: every wave owns its hidden slice; m and l are the same in all of them ------------------
    l_run += __shfl_xor(l_run, 32);
    float* part = p.part + ((size_t)b * p.n_splits + split) * p.part_stride + g.part_off;
    constexpr int PSTRIDE = C + 4;
    if (l32 < g.slots_pad) {
        if (wave == 0 && h == 0) { part[(size_t)l32 * PSTRIDE] = m_run; part[(size_t)l32 * PSTRIDE + 1] = l_run; }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<f32x4_t*>(part + (size_t)l32 * PSTRIDE + 4 + cw0 + 32 * mb + 8 * a + 4 * h) =
                    f32x4_t{acc[mb][4 * a], acc[mb][4 * a + 1], acc[mb][4 * a + 2], acc[mb][4 * a + 3]};
    }
}

// Waves per workgroup: the hidden width is split over them in 32-column blocks; eight for the 256-wide shape
// (two waves per SIMD: a wave alone issues vector instructions at half the SIMD's rate), four for the 128-wide one.
template <int C> struct MlpWaves { static constexpr int value = C >= 256 ? 8 : 4; };

template <typename E, int R, int C, bool kI8>
static hipError_t launch_mlp(const AttendParams& p, int act, hipStream_t stream) {
    constexpr int NW = MlpWaves<C>::value;
    const size_t loop_lds = 4 * (size_t)kMlpTile * (2 * R + 16) + (size_t)(NW + 1) * 64 * 16 * sizeof(float);
    const size_t stage_lds = (size_t)R * (2 * C + 32);            // first-layer weights pass through LDS at start
    const size_t lds = loop_lds > stage_lds ? loop_lds : stage_lds;
    dim3 grid(p.n_splits, p.batch, p.n_groups);
    static AttrFlag attr[2] = {false, false};
    auto kg = attend_mlp_mfma_kernel<E, R, C, KVCAR_ACT_GELU, kI8, NW>;
    auto kl = attend_mlp_mfma_kernel<E, R, C, KVCAR_ACT_LEAKY_RELU, kI8, NW>;
    const int ai = act == KVCAR_ACT_GELU ? 0 : 1;
    if (!attr[ai]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ai == 0 ? kg : kl), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr[ai] = true;
    }
    if (ai == 0) hipLaunchKernelGGL(kg, grid, dim3(64 * NW), lds, stream, p);
    else hipLaunchKernelGGL(kl, grid, dim3(64 * NW), lds, stream, p);
    return hipGetLastError();
}

// Shapes with a resident-weight instance: every group has the same (latent, hidden) widths for K and V,
// (128, 256) or (64, 128), the same activation, and at most 32 heads.
bool attend_mlp_mfma_supported(const AttendParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.n_groups < 1) return false;
    const GroupDesc& g0 = p.g[0];
    for (int i = 0; i < p.n_groups; ++i) {
        const GroupDesc& g = p.g[i];
        if (!g.k.w1 || !g.v.w1) return false;
        if (g.k.r != g0.k.r || g.v.r != g0.k.r || g.k.c != g0.k.c || g.v.c != g0.k.c) return false;
        if (g.k.act != g0.k.act || g.v.act != g0.k.act || g.k.slope != g0.k.slope || g.v.slope != g0.k.slope) return false;
        if (g.slots_pad > 32) return false;
    }
    if (g0.k.act != KVCAR_ACT_GELU && g0.k.act != KVCAR_ACT_LEAKY_RELU) return false;
    return (g0.k.r == 128 && g0.k.c == 256) || (g0.k.r == 64 && g0.k.c == 128);
}

hipError_t launch_attend_mlp_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    const int act = p.g[0].k.act;
    const bool big = p.g[0].k.r == 128;
    const bool i8 = p.g[0].k.meta != nullptr;
    if (dtype == KVCAR_BF16) {
        if (i8) return big ? launch_mlp<BF16, 128, 256, true>(p, act, stream) : launch_mlp<BF16, 64, 128, true>(p, act, stream);
        return big ? launch_mlp<BF16, 128, 256, false>(p, act, stream) : launch_mlp<BF16, 64, 128, false>(p, act, stream);
    }
    if (i8) return big ? launch_mlp<F16, 128, 256, true>(p, act, stream) : launch_mlp<F16, 64, 128, true>(p, act, stream);
    return big ? launch_mlp<F16, 128, 256, false>(p, act, stream) : launch_mlp<F16, 64, 128, false>(p, act, stream);
}

}  // namespace kvcar
