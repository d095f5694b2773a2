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
};

constexpr int kWaveTile = 32;     // tokens per wave per iteration
constexpr int kWaves = 4;

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
    __device__ explicit DimsExact(const GroupDesc&) {}
};
template <int RMAX_, int NHB_> struct DimsAny {
    static constexpr int RMAX = RMAX_, NHB = NHB_;
    static constexpr bool kExact = false;
    int rk, rv, nhb;
    __device__ explicit DimsAny(const GroupDesc& g) : rk(g.k.r), rv(g.v.r), nhb(g.slots_pad >> 4) {}
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

template <typename E, typename D>
__device__ __forceinline__ void attend_body(const AttendParams& p, const GroupDesc& g, char* lds_raw, size_t wave_lds) {
    constexpr int RMAX = D::RMAX, NHB = D::NHB;
    using G = Geo<RMAX>;
    constexpr int KS = RMAX / 32;      // k-steps of the score product
    constexpr int MB = RMAX / 16;      // 16-column blocks of the latent accumulator
    constexpr int NL = RMAX / 16;      // 128-bit loads per lane per tile

    const D d(g);
    const int split = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;

    const int rk = d.rk, rv = d.rv, nhb = d.nhb;
    const int ksteps = rk >> 5, mblocks = rv >> 4;
    const int nlk = rk >> 4, nlv = rv >> 4;
    const int cprk = rk >> 3, cprv = rv >> 3;
    const int stride_k = 2 * rk + 16, stride_v = 2 * rv + 32;

    char* my_lds = lds_raw + wave * wave_lds;
    char* lds_k = my_lds;
    char* lds_v = G::kPrefetch ? my_lds + kWaveTile * stride_k : my_lds;

    // absorbed queries of this sequence and group, resident as MFMA B operands
    u32x4_t qb[NHB][KS];
    {
        const char* qt = static_cast<const char*>(p.qt) + ((size_t)b * p.qt_stride + g.qt_off) * 2;
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (nb < nhb && s < ksteps) v = *reinterpret_cast<const u32x4_t*>(qt + ((size_t)(nb * 16 + l16) * rk + 8 * (4 * s + lg)) * 2);
                qb[nb][s] = v;
            }
    }

    f32x4_t acc[NHB][MB];
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run[NHB], l_run[NHB];
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) { m_run[nb] = -INFINITY; l_run[nb] = 0.f; }

    // Workgroup tiles (4 wave tiles = 128 tokens each) of this split.  tile_order 0: a contiguous
    // token range per split; 1: tiles dealt round-robin over the splits, so that workgroups running
    // at the same time read neighbouring addresses.
    const int wg_tiles = (p.n_ctx + kWaveTile * kWaves - 1) / (kWaveTile * kWaves);
    int j0, j1, jstep;
    if (p.tile_order == 0) {
        const int per_split = (wg_tiles + p.n_splits - 1) / p.n_splits;
        j0 = split * per_split;
        j1 = min(wg_tiles, j0 + per_split);
        jstep = 1;
    } else {
        j0 = split; j1 = wg_tiles; jstep = p.n_splits;
    }

    const char* zk = static_cast<const char*>(g.k.z) + (size_t)b * p.max_seq * rk * 2;
    const char* zv = static_cast<const char*>(g.v.z) + (size_t)b * p.max_seq * rv * 2;

    // kPrefetch: both tiles of the next iteration are in flight while this one computes.
    // Otherwise (wide rows) a tile is loaded right before it is parked and K, V take turns.
    u32x4_t stk[NL], stv[G::kPrefetch ? NL : 1];
    auto issue = [&](int j) {
        const int t0 = (j * kWaves + wave) * kWaveTile;
        const int nv = max(0, min(kWaveTile, p.n_ctx - t0));
        load_tile<NL>(stk, zk + (size_t)t0 * rk * 2, nlk, nv * cprk, nv == kWaveTile, lane);
        if constexpr (G::kPrefetch) load_tile<NL>(stv, zv + (size_t)t0 * rv * 2, nlv, nv * cprv, nv == kWaveTile, lane);
    };
    if (G::kPrefetch && j0 < j1) issue(j0);

    for (int j = j0; j < j1; j += jstep) {
        const int t0 = (j * kWaves + wave) * kWaveTile;
        const int nv = min(kWaveTile, p.n_ctx - t0);
        if (nv <= 0) break;          // wave tile past the context: only in the last workgroup tile, the last one visited

        if constexpr (!G::kPrefetch) issue(j);
        park_tile<NL>(stk, lds_k, nlk, cprk, stride_k, lane);
        if constexpr (G::kPrefetch) {
            park_tile<NL>(stv, lds_v, nlv, cprv, stride_v, lane);
            if (j + jstep < j1) issue(j + jstep);
        }

        // ---- scores: S^T[token, head] ------------------------------------------------------
        f32x4_t sT[2][NHB];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb) sT[a][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        const char* krow = lds_k + l16 * stride_k + lg * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s < ksteps) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const u32x4_t ka = *reinterpret_cast<const u32x4_t*>(krow + a * 16 * stride_k + s * 64);
#pragma unroll
                    for (int nb = 0; nb < NHB; ++nb)
                        if (nb < nhb) sT[a][nb] = Mma<E>::mfma(ka, qb[nb][s], sT[a][nb]);
                }
            }
        }
        if constexpr (!G::kPrefetch) {
            // K and V share the staging registers and the LDS region: V rows replace K rows
            // (LDS operations of one wave complete in order, so the score reads are done)
            load_tile<NL>(stk, zv + (size_t)t0 * rv * 2, nlv, nv * cprv, nv == kWaveTile, lane);
            park_tile<NL>(stk, lds_v, nlv, cprv, stride_v, lane);
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
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[nb], mx);
            alpha[nb] = __builtin_amdgcn_exp2f(m_run[nb] - m_new);     // m_run = -inf on the first tile gives 0
            rescale |= m_new != m_run[nb];
            m_run[nb] = m_new;
            float e[8];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                e[v] = __builtin_amdgcn_exp2f(sT[0][nb][v] - m_new);
                e[4 + v] = __builtin_amdgcn_exp2f(sT[1][nb][v] - m_new);
            }
            l_run[nb] = l_run[nb] * alpha[nb] + ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
            pb[nb] = u32x4_t{Mma<E>::pack2(e[0], e[1]), Mma<E>::pack2(e[2], e[3]), Mma<E>::pack2(e[4], e[5]), Mma<E>::pack2(e[6], e[7])};
        }
        // the running maxima settle after a few tiles; rescale the accumulators only when one moved
        if (__builtin_amdgcn_ballot_w64(rescale) != 0) {
#pragma unroll
            for (int nb = 0; nb < NHB; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    if (nb < nhb && mb < mblocks) acc[nb][mb] *= alpha[nb];
        }

        // ---- O^T[latent col, head] += Z_V^T . P^T --------------------------------------------
        // 16 lanes of a block supply the addresses of a 4-token x 16-column patch; the transposing
        // load hands lane i its column i for the 4 tokens
        const char* vrow = lds_v + (4 * lg + (l16 >> 2)) * stride_v + (l16 & 3) * 8;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (mb < mblocks) {
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vrow + mb * 32));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(vrow + mb * 32 + 16 * stride_v));
                const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
                const u32x4_t va = {lo2[0], lo2[1], hi2[0], hi2[1]};
#pragma unroll
                for (int nb = 0; nb < NHB; ++nb)
                    if (nb < nhb) acc[nb][mb] = Mma<E>::mfma(va, pb[nb], acc[nb][mb]);
            }
        }
    }

    // ---- merge the four waves and write one partial --------------------------------------------
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        l_run[nb] += __shfl_xor(l_run[nb], 16);
        l_run[nb] += __shfl_xor(l_run[nb], 32);
    }
    __syncthreads();                                   // every wave is done with its staging region
    float* red = reinterpret_cast<float*>(lds_raw);    // [wave][NHB*16] m, then l
    float* accs = reinterpret_cast<float*>(lds_raw) + 2 * kWaves * NHB * 16;   // [wave][NHB][MB][64][4]
    if (lane < 16) {
#pragma unroll
        for (int nb = 0; nb < NHB; ++nb) {
            red[wave * NHB * 16 + nb * 16 + lane] = m_run[nb];
            red[kWaves * NHB * 16 + wave * NHB * 16 + nb * 16 + lane] = l_run[nb];
        }
    }
    __syncthreads();
    float m_all[NHB], l_all[NHB];
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, red[w * NHB * 16 + nb * 16 + l16]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = red[w * NHB * 16 + nb * 16 + l16];
            L += mw == -INFINITY ? 0.f : red[kWaves * NHB * 16 + w * NHB * 16 + nb * 16 + l16] * exp2f(mw - M);
        }
        const float f = m_run[nb] == -INFINITY ? 0.f : exp2f(m_run[nb] - M);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            if (mb < mblocks && nb < nhb)
                *reinterpret_cast<f32x4_t*>(accs + ((size_t)((wave * NHB + nb) * MB + mb) * 64 + lane) * 4) = acc[nb][mb] * f;
        m_all[nb] = M;
        l_all[nb] = L;
    }
    __syncthreads();
    float* part = p.part + ((size_t)b * p.n_splits + split) * p.part_stride + g.part_off;
    const int pstride = rv + 4;
#pragma unroll
    for (int nb = 0; nb < NHB; ++nb) {
        if (nb >= nhb) continue;
        const int slot = nb * 16 + l16;
        if (wave == 0 && lane < 16) { part[(size_t)slot * pstride] = m_all[nb]; part[(size_t)slot * pstride + 1] = l_all[nb]; }
        // 16-column blocks are shared out over the four waves
        for (int mb = wave; mb < mblocks; mb += kWaves) {
            f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += *reinterpret_cast<const f32x4_t*>(accs + ((size_t)((w * NHB + nb) * MB + mb) * 64 + lane) * 4);
            *reinterpret_cast<f32x4_t*>(part + (size_t)slot * pstride + 4 + 16 * mb + 4 * lg) = s;
        }
    }
}

constexpr size_t mfma_lds_bytes(int rmax, int nhb) {
    size_t stage = (size_t)kWaves * (rmax <= 128 ? kWaveTile * (2 * rmax + 16) + kWaveTile * (2 * rmax + 32) : kWaveTile * (2 * rmax + 32));
    size_t merge = (size_t)(2 * kWaves * nhb * 16 + kWaves * nhb * (rmax / 16) * 64 * 4) * sizeof(float);
    return stage > merge ? stage : merge;
}

// Latent widths up to 128 (TinyLlama-class KV widths): up to two 16-head blocks per group.
template <typename E>
__global__ __launch_bounds__(256, 2) void attend_mfma_r128_kernel(AttendParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const GroupDesc& g = p.g[blockIdx.z];
    constexpr size_t wl = Geo<128>::kWaveLds;
    const int nhb = g.slots_pad >> 4;
    if (g.k.r == g.v.r) {
        const int key = g.k.r * 4 + nhb;
        switch (key) {
            case 128 * 4 + 2: attend_body<E, DimsExact<128, 2>>(p, g, lds_raw, wl); return;
            case 128 * 4 + 1: attend_body<E, DimsExact<128, 1>>(p, g, lds_raw, wl); return;
            case 96 * 4 + 2: attend_body<E, DimsExact<96, 2>>(p, g, lds_raw, wl); return;
            case 96 * 4 + 1: attend_body<E, DimsExact<96, 1>>(p, g, lds_raw, wl); return;
            case 64 * 4 + 2: attend_body<E, DimsExact<64, 2>>(p, g, lds_raw, wl); return;
            case 64 * 4 + 1: attend_body<E, DimsExact<64, 1>>(p, g, lds_raw, wl); return;
            case 32 * 4 + 2: attend_body<E, DimsExact<32, 2>>(p, g, lds_raw, wl); return;
            case 32 * 4 + 1: attend_body<E, DimsExact<32, 1>>(p, g, lds_raw, wl); return;
            default: break;
        }
    }
    attend_body<E, DimsAny<128, 2>>(p, g, lds_raw, wl);
}

// Latent widths up to 384 (GPT-2-class KV widths): one 16-head block per group.
template <typename E>
__global__ __launch_bounds__(256, 1) void attend_mfma_r384_kernel(AttendParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const GroupDesc& g = p.g[blockIdx.z];
    constexpr size_t wl = Geo<384>::kWaveLds;
    if (g.k.r == g.v.r && g.k.r == 384) { attend_body<E, DimsExact<384, 1>>(p, g, lds_raw, wl); return; }
    if (g.k.r == g.v.r && g.k.r == 288) { attend_body<E, DimsExact<288, 1>>(p, g, lds_raw, wl); return; }
    attend_body<E, DimsAny<384, 1>>(p, g, lds_raw, wl);
}

template <typename K>
static hipError_t launch_one(K kern, size_t lds, const AttendParams& p, hipStream_t stream, bool& attr_set) {
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(p.n_splits, p.batch, p.n_groups);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

bool attend_mfma_available() { return true; }

hipError_t launch_attend_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    static bool set128[2] = {false, false}, set384[2] = {false, false};
    int rmax = 0, nhb = 1;
    for (int i = 0; i < p.n_groups; ++i) {
        rmax = p.g[i].k.r > rmax ? p.g[i].k.r : rmax;
        rmax = p.g[i].v.r > rmax ? p.g[i].v.r : rmax;
        nhb = p.g[i].slots_pad / 16 > nhb ? p.g[i].slots_pad / 16 : nhb;
    }
    const int e = dtype == KVCAR_BF16 ? 0 : 1;
    if (rmax <= 128 && nhb <= 2) {
        constexpr size_t lds = mfma_lds_bytes(128, 2);
        return e == 0 ? launch_one(attend_mfma_r128_kernel<BF16>, lds, p, stream, set128[0])
                      : launch_one(attend_mfma_r128_kernel<F16>, lds, p, stream, set128[1]);
    }
    if (rmax <= 384 && nhb == 1) {
        constexpr size_t lds = mfma_lds_bytes(384, 1);
        return e == 0 ? launch_one(attend_mfma_r384_kernel<BF16>, lds, p, stream, set384[0])
                      : launch_one(attend_mfma_r384_kernel<F16>, lds, p, stream, set384[1]);
    }
    return hipErrorNotSupported;
}

}  // namespace kvcar
