// MFMA encode + append of MANY tokens through a linear encoder (gfx950, 16-bit dtypes): the prompt phase,
// where the encoder placed after K/V generation ("Network Architecture", first paragraph) sees every prompt
// token of every sequence at once and the kernel is a stream: 2 d_kv bytes in and 2 r (or r + 8) bytes out
// per token and tensor, against 2 in r multiply-adds.
//
// One workgroup = 8 waves on one compute unit, for one tensor (K or V).  The encoder matrix [in, r] is staged
// into LDS once per workgroup; after that the waves never meet again.  Each wave walks its own 16-token tiles:
//   1. the tile's input rows arrive by fully coalesced 16-byte loads (two tiles ahead, in registers) and are
//      parked in the wave's private LDS region (padded rows),
//   2. z[16 tokens, r] = x W  on v_mfma_f32_16x16x32 (A = token rows from LDS, B = the matrix by transposing
//      LDS loads),
//   3. bias, one rounding to the cache dtype (or the int8 quantiser of "Quantization", Eq. "quant", over the
//      whole row), back through the same LDS region so that the latent rows leave as 16-byte stores.
// LDS operations of one wave complete in order, so the region needs no barrier between its three uses.
#include "kvcar_device.hpp"

namespace kvcar {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct BulkMma;
template <> struct BulkMma<BF16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        bf16x2_t v = {(__bf16)lo, (__bf16)hi};          // round to nearest even
        return __builtin_bit_cast(unsigned, v);
    }
};
template <> struct BulkMma<F16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
        f16x2_t v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(unsigned, v);
    }
};

constexpr int kBulkWaves = 8;
constexpr int kBulkRows = 16;                          // tokens per wave tile
constexpr int kBulkTile = kBulkWaves * kBulkRows;      // tokens per workgroup iteration
constexpr int kBulkMaxKs = 8;                          // input width up to 256: 16-byte chunks per lane and tile
constexpr int kBulkAhead = 2;                          // tiles in flight per wave (3 and 4 measured the same)
constexpr int kBulkMinTokens = 8192;                   // below this the launch cannot fill the chip with whole workgroups
constexpr size_t kBulkLdsMax = 160 * 1024;

__host__ __device__ constexpr int bulk_stride_w(int r) { return 2 * r + 32; }
__host__ __device__ constexpr int bulk_region(int in_w, int r) { return kBulkRows * (2 * (in_w > r ? in_w : r) + 16); }

// NB: 16-column blocks of the latent (r == 16 NB exactly, NB even).
template <typename E, int NB, bool kI8>
__global__ __launch_bounds__(64 * kBulkWaves, 1) void encode_bulk_kernel(EncodeParams p, int side0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const EncodeSide& s = p.s[blockIdx.y + side0];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    constexpr int r = 16 * NB;
    const int in_w = s.in_width, ks = in_w >> 5, cpr = in_w >> 3;
    const int n_tok = p.batch * p.t_new;
    const int n_tiles = (n_tok + kBulkTile - 1) / kBulkTile;
    const int stride_w = bulk_stride_w(r), stride_x = 2 * in_w + 16;
    char* wbuf = lds;
    char* reg = lds + (size_t)in_w * stride_w + (size_t)wave * bulk_region(in_w, r);

    // this lane's chunks of a tile: chunk f = i * 64 + lane is 16 bytes of row f / cpr of the gathered input
    // (the columns of the KV heads the layer stores, 8 consecutive ones never straddling a head).  Source offsets
    // are relative to the tile's first row, so that a tile costs one 64-bit base and no per-chunk multiply.
    const int x_stride = p.d_kv * 2;
    int c_row[kBulkMaxKs], c_src[kBulkMaxKs], c_dst[kBulkMaxKs];
#pragma unroll
    for (int i = 0; i < kBulkMaxKs; ++i) {
        const int f = i * 64 + lane;
        const int row = f / cpr, col = (f - row * cpr) * 8;
        c_row[i] = row;
        c_src[i] = row * x_stride + ((int)s.heads[col / p.d_head] * p.d_head + col % p.d_head) * 2;
        c_dst[i] = row * stride_x + col * 2;
    }
    const char* x = static_cast<const char*>(s.x);
    auto issue = [&](u32x4_t (&st)[kBulkMaxKs], int tile) {
        const int t0 = tile * kBulkTile + wave * kBulkRows;
        const char* base = x + (size_t)t0 * x_stride;
        if (t0 + kBulkRows <= n_tok) {
#pragma unroll
            for (int i = 0; i < kBulkMaxKs; ++i)
                if (i < ks) st[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + c_src[i]));
        } else {
#pragma unroll
            for (int i = 0; i < kBulkMaxKs; ++i)
                if (i < ks) {
                    u32x4_t v = {0u, 0u, 0u, 0u};
                    if (t0 + c_row[i] < n_tok) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + c_src[i]));
                    st[i] = v;
                }
        }
    };

    const int step = gridDim.x;
    u32x4_t stage[kBulkAhead][kBulkMaxKs];
#pragma unroll
    for (int a = 0; a < kBulkAhead; ++a)
        if ((int)blockIdx.x + a * step < n_tiles) issue(stage[a], blockIdx.x + a * step);

    // the encoder matrix, once: rows of r elements -> padded LDS rows, eight chunks per thread in flight
    {
        constexpr int wcpr = r >> 3;
        const int total = in_w * wcpr;
        const char* w = static_cast<const char*>(s.w1);
        for (int f0 = tid; f0 < total; f0 += 8 * 64 * kBulkWaves) {
            u32x4_t t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int f = f0 + u * 64 * kBulkWaves;
                if (f < total) t[u] = *reinterpret_cast<const u32x4_t*>(w + (size_t)f * 16);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int f = f0 + u * 64 * kBulkWaves;
                if (f < total) *reinterpret_cast<u32x4_t*>(wbuf + (f / wcpr) * stride_w + (f % wcpr) * 16) = t[u];
            }
        }
    }
    // the products are formed transposed, Z^T = W^T X^T (the matrix as the first operand), so that a lane holds four
    // CONSECUTIVE latent columns 16 nb + 4 lg + v of ONE token l16: pairs convert together and leave as 8 bytes
    f32x4_t bias[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) bias[nb][v] = s.b1 ? Elem<E>::load(s.b1, 16 * nb + 4 * lg + v) : 0.f;
    __syncthreads();

    // Cache row of token t: sequence b = t / t_new at position pos(b) + t % t_new.  The division is done once per
    // tile, for its first token (the same in every lane); the rows of a tile then step through at most two
    // sequences when a sequence brings at least a tile's worth of tokens, else each row divides for itself.
    const bool long_seqs = p.t_new >= kBulkRows;
    auto cache_row = [&](int t0, int b0, int tt0, int row) -> size_t {
        int b, tt;
        if (long_seqs) {
            const bool carry = tt0 + row >= p.t_new;
            b = b0 + (carry ? 1 : 0);
            tt = tt0 + row - (carry ? p.t_new : 0);
        } else {
            b = (t0 + row) / p.t_new;
            tt = t0 + row - b * p.t_new;
        }
        return (size_t)b * p.max_seq + (p.positions ? p.positions[b] : p.pos0) + tt;
    };

    auto process = [&](u32x4_t (&st)[kBulkMaxKs], int tile, int next) {
        const int t0 = tile * kBulkTile + wave * kBulkRows;
#pragma unroll
        for (int i = 0; i < kBulkMaxKs; ++i)
            if (i < ks) *reinterpret_cast<u32x4_t*>(reg + c_dst[i]) = st[i];
        if (next < n_tiles) issue(st, next);
        if (t0 >= n_tok) return;                   // a wave tile past the end: only in the last workgroup tile
        const int b0 = __builtin_amdgcn_readfirstlane(t0 / p.t_new);
        const int tt0 = t0 - b0 * p.t_new;

        f32x4_t acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int s2 = 0; s2 < ks; ++s2) {
            const u32x4_t xa = *reinterpret_cast<const u32x4_t*>(reg + l16 * stride_x + (32 * s2 + 8 * lg) * 2);
            const char* wrow = wbuf + (32 * s2 + 8 * lg + (l16 >> 2)) * stride_w + (l16 & 3) * 8;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32 + 4 * stride_w));
                const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
                acc[nb] = BulkMma<E>::mfma(u32x4_t{lo2[0], lo2[1], hi2[0], hi2[1]}, xa, acc[nb]);
            }
        }
        // this lane: token l16, latent columns 16 nb + 4 lg + v
        if constexpr (kI8) {
            constexpr int ostride = r + 16;
            signed char* z8 = static_cast<signed char*>(s.z);
            float mn = INFINITY, mx = -INFINITY;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                acc[nb] += bias[nb];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    mn = fminf(mn, acc[nb][v]);
                    mx = fmaxf(mx, acc[nb][v]);
                }
            }
            mn = fminf(mn, __shfl_xor(mn, 16)); mx = fmaxf(mx, __shfl_xor(mx, 16));
            mn = fminf(mn, __shfl_xor(mn, 32)); mx = fmaxf(mx, __shfl_xor(mx, 32));
            const QuantParams qp = quant_params(mn, mx);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                unsigned w = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) w |= (unsigned)(unsigned char)quant_code(acc[nb][v], qp) << (8 * v);
                *reinterpret_cast<unsigned*>(reg + l16 * ostride + 16 * nb + 4 * lg) = w;
            }
            if (lg == 0 && t0 + l16 < n_tok) static_cast<RowMeta*>(s.meta)[cache_row(t0, b0, tt0, l16)] = quant_meta(qp);
            constexpr int total = kBulkRows * NB;              // 16-byte chunks of the tile's code rows
#pragma unroll
            for (int i = 0; i < (total + 63) / 64; ++i) {
                const int f = i * 64 + lane;
                const int row = f / NB, ch = f % NB;
                if (f < total && t0 + row < n_tok)
                    *reinterpret_cast<u32x4_t*>(z8 + cache_row(t0, b0, tt0, row) * r + ch * 16) = *reinterpret_cast<const u32x4_t*>(reg + row * ostride + ch * 16);
            }
        } else {
            constexpr int ostride = 2 * r + 16;
            char* z = static_cast<char*>(s.z);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const f32x4_t y = acc[nb] + bias[nb];
                *reinterpret_cast<u32x2_t*>(reg + l16 * ostride + (16 * nb + 4 * lg) * 2) = u32x2_t{BulkMma<E>::pack2(y[0], y[1]), BulkMma<E>::pack2(y[2], y[3])};
            }
            constexpr int ocpr = 2 * NB;                       // 16-byte chunks per latent row
#pragma unroll
            for (int i = 0; i < NB / 2; ++i) {
                const int f = i * 64 + lane;
                const int row = f / ocpr, ch = f % ocpr;
                if (t0 + row < n_tok)
                    *reinterpret_cast<u32x4_t*>(z + (cache_row(t0, b0, tt0, row) * r + ch * 8) * 2) = *reinterpret_cast<const u32x4_t*>(reg + row * ostride + ch * 16);
            }
        }
    };

    for (int tile = blockIdx.x; tile < n_tiles; tile += kBulkAhead * step) {
#pragma unroll
        for (int a = 0; a < kBulkAhead; ++a)
            if (tile + a * step < n_tiles) process(stage[a], tile + a * step, tile + (a + kBulkAhead) * step);
    }
}

size_t bulk_lds_bytes(const EncodeSide& s) {
    return (size_t)s.in_width * bulk_stride_w(s.r) + (size_t)kBulkWaves * bulk_region(s.in_width, s.r);
}

template <typename E, bool kI8>
hipError_t launch_bulk_nb(const EncodeParams& p, int nb, int side0, int n_sides, size_t lds, int n_cu, hipStream_t stream) {
    void (*kern)(EncodeParams, int) = nullptr;
    switch (nb) {
        case 2: kern = encode_bulk_kernel<E, 2, kI8>; break;
        case 4: kern = encode_bulk_kernel<E, 4, kI8>; break;
        case 6: kern = encode_bulk_kernel<E, 6, kI8>; break;
        case 8: kern = encode_bulk_kernel<E, 8, kI8>; break;
        default: return hipErrorInvalidValue;
    }
    static AttrFlag attr_set[5] = {false, false, false, false, false};      // per instantiation of this function template
    if (!attr_set[nb / 2]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBulkLdsMax);
        if (e != hipSuccess) return e;
        attr_set[nb / 2] = true;
    }
    const int n_tok = p.batch * p.t_new;
    const int n_tiles = (n_tok + kBulkTile - 1) / kBulkTile;
    const int per_side = n_cu > 0 ? (n_cu + n_sides - 1) / n_sides : 128;     // one workgroup per compute unit
    dim3 grid(n_tiles < per_side ? n_tiles : per_side, n_sides);
    hipLaunchKernelGGL(kern, grid, dim3(64 * kBulkWaves), lds, stream, p, side0);
    return hipGetLastError();
}

}  // namespace

// Shapes of the streaming encoder: linear, 16-bit dtype, input width a multiple of 32 up to 256 with 8-column
// chunks inside one head, latent width a multiple of 32 up to 128, matrix and wave regions within the LDS.
bool encode_bulk_supported(const EncodeParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.d_head % 8 || (long long)p.batch * p.t_new < kBulkMinTokens) return false;
    bool any = false;
    for (int i = 0; i < 2; ++i) {
        const EncodeSide& s = p.s[i];
        if (s.r == 0) continue;
        if (s.hidden > 0 || s.in_width % 32 || s.in_width < 32 || s.in_width > 32 * kBulkMaxKs || s.r % 32 || s.r > 128) return false;
        if (bulk_lds_bytes(s) > kBulkLdsMax) return false;
        any = true;
    }
    return any;
}

hipError_t launch_encode_bulk(const EncodeParams& p, int dtype, int n_cu, hipStream_t stream) {
    const bool bf = dtype == KVCAR_BF16;
    const bool i8 = p.s[0].meta != nullptr || p.s[1].meta != nullptr;
    auto go = [&](int nb, int side0, int n_sides, size_t lds) {
        if (i8) return bf ? launch_bulk_nb<BF16, true>(p, nb, side0, n_sides, lds, n_cu, stream) : launch_bulk_nb<F16, true>(p, nb, side0, n_sides, lds, n_cu, stream);
        return bf ? launch_bulk_nb<BF16, false>(p, nb, side0, n_sides, lds, n_cu, stream) : launch_bulk_nb<F16, false>(p, nb, side0, n_sides, lds, n_cu, stream);
    };
    const EncodeSide& k = p.s[0];
    const EncodeSide& v = p.s[1];
    // one launch for both tensors when their latent widths agree, else one each
    if (k.r > 0 && v.r == k.r) return go(k.r / 16, 0, 2, bulk_lds_bytes(k) > bulk_lds_bytes(v) ? bulk_lds_bytes(k) : bulk_lds_bytes(v));
    hipError_t e = hipSuccess;
    if (k.r > 0) e = go(k.r / 16, 0, 1, bulk_lds_bytes(k));
    if (e == hipSuccess && v.r > 0) e = go(v.r / 16, 1, 1, bulk_lds_bytes(v));
    return e;
}

}  // namespace kvcar
