// MFMA encode + append for gfx950 (16-bit dtypes): the encoder placed after K/V generation and the
// append of one latent row per token ("Network Architecture", first paragraph), for decode steps
// (one token per sequence) and for prefill (many tokens per sequence) alike.
//
//   linear encoder      z = x[cols] W1 + b1
//   two-layer encoder   z = act(x[cols] W1 + b1) W2 + b2
//
// One workgroup = 4 waves x 16 tokens.  A GEMM stage computes out[16 tokens, n] per wave with
// v_mfma_f32_16x16x32: the A operand is the token rows (16-byte chunks straight from global memory
// for the input vectors, from LDS for the hidden activations), the B operand is the weight matrix
// [k, n] row-major, staged through LDS in row chunks shared by the four waves and read with the
// transposing load ds_read_b64_tr_b16 (a lane needs 8 consecutive k of one column).  Hidden
// activations are kept as a bf16/fp16 pair hi + lo so that the second layer sees them to ~2^-17
// relative precision; the latent is rounded once, from the fp32 accumulator, to the cache dtype.
#include "kvcar_qtilde_mfma.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct EncMma;
template <> struct EncMma<BF16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint16_t to16(float v) { return f32_to_bf16_bits(v); }
    static __device__ __forceinline__ float from16(uint16_t b) { return bf16_bits_to_f32(b); }
};
template <> struct EncMma<F16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint16_t to16(float v) { _Float16 h = (_Float16)v; return __builtin_bit_cast(uint16_t, h); }
    static __device__ __forceinline__ float from16(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
};

constexpr int kEncWaves = 4;
constexpr int kEncTokens = 16 * kEncWaves;        // tokens per workgroup
constexpr int kWRowBytes = 64 * 1024;             // weight rows staged per chunk
constexpr int kWBufBytes = kWRowBytes + 1024;     // + slack: column blocks past a narrow matrix are read (and ignored)

// Stage rows [row0, row0 + n_rows), columns [col0, col0 + n_cols) of a row-major [k, n] weight matrix into LDS
// (padded rows of n_cols elements).
__device__ __forceinline__ void stage_weights(char* buf, const char* w, int n, int row0, int n_rows, int stride, int col0, int n_cols) {
    const int cpr = n_cols >> 3;                          // 16-byte chunks per staged row
    const unsigned inv = (1u << 20) / cpr + 1;
    const int total = n_rows * cpr;
    const char* src = w + ((size_t)row0 * n + col0) * 2;
    // eight chunks per thread in flight: a copy loop that stores each chunk before loading the next pays one
    // memory round trip per chunk
    for (int f0 = threadIdx.x; f0 < total; f0 += 8 * 256) {
        u32x4_t t[8];
        unsigned dst[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int f = f0 + u * 256;
            const unsigned row = ((unsigned)f * inv) >> 20;
            const unsigned ch = f - row * cpr;
            dst[u] = row * stride + ch * 16;
            if (f < total) t[u] = *reinterpret_cast<const u32x4_t*>(src + ((size_t)row * n + ch * 8) * 2);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (f0 + u * 256 < total) *reinterpret_cast<u32x4_t*>(buf + dst[u]) = t[u];
    }
}

// acc[nb] += A[16, 32 rows of this k-step] . W chunk, for all NB 16-column blocks.
template <typename E, int NB>
__device__ __forceinline__ void mma_kstep(f32x4_t (&acc)[NB], u32x4_t a, const char* wrow, int stride) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32 + 4 * stride));
        const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
        acc[nb] = EncMma<E>::mfma(a, u32x4_t{lo2[0], lo2[1], hi2[0], hi2[1]}, acc[nb]);
    }
}

// NB1: 16-column blocks of the first layer's output (hidden width, or latent width if linear);
// NB2: of the second layer's output (latent width; unused if linear).
// kSplit (linear encoder, rows in the model dtype): the latent columns are dealt over blockIdx.z in windows of
// 16 * NB1, each workgroup reading only its window of the weight matrix.  A decode step encodes a handful of
// tokens: without the split one workgroup per tensor streams the whole matrix (590 KB for 768 -> 384) alone.
template <typename E, int NB1, int NB2, bool kTwoLayer, bool kSplit = false>
__device__ __forceinline__ void encode_mfma_body(const EncodeParams& p, char* lds) {
    const EncodeSide& s = p.s[blockIdx.y];
    if (s.r == 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    const int n_tok = p.batch * p.t_new;
    const int tok = blockIdx.x * kEncTokens + wave * 16 + l16;      // the A-operand row of this lane
    const bool tok_ok = tok < n_tok;
    const char* xrow = static_cast<const char*>(s.x) + (size_t)(tok_ok ? tok : 0) * p.d_kv * 2;

    char* wbuf = lds;
    const int n1 = kTwoLayer ? s.hidden : s.r;
    const int col0 = kSplit ? (int)blockIdx.z * 16 * NB1 : 0;          // first output column of this workgroup
    if (kSplit && col0 >= n1) return;
    const int w1cols = kSplit ? min(16 * NB1, n1 - col0) : n1;         // staged window
    const int stride1 = 2 * w1cols + 32;

    // ---- layer 1: out1[16, n1] = x[cols] W1 ----------------------------------------------------
    f32x4_t acc1[NB1];
#pragma unroll
    for (int nb = 0; nb < NB1; ++nb) acc1[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    {
        const int rows_cap = (kWRowBytes / stride1) & ~31;
        for (int row0 = 0; row0 < s.in_width; row0 += rows_cap) {
            const int n_rows = min(rows_cap, s.in_width - row0);
            __syncthreads();                              // previous chunk fully consumed
            stage_weights(wbuf, static_cast<const char*>(s.w1), n1, row0, n_rows, stride1, col0, w1cols);
            __syncthreads();
            for (int k0 = 0; k0 < n_rows; k0 += 32) {
                const int kk = row0 + k0 + 8 * lg;        // first of this lane's 8 input columns
                const int src_col = (int)s.heads[kk / p.d_head] * p.d_head + kk % p.d_head;
                u32x4_t a = {0u, 0u, 0u, 0u};
                if (tok_ok) a = *reinterpret_cast<const u32x4_t*>(xrow + src_col * 2);
                mma_kstep<E, NB1>(acc1, a, wbuf + (k0 + 8 * lg + (l16 >> 2)) * stride1 + (l16 & 3) * 8, stride1);
            }
        }
    }

    f32x4_t* out_acc = acc1;
    const void* out_bias = s.b1;
    int n_out_blocks = NB1;
    f32x4_t acc2[kTwoLayer ? NB2 : 1];

    if constexpr (kTwoLayer) {
        // ---- hidden activations -> LDS as hi + lo, one private [16, hidden] region per wave --------
        const int stride_h = 2 * s.hidden + 16;
        char* hbuf = lds + kWBufBytes + wave * 2 * 16 * stride_h;
        char* hlo = hbuf + 16 * stride_h;
#pragma unroll
        for (int nb = 0; nb < NB1; ++nb) {
            const int col = nb * 16 + l16;
            if (col < s.hidden) {
                const float bias = s.b1 ? Elem<E>::load(s.b1, col) : 0.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float h = pinned(apply_act(acc1[nb][v] + bias, s.act, s.slope));
                    const uint16_t hi = EncMma<E>::to16(h);
                    const uint16_t lo = EncMma<E>::to16(h - EncMma<E>::from16(hi));
                    const int row = 4 * lg + v;
                    *reinterpret_cast<uint16_t*>(hbuf + row * stride_h + col * 2) = hi;
                    *reinterpret_cast<uint16_t*>(hlo + row * stride_h + col * 2) = lo;
                }
            }
        }
        // ---- layer 2: z[16, r] = h W2 ----------------------------------------------------------
#pragma unroll
        for (int nb = 0; nb < NB2; ++nb) acc2[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        const int stride2 = 2 * s.r + 32;
        const int rows_cap = (kWRowBytes / stride2) & ~31;
        for (int row0 = 0; row0 < s.hidden; row0 += rows_cap) {
            const int n_rows = min(rows_cap, s.hidden - row0);
            __syncthreads();
            stage_weights(wbuf, static_cast<const char*>(s.w2), s.r, row0, n_rows, stride2, 0, s.r);
            __syncthreads();
            for (int k0 = 0; k0 < n_rows; k0 += 32) {
                const int off = l16 * stride_h + (row0 + k0 + 8 * lg) * 2;
                const u32x4_t ah = *reinterpret_cast<const u32x4_t*>(hbuf + off);
                const u32x4_t al = *reinterpret_cast<const u32x4_t*>(hlo + off);
                const char* wrow = wbuf + (k0 + 8 * lg + (l16 >> 2)) * stride2 + (l16 & 3) * 8;
                mma_kstep<E, NB2>(acc2, ah, wrow, stride2);
                mma_kstep<E, NB2>(acc2, al, wrow, stride2);
            }
        }
        out_acc = acc2;
        out_bias = s.b2;
        n_out_blocks = NB2;
    }

    // ---- latent rows: bias, one rounding to the cache dtype, append ------------------------------
    // result layout: lane holds column 16*nb + l16 of tokens 4*lg + v
    const int tbase = blockIdx.x * kEncTokens + wave * 16 + 4 * lg;
    size_t row_off[4];
    bool row_ok[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int t = tbase + v;
        row_ok[v] = t < n_tok;
        const int b = t / p.t_new, tt = t - b * p.t_new;
        row_off[v] = ((size_t)b * p.max_seq + (p.positions && row_ok[v] ? p.positions[b] : p.pos0) + tt) * s.r;
    }
    if (s.meta) {
        // ---- int8 latents: a token's row lies in the 16 lanes of its quarter (columns 16 nb + l16) -------
        constexpr int NBO = kTwoLayer ? NB2 : NB1;
        float mn[4], mx[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) { mn[v] = INFINITY; mx[v] = -INFINITY; }
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb) {
            const int col = nb * 16 + l16;
            if (nb < n_out_blocks && col < s.r) {
                const float bias = out_bias ? Elem<E>::load(out_bias, col) : 0.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    out_acc[nb][v] += bias;
                    mn[v] = fminf(mn[v], out_acc[nb][v]);
                    mx[v] = fmaxf(mx[v], out_acc[nb][v]);
                }
            }
        }
        signed char* z8 = static_cast<signed char*>(s.z);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) {
                mn[v] = fminf(mn[v], __shfl_xor(mn[v], off));
                mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], off));
            }
            const QuantParams qp = quant_params(mn[v], mx[v]);
            if (!row_ok[v]) continue;
#pragma unroll
            for (int nb = 0; nb < NBO; ++nb) {
                const int col = nb * 16 + l16;
                if (nb < n_out_blocks && col < s.r) z8[row_off[v] + col] = quant_code(out_acc[nb][v], qp);
            }
            if (l16 == 0) static_cast<RowMeta*>(s.meta)[row_off[v] / s.r] = quant_meta(qp);
        }
        return;
    }
    uint16_t* z = static_cast<uint16_t*>(s.z);
#pragma unroll
    for (int nb = 0; nb < (kTwoLayer ? NB2 : NB1); ++nb) {
        const int col = col0 + nb * 16 + l16;
        if (nb < n_out_blocks && col < s.r) {
            const float bias = out_bias ? Elem<E>::load(out_bias, col) : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (row_ok[v]) z[row_off[v] + col] = EncMma<E>::to16(out_acc[nb][v] + bias);
        }
    }
}

template <typename E, int NB1, int NB2, bool kTwoLayer, bool kSplit = false>
__global__ __launch_bounds__(256) void encode_mfma_kernel(EncodeParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    encode_mfma_body<E, NB1, NB2, kTwoLayer, kSplit>(p, lds);
}

// A decode step's two small independent pieces in one launch: the new token's latent rows (the column-window form of
// the encoder above: workgroups blockIdx.x < enc_x) and the absorbed queries of the attention launch that follows
// (qtilde_mfma_block: the workgroups beyond, with blockIdx.y = blockIdx.z = 0, numbered (x, y, z) over a qx x qy x .. grid).
// Two launches of about 6 us each become one.
template <typename E>
__global__ __launch_bounds__(256) void encode_step_qtilde_kernel(EncodeParams p, AttendParams q, int enc_x, int qx, int qy) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if ((int)blockIdx.x < enc_x) {
        encode_mfma_body<E, 2, 1, false, true>(p, lds);
        return;
    }
    if (blockIdx.y != 0 || blockIdx.z != 0) return;
    const int id = (int)blockIdx.x - enc_x;
    qtilde_mfma_block<E>(&q, id % qx, (id / qx) % qy, id / (qx * qy), qx);
}

// Decode steps with int8 latents (linear encoder, few tokens): a row's minimum and maximum need the whole row, so
// the columns cannot be dealt over workgroups; instead a workgroup takes 16 tokens and its four waves split the
// columns (wave w: 16-column blocks w, w + 4, ..), meeting once in LDS for the row extremes.  Four times the
// workgroups of the general kernel and a quarter of the serial work per wave.
template <typename E, int NBW>
__global__ __launch_bounds__(256) void encode_i8_step_kernel(EncodeParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const EncodeSide& s = p.s[blockIdx.y];
    if (s.r == 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    const int n_tok = p.batch * p.t_new;
    const int tok = blockIdx.x * 16 + l16;                          // the A-operand row of this lane (the same in every wave)
    const bool tok_ok = tok < n_tok;
    const char* xrow = static_cast<const char*>(s.x) + (size_t)(tok_ok ? tok : 0) * p.d_kv * 2;
    char* wbuf = lds;
    float* ext = reinterpret_cast<float*>(lds + kWBufBytes);        // [4 waves][16 tokens][min, max]
    const int stride1 = 2 * s.r + 32;

    f32x4_t acc[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int rows_cap = (kWRowBytes / stride1) & ~31;
    for (int row0 = 0; row0 < s.in_width; row0 += rows_cap) {
        const int n_rows = min(rows_cap, s.in_width - row0);
        __syncthreads();
        stage_weights(wbuf, static_cast<const char*>(s.w1), s.r, row0, n_rows, stride1, 0, s.r);
        __syncthreads();
        for (int k0 = 0; k0 < n_rows; k0 += 32) {
            const int kk = row0 + k0 + 8 * lg;
            const int src_col = (int)s.heads[kk / p.d_head] * p.d_head + kk % p.d_head;
            u32x4_t a = {0u, 0u, 0u, 0u};
            if (tok_ok) a = *reinterpret_cast<const u32x4_t*>(xrow + src_col * 2);
            const char* wrow = wbuf + (k0 + 8 * lg + (l16 >> 2)) * stride1 + (l16 & 3) * 8;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                const int blk = wave + 4 * nb;                      // reads past the matrix land in the buffer's slack and are ignored
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + blk * 32));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + blk * 32 + 4 * stride1));
                const u32x2_t lo2 = __builtin_bit_cast(u32x2_t, lo), hi2 = __builtin_bit_cast(u32x2_t, hi);
                acc[nb] = EncMma<E>::mfma(a, u32x4_t{lo2[0], lo2[1], hi2[0], hi2[1]}, acc[nb]);
            }
        }
    }
    // this lane: column 16 (wave + 4 nb) + l16 of tokens 4 lg + v
    float mn[4], mx[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) { mn[v] = INFINITY; mx[v] = -INFINITY; }
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int col = 16 * (wave + 4 * nb) + l16;
        if (col < s.r) {
            const float bias = s.b1 ? Elem<E>::load(s.b1, col) : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                acc[nb][v] += bias;
                mn[v] = fminf(mn[v], acc[nb][v]);
                mx[v] = fmaxf(mx[v], acc[nb][v]);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) {
            mn[v] = fminf(mn[v], __shfl_xor(mn[v], off));
            mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], off));
        }
        if (l16 == 0) { ext[(wave * 16 + 4 * lg + v) * 2] = mn[v]; ext[(wave * 16 + 4 * lg + v) * 2 + 1] = mx[v]; }
    }
    __syncthreads();
    signed char* z8 = static_cast<signed char*>(s.z);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int tl = 4 * lg + v, t = blockIdx.x * 16 + tl;
        float lo = ext[tl * 2], hi = ext[tl * 2 + 1];
#pragma unroll
        for (int w = 1; w < 4; ++w) { lo = fminf(lo, ext[(w * 16 + tl) * 2]); hi = fmaxf(hi, ext[(w * 16 + tl) * 2 + 1]); }
        const QuantParams qp = quant_params(lo, hi);
        if (t >= n_tok) continue;
        const int b = t / p.t_new, tt = t - b * p.t_new;
        const size_t row = (size_t)b * p.max_seq + (p.positions ? p.positions[b] : p.pos0) + tt;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int col = 16 * (wave + 4 * nb) + l16;
            if (col < s.r) z8[row * s.r + col] = quant_code(acc[nb][v], qp);
        }
        if (wave == 0 && l16 == 0) static_cast<RowMeta*>(s.meta)[row] = quant_meta(qp);
    }
}


template <typename K>
static hipError_t launch_enc(K kern, size_t lds, const EncodeParams& p, hipStream_t stream, AttrFlag& attr_set, int col_windows = 1) {
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_tok = p.batch * p.t_new;
    dim3 grid((n_tok + kEncTokens - 1) / kEncTokens, 2, col_windows);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

// Shapes the MFMA encoder covers: 16-bit dtype, input width a multiple of 32 with 8-column chunks
// inside one head, latent and hidden widths multiples of 32 up to 384 / 256.
bool encode_mfma_supported(const EncodeParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.d_head % 8) return false;
    bool two = false, one = false;
    for (int i = 0; i < 2; ++i) {
        const EncodeSide& s = p.s[i];
        if (s.r == 0) continue;
        if (s.in_width % 32 || s.r % 32 || s.r > 384 || s.hidden % 32 || s.hidden > 256) return false;
        if (s.hidden > 0 && s.r > 128) return false;
        (s.hidden > 0 ? two : one) = true;
    }
    return !(two && one);      // K and V use the same kind of encoder in one launch
}

hipError_t launch_encode_mfma(const EncodeParams& p, int dtype, hipStream_t stream) {
    static AttrFlag set[8] = {false, false, false, false, false, false, false, false};
    int rmax = 0, hmax = 0;
    for (int i = 0; i < 2; ++i) { rmax = p.s[i].r > rmax ? p.s[i].r : rmax; hmax = p.s[i].hidden > hmax ? p.s[i].hidden : hmax; }
    const bool bf = dtype == KVCAR_BF16;
    if (hmax > 0) {
        const size_t lds = kWBufBytes + (size_t)kEncWaves * 2 * 16 * (2 * hmax + 16);
        return bf ? launch_enc(encode_mfma_kernel<BF16, 16, 8, true>, lds, p, stream, set[0])
                  : launch_enc(encode_mfma_kernel<F16, 16, 8, true>, lds, p, stream, set[1]);
    }
    const size_t lds = kWBufBytes;
    // few tokens (a decode step), rows in the model dtype: 32-column windows over blockIdx.z (int8 rows need the
    // whole row in one workgroup for their minimum and maximum)
    const bool i8 = p.s[0].meta != nullptr || p.s[1].meta != nullptr;
    if (i8 && (long long)p.batch * p.t_new <= 2048) {
        const size_t lds8 = kWBufBytes + 4 * 16 * 2 * sizeof(float);
        const int n_tok = p.batch * p.t_new;
        dim3 grid((n_tok + 15) / 16, 2);
        static AttrFlag set8[4] = {false, false, false, false};
        const int slot = (bf ? 0 : 2) + (rmax <= 128 ? 0 : 1);
        void (*k8)(EncodeParams) = bf ? (rmax <= 128 ? encode_i8_step_kernel<BF16, 2> : encode_i8_step_kernel<BF16, 6>)
                                      : (rmax <= 128 ? encode_i8_step_kernel<F16, 2> : encode_i8_step_kernel<F16, 6>);
        if (!set8[slot]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k8), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            set8[slot] = true;
        }
        hipLaunchKernelGGL(k8, grid, dim3(256), lds8, stream, p);
        return hipGetLastError();
    }
    if (!i8 && (long long)p.batch * p.t_new <= 2048)
        return bf ? launch_enc(encode_mfma_kernel<BF16, 2, 1, false, true>, lds, p, stream, set[6], (rmax + 31) / 32)
                  : launch_enc(encode_mfma_kernel<F16, 2, 1, false, true>, lds, p, stream, set[7], (rmax + 31) / 32);
    if (rmax <= 128)
        return bf ? launch_enc(encode_mfma_kernel<BF16, 8, 1, false>, lds, p, stream, set[2])
                  : launch_enc(encode_mfma_kernel<F16, 8, 1, false>, lds, p, stream, set[3]);
    return bf ? launch_enc(encode_mfma_kernel<BF16, 24, 1, false>, lds, p, stream, set[4])
              : launch_enc(encode_mfma_kernel<F16, 24, 1, false>, lds, p, stream, set[5]);
}

// The decode-step encoder (linear, rows in the model dtype, at most 2048 tokens) and the absorbed-query projection of `q`
// in one launch.  The caller has checked that both pieces have these forms (encode_step_qtilde_supported).
bool encode_step_qtilde_supported(const EncodeParams& p, int dtype) {
    if (!encode_mfma_supported(p, dtype) || (long long)p.batch * p.t_new > 2048) return false;
    for (int i = 0; i < 2; ++i)
        if (p.s[i].r > 0 && (p.s[i].hidden > 0 || p.s[i].meta != nullptr)) return false;
    return true;
}

hipError_t launch_encode_step_qtilde(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, int dtype, hipStream_t stream) {
    static_assert(sizeof(EncodeParams) + sizeof(AttendParams) + 16 <= 4096, "both argument blocks must fit the kernel-argument segment");
    static AttrFlag set[2] = {false, false};
    const bool bf = dtype == KVCAR_BF16;
    auto kern = bf ? encode_step_qtilde_kernel<BF16> : encode_step_qtilde_kernel<F16>;
    if (!set[bf ? 0 : 1]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        set[bf ? 0 : 1] = true;
    }
    int rmax = 0;
    for (int i = 0; i < 2; ++i) rmax = p.s[i].r > rmax ? p.s[i].r : rmax;
    const int n_tok = p.batch * p.t_new;
    const int enc_x = (n_tok + kEncTokens - 1) / kEncTokens;
    dim3 grid(enc_x + qx * qy * qz, 2, (rmax + 31) / 32);
    hipLaunchKernelGGL(kern, grid, dim3(256), kWBufBytes, stream, p, q, enc_x, qx, qy);
    return hipGetLastError();
}

}  // namespace kvcar
