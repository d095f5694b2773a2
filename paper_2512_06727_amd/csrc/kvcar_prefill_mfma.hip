// Prefill attention over the latent cache on the matrix cores (gfx950, 16-bit dtypes).
//
// A prompt chunk attends causally over the cached rows of its sequence (Introduction: the prefill phase
// produces the keys and values of all prompt tokens; they are cached as latent rows and come back through
// the decoder, "Network Architecture", 2nd paragraph; attention is Eq. 1 per token).  Unlike a decode
// step this is bound by the matrix units: T x L scores per head against L latent rows read.  Folding the
// decoder into the query (what the decode kernels do) would make every score a contraction over the
// latent width r instead of d_head - twice the work for r = 2 d_head - so here the rows are decoded
// first, ONCE per call, and a causal attention kernel runs over the decoded rows:
//
//   recon_mfma_kernel    K^^T[n, t] = W^T[n, c] . Z^T[c, t]   (v_mfma_f32_32x32x16; A = the decoder columns
//                        of one KV head through LDS and the transposing load, B = latent rows straight
//                        from global memory, dequantised in registers when they are int8 codes)
//   prefill_mfma_kernel  per workgroup: 8 waves x 32 query tokens of one head; K^ / V^ tiles of 64 rows are
//                        shared through LDS (double buffered, one barrier per tile); per 32-row half of a tile
//                          S^T[row, q] = K^ . Q^T            A = K^ rows (LDS), B = queries (registers)
//                          online softmax in base 2: a lane holds 16 rows of ONE query per half, so the
//                          reductions are in-lane plus one cross-lane step; the reference point of a query
//                          only moves when a score exceeds it by 2^8, so the accumulators are rarely rescaled
//                          O^T[d, q] += V^^T . P^T           A = V^ through the transposing load, B = P^T
//                          straight from the softmax registers (the result layout of S^T is the operand
//                          layout, with the rows of a k-step taken in the order the registers hold them)
//                        the causal limit only touches the last one or two tiles of a wave.
// Measured budget of the attention kernel on 16 x 4096 tokens (per launch, with parts removed in turn):
// matrix instructions alone would take 0.44 ms at the dense peak; LDS reads of the operands 0.40 ms, staging
// and barriers 0.19 ms, the softmax's vector instructions 0.5-0.7 ms (on this chip a matrix instruction blocks
// vector issue for about half its duration); they overlap only in part: 1.13 ms.  Hence the effort to keep
// vector work per score down to exp2 + half a conversion + half a dot2 + half a max3.
#include "kvcar_attend_mfma_body.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(16))) float f32x16_t;

template <typename E> struct Mma32;
template <> struct Mma32<BF16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma32<F16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

// acc + lo + hi for the two 16-bit elements packed in w (v_dot2 with a vector of ones: one instruction per pair).
template <typename E> struct PairSum;
template <> struct PairSum<BF16> {
    static __device__ __forceinline__ float add(float acc, unsigned w) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w), __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc, false);
    }
};
template <> struct PairSum<F16> {
    static __device__ __forceinline__ float add(float acc, unsigned w) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w), __builtin_bit_cast(f16x2_t, 0x3c003c00u), acc, false);
    }
};

// Transposing LDS load: 16 lanes supply the addresses of a 4-row x 16-column patch of 16-bit elements and
// lane i receives the 4 rows of column i.  Two patches make the 8 k-slots of a lane.
__device__ __forceinline__ u32x4_t tr_pair32(const char* p, int second_offset) {
    const s16x4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
    const s16x4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + second_offset));
    const u32x2_t a0 = __builtin_bit_cast(u32x2_t, t0), a1 = __builtin_bit_cast(u32x2_t, t1);
    return u32x4_t{a0[0], a0[1], a1[0], a1[1]};
}

// [n_rows, cpr 16-byte chunks] of a row-major matrix (row pitch src_pitch bytes) -> padded LDS rows, by the
// threads of the workgroup with eight chunks per thread in flight: a loop that stores each chunk before it loads
// the next pays one memory round trip per chunk.
__device__ __forceinline__ void recon_stage_matrix(char* dst, int dst_stride, const char* src, size_t src_pitch, int n_rows, int cpr, int tid, int n_threads) {
    const int total = n_rows * cpr;
    for (int f0 = tid; f0 < total; f0 += 8 * n_threads) {
        u32x4_t t[8];
        int off[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int f = f0 + u * n_threads;
            const int row = f / cpr, ch = f - row * cpr;
            off[u] = row * dst_stride + ch * 16;
            if (f < total) t[u] = *reinterpret_cast<const u32x4_t*>(src + (size_t)row * src_pitch + ch * 16);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (f0 + u * n_threads < total) *reinterpret_cast<u32x4_t*>(dst + off[u]) = t[u];
    }
}

// The decoded rows of one head leave a wave through LDS.  The result layout gives a lane four 8-byte pieces of one
// token's row; parked as rows of d_head elements (the wave's 32-token tiles) they go out as whole
// 16-byte chunks of contiguous memory: a tile's rows of one head are contiguous in K^ / V^.
constexpr size_t kReconLdsMax = 160 * 1024;
constexpr int kReconChunk = 256;      // tokens per workgroup: TL 32-token tiles per wave, 8 / TL waves
__host__ __device__ constexpr int recon_stage_stride(int d_head) { return 2 * d_head + 16; }
__host__ __device__ constexpr size_t recon_stage_bytes(int d_head) { return (size_t)kReconChunk * recon_stage_stride(d_head); }

// int8 rows enter the products as their codes (exact in either 16-bit dtype), so a row's scale and zero point are
// applied to the fp32 sums: x^ . W[:, n] = (sum_c u_c W[c, n] - (128 + zeropoint) S_n) / scale with u = code + 128 and
// S_n the column sums of the matrix.  Rounding the dequantised row to 16 bits first would cost about as much
// accuracy as the int8 codes themselves hold.
struct RowQuant {
    float inv;      // 1 / scale
    float sub;      // 128 + zeropoint
};

template <typename E, bool kI8>
__device__ __forceinline__ void recon_emit_block(const f32x16_t& acc, const void* bl, int col0, float out_scale, char* stage_row, char* orow,
                                                 const float* colsum, RowQuant rq) {
    // this lane: one token, decoder columns col0 + 8a + j (register 4a + j), col0 already holding the lane half's 4h;
    // colsum points at the column sums of those columns (int8 rows)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        float bias[4] = {0.f, 0.f, 0.f, 0.f};
        if (bl) {
#pragma unroll
            for (int j = 0; j < 4; ++j) bias[j] = Elem<E>::load(bl, col0 + 8 * a + j);
        }
        float v[4];
        if constexpr (kI8) {
            const f32x4_t cs = *reinterpret_cast<const f32x4_t*>(colsum + 8 * a);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = fmaf(fmaf(-rq.sub, cs[j], acc[4 * a + j]), rq.inv, bias[j]) * out_scale;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (acc[4 * a + j] + bias[j]) * out_scale;
        }
        // decoded rows are held in fp16 whatever the 16-bit model dtype (RowsOf), saturating at its range
        const u32x2_t w = {Mma<F16>::pack2(sat_half(v[0]), sat_half(v[1])), Mma<F16>::pack2(sat_half(v[2]), sat_half(v[3]))};
        if (stage_row) *reinterpret_cast<u32x2_t*>(stage_row + 16 * a) = w;
        else if (orow) *reinterpret_cast<u32x2_t*>(orow + 16 * a) = w;
    }
}

// Column sums of an [n_rows, n_cols] matrix of 16-bit elements staged in LDS (row stride in bytes), in fp32.
template <typename E>
__device__ __forceinline__ void lds_column_sums(float* out, const char* mat, int stride, int n_rows, int n_cols, int tid, int n_threads) {
    for (int n = tid; n < n_cols; n += n_threads) {
        float acc = 0.f;
        for (int c = 0; c < n_rows; ++c) acc += Elem<E>::load(mat + (size_t)c * stride, n);
        out[n] = acc;
    }
}

// The wave's parked rows of one head -> memory: tile `tile` starts at token t0; chunk f of the tile is 16 bytes at
// offset 16 f of its (contiguous) rows.
__device__ __forceinline__ void recon_flush_tile(const char* stage, int stride_o, char* tile_dst, int rows_valid, int cpr, int lane) {
    const int total = min(rows_valid, 32) * cpr;
    for (int f = lane; f < total; f += 64) {
        const int row = f / cpr, ch = f - row * cpr;
        *reinterpret_cast<u32x4_t*>(tile_dst + (size_t)f * 16) = *reinterpret_cast<const u32x4_t*>(stage + row * stride_o + ch * 16);
    }
}

// ---------------------------------------------------------------------------------------------------------
// decoded rows (linear decoder)
// ---------------------------------------------------------------------------------------------------------
typedef const __attribute__((address_space(4))) ReconParams* RArgs;
typedef const __attribute__((address_space(4))) ReconEntry* REntry;


// The wave's latent rows as B operands: tile `tile` of its 32 TL tokens; lane (token l32, half h) holds latent
// columns 16s + 8h .. +7 of k-step s, dequantised in registers when the rows are int8 codes; rows past n_rows are zero.
template <typename E, int R, bool kI8, int TL>
__device__ __forceinline__ void recon_load_rows(u32x4_t (&zb)[TL][R / 16], RowQuant (&rq)[TL], REntry e, RArgs p, int b, int tok0, int l32, int h) {
    constexpr int KS = R / 16;
    const int n_rows = p->n_rows;
#pragma unroll
    for (int tile = 0; tile < TL; ++tile) {
        const int t = tok0 + tile * 32 + l32;
        const bool valid = t < n_rows;
        const size_t row = (size_t)b * p->max_seq + (valid ? t : 0);
        rq[tile] = RowQuant{1.f, 0.f};
        if constexpr (kI8) {
            const RowMeta m = static_cast<const RowMeta*>(e->d.meta)[row];
            rq[tile].inv = 1.f / m.scale;
            rq[tile].sub = 128.f + (float)m.zeropoint;                     // codes are read as unsigned bytes u = code + 128
            const char* zr = static_cast<const char*>(e->d.z) + row * R + 8 * h;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const u32x2_t c = *reinterpret_cast<const u32x2_t*>(zr + 16 * s);
                unsigned w[4];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const unsigned x = c[i] ^ 0x80808080u;
                    w[2 * i] = Mma<E>::pack2((float)(x & 0xffu), (float)((x >> 8) & 0xffu));          // 0 .. 255: exact in 8 significant bits
                    w[2 * i + 1] = Mma<E>::pack2((float)((x >> 16) & 0xffu), (float)(x >> 24));
                }
                zb[tile][s] = valid ? u32x4_t{w[0], w[1], w[2], w[3]} : u32x4_t{0u, 0u, 0u, 0u};
            }
        } else {
            const char* zr = static_cast<const char*>(e->d.z) + (row * R + 8 * h) * 2;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (valid) v = *reinterpret_cast<const u32x4_t*>(zr + 32 * s);
                zb[tile][s] = v;
            }
        }
    }
}

// Workgroup = (256-token chunk, sequence, entry).  The wave keeps its latent rows as B operands (lane: token
// l32, latent columns 16s + 8h .. +7 of k-step s) and walks over the KV heads of the entry; per head the
// decoder slice [R, d_head] passes through LDS once for the four waves.
template <typename E, int R, bool kI8, int TL>
__global__ __launch_bounds__(64 * kReconChunk / (32 * TL)) void recon_mfma_kernel(ReconParams) {
    constexpr int NT = 64 * kReconChunk / (32 * TL);      // threads
    constexpr int KS = R / 16;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    RArgs p = (RArgs)__builtin_amdgcn_kernarg_segment_ptr();
    REntry e = &p->e[blockIdx.z];
    const int b = blockIdx.y, chunk0 = blockIdx.x * kReconChunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5, l16 = lane & 15;
    const int dh = p->d_head, n_rows = p->n_rows;
    const int stride_w = 2 * dh + 32, cpr = dh >> 3;
    const int stride_o = recon_stage_stride(dh);
    char* stage = p->staged ? lds + R * stride_w + wave * 32 * TL * stride_o : nullptr;
    float* colsum = reinterpret_cast<float*>(lds + R * stride_w + (p->staged ? kReconChunk * stride_o : 0));      // [d_head], int8 rows only

    u32x4_t zb[TL][KS];
    RowQuant rq[TL];
    recon_load_rows<E, R, kI8, TL>(zb, rq, e, p, b, chunk0 + wave * 32 * TL, l32, h);

    const char* wl = static_cast<const char*>(e->d.wl);
    const int in_width = e->d.in_width;
    char* dst = static_cast<char*>(e->which == KVCAR_K ? p->khat : p->vhat);
    const float out_scale = e->which == KVCAR_K ? p->k_scale : 1.f;      // keys carry softmax scale * log2(e) into their one rounding
    for (int hi = 0; hi < e->n_heads; ++hi) {
        const int g = e->head[hi], col = e->col[hi];
        __syncthreads();                           // the previous slice is no longer read
        recon_stage_matrix(lds, stride_w, wl + (size_t)col * 2, (size_t)in_width * 2, R, cpr, tid, NT);
        __syncthreads();
        if constexpr (kI8) {
            lds_column_sums<E>(colsum, lds, stride_w, R, dh, tid, NT);
            __syncthreads();
        }
        for (int mb = 0; mb < (dh >> 5); ++mb) {
            // A operand: row = decoder column 32 mb + l32, k-slots = latent indices 16s + 8h .. +7
            const char* wsrc = lds + (8 * h + (l16 >> 2)) * stride_w + (32 * mb + 16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
            f32x16_t acc[TL];
#pragma unroll
            for (int tile = 0; tile < TL; ++tile)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tile][v] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const u32x4_t wa = tr_pair32(wsrc + 16 * s * stride_w, 4 * stride_w);
#pragma unroll
                for (int tile = 0; tile < TL; ++tile) acc[tile] = Mma32<E>::mfma(wa, zb[tile][s], acc[tile]);
            }
            // this lane: token l32, decoder columns 32 mb + 8a + 4h + j (register 4a + j)
#pragma unroll
            for (int tile = 0; tile < TL; ++tile) {
                const int t = chunk0 + wave * 32 * TL + tile * 32 + l32;
                char* srow = stage ? stage + (tile * 32 + l32) * stride_o + (32 * mb + 4 * h) * 2 : nullptr;
                char* orow = t < n_rows ? dst + ((((size_t)b * p->n_kv_heads + g) * n_rows + t) * dh + 32 * mb + 4 * h) * 2 : nullptr;
                recon_emit_block<E, kI8>(acc[tile], e->d.bl, col + 32 * mb + 4 * h, out_scale, srow, orow, colsum + 32 * mb + 4 * h, rq[tile]);
            }
        }
        if (stage) {
#pragma unroll
            for (int tile = 0; tile < TL; ++tile) {
                const int t0 = chunk0 + wave * 32 * TL + tile * 32;
                if (t0 < n_rows)
                    recon_flush_tile(stage + tile * 32 * stride_o, stride_o, dst + (((size_t)b * p->n_kv_heads + g) * n_rows + t0) * dh * 2, n_rows - t0, cpr, lane);
            }
        }
    }
}

// Two-layer decoder (FC -> activation -> FC): the hidden rows stay in registers between the two products.
//   H^T[c, t] = W1^T . Z^T   per 32-column block of the hidden width; + b1, activation, rounded to 16 bits:
//               the result layout (lane: token l32, hidden rows 8a + 4h + j of the block) is the B-operand layout
//               of the second product with the rows of a k-step taken in register order
//   X^^T[n, t] = Wl^T[n, c] . H^T[c, t]   per KV head and 32-column block of the head
// W1 [R, C] stays in LDS for the whole workgroup; the slice [C, d_head] of the last layer passes through LDS per head.
template <typename E, int R, int C, int ACT, bool kI8, int TL>
__global__ __launch_bounds__(64 * kReconChunk / (32 * TL)) void recon_mlp_mfma_kernel(ReconParams) {
    constexpr int NT = 64 * kReconChunk / (32 * TL);      // threads
    constexpr int KS = R / 16;          // k-steps of the first product
    constexpr int CB = C / 32;          // 32-column blocks of the hidden width
    constexpr int STRIDE1 = 2 * C + 32; // LDS row stride of W1
    extern __shared__ __attribute__((aligned(16))) char lds[];
    RArgs p = (RArgs)__builtin_amdgcn_kernarg_segment_ptr();
    REntry e = &p->e[blockIdx.z];
    const int b = blockIdx.y, chunk0 = blockIdx.x * kReconChunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5, l16 = lane & 15;
    const int dh = p->d_head, n_rows = p->n_rows;
    const int stride_w = 2 * dh + 32, cpr = dh >> 3;
    char* w1_lds = lds;
    char* wl_lds = lds + R * STRIDE1;
    const int stride_o = recon_stage_stride(dh);
    char* stage = p->staged ? wl_lds + C * stride_w + wave * 32 * TL * stride_o : nullptr;
    const float slope = e->d.slope;

    u32x4_t zb[TL][KS];
    RowQuant rq[TL];
    recon_load_rows<E, R, kI8, TL>(zb, rq, e, p, b, chunk0 + wave * 32 * TL, l32, h);         // in flight while W1 is staged
    recon_stage_matrix(w1_lds, STRIDE1, static_cast<const char*>(e->d.w1), (size_t)C * 2, R, C / 8, tid, NT);
    float* b1s = reinterpret_cast<float*>(wl_lds + C * stride_w + (p->staged ? kReconChunk * stride_o : 0));      // [C] first-layer bias
    float* cs1 = b1s + C;                                                                                           // [C] column sums of W1 (int8 rows)
    for (int i = tid; i < C; i += NT) b1s[i] = e->d.b1 ? Elem<E>::load(e->d.b1, i) : 0.f;
    __syncthreads();
    if constexpr (kI8) {
        lds_column_sums<E>(cs1, w1_lds, STRIDE1, R, C, tid, NT);
        __syncthreads();
    }

    // hidden rows of the wave's two tiles as B operands of the second product: [tile][block][k-step]
    u32x4_t hb[TL][CB][2];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const char* wsrc = w1_lds + (8 * h + (l16 >> 2)) * STRIDE1 + (32 * cb + 16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
        f32x16_t acc[TL];
#pragma unroll
        for (int tile = 0; tile < TL; ++tile)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tile][v] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4_t wa = tr_pair32(wsrc + 16 * s * STRIDE1, 4 * STRIDE1);
#pragma unroll
            for (int tile = 0; tile < TL; ++tile) acc[tile] = Mma32<E>::mfma(wa, zb[tile][s], acc[tile]);
        }
        // bias of this lane's hidden rows 32 cb + 8a + 4h + j, from the fp32 copy in LDS (global loads here would all be
        // hoisted to the top of the unrolled loop and hold 16 registers per block)
        float bias[16];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4_t b4 = *reinterpret_cast<const f32x4_t*>(b1s + 32 * cb + 8 * a + 4 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) bias[4 * a + j] = b4[j];
        }
#pragma unroll
        for (int tile = 0; tile < TL; ++tile) {
            // pre-activations; int8 rows: the row's scale and zero point applied to the sums over its codes
            float pre[16];
            if constexpr (kI8) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x4_t c4 = *reinterpret_cast<const f32x4_t*>(cs1 + 32 * cb + 8 * a + 4 * h);
#pragma unroll
                    for (int j = 0; j < 4; ++j) pre[4 * a + j] = fmaf(fmaf(-rq[tile].sub, c4[j], acc[tile][4 * a + j]), rq[tile].inv, bias[4 * a + j]);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) pre[v] = acc[tile][v] + bias[v];
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                unsigned w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    w[q] = Mma<E>::pack2(fast_act<ACT>(pre[8 * s + 2 * q], slope), fast_act<ACT>(pre[8 * s + 2 * q + 1], slope));
                hb[tile][cb][s] = u32x4_t{w[0], w[1], w[2], w[3]};
            }
        }
    }

    const char* wl = static_cast<const char*>(e->d.wl);
    const int in_width = e->d.in_width;
    char* dst = static_cast<char*>(e->which == KVCAR_K ? p->khat : p->vhat);
    const float out_scale = e->which == KVCAR_K ? p->k_scale : 1.f;      // keys carry softmax scale * log2(e) into their one rounding
    for (int hi = 0; hi < e->n_heads; ++hi) {
        const int g = e->head[hi], col = e->col[hi];
        __syncthreads();                           // the previous slice is no longer read
        recon_stage_matrix(wl_lds, stride_w, wl + (size_t)col * 2, (size_t)in_width * 2, C, cpr, tid, NT);
        __syncthreads();
        for (int mb = 0; mb < (dh >> 5); ++mb) {
            // A operand: row = decoder column 32 mb + l32; k-slots of k-step s of block cb = hidden rows
            // 32 cb + 16 s + 8(e/4) + 4h + e%4
            const char* wsrc = wl_lds + (4 * h + (l16 >> 2)) * stride_w + (32 * mb + 16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
            f32x16_t acc[TL];
#pragma unroll
            for (int tile = 0; tile < TL; ++tile)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tile][v] = 0.f;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const u32x4_t wa = tr_pair32(wsrc + (32 * cb + 16 * s) * stride_w, 8 * stride_w);
#pragma unroll
                    for (int tile = 0; tile < TL; ++tile) acc[tile] = Mma32<E>::mfma(wa, hb[tile][cb][s], acc[tile]);
                }
#pragma unroll
            for (int tile = 0; tile < TL; ++tile) {
                const int t = chunk0 + wave * 32 * TL + tile * 32 + l32;
                char* srow = stage ? stage + (tile * 32 + l32) * stride_o + (32 * mb + 4 * h) * 2 : nullptr;
                char* orow = t < n_rows ? dst + ((((size_t)b * p->n_kv_heads + g) * n_rows + t) * dh + 32 * mb + 4 * h) * 2 : nullptr;
                recon_emit_block<E, false>(acc[tile], e->d.bl, col + 32 * mb + 4 * h, out_scale, srow, orow, nullptr, RowQuant{1.f, 0.f});
            }
        }
        if (stage) {
#pragma unroll
            for (int tile = 0; tile < TL; ++tile) {
                const int t0 = chunk0 + wave * 32 * TL + tile * 32;
                if (t0 < n_rows)
                    recon_flush_tile(stage + tile * 32 * stride_o, stride_o, dst + (((size_t)b * p->n_kv_heads + g) * n_rows + t0) * dh * 2, n_rows - t0, cpr, lane);
            }
        }
    }
}


static bool recon_width_ok(int r) { return r % 32 == 0 && r >= 32 && r <= 384; }      // every width a GPT-2 or TinyLlama layer can store under a reuse map

// Two-layer decoders: the (latent, hidden) shapes with an instance
static bool recon_mlp_shape_ok(const SideDesc& sd) {
    return ((sd.r == 128 && sd.c == 256) || (sd.r == 64 && sd.c == 128)) && (sd.act == KVCAR_ACT_GELU || sd.act == KVCAR_ACT_LEAKY_RELU);
}

bool recon_mfma_supported(const ReconParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.n_entries < 1) return false;
    if (p.d_head % 32 != 0) return false;
    for (int i = 0; i < p.n_entries; ++i) {
        const SideDesc& sd = p.e[i].d;
        if (sd.in_width % 8 != 0) return false;
        if (sd.w1 != nullptr) {
            if (!recon_mlp_shape_ok(sd)) return false;
            if ((size_t)sd.r * (2 * sd.c + 32) + (size_t)sd.c * (2 * p.d_head + 32) > 150 * 1024) return false;
        } else {
            if (!recon_width_ok(sd.r)) return false;
            if ((size_t)sd.r * (2 * p.d_head + 32) > 150 * 1024) return false;
        }
    }
    return true;
}

template <typename E, int R, bool kI8>
static hipError_t launch_recon_one(const ReconParams& p, hipStream_t stream) {
    size_t lds = (size_t)R * (2 * p.d_head + 32);
    const size_t sums = kI8 ? (size_t)p.d_head * sizeof(float) : 0;            // column sums of the decoder slice (int8 rows)
    ReconParams q = p;
    q.staged = lds + recon_stage_bytes(p.d_head) + sums <= kReconLdsMax ? 1 : 0;      // else the lanes store their 8-byte pieces themselves
    if (q.staged) lds += recon_stage_bytes(p.d_head);
    lds += sums;
    constexpr int TL = 2;               // four waves of 64 tokens (eight of 32 measured the same)
    auto k = recon_mfma_kernel<E, R, kI8, TL>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    dim3 grid((p.n_rows + kReconChunk - 1) / kReconChunk, p.batch, p.n_entries);
    hipLaunchKernelGGL(k, grid, dim3(64 * kReconChunk / (32 * TL)), lds, stream, q);
    return hipGetLastError();
}

template <typename E, bool kI8>
static hipError_t launch_recon_width(const ReconParams& p, int r, hipStream_t stream) {
    switch (r) {
        case 32: return launch_recon_one<E, 32, kI8>(p, stream);
        case 64: return launch_recon_one<E, 64, kI8>(p, stream);
        case 96: return launch_recon_one<E, 96, kI8>(p, stream);
        case 128: return launch_recon_one<E, 128, kI8>(p, stream);
        case 160: return launch_recon_one<E, 160, kI8>(p, stream);
        case 192: return launch_recon_one<E, 192, kI8>(p, stream);
        case 224: return launch_recon_one<E, 224, kI8>(p, stream);
        case 256: return launch_recon_one<E, 256, kI8>(p, stream);
        case 288: return launch_recon_one<E, 288, kI8>(p, stream);
        case 320: return launch_recon_one<E, 320, kI8>(p, stream);
        case 352: return launch_recon_one<E, 352, kI8>(p, stream);
        case 384: return launch_recon_one<E, 384, kI8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

template <typename E, int R, int C, int ACT, bool kI8>
static hipError_t launch_recon_mlp_one(const ReconParams& p, hipStream_t stream) {
    size_t lds = (size_t)R * (2 * C + 32) + (size_t)C * (2 * p.d_head + 32);
    ReconParams q = p;
    q.staged = lds + recon_stage_bytes(p.d_head) + 2 * C * sizeof(float) <= kReconLdsMax ? 1 : 0;
    if (q.staged) lds += recon_stage_bytes(p.d_head);
    lds += 2 * C * sizeof(float);                               // the first-layer bias and the column sums of W1 in fp32
    constexpr int TL = 1;               // eight waves of 32 tokens: two waves per SIMD overlap their matrix and vector work
    auto k = recon_mlp_mfma_kernel<E, R, C, ACT, kI8, TL>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    dim3 grid((p.n_rows + kReconChunk - 1) / kReconChunk, p.batch, p.n_entries);
    hipLaunchKernelGGL(k, grid, dim3(64 * kReconChunk / (32 * TL)), lds, stream, q);
    return hipGetLastError();
}

template <typename E, bool kI8>
static hipError_t launch_recon_mlp(const ReconParams& p, const SideDesc& sd, hipStream_t stream) {
    const bool big = sd.r == 128;
    if (sd.act == KVCAR_ACT_GELU)
        return big ? launch_recon_mlp_one<E, 128, 256, KVCAR_ACT_GELU, kI8>(p, stream) : launch_recon_mlp_one<E, 64, 128, KVCAR_ACT_GELU, kI8>(p, stream);
    return big ? launch_recon_mlp_one<E, 128, 256, KVCAR_ACT_LEAKY_RELU, kI8>(p, stream) : launch_recon_mlp_one<E, 64, 128, KVCAR_ACT_LEAKY_RELU, kI8>(p, stream);
}

// Entries of different shapes go out in launches of their own (widths and activation are template arguments).
hipError_t launch_recon_mfma(const ReconParams& p, int dtype, hipStream_t stream) {
    bool done[kMaxReconEntries] = {};
    auto same = [](const SideDesc& a, const SideDesc& b) {
        return a.r == b.r && (a.w1 != nullptr) == (b.w1 != nullptr) && (a.w1 == nullptr || (a.c == b.c && a.act == b.act));
    };
    for (int i = 0; i < p.n_entries; ++i) {
        if (done[i]) continue;
        ReconParams sub = p;
        sub.n_entries = 0;
        for (int k = i; k < p.n_entries; ++k)
            if (!done[k] && same(p.e[k].d, p.e[i].d)) { sub.e[sub.n_entries++] = p.e[k]; done[k] = true; }
        const SideDesc& sd = sub.e[0].d;
        const bool i8 = sd.meta != nullptr;
        hipError_t err;
        if (sd.w1 != nullptr) {
            if (dtype == KVCAR_BF16) err = i8 ? launch_recon_mlp<BF16, true>(sub, sd, stream) : launch_recon_mlp<BF16, false>(sub, sd, stream);
            else err = i8 ? launch_recon_mlp<F16, true>(sub, sd, stream) : launch_recon_mlp<F16, false>(sub, sd, stream);
        } else {
            if (dtype == KVCAR_BF16) err = i8 ? launch_recon_width<BF16, true>(sub, sd.r, stream) : launch_recon_width<BF16, false>(sub, sd.r, stream);
            else err = i8 ? launch_recon_width<F16, true>(sub, sd.r, stream) : launch_recon_width<F16, false>(sub, sd.r, stream);
        }
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------------------
// causal attention over the decoded rows
// ---------------------------------------------------------------------------------------------------------
constexpr int kKvTile = 64;           // decoded rows per LDS tile
constexpr float kSlack = 8.f;         // a query's softmax reference point moves when a score exceeds it by 2^kSlack
// Launch shape (measured on 16 x 4096 tokens, 32 heads of 64: TFLOP/s of the kernel):
//   one 32-query block per wave, 8 waves, 2 workgroups per CU (4 waves per SIMD)   887      <- used (970 after later savings)
//   two blocks per wave, 4 waves, 2 workgroups per CU (2 waves per SIMD)            835
//   two blocks per wave, 8 waves, 1 workgroup per CU                                779;  with 128-row tiles 808
//   two blocks per wave, 4 waves, 1 workgroup per CU (1 wave per SIMD)              485
// Workgroup indices dealt plainly instead of per XCD: 8 % slower; raising the wave priority over the matrix
// instructions: no gain.
constexpr int kPrefillQB = 1, kPrefillNW = 8;

template <int DH> struct PrefillGeo {
    static constexpr int kStrideK = 2 * DH + 16;                 // an odd number of 16-byte units: 128-bit reads hit every bank once
    static constexpr int kStrideV = DH == 64 ? 192 : 320;        // 64 or 192 modulo 256: the transposing reads hit every bank once
    static constexpr int kBuf = kKvTile * (kStrideK + kStrideV);
};

template <typename E, int DH, int QB, int NW, int OCC>
__global__ __launch_bounds__(64 * NW, OCC) void prefill_mfma_kernel(PrefillParams p, int n_qblk, int per_xcd) {
    using G = PrefillGeo<DH>;
    constexpr int KS = DH / 16;                 // k-steps of the score product
    constexpr int DB = DH / 32;                 // 32-column blocks of the output
    constexpr int TQ = NW * 32 * QB;            // query tokens per workgroup
    constexpr int NT = 64 * NW;                 // threads
    constexpr int NLD = (kKvTile * DH / 8) / NT; // 16-byte chunks per thread per tile and tensor
    static_assert(NLD * NT == kKvTile * DH / 8, "tile chunks divide over the threads");
    constexpr int CPR = DH / 8;                 // 16-byte chunks per decoded row
    extern __shared__ __attribute__((aligned(16))) char lds[];

    // Which (sequence, KV head) pair, query block and head this workgroup takes.  Hardware deals workgroup ids
    // round-robin over the 8 XCDs, each with its own L2; workgroups that share decoded rows - the query heads of
    // one pair - should meet in one L2, every XCD should get the same work, and heavy (late) query blocks should
    // start first.  per_xcd > 0: the pairs divide evenly over the XCDs; each XCD takes a contiguous run of pairs,
    // one pair after the other, heaviest blocks first.  per_xcd == 0: any other shape (e.g. one long prompt): the
    // (query block, pair) combinations, heaviest blocks first, are dealt round-robin over the XCDs, the heads of a
    // combination staying together.
    const int gq = p.n_q_heads / p.n_kv_heads;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int pair, qblk, jq;
    if (per_xcd > 0) {
        const int vid = xcd * per_xcd + slot;
        const int per_pair = gq * n_qblk;
        pair = vid / per_pair;
        const int rem = vid - pair * per_pair;
        qblk = n_qblk - 1 - rem / gq;
        jq = rem % gq;
    } else {
        const int n_pairs = p.batch * p.n_kv_heads;
        const int combo = (slot / gq) * 8 + xcd;
        if (combo >= n_pairs * n_qblk) return;
        const int rank = combo / n_pairs;
        pair = combo - rank * n_pairs;
        qblk = n_qblk - 1 - rank;
        jq = slot % gq;
    }
    const int b = pair / p.n_kv_heads, g = pair - b * p.n_kv_heads;
    const int j = g * gq + jq;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5, l16 = lane & 15;
    const int i0 = qblk * TQ + wave * 32 * QB;  // first query token of this wave

    // queries as B operands: lane (token l32 of block qb, half h) holds components 16s + 8h .. +7 (the decoded keys
    // carry scale * log2(e), so the score product comes out in log2 units).  Decoded rows are fp16 (RowsOf), so both
    // products run on the fp16 matrix instruction: a bf16 model's queries are converted here (saturating) and its
    // probabilities are packed to fp16; only the output is rounded to the model dtype.
    using W = F16;
    u32x4_t qB[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int i = i0 + 32 * qb + l32;
        const char* qrow = static_cast<const char*>(p.q) + ((((size_t)b * p.t_new + min(i, p.t_new - 1)) * p.n_q_heads + j) * DH + 8 * h) * 2;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (i < p.t_new) v = *reinterpret_cast<const u32x4_t*>(qrow + 32 * s);
            if constexpr (std::is_same<E, BF16>::value) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = Mma<F16>::pack2(sat_half(Mma<BF16>::unpack_lo(v[e])), sat_half(Mma<BF16>::unpack_hi(v[e])));
            }
            qB[qb][s] = v;
        }
    }

    const int wg_last = p.pos0 + min(p.t_new, (qblk + 1) * TQ) - 1;           // last position any query of the workgroup sees
    const int n_tiles = wg_last / kKvTile + 1;
    const int wave_tiles = i0 < p.t_new ? (p.pos0 + min(p.t_new, i0 + 32 * QB) - 1) / kKvTile + 1 : 0;
    const char* kbase = static_cast<const char*>(p.khat) + ((size_t)b * p.n_kv_heads + g) * p.n_rows * DH * 2;
    const char* vbase = static_cast<const char*>(p.vhat) + ((size_t)b * p.n_kv_heads + g) * p.n_rows * DH * 2;

    u32x4_t stk[NLD], stv[NLD];
    auto issue = [&](int jt) {
        const int valid = max(0, min(kKvTile, p.n_rows - jt * kKvTile)) * CPR;
        const size_t off = (size_t)jt * kKvTile * DH * 2;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = i * NT + tid;
            u32x4_t a = {0u, 0u, 0u, 0u}, v = {0u, 0u, 0u, 0u};
            if (f < valid) {
                a = *reinterpret_cast<const u32x4_t*>(kbase + off + (size_t)f * 16);
                v = *reinterpret_cast<const u32x4_t*>(vbase + off + (size_t)f * 16);
            }
            stk[i] = a; stv[i] = v;
        }
    };
    auto park = [&](int buf) {
        char* kl = lds + buf * G::kBuf;
        char* vl = kl + kKvTile * G::kStrideK;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = i * NT + tid;
            const int row = f / CPR, ch = f % CPR;
            *reinterpret_cast<u32x4_t*>(kl + row * G::kStrideK + ch * 16) = stk[i];
            *reinterpret_cast<u32x4_t*>(vl + row * G::kStrideV + ch * 16) = stv[i];
        }
    };

    f32x16_t acc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[qb][db][v] = 0.f;
    // -m of every query (m = the reference point of its softmax, log2 units) as the score product's initial
    // accumulator: the product then delivers score - m and the exponent needs no subtraction
    f32x16_t negm[QB];
    float l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        l_run[qb] = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) negm[qb][v] = 0.f;
    }

    issue(0);
    park(0);
    __syncthreads();
    for (int jt = 0; jt < n_tiles; ++jt) {
        if (jt + 1 < n_tiles) issue(jt + 1);
        if (jt < wave_tiles) {
            const char* kl = lds + (jt & 1) * G::kBuf;
            const char* vl = kl + kKvTile * G::kStrideK;

            const char* krow = kl + l32 * G::kStrideK + h * 16;
            const char* vrow = vl + (4 * h + (l16 >> 2)) * G::kStrideV + (16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
            // the tile in two halves of 32 rows: scores, softmax and the output product of a half need half the registers
#pragma unroll
            for (int kvb = 0; kvb < kKvTile / 32; ++kvb) {
                // ---- scores: S^T[row, q]; this lane: query l32 of block qb, rows 32 kvb + 8a + 4h + j (register 4a + j)
                f32x16_t s[QB];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const u32x4_t ka = *reinterpret_cast<const u32x4_t*>(krow + 32 * kvb * G::kStrideK + ks * 32);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) s[qb] = Mma32<W>::mfma(ka, qB[qb][ks], ks == 0 ? negm[qb] : s[qb]);
                }

                u32x4_t pb[QB][2];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    // ---- the causal limit: only where the half reaches past the block's first query
                    const int qpos0 = p.pos0 + i0 + 32 * qb;
                    const int row0 = jt * kKvTile + 32 * kvb;
                    if (row0 + 31 > qpos0) {
                        asm volatile("");             // keeps this a branch instead of 16 selects on every half
                        const int lim = qpos0 + l32 - row0 - 4 * h;      // last visible row of the half, less this lane's row offset
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (8 * (v >> 2) + (v & 3) > lim) s[qb][v] = -INFINITY;
                    }
                    // ---- online softmax in base 2.  s holds score - m.  The reference point m of a query only moves
                    // when a score exceeds it by more than kSlack: until then probabilities simply grow up to 2^kSlack,
                    // which costs nothing in fp32 / 16-bit floating point, and the accumulators need no rescaling - a
                    // rare event instead of one in most halves.  The very first half sets m (it holds row 0, which
                    // every query sees, so the maximum is finite).
                    float mx = fmaxf(fmaxf(s[qb][0], s[qb][1]), s[qb][2]);
#pragma unroll
                    for (int v = 3; v < 15; v += 2) mx = fmaxf(fmaxf(mx, s[qb][v]), s[qb][v + 1]);
                    mx = fmaxf(mx, s[qb][15]);
                    // the two lanes of a query (one per half of the wave) meet only when one of them has to move
                    const bool first = jt == 0 && kvb == 0;
                    if (__builtin_amdgcn_ballot_w64(mx > kSlack || first) != 0) {
                        mx = fmaxf(mx, __shfl_xor(mx, 32));
                        const bool moved = mx > kSlack || first;
                        const float delta = moved ? mx : 0.f;
                        const float alpha = __builtin_amdgcn_exp2f(-delta);
                        l_run[qb] *= alpha;
#pragma unroll
                        for (int db = 0; db < DB; ++db) acc[qb][db] *= alpha;
#pragma unroll
                        for (int v = 0; v < 16; ++v) { negm[qb][v] -= delta; s[qb][v] -= delta; }
                    }
                    float e[16];
#pragma unroll
                    for (int v = 0; v < 16; ++v) e[v] = __builtin_amdgcn_exp2f(s[qb][v]);
                    // k-step s2 of the half: rows 16 s2 + 8(e/4) + 4h + e%4 = registers 8 s2 .. 8 s2 + 7
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2)
                        pb[qb][s2] = u32x4_t{Mma<W>::pack2(e[8 * s2], e[8 * s2 + 1]), Mma<W>::pack2(e[8 * s2 + 2], e[8 * s2 + 3]),
                                             Mma<W>::pack2(e[8 * s2 + 4], e[8 * s2 + 5]), Mma<W>::pack2(e[8 * s2 + 6], e[8 * s2 + 7])};
                    // the denominator sums the probabilities as rounded for the product (two chains of four pairs)
                    float la = 0.f, lb = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) { la = PairSum<W>::add(la, pb[qb][0][w]); lb = PairSum<W>::add(lb, pb[qb][1][w]); }
                    l_run[qb] += la + lb;
                }

                // ---- O^T[d, q] += V^^T . P^T
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const u32x4_t va = tr_pair32(vrow + (32 * kvb + 16 * s2) * G::kStrideV + db * 64, 8 * G::kStrideV);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) acc[qb][db] = Mma32<W>::mfma(va, pb[qb][s2], acc[qb][db]);
                    }
            }
        }
        if (jt + 1 < n_tiles) park((jt + 1) & 1);
        __syncthreads();
    }

    // ---- normalise and store: this lane holds query l32 of block qb, components 32 db + 8a + 4h + j
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int i = i0 + 32 * qb + l32;
        const float l_all = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (i >= p.t_new) continue;
        const float inv = 1.f / l_all;
        char* orow = static_cast<char*>(p.out) + ((((size_t)b * p.t_new + i) * p.n_q_heads + j) * DH + 4 * h) * 2;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<u32x2_t*>(orow + (32 * db + 8 * a) * 2) =
                    u32x2_t{Mma<E>::pack2(acc[qb][db][4 * a] * inv, acc[qb][db][4 * a + 1] * inv),
                            Mma<E>::pack2(acc[qb][db][4 * a + 2] * inv, acc[qb][db][4 * a + 3] * inv)};
    }
}

bool prefill_mfma_supported(const PrefillParams& p, int dtype) {
    if (dtype == KVCAR_F32) return false;
    return p.d_head == 64 || p.d_head == 128;
}

template <typename E, int DH, int QB, int NW, int OCC>
static hipError_t launch_prefill_one(const PrefillParams& p, hipStream_t stream) {
    constexpr int TQ = NW * 32 * QB;
    const int n_qblk = (p.t_new + TQ - 1) / TQ;
    const long long total = (long long)p.batch * p.n_q_heads * n_qblk;
    if (total > (1ll << 30)) return hipErrorInvalidValue;
    const int gq = p.n_q_heads / p.n_kv_heads, n_pairs = p.batch * p.n_kv_heads;
    int per_xcd = 0, grid;
    if (n_pairs % 8 == 0) {
        per_xcd = (int)(total / 8);
        grid = (int)total;
    } else {
        const long long combos = (long long)n_pairs * n_qblk;
        grid = (int)((combos + 7) / 8 * 8 * gq);
    }
    const size_t lds = 2 * (size_t)PrefillGeo<DH>::kBuf;
    auto k = prefill_mfma_kernel<E, DH, QB, NW, OCC>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(64 * NW), lds, stream, p, n_qblk, per_xcd);
    return hipGetLastError();
}

hipError_t launch_prefill_mfma(const PrefillParams& p, int dtype, int /*n_cu*/, hipStream_t stream) {
    // d_head 128: twice the accumulators and query operands per wave, so one workgroup per compute unit
    if (p.d_head == 128) {
        if (dtype == KVCAR_BF16) return launch_prefill_one<BF16, 128, kPrefillQB, kPrefillNW, 1>(p, stream);
        return launch_prefill_one<F16, 128, kPrefillQB, kPrefillNW, 1>(p, stream);
    }
    if (dtype == KVCAR_BF16) return launch_prefill_one<BF16, 64, kPrefillQB, kPrefillNW, 2>(p, stream);
    return launch_prefill_one<F16, 64, kPrefillQB, kPrefillNW, 2>(p, stream);
}

}  // namespace kvcar
