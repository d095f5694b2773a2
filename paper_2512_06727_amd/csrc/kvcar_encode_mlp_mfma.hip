// MFMA encode + append for TWO-LAYER encoders (gfx950, 16-bit dtypes): z = act(x[cols] W1 + b1) W2 + b2
// ("Network Architecture", 2nd paragraph: the encoder is two fully connected layers with an activation
// in between), for prefill (many tokens) and decode steps alike.
//
// A wave owns 32 tokens and walks the hidden width in blocks of 32 columns:
//   H^T[hidden blk, token] = W1^T . X^T   v_mfma_f32_32x32x16 (A = a column slice of W1 read from LDS with
//                                          the transposing load, B = the token rows, resident in registers)
//   -> + b1, activation, split into a hi + lo pair of 16-bit values: the result layout IS an operand
//      layout of the second product, so the hidden activations never leave registers
//   Z^T[r, token] += W2[hidden blk, :]^T . H^T[hidden blk, token]   (A = a row slice of W2, transposing load):
//      formed transposed, so that a lane ends with consecutive latent columns of one token (8-byte stores)
// The two weight slices of a later hidden block are fetched into registers while the current block
// computes and written to another of the LDS buffers: one barrier per hidden block.
// The latent is rounded once, from the fp32 accumulator, to the cache dtype and appended.
#include "kvcar_qtilde_mfma.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct EMma;
template <> struct EMma<BF16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        bf16x2_t v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(unsigned, v);
    }
    static __device__ __forceinline__ float unpack_lo(unsigned w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float unpack_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
    static __device__ __forceinline__ uint16_t to16(float v) { return f32_to_bf16_bits(v); }
};
template <> struct EMma<F16> {
    static __device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
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

__device__ __forceinline__ u32x4_t tr_pair(const char* p, int second_offset) {
    const s16x4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
    const s16x4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + second_offset));
    const u32x2_t a0 = __builtin_bit_cast(u32x2_t, t0), a1 = __builtin_bit_cast(u32x2_t, t1);
    return u32x4_t{a0[0], a0[1], a1[0], a1[1]};
}

constexpr int kEmTokens = 128;       // tokens per workgroup (4 waves x 32)
constexpr int kW1Stride = 64 + 32;   // LDS row stride of a [in, 32] slice of W1 (bytes)

// KX: k-steps over the input width (in_width == 16 KX exactly); NBZ: 32-column blocks of the latent
// (r == 32 NBZ exactly); GELU: the activation is GELU, else leaky ReLU with the side's slope (the identity
// is slope 1). Exact compile-time shapes keep the whole hidden-block body one straight-line block: with
// run-time guards every transposing load sat in a block of its own and paid its LDS latency serially.
// kSmall (launches of a few tokens: a decode step): a workgroup takes 32 tokens and its four waves split the HIDDEN
// blocks instead of the tokens - with 16 tokens one wave would otherwise walk all blocks alone, a chain of dependent
// matrix and vector work (18 us for 256 -> 256 -> 128).  Four weight slices are staged per round, wave w computes
// block 4 round + w, the waves' partial latent rows are added in wave order through LDS and wave 0 appends them.
template <typename E, int KX, int NBZ, bool GELU, bool kSmall>
__device__ __forceinline__ void encode_mlp_mfma_body(const EncodeParams& p, int side0, char* lds) {
    const EncodeSide& s = p.s[blockIdx.y + side0];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5, l16 = lane & 15;
    const int n_tok = p.batch * p.t_new;
    const int tok0 = kSmall ? blockIdx.x * 32 : blockIdx.x * kEmTokens + wave * 32;     // first token of this wave's tile
    const int tok = tok0 + l32;                                     // the token column (B operand) of this lane
    const bool tok_ok = tok < n_tok;
    constexpr int in_w = 16 * KX, r = 32 * NBZ;
    constexpr int w2_stride = 2 * r + 32;
    constexpr int w2_off = in_w * kW1Stride;
    constexpr int buf_bytes = w2_off + 32 * w2_stride;
    const int hid = s.hidden;
    const int n_mb = hid >> 5;
    const float slope = s.act == KVCAR_ACT_LEAKY_RELU ? s.slope : 1.f;

    // token rows, resident: k-step ks holds input columns 16ks + 8h .. +7 of this lane's token
    u32x4_t xr[KX];
    {
        const char* xrow = static_cast<const char*>(s.x) + (size_t)(tok_ok ? tok : 0) * p.d_kv * 2;
        // input column 16 ks + 8 h sits in stored head hi at offset off + 8 h (d_head is a multiple of 16 here): the
        // pair (hi, off) steps along with ks, no division per k-step
        int hi = 0, off = 0;
#pragma unroll
        for (int ks = 0; ks < KX; ++ks) {
            const int src_col = (int)s.heads[hi] * p.d_head + off + 8 * h;
            u32x4_t v = *reinterpret_cast<const u32x4_t*>(xrow + src_col * 2);
            if (!tok_ok) v = u32x4_t{0u, 0u, 0u, 0u};
            xr[ks] = v;
            off += 16;
            if (off >= p.d_head) { off -= p.d_head; ++hi; }
        }
    }

    // weight slices of hidden block mb: W1[:, 32mb .. +32] (in_w rows of 64 bytes) and W2[32mb .. +32, :]
    // (32 rows of 2r bytes); 16-byte chunk f of the pair belongs to thread f % 256
    constexpr int c1 = in_w * 4, c2 = 32 * (r >> 3), cpr = r >> 3;
    constexpr int n_pre = (c1 + c2 + 255) / 256;
    auto fetch = [&](u32x4_t (&pre)[n_pre], int mb) {
#pragma unroll
        for (int i = 0; i < n_pre; ++i) {
            const int f = i * 256 + tid;
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (f < c1) {
                const int row = f >> 2, ch = f & 3;
                v = *reinterpret_cast<const u32x4_t*>(static_cast<const char*>(s.w1) + ((size_t)row * hid + 32 * mb) * 2 + ch * 16);
            } else if (f < c1 + c2) {
                const int g2 = f - c1;
                const int row = g2 / cpr, ch = g2 - row * cpr;
                v = *reinterpret_cast<const u32x4_t*>(static_cast<const char*>(s.w2) + ((size_t)(32 * mb + row) * r) * 2 + ch * 16);
            }
            pre[i] = v;
        }
    };
    auto park = [&](const u32x4_t (&pre)[n_pre], char* buf) {
#pragma unroll
        for (int i = 0; i < n_pre; ++i) {
            const int f = i * 256 + tid;
            if (f < c1) {
                const int row = f >> 2, ch = f & 3;
                *reinterpret_cast<u32x4_t*>(buf + row * kW1Stride + ch * 16) = pre[i];
            } else if (f < c1 + c2) {
                const int g2 = f - c1;
                const int row = g2 / cpr, ch = g2 - row * cpr;
                *reinterpret_cast<u32x4_t*>(buf + w2_off + row * w2_stride + ch * 16) = pre[i];
            }
        }
    };

    f32x16_t accz[NBZ];
#pragma unroll
    for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) accz[nb][v] = 0.f;

    // first-layer bias -> LDS (fp32), read from there inside the loop: a global load in the loop body
    // would queue behind the weight prefetch and serialise its latency into every block
    constexpr int NBUF = kSmall ? 4 : 2;
    float* b1s = reinterpret_cast<float*>(lds + NBUF * buf_bytes);
    for (int i = tid; i < hid; i += 256) b1s[i] = s.b1 ? Elem<E>::load(s.b1, i) : 0.f;
    float* b2s = b1s + 1024;                     // second-layer bias [r], past the largest first-layer bias
    for (int i = tid; i < r; i += 256) b2s[i] = s.b2 ? Elem<E>::load(s.b2, i) : 0.f;

    // one hidden block: hidden rows, activation, their share of the latent rows
    auto block = [&](int mb, const char* buf) {
        // bias of this lane's hidden rows 32mb + 8a + 4h + j: four 16-byte reads
        f32x4_t bq[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) bq[a] = *reinterpret_cast<const f32x4_t*>(b1s + 32 * mb + 8 * a + 4 * h);

        // ---- H^T[hidden blk, token] ------------------------------------------------------------
        f32x16_t ht;               // starts from the bias: no addition per hidden value afterwards
#pragma unroll
        for (int v = 0; v < 16; ++v) ht[v] = bq[v >> 2][v & 3];
        const char* w1row = buf + (8 * h + (l16 >> 2)) * kW1Stride + (16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
#pragma unroll
        for (int ks = 0; ks < KX; ++ks)
            ht = EMma<E>::mfma(tr_pair(w1row + 16 * ks * kW1Stride, 4 * kW1Stride), xr[ks], ht);
        // lane: token l32, hidden rows 32mb + 8a + 4h + j  (register v = 4a + j)
        u32x4_t hi[2], lo[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            unsigned wh[4], wl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float a[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int v = 8 * s2 + 2 * e + q;
                    const float x = ht[v];
                    if constexpr (GELU) a[q] = pinned(0.5f * x * (1.f + erf_rational(x * 0.70710678118654752f)));
                    else a[q] = pinned(x >= 0.f ? x : slope * x);
                }
                wh[e] = EMma<E>::pack2(a[0], a[1]);
                wl[e] = EMma<E>::pack2(a[0] - EMma<E>::unpack_lo(wh[e]), a[1] - EMma<E>::unpack_hi(wh[e]));
            }
            hi[s2] = u32x4_t{wh[0], wh[1], wh[2], wh[3]};
            lo[s2] = u32x4_t{wl[0], wl[1], wl[2], wl[3]};
        }
        // ---- Z^T[:, token] += W2[hidden blk, :]^T . H^T[hidden blk, token] (formed transposed: a lane then holds
        // consecutive latent columns of ONE token and the epilogue stores 8 bytes at a time) -----------------
        // k-slots of lane half h in k-step s2 are hidden rows 16 s2 + 4h + j and 16 s2 + 8 + 4h + j
        const char* w2base = buf + w2_off + (4 * h + (l16 >> 2)) * w2_stride + (16 * (l32 >> 4) + 4 * (l16 & 3)) * 2;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int nb = 0; nb < NBZ; ++nb) {
                const u32x4_t bw = tr_pair(w2base + 16 * s2 * w2_stride + nb * 64, 8 * w2_stride);
                accz[nb] = EMma<E>::mfma(bw, hi[s2], accz[nb]);
                accz[nb] = EMma<E>::mfma(bw, lo[s2], accz[nb]);
            }
    };

    if constexpr (kSmall) {
        u32x4_t pre[4][n_pre];
        auto fetch4 = [&](int mb0) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (mb0 + u < n_mb) fetch(pre[u], mb0 + u);
        };
        fetch4(0);
        for (int mb0 = 0; mb0 < n_mb; mb0 += 4) {
            if (mb0) __syncthreads();         // every wave is done with the previous round's slices
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (mb0 + u < n_mb) park(pre[u], lds + u * buf_bytes);
            if (mb0 + 4 < n_mb) fetch4(mb0 + 4);
            __syncthreads();
            if (mb0 + wave < n_mb) block(mb0 + wave, lds + wave * buf_bytes);
        }
        // the waves' partial latent rows, added in wave order (a fixed order); the slices' buffers are free now
        __syncthreads();
        float* part = reinterpret_cast<float*>(lds);       // [wave][NBZ][16][64]
#pragma unroll
        for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) part[((wave * NBZ + nb) * 16 + v) * 64 + lane] = accz[nb][v];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float a = part[(nb * 16 + v) * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) a += part[((w * NBZ + nb) * 16 + v) * 64 + lane];
                accz[nb][v] = a;
            }
    } else {
        u32x4_t pre[n_pre];
        fetch(pre, 0);
        for (int mb = 0; mb < n_mb; ++mb) {
            char* buf = lds + (mb & 1) * buf_bytes;
            park(pre, buf);
            if (mb + 1 < n_mb) fetch(pre, mb + 1);
            __syncthreads();      // slice mb visible; every wave is past block mb-1, whose buffer the next park reuses
            block(mb, buf);
        }
    }

    // ---- latent rows: bias, one rounding to the cache dtype, append --------------------------------
    // lane holds, for token l32 of the wave's tile, latent columns 32 nb + 8a + 4h + j (register 4a + j)
    const int t = tok;
    if (t >= n_tok) return;
    const int b = t / p.t_new, tt = t - b * p.t_new;
    const size_t row = (size_t)b * p.max_seq + (p.positions ? p.positions[b] : p.pos0) + tt;
#pragma unroll
    for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4_t b4 = *reinterpret_cast<const f32x4_t*>(b2s + 32 * nb + 8 * a + 4 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) accz[nb][4 * a + j] += b4[j];
        }
    if (s.meta) {
        // ---- int8 latents: the token's row lies in this lane and its partner in the other half ---------
        signed char* z8 = static_cast<signed char*>(s.z);
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                mn = fminf(mn, accz[nb][v]);
                mx = fmaxf(mx, accz[nb][v]);
            }
        mn = fminf(mn, __shfl_xor(mn, 32));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const QuantParams qp = quant_params(mn, mx);
#pragma unroll
        for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                unsigned w = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) w |= (unsigned)(unsigned char)quant_code(accz[nb][4 * a + j], qp) << (8 * j);
                *reinterpret_cast<unsigned*>(z8 + row * r + 32 * nb + 8 * a + 4 * h) = w;
            }
        if (h == 0) static_cast<RowMeta*>(s.meta)[row] = quant_meta(qp);
        return;
    }
    char* z = static_cast<char*>(s.z);
#pragma unroll
    for (int nb = 0; nb < NBZ; ++nb)
#pragma unroll
        for (int a = 0; a < 4; ++a)
            *reinterpret_cast<u32x2_t*>(z + (row * r + 32 * nb + 8 * a + 4 * h) * 2) =
                u32x2_t{EMma<E>::pack2(accz[nb][4 * a], accz[nb][4 * a + 1]), EMma<E>::pack2(accz[nb][4 * a + 2], accz[nb][4 * a + 3])};
}

template <typename E, int KX, int NBZ, bool GELU, bool kSmall>
__global__ __launch_bounds__(256, kSmall ? 1 : 2) void encode_mlp_mfma_kernel(EncodeParams p, int side0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    encode_mlp_mfma_body<E, KX, NBZ, GELU, kSmall>(p, side0, lds);
}

// A decode step's two small independent pieces in one launch: the new token's latent rows (the few-token form above, both
// tensors: workgroups blockIdx.x < enc_x) and the absorbed queries of the attention launch that follows
// (qtilde_mfma_block: the workgroups beyond, with blockIdx.y = 0, numbered (x, y, z) over a qx x qy x .. grid).
template <typename E, int KX, int NBZ, bool GELU>
__global__ __launch_bounds__(256, 1) void encode_mlp_step_qtilde_kernel(EncodeParams p, AttendParams q, int enc_x, int qx, int qy) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if ((int)blockIdx.x < enc_x) {
        encode_mlp_mfma_body<E, KX, NBZ, GELU, true>(p, 0, lds);
        return;
    }
    if (blockIdx.y != 0) return;
    const int id = (int)blockIdx.x - enc_x;
    qtilde_mfma_block<E>(&q, id % qx, (id / qx) % qy, id / (qx * qy), qx);
}

namespace {

struct EmShape { int kx, nbz; };
constexpr EmShape kEmShapes[] = {{4, 1}, {8, 2}, {12, 3}, {16, 4}, {16, 2}, {8, 1}};

bool em_side_ok(const EncodeSide& s) {
    if (s.hidden <= 0 || s.hidden % 32 || s.hidden > 1024) return false;
    if (s.act != KVCAR_ACT_GELU && s.act != KVCAR_ACT_LEAKY_RELU && s.act != KVCAR_ACT_NONE) return false;
    for (const EmShape& e : kEmShapes)
        if (s.in_width == 16 * e.kx && s.r == 32 * e.nbz) return true;
    return false;
}

template <typename E, int KX, int NBZ>
hipError_t em_launch_shape(const EncodeParams& p, int side0, int n_sides, bool gelu, hipStream_t stream) {
    const int n_tok = p.batch * p.t_new;
    constexpr size_t buf = (size_t)(16 * KX * kW1Stride + 32 * (64 * NBZ + 32)), biases = 4 * 1024 + 4 * 32 * NBZ;     // both biases in fp32
    // a few tokens (a decode step): 32 tokens per workgroup, the waves split the hidden blocks
    const bool small = n_tok <= kEmTokens && 4 * buf + biases <= 160 * 1024;
    dim3 grid(small ? (n_tok + 31) / 32 : (n_tok + kEmTokens - 1) / kEmTokens, n_sides);
    const size_t lds = (small ? 4 : 2) * buf + biases;
    void (*kern)(EncodeParams, int) = small ? (gelu ? encode_mlp_mfma_kernel<E, KX, NBZ, true, true> : encode_mlp_mfma_kernel<E, KX, NBZ, false, true>)
                                            : (gelu ? encode_mlp_mfma_kernel<E, KX, NBZ, true, false> : encode_mlp_mfma_kernel<E, KX, NBZ, false, false>);
    static AttrFlag attr[2][2] = {{false, false}, {false, false}};
    if (lds > 64 * 1024 && !attr[small][gelu]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (err != hipSuccess) return err;
        attr[small][gelu] = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p, side0);
    return hipGetLastError();
}

template <typename E>
hipError_t em_launch(const EncodeParams& p, int side0, int n_sides, hipStream_t stream) {
    const EncodeSide& s = p.s[side0];
    const bool gelu = s.act == KVCAR_ACT_GELU;
    const int kx = s.in_width / 16, nbz = s.r / 32;
    if (kx == 4 && nbz == 1) return em_launch_shape<E, 4, 1>(p, side0, n_sides, gelu, stream);
    if (kx == 8 && nbz == 2) return em_launch_shape<E, 8, 2>(p, side0, n_sides, gelu, stream);
    if (kx == 12 && nbz == 3) return em_launch_shape<E, 12, 3>(p, side0, n_sides, gelu, stream);
    if (kx == 16 && nbz == 4) return em_launch_shape<E, 16, 4>(p, side0, n_sides, gelu, stream);
    if (kx == 16 && nbz == 2) return em_launch_shape<E, 16, 2>(p, side0, n_sides, gelu, stream);
    if (kx == 8 && nbz == 1) return em_launch_shape<E, 8, 1>(p, side0, n_sides, gelu, stream);
    return hipErrorInvalidValue;
}

template <typename E, int KX, int NBZ>
hipError_t em_step_qtilde_shape(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, bool gelu, hipStream_t stream) {
    const int n_tok = p.batch * p.t_new;
    constexpr size_t buf = (size_t)(16 * KX * kW1Stride + 32 * (64 * NBZ + 32)), biases = 4 * 1024 + 4 * 32 * NBZ;
    const size_t lds = 4 * buf + biases;
    void (*kern)(EncodeParams, AttendParams, int, int, int) = gelu ? encode_mlp_step_qtilde_kernel<E, KX, NBZ, true> : encode_mlp_step_qtilde_kernel<E, KX, NBZ, false>;
    static AttrFlag attr[2] = {false, false};
    if (lds > 64 * 1024 && !attr[gelu]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (err != hipSuccess) return err;
        attr[gelu] = true;
    }
    const int enc_x = (n_tok + 31) / 32;
    dim3 grid(enc_x + qx * qy * qz, 2);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p, q, enc_x, qx, qy);
    return hipGetLastError();
}

// Whether a shape's few-token form applies (its four weight slices and biases fit the LDS).
template <int KX, int NBZ>
constexpr bool em_small_fits() { return 4 * (size_t)(16 * KX * kW1Stride + 32 * (64 * NBZ + 32)) + 4 * 1024 + 4 * 32 * NBZ <= 160 * 1024; }

template <typename E>
hipError_t em_step_qtilde(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, hipStream_t stream) {
    const EncodeSide& s = p.s[0];
    const bool gelu = s.act == KVCAR_ACT_GELU;
    const int kx = s.in_width / 16, nbz = s.r / 32;
    if (kx == 4 && nbz == 1) return em_step_qtilde_shape<E, 4, 1>(p, q, qx, qy, qz, gelu, stream);
    if (kx == 8 && nbz == 2) return em_step_qtilde_shape<E, 8, 2>(p, q, qx, qy, qz, gelu, stream);
    if (kx == 12 && nbz == 3) return em_step_qtilde_shape<E, 12, 3>(p, q, qx, qy, qz, gelu, stream);
    if (kx == 16 && nbz == 4) return em_step_qtilde_shape<E, 16, 4>(p, q, qx, qy, qz, gelu, stream);
    if (kx == 16 && nbz == 2) return em_step_qtilde_shape<E, 16, 2>(p, q, qx, qy, qz, gelu, stream);
    if (kx == 8 && nbz == 1) return em_step_qtilde_shape<E, 8, 1>(p, q, qx, qy, qz, gelu, stream);
    return hipErrorInvalidValue;
}

bool em_small_shape_fits(int kx, int nbz) {
    if (kx == 4 && nbz == 1) return em_small_fits<4, 1>();
    if (kx == 8 && nbz == 2) return em_small_fits<8, 2>();
    if (kx == 12 && nbz == 3) return em_small_fits<12, 3>();
    if (kx == 16 && nbz == 4) return em_small_fits<16, 4>();
    if (kx == 16 && nbz == 2) return em_small_fits<16, 2>();
    if (kx == 8 && nbz == 1) return em_small_fits<8, 1>();
    return false;
}

}  // namespace

// The few-token form for both tensors at once (same shape and activation, at most 128 tokens) can share its launch with the
// absorbed-query projection.
bool encode_mlp_step_qtilde_supported(const EncodeParams& p, int dtype) {
    if (!encode_mlp_mfma_supported(p, dtype)) return false;
    const EncodeSide &k = p.s[0], &v = p.s[1];
    if (!(k.r && v.r && k.in_width == v.in_width && k.r == v.r && (k.act == KVCAR_ACT_GELU) == (v.act == KVCAR_ACT_GELU))) return false;
    return p.batch * p.t_new <= kEmTokens && em_small_shape_fits(k.in_width / 16, k.r / 32);
}

hipError_t launch_encode_mlp_step_qtilde(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, int dtype, hipStream_t stream) {
    static_assert(sizeof(EncodeParams) + sizeof(AttendParams) + 16 <= 4096, "both argument blocks must fit the kernel-argument segment");
    return dtype == KVCAR_BF16 ? em_step_qtilde<BF16>(p, q, qx, qy, qz, stream) : em_step_qtilde<F16>(p, q, qx, qy, qz, stream);
}

// 16-bit dtype, every stored tensor two-layer with one of the compiled (input width, latent) shapes,
// 16-column chunks inside one head, hidden width a multiple of 32 up to 1024.
bool encode_mlp_mfma_supported(const EncodeParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.d_head % 16) return false;      // a 16-column k-step stays inside one head
    bool any = false;
    for (int i = 0; i < 2; ++i) {
        const EncodeSide& s = p.s[i];
        if (s.r == 0) continue;
        if (!em_side_ok(s)) return false;
        any = true;
    }
    return any;
}

// One launch covers both tensors when they share shape and activation; otherwise one launch per tensor.
hipError_t launch_encode_mlp_mfma(const EncodeParams& p, int dtype, hipStream_t stream) {
    const EncodeSide &k = p.s[0], &v = p.s[1];
    auto go = [&](int side0, int n) { return dtype == KVCAR_BF16 ? em_launch<BF16>(p, side0, n, stream) : em_launch<F16>(p, side0, n, stream); };
    if (k.r && v.r && k.in_width == v.in_width && k.r == v.r && (k.act == KVCAR_ACT_GELU) == (v.act == KVCAR_ACT_GELU)) return go(0, 2);
    hipError_t err = hipSuccess;
    if (k.r) err = go(0, 1);
    if (err == hipSuccess && v.r) err = go(1, 1);
    return err;
}

}  // namespace kvcar
