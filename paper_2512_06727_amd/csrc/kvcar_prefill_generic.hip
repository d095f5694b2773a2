// Prefill attention over the latent cache, plain-ALU kernels for any dtype, width and autoencoder (gfx950).
//
// A prompt chunk attends causally over the cached rows of its sequence (Introduction: prefill produces
// the keys and values of all prompt tokens, which go to the cache - as latent rows here - and come back
// through the decoder, "Network Architecture", 2nd paragraph; attention is Eq. 1 per token).  Two steps:
//   recon    K^[b, g, t, :] / V^[b, g, t, :] = decoder(latent row t of the layer that supplies head g),
//            the columns of head g, for t < n_rows; written once, rounded to fp16 for 16-bit models (fp32 for
//            fp32 models; see RowsOf).  The keys are multiplied by scale * log2(e) before that one rounding, so
//            scores come out in log2 units and the scale costs neither an operation per score nor a second rounding
//   attend   out[b, i, j, :] = sum_{t <= pos0 + i} softmax_t(scale q[b,i,j,:] . K^_g[t]) V^_g[t]
// These kernels serve fp32 models and shapes the matrix-core kernels do not cover.
#include "kvcar_device.hpp"

namespace kvcar {

constexpr int kReconTile = 16;     // tokens per workgroup of the plain-ALU decoder

// One workgroup: one entry (source layer and side), one sequence, 16 tokens: latent rows (dequantised when
// they are int8 codes) -> hidden rows (two-layer decoder) -> the d_head columns of every head of the entry.
template <typename E>
__global__ __launch_bounds__(256) void recon_generic_kernel(ReconParams p) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    const ReconEntry& e = p.e[blockIdx.z];
    const SideDesc& sd = e.d;
    const int b = blockIdx.y, t0 = blockIdx.x * kReconTile, tid = threadIdx.x;
    const int nt = min(kReconTile, p.n_rows - t0);
    float* zrow = lds_f;                          // [16][r]
    float* hid = lds_f + kReconTile * sd.r;       // [16][c] (two-layer decoder only)

    for (int i = tid; i < kReconTile * sd.r; i += 256) {
        const int t = i / sd.r, c = i % sd.r;
        zrow[i] = t < nt ? latent_at<E>(sd, (size_t)b * p.max_seq + t0 + t, c) : 0.f;
    }
    __syncthreads();
    const float* rows = zrow;
    if (sd.w1 != nullptr) {
        for (int i = tid; i < kReconTile * sd.c; i += 256) {
            const int t = i / sd.c, c = i % sd.c;
            float a = sd.b1 ? Elem<E>::load(sd.b1, c) : 0.f;
            for (int k = 0; k < sd.r; ++k) a = fmaf(zrow[t * sd.r + k], Elem<E>::load(sd.w1, (size_t)k * sd.c + c), a);
            hid[i] = apply_act(a, sd.act, sd.slope);
        }
        __syncthreads();
        rows = hid;
    }
    void* dst = e.which == KVCAR_K ? p.khat : p.vhat;
    const float out_scale = e.which == KVCAR_K ? p.k_scale : 1.f;     // keys carry the softmax scale (log2 units)
    const int dh = p.d_head;
    for (int hi = 0; hi < e.n_heads; ++hi) {
        const int g = e.head[hi], col = e.col[hi];
        for (int i = tid; i < kReconTile * dh; i += 256) {
            const int t = i / dh, k = i % dh;
            if (t >= nt) continue;
            float a = sd.bl ? Elem<E>::load(sd.bl, col + k) : 0.f;
            for (int c = 0; c < sd.c; ++c) a = fmaf(rows[t * sd.c + c], Elem<E>::load(sd.wl, (size_t)c * sd.in_width + col + k), a);
            Elem<typename RowsOf<E>::type>::store(dst, (((size_t)b * p.n_kv_heads + g) * p.n_rows + t0 + t) * dh + k, sat_rows<E>(a * out_scale));
        }
    }
}

hipError_t launch_recon_generic(const ReconParams& p, int dtype, hipStream_t stream) {
    size_t lds = 0;
    for (int i = 0; i < p.n_entries; ++i) {
        const SideDesc& sd = p.e[i].d;
        lds = max(lds, (size_t)kReconTile * (sd.r + (sd.w1 ? sd.c : 0)) * sizeof(float));
    }
    dim3 grid((p.n_rows + kReconTile - 1) / kReconTile, p.batch, p.n_entries);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(recon_generic_kernel<F32>, grid, dim3(256), lds, stream, p);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(recon_generic_kernel<F16>, grid, dim3(256), lds, stream, p);
    else hipLaunchKernelGGL(recon_generic_kernel<BF16>, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

// One wave: one query token of one head.  Tokens in tiles of 64: lane t computes the score of one row,
// the tile's probabilities meet in LDS, then lane d accumulates output components d, d + 64, ...
// (online softmax in base 2; the running maximum is finite after the first tile, which always holds row 0).
constexpr int kPrefillGenericDims = 4;     // d_head <= 256

template <typename E>
__global__ __launch_bounds__(64) void prefill_generic_kernel(PrefillParams p) {
    __shared__ float qs[64 * kPrefillGenericDims];
    __shared__ float ps[64];
    const int lane = threadIdx.x;
    const int i = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const int dh = p.d_head, g = j / (p.n_q_heads / p.n_kv_heads);
    const size_t qoff = (((size_t)b * p.t_new + i) * p.n_q_heads + j) * dh;
    for (int k = lane; k < dh; k += 64) qs[k] = Elem<E>::load(p.q, qoff + k);
    __syncthreads();
    const size_t row0 = ((size_t)b * p.n_kv_heads + g) * p.n_rows;
    const int n = p.pos0 + i + 1;             // rows this token sees

    float acc[kPrefillGenericDims];
#pragma unroll
    for (int u = 0; u < kPrefillGenericDims; ++u) acc[u] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    for (int t0 = 0; t0 < n; t0 += 64) {
        const int t = t0 + lane;
        float s = -INFINITY;
        if (t < n) {
            s = 0.f;
            for (int k = 0; k < dh; ++k) s = fmaf(qs[k], Elem<typename RowsOf<E>::type>::load(p.khat, (row0 + t) * dh + k), s);
        }
        float mx = s;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f(m_run - m_new);
        const float pr = t < n ? exp2f(s - m_new) : 0.f;
        float sum = pr;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        l_run = l_run * alpha + sum;
        m_run = m_new;
        __syncthreads();
        ps[lane] = pr;
        __syncthreads();
        const int nt = min(64, n - t0);
#pragma unroll
        for (int u = 0; u < kPrefillGenericDims; ++u) {
            const int d = lane + 64 * u;
            if (d < dh) {
                float a = acc[u] * alpha;
                for (int tt = 0; tt < nt; ++tt) a = fmaf(ps[tt], Elem<typename RowsOf<E>::type>::load(p.vhat, (row0 + t0 + tt) * dh + d), a);
                acc[u] = a;
            }
        }
    }
    const float inv = 1.f / l_run;
#pragma unroll
    for (int u = 0; u < kPrefillGenericDims; ++u) {
        const int d = lane + 64 * u;
        if (d < dh) Elem<E>::store(p.out, qoff + d, acc[u] * inv);
    }
}

hipError_t launch_prefill_generic(const PrefillParams& p, int dtype, hipStream_t stream) {
    if (p.d_head > 64 * kPrefillGenericDims) return hipErrorInvalidValue;
    dim3 grid(p.t_new, p.n_q_heads, p.batch);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(prefill_generic_kernel<F32>, grid, dim3(64), 0, stream, p);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(prefill_generic_kernel<F16>, grid, dim3(64), 0, stream, p);
    else hipLaunchKernelGGL(prefill_generic_kernel<BF16>, grid, dim3(64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace kvcar
