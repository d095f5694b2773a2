// Reuse-map selection statistic (Algorithm 2, steps 1-2; Methodology, the paragraph on key and value
// reuse): the L1 distance between the same head of adjacent layers, averaged over the tokens of a
// calibration batch.  Which heads are then reused is the caller's threshold decision.
//
//   dist[g] = mean over tokens t and components k < d_head of | cur[t, g, k] - prev[t, g, k] |
//
// An HBM-bound reduction: both tensors are read once with 16-byte loads.  A lane keeps one 16-byte
// column chunk (so one head) for all its rows; a workgroup reduces its lanes per head in a fixed
// order and writes one partial per head; a second, tiny kernel adds the partials in a fixed order in
// double precision: the result does not depend on scheduling.
#include "kvcar_device.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(4))) unsigned sel_u32x4_t;

template <typename E> struct SelChunk;      // sum of |a - b| over one 16-byte chunk
template <> struct SelChunk<F32> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ float absdiff(sel_u32x4_t a, sel_u32x4_t b) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) s += fabsf(__uint_as_float(a[i]) - __uint_as_float(b[i]));
        return s;
    }
};
template <> struct SelChunk<BF16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ float absdiff(sel_u32x4_t a, sel_u32x4_t b) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s += fabsf(__uint_as_float(a[i] << 16) - __uint_as_float(b[i] << 16));
            s += fabsf(__uint_as_float(a[i] & 0xffff0000u) - __uint_as_float(b[i] & 0xffff0000u));
        }
        return s;
    }
};
template <> struct SelChunk<F16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ float half_at(unsigned w, int hi) {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(hi ? w >> 16 : w & 0xffffu));
    }
    static __device__ __forceinline__ float absdiff(sel_u32x4_t a, sel_u32x4_t b) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s += fabsf(pinned(half_at(a[i], 0) - half_at(b[i], 0)));
            s += fabsf(pinned(half_at(a[i], 1) - half_at(b[i], 1)));
        }
        return s;
    }
};

constexpr int kSelThreads = 256;
constexpr int kSelUnroll = 8;

// grid.x workgroups share the tokens; partial[wg][head] = sum over the workgroup's tokens.
template <typename E>
__global__ __launch_bounds__(kSelThreads) void head_l1_partial_kernel(const char* __restrict__ prev, const char* __restrict__ cur, size_t n_tokens,
                                                                      int n_kv_heads, int d_head, float* __restrict__ partial) {
    __shared__ float lane_sum[kSelThreads];
    __shared__ int lane_head[kSelThreads];
    constexpr int EL = SelChunk<E>::kElems;
    const int cpr = n_kv_heads * d_head / EL;                 // 16-byte chunks per token row
    const size_t row_bytes = (size_t)cpr * 16;
    const int tid = threadIdx.x;
    float* out = partial + (size_t)blockIdx.x * n_kv_heads;
    for (int h = tid; h < n_kv_heads; h += kSelThreads) out[h] = 0.f;

    // column blocks of up to 256 chunks; inside a block a lane owns chunk c0 + tid % w of rows tid / w, + rows_per_pass, ...
    for (int c0 = 0; c0 < cpr; c0 += kSelThreads) {
        const int w = min(kSelThreads, cpr - c0);
        const int rows_per_pass = kSelThreads / w;
        const int r_in = tid / w, ch = c0 + tid - r_in * w;
        const bool active = r_in < rows_per_pass;
        float acc = 0.f;
        if (active) {
            // kSelUnroll independent row pairs in flight per lane
            const size_t off = (size_t)ch * 16;
            // a contiguous token range per workgroup
            const size_t per_wg = (n_tokens + gridDim.x - 1) / gridDim.x;
            const size_t step = rows_per_pass;
            size_t t = (size_t)blockIdx.x * per_wg + r_in;
            const size_t n_end = (size_t)(blockIdx.x + 1) * per_wg < n_tokens ? (size_t)(blockIdx.x + 1) * per_wg : n_tokens;
            for (; t + (kSelUnroll - 1) * step < n_end; t += kSelUnroll * step) {
                sel_u32x4_t a[kSelUnroll], b[kSelUnroll];
#pragma unroll
                for (int u = 0; u < kSelUnroll; ++u) {
                    const size_t o = (t + u * step) * row_bytes + off;
                    a[u] = __builtin_nontemporal_load(reinterpret_cast<const sel_u32x4_t*>(prev + o));
                    b[u] = __builtin_nontemporal_load(reinterpret_cast<const sel_u32x4_t*>(cur + o));
                }
#pragma unroll
                for (int u = 0; u < kSelUnroll; ++u) acc += SelChunk<E>::absdiff(a[u], b[u]);
            }
            for (; t < n_end; t += step) {
                const size_t o = t * row_bytes + off;
                acc += SelChunk<E>::absdiff(__builtin_nontemporal_load(reinterpret_cast<const sel_u32x4_t*>(prev + o)),
                                            __builtin_nontemporal_load(reinterpret_cast<const sel_u32x4_t*>(cur + o)));
            }
        }
        __syncthreads();                         // the previous column block's reduction is done
        lane_sum[tid] = acc;
        lane_head[tid] = active ? ch * EL / d_head : -1;
        __syncthreads();
        // one thread per head adds that head's lanes in lane order
        for (int h = tid; h < n_kv_heads; h += kSelThreads) {
            float s = 0.f;
            for (int l = 0; l < kSelThreads; ++l)
                if (lane_head[l] == h) s += lane_sum[l];
            out[h] += s;
        }
    }
}

// dist[h] (+)= sum over workgroups of partial[wg][h] / (n_tokens * d_head)
__global__ void head_l1_final_kernel(const float* __restrict__ partial, int n_wg, int n_kv_heads, double inv_count, int accumulate,
                                     float* __restrict__ dist) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= n_kv_heads) return;
    double s = 0.0;
    for (int i = 0; i < n_wg; ++i) s += (double)partial[(size_t)i * n_kv_heads + h];
    const float v = (float)(s * inv_count);
    dist[h] = accumulate ? dist[h] + v : v;
}

int head_l1_workgroups(size_t n_tokens, int n_cu) {
    // one long-lived workgroup per compute unit measured best (the per-workgroup reduction at the end is serial)
    const size_t want = (size_t)(n_cu > 0 ? n_cu : 256);
    const size_t by_tokens = (n_tokens + 15) / 16;           // at least 16 token rows per workgroup
    const size_t n = want < by_tokens ? want : by_tokens;
    return (int)(n < 1 ? 1 : n);
}

hipError_t launch_head_l1(const void* prev, const void* cur, int dtype, size_t n_tokens, int n_kv_heads, int d_head, int accumulate, float* dist,
                          float* partial, int n_wg, hipStream_t stream) {
    const char* a = static_cast<const char*>(prev);
    const char* b = static_cast<const char*>(cur);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(head_l1_partial_kernel<F32>, dim3(n_wg), dim3(kSelThreads), 0, stream, a, b, n_tokens, n_kv_heads, d_head, partial);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(head_l1_partial_kernel<F16>, dim3(n_wg), dim3(kSelThreads), 0, stream, a, b, n_tokens, n_kv_heads, d_head, partial);
    else hipLaunchKernelGGL(head_l1_partial_kernel<BF16>, dim3(n_wg), dim3(kSelThreads), 0, stream, a, b, n_tokens, n_kv_heads, d_head, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const double inv = 1.0 / ((double)n_tokens * d_head);
    hipLaunchKernelGGL(head_l1_final_kernel, dim3((n_kv_heads + 63) / 64), dim3(64), 0, stream, partial, n_wg, n_kv_heads, inv, accumulate, dist);
    return hipGetLastError();
}

}  // namespace kvcar
