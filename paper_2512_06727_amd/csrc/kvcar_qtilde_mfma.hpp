// The absorbed-query projection on the matrix cores as a per-workgroup function (gfx950, 16-bit dtypes), shared by its own
// kernel and by the decode-step encoder kernel that runs it in the same launch (two small independent pieces of a layer's
// step: the new token's latent rows and the absorbed queries).
#pragma once
#include "kvcar_device.hpp"

namespace kvcar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

template <typename E> struct PMma;
template <> struct PMma<BF16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint16_t to16(float v) { return f32_to_bf16_bits(v); }
    static __device__ __forceinline__ float from16(uint16_t b) { return bf16_bits_to_f32(b); }
};
template <> struct PMma<F16> {
    static __device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint16_t to16(float v) { _Float16 h = (_Float16)v; return __builtin_bit_cast(uint16_t, h); }
    static __device__ __forceinline__ float from16(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
};

// Slots of a group that share a KV head are consecutive and share a column offset.  Finds the
// `which`-th such run of `col`; returns false if there are fewer runs.  The host's table of runs answers
// directly when the group has at most kMaxSeg of them; otherwise the column table is walked.
__device__ __forceinline__ bool find_segment(const short* col, int n_slots, int n_seg, const short* seg_lo, const short* seg_hi, int which, int& s0,
                                             int& len) {
    if (n_seg > 0) {
        if (which >= n_seg) return false;
        s0 = seg_lo[which];
        len = seg_hi[which] - s0;
        return true;
    }
    int seg = -1, start = 0;
    for (int s = 0; s <= n_slots; ++s) {
        if (s == n_slots || (s > 0 && col[s] != col[s - 1])) {
            if (s > 0) {
                ++seg;
                if (seg == which) { s0 = start; len = s - start; return true; }
            }
            start = s;
        }
    }
    return false;
}

// ---------------------------------------------------------------------------------------------
// absorbed queries.  grid = (16-row blocks, segment, group); rows are (sequence, head) pairs.
// Both MFMA operands come straight from global memory: a lane needs 8 consecutive k of one query
// row (A) and 8 consecutive k of one decoder-matrix row (B), both contiguous.
// Segment index == number of segments is the zero-fill of the group's padding slots.
// ---------------------------------------------------------------------------------------------
// One workgroup's share, as a function: block (bx, by, bz) of a grid whose x extent is grid_x.  P is a pointer to the launch's
// AttendParams (in kernel arguments: generic or constant address space).
template <typename E, typename P>
__device__ __forceinline__ void qtilde_mfma_block(P pp, int bx, int by, int bz, int grid_x) {
    const auto& p = *pp;
    const auto& g = p.g[bz];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    const int rk = g.k.c;            // contraction width of the score product: latent (linear decoder) or hidden width
    int s0 = 0, len = 0;
    if (!find_segment(g.k_col, g.n_slots, g.n_kseg, g.kseg_lo, g.kseg_hi, by, s0, len)) {
        int dummy0, dummy1;
        const bool is_pad_pass = (by == 0) ? false : find_segment(g.k_col, g.n_slots, g.n_kseg, g.kseg_lo, g.kseg_hi, by - 1, dummy0, dummy1);
        if (!is_pad_pass || g.slots_pad == g.n_slots) return;
        // zero the padding slots of every sequence (rows of qt the attention kernel loads but ignores)
        const int pad = g.slots_pad - g.n_slots;
        const int chunks = pad * rk / 8;                          // 16-byte chunks per sequence
        const int total = p.batch * chunks;
        for (int i = bx * 256 + threadIdx.x; i < total; i += grid_x * 256) {
            const int b = i / chunks, c = i - b * chunks;
            char* dst = static_cast<char*>(p.qt) + ((size_t)b * p.qt_stride + g.qt_off + (size_t)g.n_slots * rk) * 2 + (size_t)c * 16;
            *reinterpret_cast<u32x4_t*>(dst) = u32x4_t{0u, 0u, 0u, 0u};
        }
        return;
    }
    const int rows = p.batch * len;
    const int row0 = bx * 16;                 // the four waves share the rows and deal out the column blocks
    if (row0 >= rows) return;
    const int col = g.k_col[s0];
    const int dh = p.d_head;

    // A operand: query rows (d_head <= 128: at most four k-steps, loaded once)
    const int arow = row0 + l16;
    const int ab = arow / len, ai = arow - ab * len;
    const bool a_ok = arow < rows;
    const char* qrow = static_cast<const char*>(p.q) + ((size_t)(a_ok ? ab : 0) * p.n_q_heads + g.q_head[s0 + (a_ok ? ai : 0)]) * dh * 2;
    u32x4_t a[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        a[ks] = u32x4_t{0u, 0u, 0u, 0u};
        if (a_ok && ks * 32 < dh) a[ks] = *reinterpret_cast<const u32x4_t*>(qrow + (ks * 32 + 8 * lg) * 2);
    }
    // result rows of this lane
    size_t orow[4];
    bool ook[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int r = row0 + 4 * lg + v;
        ook[v] = r < rows;
        const int b = r / len, i = r - b * len;
        orow[v] = (size_t)b * p.qt_stride + g.qt_off + (size_t)(s0 + i) * rk;
    }
    uint16_t* qt = static_cast<uint16_t*>(p.qt);
    const char* wl = static_cast<const char*>(g.k.wl);
    for (int nb = wave; nb < (rk >> 4); nb += 4) {
        const char* wrow = wl + ((size_t)(nb * 16 + l16) * g.k.in_width + col) * 2;
        u32x4_t bw[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            if (ks * 32 < dh) bw[ks] = *reinterpret_cast<const u32x4_t*>(wrow + (ks * 32 + 8 * lg) * 2);
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            if (ks * 32 < dh) acc = PMma<E>::mfma(a[ks], bw[ks], acc);
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (ook[v]) qt[orow[v] + nb * 16 + l16] = PMma<E>::to16(acc[v] * p.scale_log2e);
    }
}

}  // namespace kvcar
