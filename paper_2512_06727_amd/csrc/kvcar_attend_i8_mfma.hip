// MFMA attention over int8 latent rows ("Quantization", Eq. "quant"; gfx950, 16-bit model dtypes, linear
// decoders, latent width 32 / 64 / 96 / 128 equal for K and V).  Same loop as the 16-bit kernel
// (kvcar_attend_mfma_body.hpp): the code bytes become fp16 operands on their way into LDS and the
// per-row scale and zero point are applied to the scores and folded into the probabilities.
#include "kvcar_attend_mfma_body.hpp"

namespace kvcar {

constexpr size_t kI8WaveLds = Geo<128>::kWaveLds + 512;      // + 1/scale, off/scale, 256/scale of the tile's rows

template <typename E>
__global__ __launch_bounds__(256, 2) void attend_i8_mfma_r128_kernel(AttendParams p_by_value) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    (void)p_by_value;
    KArgs p = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const WgCoords wc = wg_coords(p);
    KGroup g = &p->g[wc.z];
    const int key = g->k.r * 4 + (g->slots_pad >> 4);
    if (p->fused == 4) {                      // several splits in one launch: the last workgroup to arrive merges and decodes
        switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, true, kWaves, true, true>(p, g, wc, lds_raw, kI8WaveLds); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: return;
        }
    }
    if (p->fused == 3) {                      // several splits, absorbed queries computed here
        switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, true, kWaves, true>(p, g, wc, lds_raw, kI8WaveLds); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: return;
        }
    }
    if (p->fused) {
        switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, true, true>(p, g, wc, lds_raw, kI8WaveLds); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: return;
        }
    }
    switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, true>(p, g, wc, lds_raw, kI8WaveLds); return;
        KVCAR_EXACT_SHAPES(X)
#undef X
        default: return;
    }
}

// Eight waves per workgroup (the one-launch forms): for launches with no more workgroups than compute units.
template <typename E>
__global__ __launch_bounds__(512, 1) void attend_i8_mfma_r128_w8_kernel(AttendParams p_by_value) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    (void)p_by_value;
    KArgs p = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const WgCoords wc = wg_coords(p);
    KGroup g = &p->g[wc.z];
    if (p->fused == 5) {                      // several splits in one launch (the last workgroup merges), eight waves
        switch (g->k.r * 4 + (g->slots_pad >> 4)) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, true, 8, true, true>(p, g, wc, lds_raw, kI8WaveLds); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: return;
        }
    }
    switch (g->k.r * 4 + (g->slots_pad >> 4)) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, true, true, 8>(p, g, wc, lds_raw, kI8WaveLds); return;
        KVCAR_EXACT_SHAPES(X)
#undef X
        default: return;
    }
}

// Every group: int8 rows with metadata, linear decoders, K and V latent widths equal and one of 32 / 64 / 96 / 128,
// at most 32 query heads.
bool attend_i8_mfma_supported(const AttendParams& p, int dtype) {
    if (dtype == KVCAR_F32) return false;
    for (int i = 0; i < p.n_groups; ++i) {
        const GroupDesc& g = p.g[i];
        if (!g.k.meta || !g.v.meta || g.k.w1 || g.v.w1) return false;
        if (g.k.r != g.v.r || !exact_shape(g.k.r, g.slots_pad / 16)) return false;      // every form of this kernel is compiled for the exact shapes only
    }
    return true;
}

hipError_t launch_attend_i8_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    static AttrFlag attr[2] = {false, false}, attr8[2] = {false, false};
    if (!attend_i8_mfma_supported(p, dtype)) return hipErrorNotSupported;
    if (p.fused == 2 || p.fused == 5) {
        const size_t epi8 = 2048 + 32 * 132 * 4 + 128 * (2 * (size_t)p.d_head + 32);
        size_t lds8 = 8 * kI8WaveLds + 2 * 4 * 64 * 16;              // + swapped query operands (the new token's codes of append-and-attend sit in the waves' spare bytes)
        lds8 = lds8 > epi8 ? lds8 : epi8;
        const int e8 = dtype == KVCAR_BF16 ? 0 : 1;
        auto kern8 = e8 == 0 ? attend_i8_mfma_r128_w8_kernel<BF16> : attend_i8_mfma_r128_w8_kernel<F16>;
        if (!attr8[e8]) {
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern8), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (err != hipSuccess) return err;
            attr8[e8] = true;
        }
        hipLaunchKernelGGL(kern8, dim3(p.n_splits, p.batch, p.n_groups), dim3(512), lds8, stream, p);
        return hipGetLastError();
    }
    const size_t epi = 1024 + 32 * 132 * 4 + 128 * (2 * (size_t)p.d_head + 32);
    const size_t merge = mfma_lds_bytes(128, 2);
    size_t lds = kWaves * kI8WaveLds + (p.fused ? 2 * 4 * 64 * 16 : 0);       // two workgroups of 81920 bytes fill a compute unit's LDS exactly
    lds = lds > merge ? lds : merge;
    lds = lds > epi ? lds : epi;
    const int e = dtype == KVCAR_BF16 ? 0 : 1;
    auto kern = e == 0 ? attend_i8_mfma_r128_kernel<BF16> : attend_i8_mfma_r128_kernel<F16>;
    if (!attr[e]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (err != hipSuccess) return err;
        attr[e] = true;
    }
    dim3 grid(p.n_splits, p.batch, p.n_groups);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

}  // namespace kvcar
