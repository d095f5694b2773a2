// Kernels and launchers of the MFMA attention over latent rows held in the model dtype (gfx950).
// The loop itself lives in kvcar_attend_mfma_body.hpp.
#include "kvcar_attend_mfma_body.hpp"

namespace kvcar {

// Latent widths up to 128 (TinyLlama-class KV widths): up to two 16-head blocks per group.
template <typename E>
__global__ __launch_bounds__(256, 2) void attend_mfma_r128_kernel(AttendParams p_by_value) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    (void)p_by_value;
    KArgs p = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const WgCoords wc = wg_coords(p);
    KGroup g = &p->g[wc.z];
    constexpr size_t wl = Geo<128>::kWaveLds;
    const int nhb = g->slots_pad >> 4;
    if (g->k.r == g->v.r) {
        const int key = g->k.r * 4 + nhb;
        if (p->fused == 1) {                  // the host only asks for this with exact shapes in every group
            switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, true>(p, g, wc, lds_raw, wl); return;
                KVCAR_EXACT_SHAPES(X)
#undef X
                default: return;
            }
        }
        if (p->fused == 4) {                  // several splits in one launch: the last workgroup to arrive merges and decodes
            switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, false, kWaves, true, true>(p, g, wc, lds_raw, wl); return;
                KVCAR_EXACT_SHAPES(X)
#undef X
                default: return;
            }
        }
        if (p->fused == 3) {                  // several splits, absorbed queries computed here
            switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, false, kWaves, true>(p, g, wc, lds_raw, wl); return;
                KVCAR_EXACT_SHAPES(X)
#undef X
                default: return;
            }
        }
        switch (key) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false>(p, g, wc, lds_raw, wl); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: break;
        }
    }
    attend_body<E, DimsAny<128, 2>, false>(p, g, wc, lds_raw, wl);
}

// Fused single-split variant with eight waves per workgroup, for launches with no more workgroups
// than compute units: a four-wave workgroup alone on a compute unit leaves one wave per SIMD, which
// cannot overlap its loads, MFMA and vector work with anything.
template <typename E>
__global__ __launch_bounds__(512, 1) void attend_mfma_r128_w8_kernel(AttendParams p_by_value) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    (void)p_by_value;
    KArgs p = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const WgCoords wc = wg_coords(p);
    KGroup g = &p->g[wc.z];
    constexpr size_t wl = Geo<128>::kWaveLds;
    if (p->fused == 5) {                      // several splits in one launch (the last workgroup merges), eight waves
        switch (g->k.r * 4 + (g->slots_pad >> 4)) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, false, false, 8, true, true>(p, g, wc, lds_raw, wl); return;
            KVCAR_EXACT_SHAPES(X)
#undef X
            default: return;
        }
    }
    switch (g->k.r * 4 + (g->slots_pad >> 4)) {
#define X(R, N) case R * 4 + N: attend_body<E, DimsExact<R, N>, true, false, 8>(p, g, wc, lds_raw, wl); return;
        KVCAR_EXACT_SHAPES(X)
#undef X
        default: return;
    }
}

// Latent widths up to 384 (GPT-2-class KV widths): one 16-head block per group.
template <typename E>
__global__ __launch_bounds__(256, 1) void attend_mfma_r384_kernel(AttendParams p_by_value) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    (void)p_by_value;
    KArgs p = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const WgCoords wc = wg_coords(p);
    KGroup g = &p->g[wc.z];
    constexpr size_t wl = Geo<384>::kWaveLds;
    if (g->k.r == g->v.r && g->k.r == 384) { attend_body<E, DimsExact<384, 1>, false>(p, g, wc, lds_raw, wl); return; }
    if (g->k.r == g->v.r && g->k.r == 288) { attend_body<E, DimsExact<288, 1>, false>(p, g, wc, lds_raw, wl); return; }
    attend_body<E, DimsAny<384, 1>, false>(p, g, wc, lds_raw, wl);
}

template <typename K>
static hipError_t launch_one(K kern, size_t lds, const AttendParams& p, hipStream_t stream, AttrFlag& attr_set, int threads = 256) {
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(p.n_splits, p.batch, p.n_groups);
    hipLaunchKernelGGL(kern, grid, dim3(threads), lds, stream, p);
    return hipGetLastError();
}

bool attend_mfma_available() { return true; }

hipError_t launch_attend_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    static AttrFlag set128[2] = {false, false}, set384[2] = {false, false}, set128w8[2] = {false, false};
    int rmax = 0, nhb = 1;
    for (int i = 0; i < p.n_groups; ++i) {
        rmax = p.g[i].k.r > rmax ? p.g[i].k.r : rmax;
        rmax = p.g[i].v.r > rmax ? p.g[i].v.r : rmax;
        nhb = p.g[i].slots_pad / 16 > nhb ? p.g[i].slots_pad / 16 : nhb;
    }
    const int e = dtype == KVCAR_BF16 ? 0 : 1;
    // the fused and prologue forms exist for the exact shapes only: a group outside them would find no instance
    if (p.fused != 0)
        for (int i = 0; i < p.n_groups; ++i)
            if (p.g[i].k.r != p.g[i].v.r || !exact_shape(p.g[i].k.r, p.g[i].slots_pad / 16)) return hipErrorNotSupported;
    if (rmax <= 128 && nhb <= 2 && (p.fused == 2 || p.fused == 5)) {
        // eight waves: staging regions + swapped query operands, or the epilogue's exchange area (m, l of
        // eight waves) + latent sums + one decoder slice
        const size_t epi = 2048 + 32 * 132 * 4 + 128 * (2 * (size_t)p.d_head + 32);
        const size_t stage = 8 * Geo<128>::kWaveLds + 2 * 4 * 64 * 16 + 512;      // + the new token's rows (append-and-attend)
        const size_t lds = epi > stage ? epi : stage;
        return e == 0 ? launch_one(attend_mfma_r128_w8_kernel<BF16>, lds, p, stream, set128w8[0], 512)
                      : launch_one(attend_mfma_r128_w8_kernel<F16>, lds, p, stream, set128w8[1], 512);
    }
    if (rmax <= 128 && nhb <= 2) {
        // fused: + normalised latent sums [32][132] fp32 + one decoder-matrix slice [128][2*d_head+32]
        // fused epilogue: exchange area + latent sums [32][132] fp32 + one decoder slice [128][2*d_head+32]
        const size_t epi = 1024 + 32 * 132 * 4 + 128 * (2 * (size_t)p.d_head + 32);
        const size_t stage = mfma_lds_bytes(128, 2) + (p.fused ? 2 * 4 * 64 * 16 + 512 : 0);   // + swapped query operands + the new token's rows (append-and-attend)
        const size_t lds = epi > stage ? epi : stage;
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
