// Device-side helpers: element types, conversions, activations (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvcar_internal.hpp"

namespace kvcar {

struct F32 { using type = float; };
struct F16 { using type = _Float16; };
struct BF16 { using type = uint16_t; };   // raw bf16 bits

template <typename E> struct Elem;

template <> struct Elem<F32> {
    using T = float;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return static_cast<const float*>(p)[i]; }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { static_cast<float*>(p)[i] = v; }
};

template <> struct Elem<F16> {
    using T = _Float16;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return (float)static_cast<const _Float16*>(p)[i]; }
    // fp32 -> fp16 conversion rounds to nearest even
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { static_cast<_Float16*>(p)[i] = (_Float16)v; }
};

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <> struct Elem<BF16> {
    using T = uint16_t;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[i]); }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { static_cast<uint16_t*>(p)[i] = f32_to_bf16_bits(v); }
};

// The dtype in which prefill attention holds the decoded rows K^ / V^ between its two kernels: fp32 for fp32 models,
// fp16 for both 16-bit dtypes.  A bf16 model's decoded rows would otherwise carry bf16's 8-bit rounding into every
// prompt score (q . dK^ grows with the query's size and the row width); fp16 keeps 11 bits at the same cost.  Its
// range ends at 65504: decoded values (the keys after the softmax scale) and queries beyond that saturate.
template <typename E> struct RowsOf { using type = F16; };
template <> struct RowsOf<F32> { using type = F32; };
constexpr float kHalfMax = 65504.f;
__device__ __forceinline__ float sat_half(float x) { return __builtin_amdgcn_fmed3f(x, -kHalfMax, kHalfMax); }
template <typename E> __device__ __forceinline__ float sat_rows(float x) { return sat_half(x); }
template <> __device__ __forceinline__ float sat_rows<F32>(float x) { return x; }

// Element c of latent row `row` of a cache side: as stored, or dequantised from its int8 code
// (x^ = (code - zeropoint) / scale, Eq. "quant").
template <typename E>
__device__ __forceinline__ float latent_at(const SideDesc& sd, size_t row, int c) {
    if (sd.meta == nullptr) return Elem<E>::load(sd.z, row * sd.r + c);
    const RowMeta m = static_cast<const RowMeta*>(sd.meta)[row];
    const int code = static_cast<const signed char*>(sd.z)[row * sd.r + c];
    return (float)(code - m.zeropoint) / m.scale;
}

// Activation between the two fully connected layers of an encoder / decoder.
__device__ __forceinline__ float apply_act(float x, int act, float slope) {
    if (act == KVCAR_ACT_LEAKY_RELU) return x >= 0.f ? x : slope * x;
    if (act == KVCAR_ACT_GELU) return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    return x;
}

// erf by the rational-times-Gaussian form (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7): for GELU in
// kernels whose result is rounded to 16 bits afterwards.
__device__ __forceinline__ float erf_rational(float x) {
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
    return copysignf(fmaf(-p * t, e, 1.0f), x);
}

// Pins a value in a register as the compiler sees it.  A value that is split into a 16-bit hi part and
// the remainder lo = x - hi must round to hi ONCE: when x is the product of two registers the compiler
// may fold the multiply into the conversion (one rounding of the exact product) at one use and convert
// the fp32 product (two roundings) at another, and near a rounding tie hi + lo is then off by a whole
// unit in hi's last place.  Passing x through here first makes every use see the same fp32 value.
__device__ __forceinline__ float pinned(float x) {
    asm("" : "+v"(x));
    return x;
}

// int8 quantisation of one latent row ("Quantization", Eq. "quant"), one fp32 operation per step:
//   scale = 255 / (max - min);  zeropoint = -round(scale * min) - 128;  code = round(scale * x + zeropoint)
// round = half to even, codes saturate to [-128, 127]; a row of equal values uses |x| as its range, an
// all-zero row 1.  Products are pinned so that none is fused into the add that follows.
struct QuantParams {
    float scale, zp;       // zp holds the integer zero point as a float
};
__device__ __forceinline__ QuantParams quant_params(float mn, float mx) {
    float rng = mx - mn;
    if (rng == 0.f) rng = fabsf(mx);
    if (rng == 0.f) rng = 1.f;
    QuantParams q;
    q.scale = 255.f / rng;                                  // correctly rounded fp32 division
    q.zp = -rintf(pinned(q.scale * mn)) - 128.f;
    return q;
}
__device__ __forceinline__ signed char quant_code(float x, const QuantParams& q) {
    const float c = rintf(pinned(q.scale * x) + q.zp);
    return (signed char)(int)fminf(fmaxf(c, -128.f), 127.f);
}
__device__ __forceinline__ RowMeta quant_meta(const QuantParams& q) {
    return RowMeta{q.scale, (int)fminf(fmaxf(q.zp, -2147483648.f), 2147483520.f)};
}

__device__ __forceinline__ float apply_act_fast(float x, int act, float slope) {
    if (act == KVCAR_ACT_LEAKY_RELU) return x >= 0.f ? x : slope * x;
    if (act == KVCAR_ACT_GELU) return 0.5f * x * (1.f + erf_rational(x * 0.70710678118654752f));
    return x;
}

// GELU(x) = x * Phi(x) with Phi(x) = 0.5 + x R(x^2), R a degree-8 polynomial fitted on |x| <= 4 (least
// squares on Chebyshev nodes, weighted by x); beyond that Phi is held at its value at +-4.  |Phi error|
// <= 3.1e-5, i.e. |GELU error| <= 3.1e-5 |x|: two orders below the 16-bit rounding applied right after.
// No transcendental instruction: 8 FMAs, a clamp and three multiplies.
__device__ __forceinline__ float fast_gelu(float x) {
    const float xc = __builtin_amdgcn_fmed3f(x, -4.0f, 4.0f);
    const float s = xc * xc;
    float r = 7.804710350223232e-11f;
    r = fmaf(r, s, -6.827684195798156e-09f);
    r = fmaf(r, s, 2.666981799848145e-07f);
    r = fmaf(r, s, -6.222018782864325e-06f);
    r = fmaf(r, s, 9.829134069150314e-05f);
    r = fmaf(r, s, -0.0011309664696455002f);
    r = fmaf(r, s, 0.009869969449937344f);
    r = fmaf(r, s, -0.06640204787254333f);
    r = fmaf(r, s, 0.39891988039016724f);
    return x * fmaf(xc, r, 0.5f);
}

template <int ACT>
__device__ __forceinline__ float fast_act(float x, float slope) {
    if (ACT == KVCAR_ACT_LEAKY_RELU) return x >= 0.f ? x : slope * x;
    if (ACT == KVCAR_ACT_GELU) return fast_gelu(x);
    return x;
}

}  // namespace kvcar
