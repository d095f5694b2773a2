// Plain-ALU kernels of libkvcar: encode+append, absorbed-query prologue, attention over the latent
// cache (any dtype, linear or two-layer decoders), split merge + last-decoder-layer epilogue.
// They are the only kernels for fp32 and for shapes the MFMA kernels do not cover.
//
// Decoder handling ("Network Architecture": the decoder expands every cached row at every step):
// the decoder's last layer is linear, x^ = h W + b, so for a query head with columns C of KV head g
//   q . x^[C]            = (W[:,C] q) . h + const      -> the constant cancels in the softmax
//   sum_t p_t x^_t[C]    = (sum_t p_t h_t) W[:,C] + b[C]
// where h is the latent row itself (linear decoder) or act(z W1 + b1) (two-layer decoder).  The
// kernels therefore attend over rows h_t and apply W once per head before and after.
#include <algorithm>

#include "kvcar_device.hpp"

namespace kvcar {

// ---------------------------------------------------------------------------------------------
// encode + append:  z = x[cols] W1 + b1            (linear encoder)
//                   z = act(x[cols] W1 + b1) W2 + b2 (two fully connected layers)
// One workgroup handles kTok tokens of one tensor (K or V).
// ---------------------------------------------------------------------------------------------
constexpr int kEncTok = 8;

template <typename E>
__global__ __launch_bounds__(256) void encode_generic_kernel(EncodeParams p) {
    extern __shared__ float smem[];
    const EncodeSide& s = p.s[blockIdx.y];
    if (s.r == 0) return;
    const int n_tok = p.batch * p.t_new;
    const int tok0 = blockIdx.x * kEncTok;
    const int nt = min(kEncTok, n_tok - tok0);
    float* xs = smem;                              // [kEncTok][in_width]
    float* hs = smem + kEncTok * s.in_width;       // [kEncTok][hidden]
    float* zs = hs + kEncTok * s.hidden;           // [kEncTok][r] (int8 latents only)
    const int tid = threadIdx.x;

    for (int i = tid; i < nt * s.in_width; i += 256) {
        const int t = i / s.in_width, c = i % s.in_width;
        const int src_col = (int)s.heads[c / p.d_head] * p.d_head + c % p.d_head;
        xs[t * s.in_width + c] = Elem<E>::load(s.x, (size_t)(tok0 + t) * p.d_kv + src_col);
    }
    __syncthreads();

    const float* in = xs;
    int in_w = s.in_width;
    if (s.hidden > 0) {
        for (int i = tid; i < nt * s.hidden; i += 256) {
            const int t = i / s.hidden, c = i % s.hidden;
            float a = s.b1 ? Elem<E>::load(s.b1, c) : 0.f;
#pragma unroll 16
            for (int k = 0; k < s.in_width; ++k) a = fmaf(xs[t * s.in_width + k], Elem<E>::load(s.w1, (size_t)k * s.hidden + c), a);
            hs[t * s.hidden + c] = apply_act(a, s.act, s.slope);
        }
        __syncthreads();
        in = hs;
        in_w = s.hidden;
    }
    const void* w = s.hidden > 0 ? s.w2 : s.w1;
    const void* bias = s.hidden > 0 ? s.b2 : s.b1;
    for (int i = tid; i < nt * s.r; i += 256) {
        const int t = i / s.r, c = i % s.r;
        float a = bias ? Elem<E>::load(bias, c) : 0.f;
#pragma unroll 16
        for (int k = 0; k < in_w; ++k) a = fmaf(in[t * in_w + k], Elem<E>::load(w, (size_t)k * s.r + c), a);
        if (s.meta) { zs[t * s.r + c] = a; continue; }
        const int tok = tok0 + t;
        const int b = tok / p.t_new, tt = tok % p.t_new;
        Elem<E>::store(s.z, ((size_t)b * p.max_seq + (p.positions ? p.positions[b] : p.pos0) + tt) * s.r + c, a);
    }
    if (s.meta == nullptr) return;

    // ---- int8 latents ("Quantization", Eq. "quant"): 32 lanes per token row -------------------------
    __syncthreads();
    const int t = tid >> 5, j = tid & 31;
    if (t >= nt) return;
    const float* zr = zs + t * s.r;
    float mn = INFINITY, mx = -INFINITY;
    for (int c = j; c < s.r; c += 32) { mn = fminf(mn, zr[c]); mx = fmaxf(mx, zr[c]); }
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, off));
        mx = fmaxf(mx, __shfl_xor(mx, off));
    }
    const QuantParams qp = quant_params(mn, mx);
    const int tok = tok0 + t;
    const int b = tok / p.t_new, tt = tok % p.t_new;
    const size_t row = (size_t)b * p.max_seq + (p.positions ? p.positions[b] : p.pos0) + tt;
    signed char* codes = static_cast<signed char*>(s.z) + row * s.r;
    for (int c = j; c < s.r; c += 32) codes[c] = quant_code(zr[c], qp);
    if (j == 0) static_cast<RowMeta*>(s.meta)[row] = quant_meta(qp);
}

hipError_t launch_encode_generic(const EncodeParams& p, int dtype, hipStream_t stream) {
    const int n_tok = p.batch * p.t_new;
    dim3 grid((n_tok + kEncTok - 1) / kEncTok, 2);
    size_t lds = 0;
    for (int i = 0; i < 2; ++i) {
        size_t need = (size_t)kEncTok * (p.s[i].in_width + p.s[i].hidden + (p.s[i].meta ? p.s[i].r : 0)) * sizeof(float);
        lds = need > lds ? need : lds;
    }
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(encode_generic_kernel<F32>, grid, dim3(256), lds, stream, p);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(encode_generic_kernel<F16>, grid, dim3(256), lds, stream, p);
    else hipLaunchKernelGGL(encode_generic_kernel<BF16>, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// absorbed queries:  qt[b][group][slot][c] = scale*log2(e) * sum_k Wl_K[c, col(slot)+k] q[b, head(slot), k]
// stored as fp32 (plain-ALU attention) or in the 16-bit dtype (MFMA attention).  Padding slots = 0.
// ---------------------------------------------------------------------------------------------
template <typename E, bool kF32Out>
__global__ __launch_bounds__(256) void qtilde_kernel(AttendParams p) {
    extern __shared__ float smem[];
    const GroupDesc& g = p.g[blockIdx.y];
    const int b = blockIdx.x;
    const int dh = p.d_head;
    float* qs = smem;                                   // [n_slots][d_head]
    for (int i = threadIdx.x; i < g.n_slots * dh; i += 256) {
        const int s = i / dh, k = i % dh;
        qs[i] = Elem<E>::load(p.q, ((size_t)b * p.n_q_heads + g.q_head[s]) * dh + k);
    }
    __syncthreads();
    const int c_w = g.k.c;
    const size_t base = (size_t)b * p.qt_stride + g.qt_off;
    // the (slot, column) items are dealt over blockIdx.z: a single sequence would otherwise leave one workgroup with all of them
    for (int i = blockIdx.z * 256 + threadIdx.x; i < g.slots_pad * c_w; i += 256 * gridDim.z) {
        const int s = i / c_w, c = i % c_w;
        float a = 0.f;
        if (s < g.n_slots) {
            const size_t wrow = (size_t)c * g.k.in_width + g.k_col[s];
#pragma unroll 16
            for (int k = 0; k < dh; ++k) a = fmaf(Elem<E>::load(g.k.wl, wrow + k), qs[s * dh + k], a);
            a *= p.scale_log2e;
        }
        if (kF32Out) static_cast<float*>(p.qt)[base + i] = a;
        else Elem<E>::store(p.qt, base + i, a);
    }
}

hipError_t launch_qtilde(const AttendParams& p, int dtype, bool qt_f32, hipStream_t stream) {
    int items = 0;
    for (int i = 0; i < p.n_groups; ++i) items = std::max(items, p.g[i].slots_pad * p.g[i].k.c);
    const int nz = std::max(1, std::min(16, std::min((items + 255) / 256, 512 / std::max(1, p.batch * p.n_groups))));     // a few hundred workgroups at most
    dim3 grid(p.batch, p.n_groups, nz);
    size_t lds = (size_t)kMaxSlots * p.d_head * sizeof(float);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL((qtilde_kernel<F32, true>), grid, dim3(256), lds, stream, p);
    else if (dtype == KVCAR_F16) {
        if (qt_f32) hipLaunchKernelGGL((qtilde_kernel<F16, true>), grid, dim3(256), lds, stream, p);
        else hipLaunchKernelGGL((qtilde_kernel<F16, false>), grid, dim3(256), lds, stream, p);
    } else {
        if (qt_f32) hipLaunchKernelGGL((qtilde_kernel<BF16, true>), grid, dim3(256), lds, stream, p);
        else hipLaunchKernelGGL((qtilde_kernel<BF16, false>), grid, dim3(256), lds, stream, p);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// plain-ALU attention over rows h_t, one workgroup per (split, sequence, group).
// Partial written per (b, split, group): for each slot  [m, l, -, -, o[0..cv)]  with scores in log2 units.
// ---------------------------------------------------------------------------------------------
// `codes` (keys over int8 rows through a linear decoder): the rows are left as their integer codes and the tile's
// scales and zero points go to inv / zp; the caller applies them to the finished dot products (see there).
template <typename E>
__device__ void load_rows(const SideDesc& sd, float* rows, float* zrow, int b, int t0, int nt, int max_seq, bool codes = false, float* inv = nullptr,
                          int* zp = nullptr) {
    // rows [kGenericTile][c+1]; rows of tokens >= nt are zero
    const int tid = threadIdx.x;
    const int ld = sd.c + 1;
    if (codes) {
        for (int i = tid; i < kGenericTile * sd.c; i += 256) {
            const int t = i / sd.c, c = i % sd.c;
            rows[t * ld + c] = t < nt ? (float)static_cast<const signed char*>(sd.z)[((size_t)b * max_seq + t0 + t) * sd.r + c] : 0.f;
        }
        if (tid < kGenericTile) {
            const RowMeta m = tid < nt ? static_cast<const RowMeta*>(sd.meta)[(size_t)b * max_seq + t0 + tid] : RowMeta{1.f, 0};
            inv[tid] = 1.f / m.scale;
            zp[tid] = m.zeropoint;
        }
        return;
    }
    if (sd.w1 == nullptr) {
        for (int i = tid; i < kGenericTile * sd.c; i += 256) {
            const int t = i / sd.c, c = i % sd.c;
            rows[t * ld + c] = t < nt ? latent_at<E>(sd, (size_t)b * max_seq + t0 + t, c) : 0.f;
        }
        return;
    }
    for (int i = tid; i < kGenericTile * sd.r; i += 256) {
        const int t = i / sd.r, c = i % sd.r;
        zrow[i] = t < nt ? latent_at<E>(sd, (size_t)b * max_seq + t0 + t, c) : 0.f;
    }
    __syncthreads();
    for (int i = tid; i < kGenericTile * sd.c; i += 256) {
        const int t = i / sd.c, c = i % sd.c;
        float a = sd.b1 ? Elem<E>::load(sd.b1, c) : 0.f;
#pragma unroll 16
        for (int k = 0; k < sd.r; ++k) a = fmaf(zrow[t * sd.r + k], Elem<E>::load(sd.w1, (size_t)k * sd.c + c), a);
        rows[t * ld + c] = t < nt ? apply_act(a, sd.act, sd.slope) : 0.f;
    }
    __syncthreads();   // zrow is reused by the next call
}

size_t attend_generic_lds_bytes(const GroupDesc& g) {
    size_t zr = 0;
    if (g.k.w1) zr = g.k.r;
    if (g.v.w1 && (size_t)g.v.r > zr) zr = g.v.r;
    size_t f = (size_t)g.n_slots * g.k.c + (size_t)kGenericTile * (g.k.c + 1) + (size_t)kGenericTile * (g.v.c + 1) +
               (size_t)kGenericTile * zr + (size_t)g.n_slots * kGenericTile + 3 * (size_t)g.n_slots;
    f += 2 * (size_t)g.n_slots + 2 * kGenericTile + 2;      // int8 key rows: the slots' query sums (fp64) and the tile's scales and zero points
    return f * sizeof(float);
}

template <typename E>
__global__ __launch_bounds__(256) void attend_generic_kernel(AttendParams p) {
    extern __shared__ float smem[];
    const GroupDesc& g = p.g[blockIdx.z];
    const int split = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    const int ns = g.n_slots, ck = g.k.c, cv = g.v.c;
    const int n_ctx = p.seq_lens ? min(p.seq_lens[b], p.n_ctx) : p.n_ctx;
    int zr = 0;
    if (g.k.w1) zr = g.k.r;
    if (g.v.w1 && g.v.r > zr) zr = g.v.r;

    float* qt = smem;                                   // [ns][ck]
    float* rk = qt + ns * ck;                           // [tile][ck+1]
    float* rv = rk + kGenericTile * (ck + 1);           // [tile][cv+1]
    float* zrow = rv + kGenericTile * (cv + 1);         // [tile][zr]
    float* sc = zrow + kGenericTile * zr;               // [ns][tile]
    float* m_s = sc + ns * kGenericTile;                // [ns]
    float* l_s = m_s + ns;
    float* a_s = l_s + ns;
    // Keys over int8 rows through a linear decoder: score = (sum_c qt_c code_c - zeropoint sum_c qt_c) / scale.  A row far
    // from zero has a large zero point, and the second term - the same for every token up to the rows' own offsets,
    // so softmax only sees differences of it - is then far larger than the score: the difference is formed in fp64 from
    // the fp32 dot product over the codes and the slot's query sum (fp64).  Dequantising the row in fp32 first would
    // round away part of every code once |zeropoint| passes 2^20.
    const bool k_codes = g.k.meta != nullptr && g.k.w1 == nullptr;
    float* inv_k = a_s + ns;                            // [tile]
    int* zp_k = reinterpret_cast<int*>(inv_k + kGenericTile);
    double* qsum = reinterpret_cast<double*>((reinterpret_cast<uintptr_t>(zp_k + kGenericTile) + 7) & ~(uintptr_t)7);      // [ns]

    const float* qsrc = static_cast<const float*>(p.qt) + (size_t)b * p.qt_stride + g.qt_off;
    for (int i = tid; i < ns * ck; i += 256) qt[i] = qsrc[i];
    if (tid < ns) { m_s[tid] = -INFINITY; l_s[tid] = 0.f; }
    if (k_codes) {
        __syncthreads();
        if (tid < ns) {
            double a = 0.0;
            for (int c = 0; c < ck; ++c) a += (double)qt[tid * ck + c];
            qsum[tid] = a;
        }
    }

    float acc[kGenericAcc];
#pragma unroll
    for (int i = 0; i < kGenericAcc; ++i) acc[i] = 0.f;
    const int n_out = ns * cv;

    // contiguous token range of this split, in whole tiles
    const int tiles = (n_ctx + kGenericTile - 1) / kGenericTile;
    const int tiles_per = (tiles + p.n_splits - 1) / p.n_splits;
    const int tile0 = split * tiles_per;
    const int tile1 = min(tiles, tile0 + tiles_per);
    __syncthreads();

    for (int tile = tile0; tile < tile1; ++tile) {
        const int t0 = tile * kGenericTile;
        const int nt = min(kGenericTile, n_ctx - t0);
        load_rows<E>(g.k, rk, zrow, b, t0, nt, p.max_seq, k_codes, inv_k, zp_k);
        load_rows<E>(g.v, rv, zrow, b, t0, nt, p.max_seq);
        __syncthreads();
        for (int i = tid; i < ns * kGenericTile; i += 256) {
            const int s = i / kGenericTile, t = i % kGenericTile;
            float a = 0.f;
            for (int c = 0; c < ck; ++c) a = fmaf(qt[s * ck + c], rk[t * (ck + 1) + c], a);
            if (k_codes) a = (float)((double)a - (double)zp_k[t] * qsum[s]) * inv_k[t];
            sc[i] = t < nt ? a : -INFINITY;
        }
        __syncthreads();
        if (tid < ns) {
            float mx = m_s[tid];
            for (int t = 0; t < kGenericTile; ++t) mx = fmaxf(mx, sc[tid * kGenericTile + t]);
            const float alpha = exp2f(m_s[tid] - mx);     // m = -inf on the first tile gives 0
            float sum = 0.f;
            for (int t = 0; t < kGenericTile; ++t) {
                const float e = exp2f(sc[tid * kGenericTile + t] - mx);
                sc[tid * kGenericTile + t] = e;
                sum += e;
            }
            l_s[tid] = l_s[tid] * alpha + sum;
            m_s[tid] = mx;
            a_s[tid] = alpha;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kGenericAcc; ++i) {
            const int o = tid + i * 256;
            if (o < n_out) {
                const int s = o / cv, c = o % cv;
                float a = acc[i] * a_s[s];
                for (int t = 0; t < kGenericTile; ++t) a = fmaf(sc[s * kGenericTile + t], rv[t * (cv + 1) + c], a);
                acc[i] = a;
            }
        }
        __syncthreads();
    }

    float* part = p.part + ((size_t)b * p.n_splits + split) * p.part_stride + g.part_off;
    if (tid < ns) { part[tid * (cv + 4)] = m_s[tid]; part[tid * (cv + 4) + 1] = l_s[tid]; }
#pragma unroll
    for (int i = 0; i < kGenericAcc; ++i) {
        const int o = tid + i * 256;
        if (o < n_out) { const int s = o / cv, c = o % cv; part[s * (cv + 4) + 4 + c] = acc[i]; }
    }
}

hipError_t launch_attend_generic(const AttendParams& p, int dtype, hipStream_t stream) {
    size_t lds = 0;
    for (int i = 0; i < p.n_groups; ++i) { size_t n = attend_generic_lds_bytes(p.g[i]); lds = n > lds ? n : lds; }
    dim3 grid(p.n_splits, p.batch, p.n_groups);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(attend_generic_kernel<F32>, grid, dim3(256), lds, stream, p);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(attend_generic_kernel<F16>, grid, dim3(256), lds, stream, p);
    else hipLaunchKernelGGL(attend_generic_kernel<BF16>, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// split merge + epilogue: one workgroup per (sequence, group, slot)
//   M = max_i m_i,  L = sum_i l_i 2^(m_i-M),  o_lat = sum_i o_i 2^(m_i-M) / L
//   out[b, head, k] = sum_c o_lat[c] Wl_V[c, col+k] + bl_V[col+k]   rounded once to dtype
// With the current token's exact row ("Network Architecture", 2nd paragraph: the decoded rows are
// concatenated with the current key and value vectors) one more softmax term joins the merge:
//   s = scale q . k_cur[head],  p = 2^(s-M'),  M' = max(M, s),  L' = L 2^(M-M') + p
//   out = ((L 2^(M-M')) (o_lat W + b) + p v_cur[head]) / L'
// ---------------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(64) void combine_kernel(AttendParams p) {
    __shared__ float olat[kMaxRow];
    const GroupDesc& g = p.g[blockIdx.z];
    const int b = blockIdx.x, s = blockIdx.y;
    if (s >= g.n_slots) return;
    const int cv = g.v.c;
    const int tid = threadIdx.x;
    const float* base = p.part + (size_t)b * p.n_splits * p.part_stride + g.part_off + (size_t)s * (cv + 4);
    float M = -INFINITY;
    for (int i = 0; i < p.n_splits; ++i) M = fmaxf(M, base[(size_t)i * p.part_stride]);
    float L = 0.f;
    for (int i = 0; i < p.n_splits; ++i) {
        const float m_i = base[(size_t)i * p.part_stride];
        L += base[(size_t)i * p.part_stride + 1] * (m_i == -INFINITY ? 0.f : exp2f(m_i - M));
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    float w_cached = 1.f, w_cur = 0.f;                 // weights of the cached part and of the exact current row
    const int kvh = g.q_head[s] / p.gq;
    if (p.k_cur) {
        // the bias of the last K decoder layer shifts every cached score of the head by q . b and was left
        // out of them (it cancels among cached rows): the exact row's score is lowered by it instead
        float d = 0.f;
        for (int k = tid; k < p.d_head; k += 64)
            d = fmaf(Elem<E>::load(p.q, ((size_t)b * p.n_q_heads + g.q_head[s]) * p.d_head + k),
                     Elem<E>::load(p.k_cur, ((size_t)b * (p.n_q_heads / p.gq) + kvh) * p.d_head + k) -
                         (g.k.bl ? Elem<E>::load(g.k.bl, g.k_col[s] + k) : 0.f), d);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) d += __shfl_xor(d, off);
        const float s_cur = d * p.scale_log2e;
        const float M2 = fmaxf(M, s_cur);
        const float lc = M == -INFINITY ? 0.f : L * exp2f(M - M2);
        const float pc = exp2f(s_cur - M2);
        w_cached = lc / (lc + pc);
        w_cur = pc / (lc + pc);
    }
    for (int c = tid; c < cv; c += 64) {
        float a = 0.f;
        for (int i = 0; i < p.n_splits; ++i) {
            const float m_i = base[(size_t)i * p.part_stride];
            if (m_i != -INFINITY) a = fmaf(base[(size_t)i * p.part_stride + 4 + c], exp2f(m_i - M), a);
        }
        olat[c] = a * inv;
    }
    __syncthreads();
    const int col = g.v_col[s];
    for (int k = tid; k < p.d_head; k += 64) {
        float a = g.v.bl ? Elem<E>::load(g.v.bl, col + k) : 0.f;
#pragma unroll 16
        for (int c = 0; c < cv; ++c) a = fmaf(olat[c], Elem<E>::load(g.v.wl, (size_t)c * g.v.in_width + col + k), a);
        if (p.v_cur) a = w_cached * a + w_cur * Elem<E>::load(p.v_cur, ((size_t)b * (p.n_q_heads / p.gq) + kvh) * p.d_head + k);
        Elem<E>::store(p.out, ((size_t)b * p.n_q_heads + g.q_head[s]) * p.d_head + k, a);
    }
}

hipError_t launch_combine(const AttendParams& p, int dtype, hipStream_t stream) {
    int max_slots = 0;
    for (int i = 0; i < p.n_groups; ++i) max_slots = p.g[i].n_slots > max_slots ? p.g[i].n_slots : max_slots;
    dim3 grid(p.batch, max_slots, p.n_groups);
    if (dtype == KVCAR_F32) hipLaunchKernelGGL(combine_kernel<F32>, grid, dim3(64), 0, stream, p);
    else if (dtype == KVCAR_F16) hipLaunchKernelGGL(combine_kernel<F16>, grid, dim3(64), 0, stream, p);
    else hipLaunchKernelGGL(combine_kernel<BF16>, grid, dim3(64), 0, stream, p);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// Read-only streaming probe: every lane folds 16-byte non-temporal loads into a checksum; one
// word per workgroup is written so that the loads cannot be dropped.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned probe_u32x4_t;

__global__ __launch_bounds__(512) void stream_read_kernel(const probe_u32x4_t* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
    probe_u32x4_t acc = {0u, 0u, 0u, 0u};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const unsigned x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9e3779b9u && sink) sink[blockIdx.x] = x;     // practically never true: keeps the loads alive
}

hipError_t launch_stream_read(const void* src, size_t bytes, int n_blocks, int block, unsigned* sink, hipStream_t stream) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_blocks), dim3(block), 0, stream, static_cast<const probe_u32x4_t*>(src), bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace kvcar
