// MFMA kernels for the two small projections around the attention kernel (gfx950, 16-bit dtypes):
//
//   absorbed queries   qt[(b,slot), c]  = scale*log2(e) * sum_k q[(b,slot), k] * Wl_K[c, col+k]
//   output epilogue    out[(b,slot), k] = sum_c o[(b,slot), c] * Wl_V[c, col+k] + bl_V[col+k]
//                      with o = the split partials merged and normalised
//
// i.e. the last (linear) decoder layer applied to the query instead of to every cached key row,
// and to the softmax-weighted latent sum instead of to every cached value row ("Network
// Architecture", 2nd paragraph, restated by linearity).  Query heads that share a KV head share the
// 64-column slice of the decoder matrix, so rows (sequence, head) are batched per KV head into
// 16-row MFMA blocks: [B*heads, d_head] x [d_head, r] and [B*heads, r] x [r, d_head].
#include "kvcar_qtilde_mfma.hpp"

namespace kvcar {

template <typename E>
__global__ __launch_bounds__(256) void qtilde_mfma_kernel(AttendParams p) {
    qtilde_mfma_block<E>(&p, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.x);
}

// ---------------------------------------------------------------------------------------------
// split merge + output epilogue.  grid = (row blocks, segment, group); a workgroup owns 4, 16 or 64 rows
// (sequence, head) of one KV head (the launcher picks: few rows per workgroup when the launch is small).
//   phase 0  the decoder-matrix slice [r, d_head] of the KV head is staged in LDS (read later with
//            the transposing load: a lane needs 8 consecutive c of one output column)
//   phase 1  all threads merge the split partials of the workgroup's rows into LDS:
//            o = sum_i o_i 2^(m_i-M) / sum_i l_i 2^(m_i-M)
//   phase 2  out = o . W with MFMA, o fed as a hi + lo pair of 16-bit values (accurate to ~2^-17)
// ---------------------------------------------------------------------------------------------
constexpr int kCombMaxSplits = 32;

template <typename E, int NBO, int kPf, int kDepth = 4>
__global__ __launch_bounds__(256) void combine_mfma_kernel(AttendParams p, int rows_per_wg) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const GroupDesc& g = p.g[blockIdx.z];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    int s0 = 0, len = 0;
    if (!find_segment(g.v_col, g.n_slots, g.n_vseg, g.vseg_lo, g.vseg_hi, blockIdx.y, s0, len)) return;
    const int rows = p.batch * len;
    const int wg_row0 = blockIdx.x * rows_per_wg;
    if (wg_row0 >= rows) return;
    const int rv = g.v.c, dh = p.d_head;      // rows of the last decoder layer: latent or hidden width
    const int col = g.v_col[s0];
    const int stride_w = 2 * dh + 32;
    const int pstride = rv + 4;
    const int ns = p.n_splits;

    char* wbuf = lds;                                                   // [rv][stride_w]
    float* om = reinterpret_cast<float*>(lds + (size_t)rv * stride_w + 1024);   // [rows_per_wg][rv + 4]
    float* wts = om + (size_t)rows_per_wg * pstride;                    // [rows_per_wg][ns]

    // Small launches are a chain of memory round trips (decoder slice, (m, l) pairs, latent sums): when a thread
    // has at most kPf items of phase 1b, their first kDepth splits (4, or 16 for launches of a few rows) are
    // requested here, before anything waits on memory, so that the three share one round trip.
    const int c4n = rv >> 2;
    constexpr bool prefetch = kPf > 0;                      // the launcher picks kPf >= items per thread, or 0
    f32x4_t xp[kPf > 0 ? kPf : 1][kDepth];
    if constexpr (prefetch) {
#pragma unroll
        for (int it = 0; it < kPf; ++it) {
            const int idx = it * 256 + threadIdx.x;
            const int r = idx / c4n, c4 = idx - r * c4n;
            const int row = wg_row0 + r;
            const bool live = idx < rows_per_wg * c4n && row < rows;
            const int b = live ? row / len : 0, i = live ? row - b * len : 0;
            const float* prow = p.part + (size_t)b * ns * p.part_stride + g.part_off + (size_t)(s0 + i) * pstride + 4 + 4 * (live ? c4 : 0);
#pragma unroll
            for (int u = 0; u < kDepth; ++u)
                xp[it][u] = live && u < ns ? *reinterpret_cast<const f32x4_t*>(prow + (size_t)u * p.part_stride) : f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
    }
    // the (m, l) pair of (row, split) number threadIdx.x joins the same round trip
    float pm = -INFINITY, pl = 0.f;
    {
        const int idx = threadIdx.x;
        const int r = idx / ns, k = idx - r * ns;
        const int row = wg_row0 + r;
        if (idx < rows_per_wg * ns && row < rows) {
            const int b = row / len, i = row - b * len;
            const float* prow = p.part + ((size_t)b * ns + k) * p.part_stride + g.part_off + (size_t)(s0 + i) * pstride;
            pm = prow[0];
            pl = prow[1];
        }
    }
    {   // phase 0
        const int cpr = dh >> 3;                             // 4, 8, 12 or 16 pieces of 16 bytes per row
        const unsigned inv_cpr = (65536u + cpr - 1) / cpr;   // f / cpr == (f * inv_cpr) >> 16 for f < 8192 at these values
        const int total = rv * cpr;
        const char* src = static_cast<const char*>(g.v.wl);
        // eight chunks per thread in flight (a load-store-load-store loop pays one round trip per chunk)
        for (int f0 = threadIdx.x; f0 < total; f0 += 8 * 256) {
            u32x4_t t[8];
            int dst[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int f = f0 + u * 256;
                const int row = (int)(((unsigned)f * inv_cpr) >> 16), ch = f - row * cpr;
                dst[u] = row * stride_w + ch * 16;
                if (f < total) t[u] = *reinterpret_cast<const u32x4_t*>(src + ((size_t)row * g.v.in_width + col) * 2 + ch * 16);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (f0 + u * 256 < total) *reinterpret_cast<u32x4_t*>(wbuf + dst[u]) = t[u];
        }
    }
    // phase 1a: per-row merge weights.  All (row, split) pairs fetch their m and l at once (a serial
    // loop over the splits would pay one memory latency per split), then one thread per row reduces.
    float* ml = wts + (size_t)rows_per_wg * ns;                         // [rows_per_wg][ns][2]
    float* ab = ml + 2 * (size_t)rows_per_wg * ns;                      // [rows_per_wg][2]: weights of bias and of the exact current row
    if (threadIdx.x < rows_per_wg * ns) {
        ml[2 * threadIdx.x] = pm;
        ml[2 * threadIdx.x + 1] = pl;
    }
    for (int idx = threadIdx.x + 256; idx < rows_per_wg * ns; idx += 256) {
        const int r = idx / ns, k = idx - r * ns;
        const int row = wg_row0 + r;
        float m_k = -INFINITY, l_k = 0.f;
        if (row < rows) {
            const int b = row / len, i = row - b * len;
            const float* prow = p.part + ((size_t)b * ns + k) * p.part_stride + g.part_off + (size_t)(s0 + i) * pstride;
            m_k = prow[0];
            l_k = prow[1];
        }
        ml[2 * idx] = m_k;
        ml[2 * idx + 1] = l_k;
    }
    __syncthreads();
    // With the current token's exact row (k_cur, v_cur) one more softmax term joins the merge:
    // s = scale q . k_cur[head], weight 2^(s-M); the output is (L (o W + b) + 2^(s-M) v_cur) / (L + 2^(s-M)).
    for (int r = threadIdx.x; r < rows_per_wg; r += 256) {
        float M = -INFINITY;
        for (int k = 0; k < ns; ++k) M = fmaxf(M, ml[2 * (r * ns + k)]);
        float s_cur = -INFINITY;
        const int row = wg_row0 + r;
        if (p.k_cur && row < rows) {
            const int b = row / len, i = row - b * len;
            const int head = g.q_head[s0 + i];
            const size_t qo = ((size_t)b * p.n_q_heads + head) * dh, ko = ((size_t)b * (p.n_q_heads / p.gq) + head / p.gq) * dh;
            float d = 0.f;
            // the K decoder's last-layer bias was left out of the cached scores (it cancels among them):
            // the exact row's score is lowered by q . b instead
            const int kcol = g.k_col[s0 + i];
            for (int k = 0; k < dh; ++k)
                d = fmaf(Elem<E>::load(p.q, qo + k), Elem<E>::load(p.k_cur, ko + k) - (g.k.bl ? Elem<E>::load(g.k.bl, kcol + k) : 0.f), d);
            s_cur = d * p.scale_log2e;
            M = fmaxf(M, s_cur);
        }
        float L = 0.f;
        for (int k = 0; k < ns; ++k) {
            const float m_k = ml[2 * (r * ns + k)];
            const float e = m_k == -INFINITY ? 0.f : exp2f(m_k - M);
            wts[r * ns + k] = e;
            L += ml[2 * (r * ns + k) + 1] * e;
        }
        const float pc = s_cur == -INFINITY ? 0.f : exp2f(s_cur - M);
        const float inv = L + pc > 0.f ? 1.f / (L + pc) : 0.f;
        for (int k = 0; k < ns; ++k) wts[r * ns + k] *= inv;
        ab[2 * r] = p.k_cur ? L * inv : 1.f;
        ab[2 * r + 1] = pc * inv;
    }
    __syncthreads();
    // phase 1b: merged, normalised latent sums
    if constexpr (prefetch) {
#pragma unroll
        for (int it = 0; it < kPf; ++it) {
            const int idx = it * 256 + threadIdx.x;
            if (idx >= rows_per_wg * c4n) continue;
            const int r = idx / c4n, c4 = idx - r * c4n;
            const int row = wg_row0 + r;
            f32x4_t a = {0.f, 0.f, 0.f, 0.f};
            if (row < rows) {
#pragma unroll
                for (int u = 0; u < kDepth; ++u)
                    if (u < ns) a += xp[it][u] * wts[r * ns + u];
                const int b = row / len, i = row - b * len;
                const float* prow = p.part + (size_t)b * ns * p.part_stride + g.part_off + (size_t)(s0 + i) * pstride + 4 + 4 * c4;
                for (int k = kDepth; k < ns; k += 4) {
                    f32x4_t x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        x[u] = k + u < ns ? *reinterpret_cast<const f32x4_t*>(prow + (size_t)(k + u) * p.part_stride) : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (k + u < ns) a += x[u] * wts[r * ns + k + u];
                }
            }
            *reinterpret_cast<f32x4_t*>(om + (size_t)r * pstride + 4 * c4) = a;
        }
    } else {
        for (int idx = threadIdx.x; idx < rows_per_wg * c4n; idx += 256) {
            const int r = idx / c4n, c4 = idx - r * c4n;
            const int row = wg_row0 + r;
            f32x4_t a = {0.f, 0.f, 0.f, 0.f};
            if (row < rows) {
                const int b = row / len, i = row - b * len;
                const float* prow = p.part + (size_t)b * ns * p.part_stride + g.part_off + (size_t)(s0 + i) * pstride + 4 + 4 * c4;
                // four partials in flight at a time (a load inside a one-at-a-time loop pays its latency each turn)
                for (int k = 0; k < ns; k += 4) {
                    f32x4_t x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        x[u] = k + u < ns ? *reinterpret_cast<const f32x4_t*>(prow + (size_t)(k + u) * p.part_stride) : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (k + u < ns) a += x[u] * wts[r * ns + k + u];
                }
            }
            *reinterpret_cast<f32x4_t*>(om + (size_t)r * pstride + 4 * c4) = a;
        }
    }
    __syncthreads();

    // phase 2.  Workgroups of up to 16 rows have one row block: its k-steps are dealt over the four waves, whose
    // partial products wave 0 adds in wave order (the decoder slice's buffer takes them once every wave has read it).
    const int nbo = dh >> 4;
    const bool ksplit = rows_per_wg <= 16 && rv >= 128 && (size_t)rv * stride_w >= (size_t)nbo * 4 * 1024;
    const int row0 = ksplit ? 0 : wave * 16;          // within the workgroup
    if (!ksplit && (row0 >= rows_per_wg || wg_row0 + row0 >= rows)) return;
    f32x4_t acc[NBO];
#pragma unroll
    for (int nb = 0; nb < NBO; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const float* arow = om + (size_t)min(row0 + l16, rows_per_wg - 1) * pstride;      // workgroups of fewer than 16 rows: the block's other rows are not stored
    for (int k0 = ksplit ? 32 * wave : 0; k0 < rv; k0 += ksplit ? 128 : 32) {
        const f32x4_t x0 = *reinterpret_cast<const f32x4_t*>(arow + k0 + 8 * lg);
        const f32x4_t x1 = *reinterpret_cast<const f32x4_t*>(arow + k0 + 8 * lg + 4);
        const float o[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
        unsigned hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint16_t h0 = PMma<E>::to16(o[2 * e]), h1 = PMma<E>::to16(o[2 * e + 1]);
            const uint16_t l0 = PMma<E>::to16(o[2 * e] - PMma<E>::from16(h0)), l1 = PMma<E>::to16(o[2 * e + 1] - PMma<E>::from16(h1));
            hi[e] = (unsigned)h0 | ((unsigned)h1 << 16);
            lo[e] = (unsigned)l0 | ((unsigned)l1 << 16);
        }
        const u32x4_t ah = {hi[0], hi[1], hi[2], hi[3]}, al = {lo[0], lo[1], lo[2], lo[3]};
        const char* wrow = wbuf + (k0 + 8 * lg + (l16 >> 2)) * stride_w + (l16 & 3) * 8;
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb) {
            if (nb < nbo) {
                const s16x4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32));
                const s16x4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(wrow + nb * 32 + 4 * stride_w));
                const u32x2_t a0 = __builtin_bit_cast(u32x2_t, t0), a1 = __builtin_bit_cast(u32x2_t, t1);
                const u32x4_t bw = {a0[0], a0[1], a1[0], a1[1]};
                acc[nb] = PMma<E>::mfma(ah, bw, acc[nb]);
                acc[nb] = PMma<E>::mfma(al, bw, acc[nb]);
            }
        }
    }
    if (ksplit) {
        __syncthreads();                                   // every wave is done with the decoder slice
        f32x4_t* part2 = reinterpret_cast<f32x4_t*>(wbuf); // [wave][nbo][64]
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb)
            if (nb < nbo) part2[(wave * nbo + nb) * 64 + lane] = acc[nb];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb)
            if (nb < nbo) {
                f32x4_t a = part2[nb * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) a += part2[(w * nbo + nb) * 64 + lane];
                acc[nb] = a;
            }
    }
    // epilogue: bias, one rounding, store; this lane holds output column 16*nb + l16 of rows 4*lg + v
    uint16_t* out = static_cast<uint16_t*>(p.out);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int rl = row0 + 4 * lg + v;
        const int r = wg_row0 + rl;
        if (rl >= rows_per_wg || r >= rows) continue;
        const int b = r / len, i = r - b * len;
        const size_t base = ((size_t)b * p.n_q_heads + g.q_head[s0 + i]) * dh;
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb) {
            if (nb < nbo) {
                const int k = nb * 16 + l16;
                const float bias = g.v.bl ? Elem<E>::load(g.v.bl, col + k) : 0.f;
                float y = acc[nb][v] + ab[2 * rl] * bias;
                if (p.v_cur) y += ab[2 * rl + 1] * Elem<E>::load(p.v_cur, ((size_t)b * (p.n_q_heads / p.gq) + g.q_head[s0 + i] / p.gq) * dh + k);
                out[base + k] = PMma<E>::to16(y);
            }
        }
    }
}

// d_head a multiple of 32 (k-steps of the query product, column blocks of the output), up to 128;
// latent widths multiples of 32.
bool proj_mfma_supported(const AttendParams& p, int dtype) {
    if (dtype == KVCAR_F32 || p.d_head % 32 || p.d_head > 128 || p.n_splits > kCombMaxSplits) return false;
    for (int i = 0; i < p.n_groups; ++i)
        if (p.g[i].k.c % 32 || p.g[i].v.c % 32) return false;
    return true;
}

static int max_segments(const AttendParams& p, bool use_k, int& max_len) {
    int mx = 0;
    max_len = 1;
    for (int i = 0; i < p.n_groups; ++i) {
        const short* col = use_k ? p.g[i].k_col : p.g[i].v_col;
        int segs = 0, run = 0;
        for (int s = 0; s < p.g[i].n_slots; ++s) {
            if (s == 0 || col[s] != col[s - 1]) { ++segs; run = 0; }
            ++run;
            max_len = run > max_len ? run : max_len;
        }
        mx = segs > mx ? segs : mx;
    }
    return mx;
}

// Grid of the absorbed-query projection: (16-row blocks, segments + 1, groups); +1: zero-fill of padding slots.
void qtilde_mfma_grid(const AttendParams& p, int& qx, int& qy, int& qz) {
    int max_len;
    const int segs = max_segments(p, true, max_len);
    qx = (p.batch * max_len + 15) / 16;
    qy = segs + 1;
    qz = p.n_groups;
}

hipError_t launch_qtilde_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    int qx, qy, qz;
    qtilde_mfma_grid(p, qx, qy, qz);
    dim3 grid(qx, qy, qz);
    if (dtype == KVCAR_BF16) hipLaunchKernelGGL(qtilde_mfma_kernel<BF16>, grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(qtilde_mfma_kernel<F16>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_combine_mfma(const AttendParams& p, int dtype, hipStream_t stream) {
    int max_len, rmax = 0;
    const int segs = max_segments(p, false, max_len);
    for (int i = 0; i < p.n_groups; ++i) rmax = p.g[i].v.c > rmax ? p.g[i].v.c : rmax;
    // 64 rows per workgroup for narrow rows; 16 when the launch is small (more workgroups, and few enough items
    // per thread for the kernel to request everything at once); 4 when even that leaves most of the chip idle (a few
    // sequences: every thread then has one or two items and requests all their splits, up to 16, in one go)
    const long long rows_all = (long long)p.batch * max_len * segs * p.n_groups;
    int rows_per_wg = rmax <= 128 && rows_all > 64 * 64 ? 64 : 16;
    if (rows_per_wg == 16 && rows_all <= 16 * 64 && (4 * (rmax >> 2) + 255) / 256 <= 2) rows_per_wg = 4;
    const size_t lds = (size_t)rmax * (2 * p.d_head + 32) + 1024 + (size_t)rows_per_wg * (rmax + 4 + 3 * p.n_splits + 2) * sizeof(float);
    dim3 grid((p.batch * max_len + rows_per_wg - 1) / rows_per_wg, segs, p.n_groups);
    const int items = (rows_per_wg * (rmax >> 2) + 255) / 256;        // phase-1b items per thread
    const bool deep = rows_per_wg == 4 && p.n_splits > 4;             // all splits (up to 16) of an item in flight
    const int pf = items <= 2 ? 2 : items <= 6 ? 6 : 0;
    void (*kern)(AttendParams, int);
    if (dtype == KVCAR_BF16) kern = deep ? combine_mfma_kernel<BF16, 8, 2, 16> : pf == 2 ? combine_mfma_kernel<BF16, 8, 2> : pf == 6 ? combine_mfma_kernel<BF16, 8, 6> : combine_mfma_kernel<BF16, 8, 0>;
    else kern = deep ? combine_mfma_kernel<F16, 8, 2, 16> : pf == 2 ? combine_mfma_kernel<F16, 8, 2> : pf == 6 ? combine_mfma_kernel<F16, 8, 6> : combine_mfma_kernel<F16, 8, 0>;
    const int slot = (dtype == KVCAR_BF16 ? 0 : 4) + (deep ? 3 : pf == 2 ? 1 : pf == 6 ? 2 : 0);
    static AttrFlag attr[8] = {};
    if (!attr[slot]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (err != hipSuccess) return err;
        attr[slot] = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p, rows_per_wg);
    return hipGetLastError();
}

}  // namespace kvcar
