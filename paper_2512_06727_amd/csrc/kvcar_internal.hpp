// Internal declarations shared by the host code and the kernels of libkvcar (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "kvcar.h"

namespace kvcar {

// "This kernel's dynamic-LDS limit has been raised" flags of the launchers: process-wide, set once; two host threads
// that launch at the same moment may both set the attribute, which is harmless.
using AttrFlag = std::atomic<bool>;

constexpr int kMaxSlots = 32;       // query heads served by one group
constexpr int kMaxGroups = 8;       // groups per attention launch
constexpr int kMaxKvHeads = 64;     // bound on n_kv_heads (head lists live in kernel arguments)
constexpr int kGenericTile = 16;    // tokens per tile of the plain-ALU attention kernel
constexpr int kGenericAcc = 48;     // accumulators per thread of the plain-ALU attention kernel
constexpr int kMaxRow = 384;        // widest latent / hidden row any kernel handles
constexpr int kArriveMaxSplits = 128;  // most splits the one-launch form's last workgroup merges
constexpr int kArrivePitch = 32;       // 8-byte words between two arrival counters: 256 bytes apart, so that the atomic
                                       // operations of different (sequence, group) pairs spread over the memory channels
constexpr float kLog2e = 1.4426950408889634f;

// Scale and zero point of one int8 latent row.
struct RowMeta {
    float scale;
    int zeropoint;
};

// One side (keys or values) of a group: where its rows come from and how they are decoded.
struct SideDesc {
    const void* z;        // source layer's latent cache [max_batch, max_seq, r]
    const void* meta;     // int8 latents: {float scale; int zeropoint} per row [max_batch, max_seq]; else null
    const void* w1;       // first decoder layer [r, c] (two-layer decoder only, else null)
    const void* b1;       // its bias or null
    const void* wl;       // last decoder layer [c, in_width]
    const void* bl;       // its bias or null
    int r;                // latent row width
    int c;                // contraction width: r (linear decoder) or hidden width
    int in_width;         // row stride of wl
    int act;              // kvcar_act between the two layers
    float slope;
};

// A group: query heads of one layer that read the same (K source layer, V source layer).
struct GroupDesc {
    SideDesc k, v;
    int n_slots;                   // query heads in the group (<= kMaxSlots)
    int slots_pad;                 // n_slots rounded up to 16
    int qt_off;                    // element offset of the group's absorbed queries, per sequence
    int part_off;                  // float offset of the group's partials, per (sequence, split)
    short q_head[kMaxSlots];       // query head of each slot
    short k_col[kMaxSlots];        // first column of the slot's KV head in k.wl
    short v_col[kMaxSlots];        // same for v.wl
    // Runs of slots with the same KV head (slots are ordered by KV head), worked out on the host so that the
    // fused kernels read a handful of scalars instead of walking the tables above: [lo, hi) and the column.
    // n = 0 when there are more than kMaxSeg runs (then no fused kernel is used).
    short n_kseg, n_vseg;
    short kseg_lo[4], kseg_hi[4], kseg_col[4];
    short vseg_lo[4], vseg_hi[4], vseg_col[4];
    // Append-and-attend: bit 0 / 1 = this group's key / value rows come from the layer whose new token the launch
    // encodes (so its last row is the one being appended); bit 2 / 3 = this group's workgroup also writes that row to
    // the cache (one group per side does).
    short append;
    // Per-head autoencoders: the block of the source's head-major cache this group reads on the key / value side (the
    // position of its KV head among the covered heads), else -1; and the group's first KV head.
    short app_slice[2];
    short app_head;
};
constexpr int kMaxSeg = 4;

constexpr int kAppendMaxHeads = 16;  // KV heads a layer may have for the in-kernel encoder of append-and-attend

// One side (keys or values) of the token that append-and-attend encodes inside the attention kernel: a linear encoder.
struct AppendSide {
    const void* x;        // [batch, d_kv]: the new token's vectors
    void* z;              // the layer's own cache [max_batch, max_seq, r]
    void* meta;           // int8 latents: {float scale; int zeropoint} per row of that cache; else null
    const void* w;        // encoder matrix [in_width, r]
    const void* b;        // its bias or null
    int in_width, r;      // r = 0: the layer stores nothing on this side
    unsigned char heads[kAppendMaxHeads];   // KV heads whose columns form the encoder input, in order
    // Per-head autoencoders: bytes between two heads' blocks of the cache, and in_width = d_head, r = one head's latent
    // width; a group then encodes its own head (GroupDesc::app_head) with the app_slice-th [in_width, r] matrix of w,
    // the app_slice-th r entries of b, into the app_slice-th block of z.  0 = one dense autoencoder.
    long long head_block;
};

struct AttendParams {
    GroupDesc g[kMaxGroups];
    const void* q;        // [batch, H_q, d_head]
    void* out;            // [batch, H_q, d_head]
    void* qt;             // workspace: absorbed queries
    float* part;          // workspace: split partials
    int n_groups;
    int batch, n_ctx, n_splits;
    int n_q_heads, d_head;
    int max_seq;
    int qt_stride;        // absorbed-query elements per sequence (all groups)
    int part_stride;      // partial floats per (sequence, split) (all groups)
    float scale_log2e;    // softmax scale * log2(e)
    int tile_order;       // MFMA kernel: 0 = contiguous token range per split, 1 = tiles dealt round-robin
    int fused;            // MFMA kernel: 1 = absorbed queries and output epilogue computed inside (single split); 2 = the
                          // eight-wave variant of that; 3 = several splits, absorbed queries computed inside, partials to the
                          // merge kernel; 4 = several splits, the last workgroup to arrive merges and decodes (one launch);
                          // 5 = the eight-wave variant of that
    unsigned long long* arrive;   // fused == 4, 5: arrival counter of (sequence b, group z of this launch) at [(b * arrive_stride + z) * kArrivePitch]:
    int arrive_stride;            //   {tag : 32, count : 32}; valid only while the tag equals `epoch`
    unsigned epoch;               //   tag of this launch (never 0)
    int append;                   // 1 = append-and-attend: the new token (position n_ctx - 1 of every sequence) is encoded in
    AppendSide enc[2];            //   this kernel, written to the cache and attended to as the context's last row
    int gq;               // query heads per KV head
    int colocate;         // 1 = groups of this launch read the same rows: the groups of a (split, sequence) share an XCD
    const int* seq_lens;  // per-sequence context length [batch] (ragged batch), or null: n_ctx for all
    const void* k_cur;    // exact key / value row of the current token [batch, H_kv * d_head], attended as one
    const void* v_cur;    //   more row after the cached ones; or both null
};

// Kernel arguments travel in the kernel-argument segment, which holds at most 4 KB.
static_assert(sizeof(AttendParams) <= 4096, "AttendParams must fit the kernel-argument segment");

struct EncodeSide {
    const void* x;        // [batch, t_new, d_kv]
    void* z;              // cache [max_batch, max_seq, r]
    void* meta;           // int8 latents: {float scale; int zeropoint} per row; else null
    const void* w1; const void* b1;   // [in, hidden or r]
    const void* w2; const void* b2;   // [hidden, r] or null
    int in_width, hidden, r, act, n_heads;
    float slope;
    unsigned char heads[kMaxKvHeads]; // KV heads whose columns form the encoder input
};

struct EncodeParams {
    EncodeSide s[2];
    int batch, t_new, pos0, max_seq, d_kv, d_head;
    const int* positions; // per-sequence first position [batch] (ragged batch), or null: pos0 for all
};

// Launchers (defined next to their kernels). All enqueue on `stream` and return hipGetLastError().
hipError_t launch_encode_generic(const EncodeParams& p, int dtype, hipStream_t stream);
hipError_t launch_qtilde(const AttendParams& p, int dtype, bool qt_f32, hipStream_t stream);
hipError_t launch_attend_generic(const AttendParams& p, int dtype, hipStream_t stream);
hipError_t launch_combine(const AttendParams& p, int dtype, hipStream_t stream);
size_t attend_generic_lds_bytes(const GroupDesc& g);

// MFMA encoder (16-bit dtypes, widths that are multiples of 32).
bool encode_mfma_supported(const EncodeParams& p, int dtype);
hipError_t launch_encode_mfma(const EncodeParams& p, int dtype, hipStream_t stream);
bool encode_bulk_supported(const EncodeParams& p, int dtype);
hipError_t launch_encode_bulk(const EncodeParams& p, int dtype, int n_cu, hipStream_t stream);

// MFMA encoder for two-layer encoders (32-token waves, hidden activations kept in registers).
bool encode_mlp_mfma_supported(const EncodeParams& p, int dtype);
hipError_t launch_encode_mlp_mfma(const EncodeParams& p, int dtype, hipStream_t stream);

// MFMA versions of the absorbed-query prologue and the merge + output epilogue.
bool proj_mfma_supported(const AttendParams& p, int dtype);
hipError_t launch_qtilde_mfma(const AttendParams& p, int dtype, hipStream_t stream);
hipError_t launch_combine_mfma(const AttendParams& p, int dtype, hipStream_t stream);
void qtilde_mfma_grid(const AttendParams& p, int& qx, int& qy, int& qz);
// The decode-step encoder (linear, rows in the model dtype) and the absorbed-query projection in one launch.
bool encode_step_qtilde_supported(const EncodeParams& p, int dtype);
hipError_t launch_encode_step_qtilde(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, int dtype, hipStream_t stream);
// The same for the few-token form of the two-layer encoder.
bool encode_mlp_step_qtilde_supported(const EncodeParams& p, int dtype);
hipError_t launch_encode_mlp_step_qtilde(const EncodeParams& p, const AttendParams& q, int qx, int qy, int qz, int dtype, hipStream_t stream);

// MFMA attention for two-layer decoders (resident first-layer weights).
bool attend_mlp_mfma_supported(const AttendParams& p, int dtype);
hipError_t launch_attend_mlp_mfma(const AttendParams& p, int dtype, hipStream_t stream);

// MFMA path (16-bit dtypes, linear decoders, widths that are multiples of 32).
bool attend_mfma_available();
hipError_t launch_attend_mfma(const AttendParams& p, int dtype, hipStream_t stream);

// MFMA attention over int8 latent rows (linear decoders, equal K / V widths of 32..128).
bool attend_i8_mfma_supported(const AttendParams& p, int dtype);
hipError_t launch_attend_i8_mfma(const AttendParams& p, int dtype, hipStream_t stream);

// Reuse-map selection statistic: per-head mean L1 distance between two [n_tokens, H_kv * d_head] tensors.
int head_l1_workgroups(size_t n_tokens, int n_cu);
hipError_t launch_head_l1(const void* prev, const void* cur, int dtype, size_t n_tokens, int n_kv_heads, int d_head, int accumulate, float* dist,
                          float* partial, int n_wg, hipStream_t stream);

// ---- prefill attention: decode every needed row once, then causal attention over the decoded rows ----------
constexpr int kMaxReconHeads = 16;     // KV heads per entry
constexpr int kMaxReconEntries = 8;    // entries per launch

// One source (layer, K or V) whose cached rows are decoded, with the KV heads of the attending layer that take it.
struct ReconEntry {
    SideDesc d;
    int which;                    // KVCAR_K / KVCAR_V: which of the two decoded tensors the heads go to
    int n_heads;
    short head[kMaxReconHeads];   // KV head index in the attending layer
    short col[kMaxReconHeads];    // first column of that head in d.wl
};

struct ReconParams {
    ReconEntry e[kMaxReconEntries];
    int n_entries;
    void* khat;                   // decoded keys   [batch, H_kv, n_rows, d_head]
    void* vhat;                   // decoded values [batch, H_kv, n_rows, d_head]
    int batch, n_rows, max_seq, n_kv_heads, d_head;
    float k_scale;                // softmax scale * log2(e), multiplied into the decoded keys before their one rounding
    int staged;                   // set by the MFMA launcher: rows leave through an LDS staging area as 16-byte chunks
};

struct PrefillParams {
    const void* q;                // [batch, t_new, H_q, d_head]
    void* out;                    // [batch, t_new, H_q, d_head]
    const void* khat;             // decoded keys, already multiplied by softmax scale * log2(e): scores come out in log2 units
    const void* vhat;
    int batch, t_new, pos0, n_rows;
    int n_q_heads, n_kv_heads, d_head;
};

hipError_t launch_recon_generic(const ReconParams& p, int dtype, hipStream_t stream);
hipError_t launch_prefill_generic(const PrefillParams& p, int dtype, hipStream_t stream);
// MFMA versions (16-bit dtypes): decoded rows for linear decoders with latent widths that are multiples of 32;
// causal attention for d_head = 64 or 128.
bool recon_mfma_supported(const ReconParams& p, int dtype);
hipError_t launch_recon_mfma(const ReconParams& p, int dtype, hipStream_t stream);
bool prefill_mfma_supported(const PrefillParams& p, int dtype);
hipError_t launch_prefill_mfma(const PrefillParams& p, int dtype, int n_cu, hipStream_t stream);

hipError_t launch_stream_read(const void* src, size_t bytes, int n_blocks, int block, unsigned* sink, hipStream_t stream);

}  // namespace kvcar
