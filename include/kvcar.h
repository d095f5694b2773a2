/*
 * kvcar.h - C ABI of libkvcar: the decode-time hot path of KV-CAR on one MI355X (gfx950).
 *
 * KV-CAR (arxiv 2512.06727) stores, per transformer layer, an autoencoder *latent* of every
 * token's key vector and value vector instead of the vectors themselves, and lets selected heads
 * of a layer take the previous layer's keys/values instead of storing their own.  This library
 * implements the two operations a decode step needs per layer:
 *
 *   kvcar_encode_append     encoder after K/V generation + append of one latent row per token to
 *                           the layer's latent KV cache   (Methodology, "Network Architecture",
 *                           first paragraph)
 *   kvcar_decode_attention  decoder applied to every cached latent row at retrieval, followed by
 *                           scaled-dot-product attention per head   ("Network Architecture",
 *                           second paragraph; Background, Eq. 1), with inter-layer head reuse
 *                           ("Network Architecture", third paragraph) resolved while addressing
 *   kvcar_set_reuse_map     the per-layer boolean map of reused K heads and V heads
 * and, for the prompt, kvcar_prefill_attention (causal attention of a chunk over the same caches).
 *
 * Conventions
 *   - Pure C.  Every function returns a kvcar_status (0 = OK, negative = error); nothing throws
 *     (a failed host allocation inside the library comes back as KVCAR_ERR_NOMEM).
 *   - "dev" pointers are device (HBM) addresses owned by the caller (e.g. PyTorch tensors); they
 *     must be 16-byte aligned and stay valid until the work enqueued on `stream` has finished.
 *     "host" pointers are read during the call and not retained.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  No call
 *     synchronises the device or allocates device memory; kernels are only enqueued.
 *   - Elements (activations, weights, cache, output) share one dtype; accumulation is fp32.
 *   - Weight matrices are row-major [in_features, out_features]; biases may be NULL.
 *   - The library owns only its host-side context.  The context holds no sequence positions:
 *     positions are explicit arguments, so calls can be replayed.
 *   - kvcar_encode_append / kvcar_decode_attention treat all sequences of a batch alike (same position, same
 *     context length); kvcar_encode_append_at / kvcar_decode_attention_ex take per-sequence positions and lengths.
 *   - Layers are 0-indexed.  KVCAR_K = keys, KVCAR_V = values.
 *
 * Latent cache layout (library-defined, caller-allocated): for layer N and tensor `which`
 *   Z[b][t][c],  b < max_batch, t < max_seq, c < r   row-major, r = latent_width of that
 *   layer-tensor; one row is r * sizeof(dtype) bytes; kvcar_cache_bytes gives the total.
 *
 * int8 latents (kvcar_config.latent_format = KVCAR_LATENT_INT8; Methodology, "Quantization",
 * Eq. "quant"): kvcar_encode_append quantises every latent row after the encoder,
 *   scale = 255 / (max(x) - min(x)),  zeropoint = -round(scale * min(x)) - 128,
 *   code  = round(scale * x + zeropoint)   saturated to [-128, 127],
 * over the r elements x of the row (fp32 encoder output, round = half to even, every operation
 * one fp32 operation; a row of equal values uses |x| as its range, or 1 if x = 0), and
 * kvcar_decode_attention dequantises, x^ = (code - zeropoint) / scale, before the decoder.
 * The cache of (layer, which) is then one buffer holding
 *   codes  int8  Z8[b][t][c]            at byte offset 0, followed at the next multiple of 256 by
 *   meta   M[b][t] = { float scale; int32 zeropoint; }   8 bytes per row;
 * r must be a multiple of 16.  Activations, weights and outputs keep the configured dtype.
 * The matrix-core attention kernel for int8 rows feeds codes, 1/scale and the zero point to fp16
 * operands: it expects |zeropoint| < 2^23 and max(x) - min(x) < 6e4 in every row (far outside what
 * latent activations reach; a row of nearly equal values 1e5 times larger than their spread would
 * violate the first).  Beyond these limits it saturates the operands: its result stays finite but is
 * no longer the method's.  A caller whose latents can look like that sets kvcar_tuning.force_generic:
 * the plain-ALU kernels take a key row's zero point out of the scores in fp64 and dequantise value
 * rows in fp32, which is exact for |zeropoint| <= 2^24.
 */
#ifndef KVCAR_H
#define KVCAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvcar_ctx kvcar_ctx;

typedef enum {
    KVCAR_OK = 0,
    KVCAR_ERR_ARG = -1,          /* null / misaligned pointer, index out of range          */
    KVCAR_ERR_SHAPE = -2,        /* widths inconsistent with the model or the reuse map    */
    KVCAR_ERR_CAPACITY = -3,     /* batch, position or context beyond max_batch / max_seq  */
    KVCAR_ERR_REUSE = -4,        /* layer 0 asked to reuse; source layer lacks the head    */
    KVCAR_ERR_UNSUPPORTED = -5,  /* no kernel for this dtype / width combination           */
    KVCAR_ERR_STATE = -6,        /* autoencoder or cache of a needed layer not set / bound */
    KVCAR_ERR_HIP = -7,          /* a HIP runtime call failed                               */
    KVCAR_ERR_WORKSPACE = -8,    /* workspace too small                                     */
    KVCAR_ERR_NOMEM = -9         /* a host allocation inside the library failed             */
} kvcar_status;

typedef enum { KVCAR_F32 = 0, KVCAR_F16 = 1, KVCAR_BF16 = 2 } kvcar_dtype;

/* How latent rows are held in the cache: in the model dtype, or as int8 codes with a scale and
 * a zero point per row ("Quantization", Eq. "quant"). */
typedef enum { KVCAR_LATENT_DTYPE = 0, KVCAR_LATENT_INT8 = 1 } kvcar_latent_format;

/* Activation between the two fully connected layers of an encoder / decoder.  NONE = the
 * autoencoder is a single linear map each way. */
typedef enum { KVCAR_ACT_NONE = 0, KVCAR_ACT_LEAKY_RELU = 1, KVCAR_ACT_GELU = 2 } kvcar_act;
/* GELU is x Phi(x) with the normal distribution function Phi (the erf form, not the tanh form).  Encoders and
 * the plain-ALU kernels evaluate erf to 1.5e-7; the matrix-core kernels that rebuild hidden rows of a two-layer
 * decoder (decode and prefill attention) use a polynomial for Phi with |GELU error| <= 3.1e-5 |x|, below the
 * 16-bit rounding those hidden rows receive next. */

enum { KVCAR_K = 0, KVCAR_V = 1 };

/* Model shape.  D_kv = n_kv_heads * d_head is the width of one token's key (or value) vector. */
typedef struct {
    int n_layers;
    int n_q_heads;      /* H_q; must be a multiple of n_kv_heads (grouped-query attention)   */
    int n_kv_heads;     /* H_kv                                                               */
    int d_head;
    int max_batch;
    int max_seq;        /* capacity of every latent cache, in tokens                          */
    int dtype;          /* kvcar_dtype                                                        */
    float softmax_scale; /* 0 => 1/sqrt(d_head), the scaling of Eq. 1                         */
    int latent_format;  /* kvcar_latent_format; 0 = rows in `dtype`                           */
} kvcar_config;

/*
 * Autoencoder of one layer for K or for V ("Network Architecture": encoder D -> d placed after
 * K/V generation, mirrored decoder d -> D applied at retrieval; two fully connected layers with
 * an activation in between, or a single linear map when hidden_width == 0.  A batch-norm between
 * the layers is folded into w1/b1 by the caller).
 *
 *   in_width      width of the encoder input / decoder output.  Either D_kv (the autoencoder
 *                 covers every head; columns of reused heads are ignored on decode), or
 *                 n_stored * d_head where the stored heads are the layer's non-reused heads in
 *                 increasing order (the autoencoder covers only what the layer stores).
 *   latent_width  r, the row width of this layer-tensor's cache.  0 is allowed only when
 *                 in_width == 0 (a layer that stores nothing for this tensor).
 *   enc_w1 [in_width, hidden or latent], enc_b1; enc_w2 [hidden, latent], enc_b2 (hidden > 0)
 *   dec_w1 [latent, hidden or in_width], dec_b1; dec_w2 [hidden, in_width], dec_b2 (hidden > 0)
 *   All weight pointers are dev pointers that must outlive every call using the context.
 *
 *   per_head      0: one autoencoder over the whole vector, as in the paper (every head's keys depend on the
 *                 whole latent row).  1: a block-diagonal autoencoder, one d_head -> r_h -> d_head pair per
 *                 covered head, r_h = latent_width / n_covered (an extension: the paper's autoencoder is dense).
 *                 A head that reuses an earlier layer's keys or values then reads only that head's latent
 *                 rows of the source layer.  Linear autoencoders and latent rows in `dtype` only; r_h rows must
 *                 be a multiple of 16 bytes.  Layouts, with i the position of the head among the covered heads:
 *                   enc_w1 [n_covered][d_head][r_h], enc_b1 [n_covered][r_h]
 *                   dec_w1 [n_covered][r_h][d_head], dec_b1 [n_covered][d_head]
 *                 and the cache of this layer-tensor is head-major, Z[i][b][t][r_h] (b < max_batch,
 *                 t < max_seq): a head's rows of one sequence are contiguous.  kvcar_cache_bytes is unchanged.
 */
typedef struct {
    int in_width;
    int hidden_width;
    int latent_width;
    int act;            /* kvcar_act; must be NONE iff hidden_width == 0 */
    float leaky_slope;
    const void *enc_w1, *enc_b1, *enc_w2, *enc_b2;
    const void *dec_w1, *dec_b1, *dec_w2, *dec_b2;
    int per_head;       /* 0 or 1, see above */
} kvcar_ae_desc;

/* Launch tuning; all zero = library defaults. */
typedef struct {
    int n_splits;       /* token-range splits per sequence in decode_attention; 0 = automatic */
    int force_generic;  /* 1 = use the plain-ALU kernels even where an MFMA kernel exists     */
    int tile_order;     /* MFMA attention: 0 = library default, 1 = each split owns a contiguous
                           token range, 2 = 128-token tiles dealt round-robin over the splits    */
    int no_fuse;        /* 1 = always run prologue / attention / epilogue as separate kernels     */
    int wg_waves;       /* one-launch attention kernels (one split, or several with the last workgroup merging):
                           0 = automatic (eight waves per workgroup when the launch has no more workgroups
                           than compute units, else four), 4 or 8                                    */
    int no_bulk_encode; /* 1 = prompt-sized encode calls take the general encoder kernel, not the
                           streaming one (linear encoders, 8192 tokens or more)                      */
    int no_arrive;      /* 1 = with several splits the partials always go to a separate merge kernel; default: where the
                           shapes allow, one launch whose last workgroup per (sequence, group) merges and decodes */
    int no_colocate;    /* 1 = workgroups take (split, sequence, group) in launch order even where groups of the launch
                           read the same rows; default: such launches, if they read no more than about 320 MB, place the
                           groups of a (split, sequence) on one XCD, whose L2 then serves the repeated reads */
    int group_slots;    /* matrix-core attention over rows up to 128 wide: most query heads one workgroup serves: 8, 16 or
                           32; 0 = automatic (launches that would then still read no more than about 320 MB - bound by latency, not
                           by bandwidth - give every KV head a group of its own where that keeps the layer one launch: less
                           prologue, partial and epilogue per workgroup, at the price of reading a source's rows once per
                           group; larger launches keep up to 32 heads per workgroup) */
} kvcar_tuning;

/* Create / destroy a context.  ERR_ARG on null pointers, ERR_SHAPE on non-positive sizes or
 * n_q_heads % n_kv_heads != 0, ERR_UNSUPPORTED on an unknown dtype or latent format, more than 64 KV heads,
 * n_q_heads > 32767 or n_kv_heads * d_head > 32767. */
int kvcar_create(const kvcar_config *cfg, kvcar_ctx **out);
int kvcar_destroy(kvcar_ctx *ctx);

/*
 * Inter-layer head reuse ("Network Architecture", third paragraph): k_reuse[g] != 0 means KV head g
 * of `layer` takes the keys of head g of the previous layer instead of storing its own; v_reuse
 * likewise for values.  Both are host arrays of n_kv_heads bytes.  "The previous layer's" tensor
 * is whatever that layer itself uses, so chains resolve to the nearest earlier layer whose bit is
 * clear.  Layer 0 cannot reuse: ERR_REUSE.  Changing a layer's map invalidates the autoencoders
 * set for that layer (set them again).  Default: nothing reused.
 */
int kvcar_set_reuse_map(kvcar_ctx *ctx, int layer, const uint8_t *k_reuse, const uint8_t *v_reuse);

/* Layer that supplies head `kv_head` of `layer` for tensor `which` under the current maps. */
int kvcar_resolve_source(const kvcar_ctx *ctx, int layer, int which, int kv_head, int *src_layer);

/* Set the autoencoder of (layer, which).  ERR_SHAPE if in_width matches neither form above or
 * widths are inconsistent (per_head: latent_width not a multiple of the covered heads); ERR_ARG on null /
 * misaligned required pointers or per_head outside {0, 1}; ERR_UNSUPPORTED for per_head with a hidden layer,
 * with int8 latents, or with head rows that are not a multiple of 16 bytes. */
int kvcar_set_autoencoder(kvcar_ctx *ctx, int layer, int which, const kvcar_ae_desc *desc);

/* Bytes of the latent cache of (layer, which): max_batch * max_seq * latent_width * sizeof(dtype)
 * (Eq. 3 with d_model replaced by what the layer-tensor stores); with int8 latents the codes
 * (one byte per element, padded to a multiple of 256 bytes) plus 8 bytes of scale and zero point
 * per row.  Needs the autoencoder set. */
int kvcar_cache_bytes(const kvcar_ctx *ctx, int layer, int which, size_t *bytes);

/* Bind caller-allocated device memory as the cache of (layer, which).  ERR_CAPACITY if `bytes`
 * is smaller than kvcar_cache_bytes.  A zero-width cache needs no binding. */
int kvcar_bind_cache(kvcar_ctx *ctx, int layer, int which, void *dev, size_t bytes);

int kvcar_set_tuning(kvcar_ctx *ctx, const kvcar_tuning *tuning);

/* Workspace (device bytes) that kvcar_decode_attention needs for `batch` sequences of `n_ctx`
 * cached tokens, maximised over layers under the current maps, autoencoders and tuning.  The launch plan (splits per
 * sequence, query heads per workgroup) follows the sizes of the call, so the need is not monotonic in batch or n_ctx:
 * ask for the sizes of the call, or take the largest answer over the sizes to come; a workspace that is too small is
 * refused with KVCAR_ERR_WORKSPACE before anything is enqueued. */
int kvcar_workspace_bytes(const kvcar_ctx *ctx, int batch, int n_ctx, size_t *bytes);

/*
 * Encode the new tokens' key and value vectors and append the latent rows to the layer's caches.
 *   k_new, v_new  dev [batch, t_new, D_kv] row-major (full-width vectors; only the columns the
 *                 layer's autoencoder covers are read)
 *   rows are written at positions [pos0, pos0 + t_new) of sequences 0..batch-1, rounded once
 *   (nearest-even) from the fp32 result to the cache dtype.  Other rows are not touched.
 * ERR_CAPACITY if batch > max_batch or pos0 + t_new > max_seq; ERR_STATE if an autoencoder or a
 * non-empty cache of this layer is not set / bound.
 */
int kvcar_encode_append(kvcar_ctx *ctx, int layer, const void *k_new, const void *v_new,
                        int batch, int pos0, int t_new, void *stream);

/*
 * One decode step of attention for `layer` over cached tokens 0..n_ctx-1 of every sequence:
 * for each query head j (KV head g = j / (H_q/H_kv)), K^_g[t] and V^_g[t] are the decoder outputs
 * of the latent rows of the layer that supplies head g (reuse map), and
 *   out[b, j, :] = sum_t softmax_t(scale * q[b,j,:] . K^_g[t]) V^_g[t]            (Eq. 1)
 *   q    dev [batch, H_q, d_head]      out  dev [batch, H_q, d_head] (rounded once to dtype)
 * The decoded K^/V^ are never written to memory; with a linear last decoder layer that layer is
 * applied to the query and to the weighted latent sum instead of to every row (same result up to
 * rounding order).  `workspace` is dev scratch of at least kvcar_workspace_bytes(batch, n_ctx).
 * ERR_CAPACITY if batch > max_batch or n_ctx > max_seq or n_ctx < 1; ERR_STATE if a source
 * layer's autoencoder / cache is missing; ERR_REUSE if a source layer's autoencoder does not
 * cover a head taken from it; ERR_WORKSPACE if workspace_bytes is too small.
 */
int kvcar_decode_attention(kvcar_ctx *ctx, int layer, const void *q, void *out,
                           int batch, int n_ctx, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Extensions of a decode step.  All pointers may be NULL (then the call equals the plain one).
 *   seq_lens  dev int32 [batch]: per-sequence context length (ragged batch); sequence b attends over
 *             its first min(seq_lens[b], n_ctx) cached rows.  n_ctx stays the upper bound the launch
 *             is sized for.  A length of 0 is allowed only together with k_cur / v_cur.
 *   k_cur, v_cur  dev [batch, H_kv * d_head] in the model dtype, both or neither: the paper's form of
 *             the step ("Network Architecture", 2nd paragraph): the decoded rows of the cached tokens
 *             are concatenated with the current token's exact key and value vectors, so attention
 *             runs over the cached rows plus this one row, which never passed the autoencoder.
 *             Column block g holds the vector KV head g of this layer uses (for a reused head: the
 *             source layer's).  With these, n_ctx = 0 (nothing cached yet) is accepted.
 */
typedef struct {
    const int32_t *seq_lens;
    const void *k_cur;
    const void *v_cur;
} kvcar_step_ext;

/* kvcar_decode_attention with the extensions above.  Same arguments, errors and workspace; ERR_ARG
 * if only one of k_cur / v_cur is given or a pointer is misaligned. */
int kvcar_decode_attention_ex(kvcar_ctx *ctx, int layer, const void *q, void *out, int batch, int n_ctx,
                              const kvcar_step_ext *ext, void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvcar_decode_attention for callers that cannot allocate device memory and have no workspace to pass: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result
 * and errors as kvcar_decode_attention, without the workspace: the scratch memory of the call (absorbed queries
 * and split partials) is a static device buffer of KVCAR_STATIC_SCRATCH_BYTES bytes inside the library, which
 * every GPU the library runs on holds until the process ends.  The call allocates nothing on the device, creates
 * no events (kvcar_profile_enable is ignored by it) and, like the other calls, does not synchronise.
 * KVCAR_ERR_WORKSPACE if the call needs more scratch memory than the buffer holds
 * (kvcar_workspace_bytes(batch, n_ctx) tells how much; the long-context single-split form needs none),
 * KVCAR_ERR_HIP if the buffer's address cannot be obtained.  The buffer's address on a device is looked up once,
 * in kvcar_create on that device or else in the first such call there.  All such calls on one GPU share the one
 * buffer, whatever their context or stream: calls that may overlap on a GPU (different streams, no ordering
 * between them) race on it and give wrong results; calls on one stream are safe.  Nothing in it needs to start
 * from zero: every call writes what it later reads.
 */
#define KVCAR_STATIC_SCRATCH_BYTES (32u << 20)
int kvcar_decode_attention_static(kvcar_ctx *ctx, int layer, const void *q, void *out, int batch, int n_ctx,
                                  void *stream);

/*
 * One decode step of a layer in one call: kvcar_encode_append(layer, k_new, v_new, batch, pos, 1) followed by
 * kvcar_decode_attention(layer, q, out, batch, pos + 1, ..) - the encoder after K/V generation, the append, and
 * attention over the cache including the row just appended ("Network Architecture", 1st and 2nd paragraphs; Eq. 1).
 *   k_new, v_new  dev [batch, D_kv]: the new token's key and value vectors of every sequence
 *   pos           position the rows are written at; attention then runs over rows 0 .. pos
 * Where the launch planned for the attention can take the encoder in (matrix-core kernels over rows in the model
 * dtype or int8 codes, linear encoders with in_width <= 256 and latent_width <= 128 - per head with per_head
 * autoencoders -, at most 16 KV heads, tuning without no_fuse / tile_order 2) the whole step of the layer is ONE kernel:
 * the workgroup that reaches the end of a sequence's context encodes that sequence's new rows (and quantises them, with
 * int8 latents), writes them to the caches and attends to them; otherwise the call enqueues what the two separate calls
 * would - except that the encoder of a few tokens and the projection of the absorbed queries, two small independent
 * launches, become one where both have their matrix-core forms (GPT-2-shaped and two-layer configurations).  Results equal those of the two calls up to the order of the encoder's fp32 sums (the row written may differ in
 * the last place of the cache dtype - by one in an int8 code - on a small fraction of elements).
 * Arguments, workspace (kvcar_workspace_bytes(batch, pos + 1)) and errors as for the two calls.
 */
int kvcar_append_attend(kvcar_ctx *ctx, int layer, const void *k_new, const void *v_new, const void *q, void *out,
                        int batch, int pos, void *workspace, size_t workspace_bytes, void *stream);

/* kvcar_encode_append for a ragged batch: sequence b's t_new rows land at positions
 * [positions[b], positions[b] + t_new) (positions: dev int32 [batch]).  The caller guarantees
 * positions[b] + t_new <= max_seq (device data is not checked). */
int kvcar_encode_append_at(kvcar_ctx *ctx, int layer, const void *k_new, const void *v_new, int batch,
                           const int32_t *positions, int t_new, void *stream);

/*
 * Prefill attention over the latent cache (Introduction: in the prefill phase the whole prompt is
 * processed and the keys and values of all its tokens go to the KV cache - here as latent rows;
 * "Network Architecture", 2nd paragraph: the decoder rebuilds them on retrieval; Eq. 1 per token, each
 * token attending to the rows up to and including its own).  For a chunk of t_new query tokens per
 * sequence, token i sitting at position pos0 + i, whose latent rows - like those of all earlier
 * positions - are already in the caches (kvcar_encode_append):
 *   out[b, i, j, :] = sum_{t <= pos0 + i} softmax_t(scale * q[b,i,j,:] . K^_g[t]) V^_g[t],   g = j / (H_q/H_kv)
 *   q    dev [batch, t_new, H_q, d_head]      out  dev [batch, t_new, H_q, d_head] (rounded once to dtype)
 * K^_g / V^_g as in kvcar_decode_attention (source layer by the reuse map).  This equals t_new decode
 * steps with n_ctx = pos0 + i + 1 up to rounding.  Unlike a decode step, a prompt chunk is bound by the
 * matrix units, not by reading the cache, so the decoder is not folded into the query (that would double
 * the products per score): the rows 0 .. pos0 + t_new - 1 of every KV head are decoded ONCE per call into
 * `workspace` and a causal attention kernel runs over them.  The decoded rows are an internal
 * approximation, not a step of the method: they are held in fp16 for both 16-bit model dtypes (11-bit
 * significands; bf16's 8 bits would put the rounding of every key into every prompt score), in fp32 for
 * fp32 models, the keys carrying the softmax scale into that one rounding.  fp16's range applies: |q|,
 * |scale * log2(e) * K^| and |V^| beyond 65504 saturate.  Nothing outlives the call: the workspace may be reused at once by
 * the next layer.  kvcar_prefill_workspace_bytes(batch, n_rows) gives its size for n_rows = pos0 + t_new
 * (2 * batch * n_rows * H_kv * d_head elements).
 * ERR_CAPACITY if batch > max_batch or pos0 + t_new > max_seq; ERR_ARG if t_new < 1, pos0 < 0 or a
 * pointer is null / misaligned; ERR_STATE / ERR_REUSE as for a decode step; ERR_WORKSPACE;
 * ERR_UNSUPPORTED if d_head > 256.
 */
int kvcar_prefill_workspace_bytes(const kvcar_ctx *ctx, int batch, int n_rows, size_t *bytes);
int kvcar_prefill_attention(kvcar_ctx *ctx, int layer, const void *q, void *out, int batch, int pos0, int t_new,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * What kvcar_decode_attention would launch for (layer, batch, n_ctx) under the current maps,
 * autoencoders and tuning.  A "group" is the set of query heads of the layer that read the same
 * (K source layer, V source layer) - with per_head autoencoders, the query heads of one KV head; each
 * distinct source's latent rows are streamed once per group.
 */
typedef struct {
    int uses_mfma;          /* 1 = MFMA kernels, 0 = plain-ALU kernels                          */
    int n_groups;
    int n_splits;           /* token-range splits per sequence                                  */
    int n_launches;         /* attention-kernel launches (groups are batched 8 per launch)      */
    int fused;              /* 1 = one split and prologue and epilogue run inside the attention kernel; 2 = several
                               splits in one launch: the last workgroup of a (sequence, group) merges and decodes
                               (its arrival counters lie in the workspace and need no initial state);
                               0 = separate kernels                                             */
    size_t workspace_bytes;
    size_t latent_bytes;    /* bytes of latent rows the attention kernel reads for this call    */
    int append_in_kernel;   /* 1 = kvcar_append_attend at this size encodes the new token inside the
                               attention kernel (one launch for the layer's whole step)         */
} kvcar_plan_info;
int kvcar_describe_plan(const kvcar_ctx *ctx, int layer, int batch, int n_ctx, kvcar_plan_info *out);

/*
 * Which encoder kernel kvcar_encode_append(layer, batch, .., t_new) would take with the current
 * autoencoders and tuning (host-only, nothing is launched; caches need not be bound).  ERR_ARG / ERR_CAPACITY
 * / ERR_STATE as for the call itself.
 */
enum {
    KVCAR_ENC_NONE = 0,            /* the layer stores nothing: no launch                                   */
    KVCAR_ENC_PLAIN = 1,           /* plain-ALU kernel (fp32 models, shapes without an MFMA kernel)          */
    KVCAR_ENC_MFMA = 2,            /* general MFMA kernel (linear, or two layers of any covered shape)       */
    KVCAR_ENC_MFMA_TWO_LAYER = 3,  /* two-layer encoder of one of the exact shapes with resident token rows  */
    KVCAR_ENC_MFMA_STREAM = 4      /* streaming kernel for prompt-sized calls through a linear encoder       */
};
int kvcar_describe_encode(const kvcar_ctx *ctx, int layer, int batch, int t_new, int *kernel);

/*
 * Optional timing of the attention kernel (the kernel that streams the latent cache; for
 * kvcar_prefill_attention the causal attention kernel).  While enabled, kvcar_decode_attention and
 * kvcar_prefill_attention record a HIP event before and after that kernel on the caller's stream.
 * kvcar_profile_read waits for the recorded events (this is the only call that blocks on
 * the device), returns the summed kernel time in milliseconds and the number of launches since the
 * last reset, and resets the counters.
 */
int kvcar_profile_enable(kvcar_ctx *ctx, int enable);
int kvcar_profile_read(kvcar_ctx *ctx, double *attend_ms, long *n_launches);

/*
 * Reuse-map selection statistic (Algorithm 2, steps 1-2; Methodology, the paragraph on key and value
 * reuse: the L1 norm between heads of adjacent layers, averaged over mini-batches, is what the reuse
 * threshold is applied to).  For two dev tensors [n_tokens, n_kv_heads * d_head] in `dtype` (the keys,
 * or the values, of layer N-1 and of layer N for the same tokens):
 *   dist[g] = mean over tokens t and components k < d_head of | x_cur[t, g, k] - x_prev[t, g, k] |
 * written to dist (dev fp32 [n_kv_heads]); with accumulate != 0 the result is added to what dist holds,
 * so that a caller sums mini-batches and divides by their number.  Choosing the threshold and filling
 * kvcar_set_reuse_map stay with the caller.  The result does not depend on scheduling (fixed reduction
 * order).  workspace: dev, 16-byte aligned, kvcar_head_l1_workspace_bytes bytes.  Stateless: no context.
 * ERR_ARG on null / misaligned pointers or n_tokens == 0, ERR_SHAPE if a row is not a multiple of
 * 16 bytes or d_head is not a multiple of the elements in 16 bytes, ERR_UNSUPPORTED on an unknown
 * dtype or more than 1024 heads, ERR_WORKSPACE, ERR_HIP.
 */
int kvcar_head_l1_workspace_bytes(size_t n_tokens, int n_kv_heads, size_t *bytes);
int kvcar_head_l1_distance(const void *x_prev, const void *x_cur, int dtype, size_t n_tokens, int n_kv_heads,
                           int d_head, int accumulate, float *dist, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Read-only streaming ceiling of the device: a kernel with no arithmetic reads `bytes` bytes of
 * `dev_buf` (device memory, 16-byte aligned, bytes a multiple of 16) `repeats` times with 16-byte
 * non-temporal loads, one grid-stride sweep per repeat, timed with HIP events on `stream`, for a
 * few launch shapes.  Writes the best achieved GB/s (1e9 bytes per second) to *gb_per_s.  This is the bandwidth a kernel
 * that only reads can reach on this GPU: the attention kernel's rate is reported against it as
 * well as against the published peak.  Blocks until the kernels have finished.  The buffer is
 * not modified.  KVCAR_ERR_ARG for null / misaligned arguments, KVCAR_ERR_HIP if a HIP call fails.
 */
int kvcar_probe_read_bandwidth(const void *dev_buf, size_t bytes, int repeats, void *stream, double *gb_per_s);

/* Human-readable name of a status code (static string). */
const char *kvcar_status_string(int status);

/* Text of the last error recorded in this context (valid until the next call on it). */
const char *kvcar_last_error(const kvcar_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* KVCAR_H */
