/*
 * cacheblend.h -- C ABI of the MI355X (gfx950) CacheBlend KV-cache fusor.
 *
 * The library fuses N independently pre-computed per-chunk KV caches into the KV
 * cache of the concatenated input (paper Sec. 4): the cached keys are first moved
 * to their positions in the concatenation (Sec. 4.3 footnote, Appendix A), then,
 * layer by layer, only a small and shrinking set of high-KV-deviation (HKVD)
 * tokens is recomputed (Sec. 4.2, 4.3) while every other token's K/V is reused.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says HOST.
 *   - All buffers are owned by the caller.  The library allocates only the
 *     cb_ctx (a host struct plus one device table of rotary cos/sin values) in
 *     cb_create and releases it in cb_destroy.
 *   - Storage type T = cb_model_desc.dtype (float or bfloat16) for weights, the
 *     layer-0 input x, and the K/V caches.  The residual stream that crosses the
 *     per-layer boundary (h_in / h_out / final_hidden) is always float.
 *   - Weight matrices are row-major [out_features, in_features] (y = x W^T).
 *   - A layer's K cache and V cache are separate arrays [n_tokens, n_kv_heads,
 *     head_dim] of T, token-major; row p holds the token at global position p.
 *   - Alignment: device pointers to tensors (weights, x, caches, h_in / h_out, final_hidden,
 *     logits) must be multiples of 16 bytes, index and deviation arrays of 4 bytes, workspaces of
 *     256 bytes; anything else is refused with CB_EINVAL before any launch.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising the device.  Results are
 *     valid once the caller has synchronised the stream.
 *   - Return value: CB_OK (0) or a negative cb_status.  Arguments are validated
 *     before the first launch, so a failing call leaves every buffer untouched
 *     (CB_EHIP, a launch failure reported by the runtime, is the exception).
 *   - One cb_ctx serves one stream at a time; calls on the same ctx must not
 *     overlap.  Different ctx objects are independent.
 */
#ifndef CACHEBLEND_H
#define CACHEBLEND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CB_OK = 0,
  CB_EINVAL = -1,       /* bad shape / argument */
  CB_ENULL = -2,        /* required pointer is NULL */
  CB_EWORKSPACE = -3,   /* workspace too small */
  CB_EUNSUPPORTED = -4, /* geometry the kernels do not cover */
  CB_EHIP = -5,         /* HIP runtime reported an error */
  CB_ENOMEM = -6        /* allocation of the ctx failed */
} cb_status;

typedef enum { CB_F32 = 0, CB_BF16 = 1 } cb_dtype;

/* Which two channels of a head one 2x2 block of the rotary matrix (Appendix A) acts on:
 * the adjacent pair (2i, 2i+1), as the paper writes it, or (i, i + head_dim/2), the
 * order in which many checkpoints store their query/key projections.  Same matrix,
 * channels renumbered; the caches a caller hands in must be in the same order. */
typedef enum { CB_ROPE_ADJACENT = 0, CB_ROPE_HALF = 1 } cb_rope_layout;

/* How the seven projection matrices of a layer are stored (Sec. 7.1 serves its two larger models
 * with 8-bit weights; the paper names no scheme, this is weight-only symmetric int8):
 *   CB_W_NATIVE  elements of storage type T
 *   CB_W_INT8    int8 elements q with one float scale per OUTPUT feature (row of the [out, in]
 *                matrix): w[o][i] = q[o][i] * scale[o].  Needs dtype == CB_BF16.  Arithmetic stays
 *                bf16 x bf16 -> float on the matrix cores.  A projection whose input width is a multiple
 *                of 64 reads the bytes itself: they travel as bytes through HBM, L2 and LDS, are expanded
 *                to bf16 in registers (exact: |q| <= 128) and the float sums are multiplied by scale[o].
 *                Any other input width: the matrix is expanded to bf16(q * scale) into the workspace right
 *                before its projection runs.  Either way HBM holds one byte per weight.
 * Norm gains, the final norm and the vocabulary matrix of cb_first_token are always of type T. */
typedef enum { CB_W_NATIVE = 0, CB_W_INT8 = 1 } cb_weight_format;

/* Decoder geometry (RMSNorm, grouped-query attention, rotary embedding as in
 * Appendix A, SwiGLU MLP, no biases). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff;
  float rms_eps, rope_theta;
  int32_t dtype;         /* cb_dtype */
  int32_t rope_layout;   /* cb_rope_layout */
  int32_t weight_format; /* cb_weight_format */
} cb_model_desc;

/* One layer's weights: norm gains of storage type T; matrices of T, or int8 with the scale arrays
 * below when weight_format == CB_W_INT8 (the scale pointers are ignored otherwise). */
typedef struct {
  const void *attn_norm;      /* [d_model] */
  const void *wq, *wk, *wv;   /* [Hq*dh, d], [Hkv*dh, d], [Hkv*dh, d] */
  const void *wo;             /* [d, Hq*dh] */
  const void *mlp_norm;       /* [d_model] */
  const void *w_gate, *w_up;  /* [d_ff, d] */
  const void *w_down;         /* [d, d_ff] */
  /* CB_W_INT8: float scale per output feature of the matrix of the same name */
  const float *wq_scale, *wk_scale, *wv_scale;   /* [Hq*dh], [Hkv*dh], [Hkv*dh] */
  const float *wo_scale;                         /* [d] */
  const float *w_gate_scale, *w_up_scale;        /* [d_ff] */
  const float *w_down_scale;                     /* [d] */
} cb_layer_weights;

typedef struct cb_ctx cb_ctx;

/* Creates a context for one model geometry; positions 0 .. max_tokens-1 are
 * covered by the rotary table.  desc and out are HOST pointers. */
int cb_create(const cb_model_desc *desc, int32_t max_tokens, cb_ctx **out);
void cb_destroy(cb_ctx *ctx);
const char *cb_strerror(int status);

/* Bytes of workspace cb_fuse_layer needs for calls with n_rows <= max_rows. */
size_t cb_layer_workspace_bytes(const cb_ctx *ctx, int32_t max_rows);
/* Bytes of workspace cb_fuse_prefill needs for n_tokens = context + suffix. */
size_t cb_prefill_workspace_bytes(const cb_ctx *ctx, int32_t n_tokens);

/* Gradual-filtering schedule (Sec. 4.3): keep_counts[0] = n_ctx; for l >= 1 the
 * kept fraction falls from r1 on layer 1 to (3r - r1)/2 on the last layer along
 * (1-t)^2, so it averages r; counts are ceil(fraction * n_ctx), non-increasing.
 * r1 <= 0 selects r1 = 2r; flat != 0 gives ceil(r * n_ctx) on every layer >= 1.
 * keep_counts: HOST int32[n_layers]. */
int cb_default_schedule(int32_t n_layers, int32_t n_ctx, double r, double r1, int32_t flat,
                        int32_t *keep_counts);

/* Positional recovery of cached keys (Sec. 4.3 footnote; Appendix A).
 * Chunk c was prefilled at positions 0.., so its cached keys carry R(t); this
 * multiplies rows [o_c, o_{c+1}) of every given layer's K cache by R(o_c), in
 * place.  Chunk 0 and all V caches are not touched.
 *   k_cache_layers : HOST array [n_layers] of device base pointers (T [*, Hkv, dh])
 *   layer_begin/end: half-open layer range to process
 *   chunk_offsets  : HOST int32[n_chunks + 1], o_0 = 0 < o_1 < ... <= max_tokens */
int cb_realign_rope(cb_ctx *ctx, void *const *k_cache_layers, int32_t layer_begin,
                    int32_t layer_end, const int32_t *chunk_offsets, int32_t n_chunks,
                    void *stream);

/* One layer of selective recompute (Sec. 4.2 workflow; Sec. 6 prefill_layer with
 * its check_flag / HKVD_indices).
 *   h_in    : float [n_rows, d]   this layer's input for the rows that survived
 *   row_pos : int32 [n_rows]      their global positions, strictly ascending;
 *                                 the LAST n_suffix rows are the suffix (never
 *                                 candidates, always kept)
 *   k_cache, v_cache : T [n_tokens_total, Hkv, dh]; in: re-aligned pre-computed
 *                      rows (rows of the suffix may hold anything); out: rows of
 *                      the kept tokens overwritten with their new K/V, all other
 *                      rows unchanged
 *   k_keep  : number of context rows to keep, 0 <= k_keep <= n_rows - n_suffix.
 *             k_keep == n_rows - n_suffix without forced_sel means "no check":
 *             the deviation and top-k steps are skipped.
 *   forced_sel : NULL, or int32 [k_keep] strictly ascending positions taken from
 *             row_pos's context part, kept instead of the top-k (the deviation is
 *             still computed).  Positions that are not candidates give undefined
 *             selections but no out-of-bounds access.
 *   h_out   : float [k_keep + n_suffix, d]   next layer's input
 *   pos_out : int32 [k_keep + n_suffix]      positions of those rows, ascending
 *   dev_out : NULL, or float [n_rows - n_suffix]: squared L2 deviation of each
 *             candidate's new K/V from its cached K/V, in row order (written only
 *             when the check runs)
 * Kept = the k_keep candidates with the largest deviation, equal values going
 * to the lower position.  h_out/pos_out must not alias h_in/row_pos. */
int cb_fuse_layer(cb_ctx *ctx, int32_t layer, const cb_layer_weights *weights /*HOST*/,
                  const float *h_in, const int32_t *row_pos, int32_t n_rows, int32_t n_suffix,
                  void *k_cache, void *v_cache, int32_t n_tokens_total, int32_t k_keep,
                  const int32_t *forced_sel, float *h_out, int32_t *pos_out, float *dev_out,
                  void *workspace, size_t workspace_bytes, void *stream);

/* cb_fuse_layer for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, results and validation, minus the
 * workspace -- the layer's intermediates live in an array of CB_STATIC_SCRATCH_BYTES built into the
 * library (one copy per GPU, held until the process ends).  The call allocates nothing on the device or
 * through the HIP runtime.  A call whose cb_layer_workspace_bytes(ctx, n_rows) exceeds CB_STATIC_SCRATCH_BYTES is
 * refused with CB_EWORKSPACE before any launch; the ctx must have been created on the device that is
 * current (else CB_EINVAL).  Every call on a GPU shares that GPU's array: calls that overlap in time on
 * one GPU (two streams, two ctx objects, two threads) race on it.  The array keeps the last call's
 * contents; nothing in it has to start at zero, every region is written before it is read.  Per-launch
 * timing (cb_profile_enable) is suspended during the call. */
#define CB_STATIC_SCRATCH_BYTES (128u << 20)
size_t cb_static_scratch_bytes(void);
int cb_fuse_layer_static(cb_ctx *ctx, int32_t layer, const cb_layer_weights *weights /*HOST*/,
                         const float *h_in, const int32_t *row_pos, int32_t n_rows, int32_t n_suffix,
                         void *k_cache, void *v_cache, int32_t n_tokens_total, int32_t k_keep,
                         const int32_t *forced_sel, float *h_out, int32_t *pos_out, float *dev_out,
                         void *stream);

/* Whole fusing pass (Sec. 4; Sec. 5.1 "fusor"): cb_realign_rope on layers 1 .. L-1 (layer 0
 * keeps, i.e. recomputes, every context row, so its pre-computed K/V is never read), then
 * cb_fuse_layer for layers 0 .. L-1, each layer's survivors feeding the next.
 *   layers        : HOST array [L] of cb_layer_weights
 *   x             : T [n_ctx + n_suffix, d] layer-0 input, context tokens chunk
 *                   after chunk, then the suffix
 *   chunk_lens    : HOST int32[n_chunks], each >= 1
 *   k_cache_layers, v_cache_layers : HOST arrays [L] of device pointers to
 *                   T [n_ctx + n_suffix, Hkv, dh]; rows [0, n_ctx) hold the chunks'
 *                   pre-computed K/V as cached at positions 0.. (NOT re-aligned)
 *   keep_counts   : HOST int32[L], keep_counts[0] == n_ctx, non-increasing
 *   forced_sel    : NULL, or HOST array [L] of (NULL | device int32[keep_counts[l]])
 *   final_hidden  : float [n_suffix, d] residual stream after the last layer
 *   sel_dump      : NULL, or HOST array [L] of (NULL | device int32[keep_counts[l]])
 *                   receiving the kept context positions of layer l
 *   dev_dump      : NULL, or HOST array [L] of (NULL | device float[candidates of
 *                   layer l]) receiving that layer's deviation vector */
int cb_fuse_prefill(cb_ctx *ctx, const cb_layer_weights *layers, const void *x,
                    const int32_t *chunk_lens, int32_t n_chunks, int32_t n_suffix,
                    void *const *k_cache_layers, void *const *v_cache_layers,
                    const int32_t *keep_counts, const int32_t *const *forced_sel,
                    float *final_hidden, int32_t *const *sel_dump, float *const *dev_dump,
                    void *workspace, size_t workspace_bytes, void *stream);

/* The same pass with the pre-computed caches still in HOST memory (Sec. 5: pipelining KV
 * loading and recompute).  The copies are queued on copy_stream in layer order, a few layers
 * ahead of the launches of the layer that needs them; on `stream`, layer l waits for its own copy
 * only, is re-aligned and fused, so loading layer l+1.. overlaps the recompute of layer l.  Layer 0 recomputes every row and reads none of
 * its cached K/V, so k_host_layers[0] / v_host_layers[0] are not loaded (they must still be non-NULL).
 *   k_host_layers, v_host_layers : HOST arrays [L] of HOST pointers to T [n_ctx, Hkv, dh], each
 *                   chunk cached at positions 0..; pinned memory if the copies are to overlap
 *   k_cache_layers, v_cache_layers : HOST arrays [L] of device pointers to
 *                   T [n_ctx + n_suffix, Hkv, dh]; receive the loaded rows and end as the fused caches
 *   stream, copy_stream : two different streams of the same (default) priority; copy_stream first
 *                   waits for the work already queued on stream.  All work, copies included, has
 *                   completed once `stream` has been synchronised.
 * Other arguments, validation and results as cb_fuse_prefill (without forced selections and dumps).
 * The host buffers must stay valid and unchanged until then. */
int cb_fuse_prefill_pipelined(cb_ctx *ctx, const cb_layer_weights *layers, const void *x,
                              const int32_t *chunk_lens, int32_t n_chunks, int32_t n_suffix,
                              const void *const *k_host_layers, const void *const *v_host_layers,
                              void *const *k_cache_layers, void *const *v_cache_layers,
                              const int32_t *keep_counts, float *final_hidden, void *workspace,
                              size_t workspace_bytes, void *stream, void *copy_stream);

/* Several requests in one pass (Sec. 7 sensitivity analysis, the batch-size paragraph): the projections and the MLP run on
 * the stacked rows of all requests, selection and attention per request.  Request b contributes
 * n_chunks[b] chunks and n_suffix[b] query tokens; T_b = its context + suffix length.
 *   x             : T [sum_b T_b, d], request after request, each: context chunks then suffix
 *   chunk_lens    : HOST int32[sum_b n_chunks[b]], the requests' chunk lengths one after another
 *   n_chunks, n_suffix : HOST int32[n_requests]
 *   k_cache_layers, v_cache_layers : HOST arrays [L] of device pointers to
 *                   T [n_requests * cache_stride, Hkv, dh]; request b owns rows
 *                   [b * cache_stride, b * cache_stride + T_b), laid out as for cb_fuse_prefill
 *   cache_stride  : rows between two requests' slabs, >= max_b T_b
 *   keep_counts   : HOST int32[n_requests * L], keep_counts[b * L + l]; per request as in cb_fuse_prefill
 *   final_hidden  : float [sum_b n_suffix[b], d], request after request
 *   sel_dump      : NULL, or HOST array [n_requests * L] of (NULL | device int32[keep_counts[b * L + l]])
 *   dev_dump      : NULL, or HOST array [L] of (NULL | device float[rows entering layer l]): the
 *                   deviation of every stacked row in row order (values at suffix rows are meaningless)
 * Each request's results equal those of its own cb_fuse_prefill call up to the summation order of
 * the projections. */
size_t cb_batched_workspace_bytes(const cb_ctx *ctx, int32_t total_tokens);
int cb_fuse_prefill_batched(cb_ctx *ctx, const cb_layer_weights *layers, int32_t n_requests, const void *x,
                            const int32_t *chunk_lens, const int32_t *n_chunks, const int32_t *n_suffix,
                            void *const *k_cache_layers, void *const *v_cache_layers, int32_t cache_stride,
                            const int32_t *keep_counts, float *final_hidden, int32_t *const *sel_dump,
                            float *const *dev_dump, void *workspace, size_t workspace_bytes, void *stream);

/* First token (Sec. 2: the prefill phase ends when the first token is generated):
 * RMSNorm of the LAST row of final_hidden, vocabulary projection, greedy pick.
 *   final_hidden : float [n_suffix, d] as cb_fuse_prefill leaves it, n_suffix >= 1
 *   final_norm   : T [d] gain of the final RMSNorm (eps = desc.rms_eps)
 *   lm_head      : T [vocab, d] row-major
 *   logits       : float [vocab] (out)
 *   token        : int32 [1] (out, device): smallest index among the largest logits
 * Needs d_model % 8 == 0 and d_model <= 16384 (else CB_EUNSUPPORTED). */
int cb_first_token(cb_ctx *ctx, const float *final_hidden, int32_t n_suffix, const void *final_norm,
                   const void *lm_head, int32_t vocab, float *logits, int32_t *token, void *stream);

/* Loading controller (Sec. 5.1).  Plain host arithmetic, no ctx, no device work.
 * cb_recompute_delay: T_recompute = ratio x profiled full-prefill delay (first footnote).
 * cb_load_delay     : T_load = per-token KV bytes x tokens / device throughput, in seconds
 *                     (second footnote); non-positive throughput gives +infinity.
 * cb_pick_recompute_ratio: the ratio at which recompute takes as long as loading, clamped
 *                     to [min_ratio, 1] (min_ratio = the paper's quality floor r*, 0.15).
 * cb_pick_storage_device: index of the cheapest of n devices whose loading delay does not
 *                     exceed recompute_delay (ties -> lower index), -1 if there is none.
 *                     load_delays, costs: HOST double[n]. */
double cb_recompute_delay(double ratio, double prefill_delay);
double cb_load_delay(double per_token_kv_bytes, double n_tokens, double throughput_bytes_per_s);
double cb_pick_recompute_ratio(double prefill_delay, double load_delay, double min_ratio);
int32_t cb_pick_storage_device(double recompute_delay, const double *load_delays, const double *costs,
                               int32_t n);

/* Instrumentation for benchmarks (no operation of the paper): HIP-event timing per kernel class.
 * Classes: projections' main launches; attention (+ merge of key-range pieces); re-alignment; the K/V
 * projection's finish launch that also computes the deviation; selection + cache update; stand-alone
 * RMSNorm; copies and conversions; the other finish launches (sum of parked sums + residual + norm, SwiGLU
 * tail); first-token head; and two PHASES of cb_fuse_prefill / cb_fuse_prefill_pipelined that span many
 * launches: everything up to the end of layer 0 (input conversion, re-alignment, the full first layer), and
 * the selective layers 1 .. L-1 with the final copy. */
enum { CB_PROF_GEMM = 0, CB_PROF_ATTN = 1, CB_PROF_REALIGN = 2, CB_PROF_DEV = 3,
       CB_PROF_TOPK = 4, CB_PROF_NORM = 5, CB_PROF_OTHER = 6, CB_PROF_REDUCE = 7,
       CB_PROF_HEAD = 8, CB_PROF_PHASE_FIRST = 9, CB_PROF_PHASE_SELECTIVE = 10, CB_PROF_NCLASS = 11 };
/* enable = 1: every later launch on ctx is bracketed by a pair of HIP events on its stream (this
 * slows the pass a little; do not time whole calls meanwhile).  enable = 2: only the two phases are
 * bracketed (three events per call: whole-call timing stays valid).  enable = 0: off. */
int cb_profile_enable(cb_ctx *ctx, int32_t enable);
/* Synchronises the events recorded since the last read, adds up milliseconds,
 * launch counts, algorithmic flops and algorithmic bytes per class into HOST
 * arrays of CB_PROF_NCLASS entries each, and resets the record. */
int cb_profile_read(cb_ctx *ctx, double *ms, int64_t *launches, double *flops, double *bytes);

#ifdef __cplusplus
}
#endif
#endif /* CACHEBLEND_H */
