// Host-side launchers of the gfx950 kernels (one .hip file per kernel family).
// dtype: 0 = float storage, 1 = bfloat16 storage (cb_dtype).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cb {

// Device table of the requests stacked in one layer call, kSegInts ints per request (+ one closing
// entry whose kSegQwg is the total): where its rows enter (kSegInOff) and how many of them are
// candidates / kept / suffix rows, where its kept rows start in the output (kSegOutOff), its first
// attention query workgroup (kSegQwg) and the first row of its slab in the cache arrays.
enum { kSegInOff = 0, kSegCand = 1, kSegKeep = 2, kSegSuffix = 3, kSegOutOff = 4, kSegQwg = 5, kSegCacheRow = 6,
       kSegInts = 8 };

// ---- elementwise.hip -------------------------------------------------------
// In-place rotation of cached keys of chunks >= 1 by their offsets.
// rope_tab: float2 [max_tokens][head_dim/2] = (cos, sin)(p * theta_i).
// rope_half: rotary block i acts on channels (i, i + head_dim/2) of a head instead of (2i, 2i+1).
hipError_t launch_realign(int dtype, void *const *k_layers_host, int n_layers,
                          const int32_t *chunk_offsets_host, int n_chunks, int kv_dim,
                          int head_dim, int rope_half, const float2 *rope_tab, hipStream_t s);
hipError_t launch_to_f32(int dtype, const void *x, float *out, size_t n, hipStream_t s);
// out[r][c] = bf16(q[r][c] * scale[r]) for an int8 matrix [rows, cols], cols % 16 == 0.
hipError_t launch_dequant_int8(const void *q, const float *scale, void *out, int rows, int cols, hipStream_t s);
// out[r] = rmsnorm(h[r]) * gain, r < n_rows; out has storage type and row pitch ld_out;
// lo_off > 0: the rounding remainder of every value is stored lo_off elements after it.
hipError_t launch_rmsnorm(int dtype, const float *h, const void *gain, void *out, int ld_out, int lo_off,
                          int n_rows, int d, float eps, hipStream_t s);
// K[pos_out[i]] = kvnew[sel_rows[i]][:kv_dim], V[...] = kvnew[...][kv_dim:], i < m.
hipError_t launch_scatter_kv(int dtype, const void *kvnew, const int32_t *sel_rows,
                             const int32_t *pos_out, int m, void *k_cache, void *v_cache,
                             int kv_dim, hipStream_t s);
// out[i] = in[first_row + i] for n_rows rows of width d (float).
hipError_t launch_copy_rows_f32(const float *in, float *out, size_t n, hipStream_t s);

// ---- select.hip ------------------------------------------------------------
// Keep the k largest of dev[0..n_cand) (ties -> lower index); sel_rows[0..k) = row_base + kept
// row indices ascending, then the n_suffix rows row_base + n_cand ..; pos_out[i] = row_pos of
// that row and cache_row_out[i] (nullable) = its cache row (cache_row, NULL: row_pos; both indexed
// without row_base).  With kvnew != NULL the same launch copies the kept rows' new K/V
// (kvnew[row_base + i] = [K | V], kv_row_bytes each, a multiple of 16) into rows cache_row of kc / vc.
// segs (device, NULL: one request): the request table; the arrays are then the stacked ones of all
// n_segs requests, each request's counts and offsets come from its entry (n_cand, k, n_suffix, row_base
// are ignored) and max_out is the largest k + n_suffix of any request.
hipError_t launch_topk_scatter(const float *dev, int n_cand, int k, int n_suffix, const int32_t *row_pos,
                               const int32_t *cache_row, int32_t *sel_rows, int32_t *pos_out,
                               int32_t *cache_row_out, int row_base, const void *kvnew, void *kc, void *vc,
                               int kv_row_bytes, hipStream_t s, const int32_t *segs = nullptr, int n_segs = 0,
                               int max_out = 0);
// out[i] = src[idx[i]], i < n.
hipError_t launch_gather_i32(const int32_t *src, const int32_t *idx, int n, int32_t *out, hipStream_t s);
// Same outputs from a given ascending list of positions (lower-bound search in row_pos).
hipError_t launch_forced_map(const int32_t *forced, int k, const int32_t *row_pos, int n_cand,
                             int n_suffix, int32_t *sel_rows, int32_t *pos_out, hipStream_t s);

// ---- gemm.hip --------------------------------------------------------------
enum { EPI_SEG = 0, EPI_SWIGLU = 1, EPI_F32 = 2 };
struct GemmSeg {
  const void *w;           // [n, K] row-major weights of this column segment
  int n;                   // number of output columns in the segment
  void *dst;               // EPI_SEG: destination base (storage type)
  int ld_dst;              // destination row pitch in elements
  const int32_t *row_map;  // EPI_SEG: destination row = row_map[r] (NULL: r)
  int rope;                // EPI_SEG: rotate adjacent column pairs by row_pos[r]
  const void *dev_cache;   // EPI_SEG with dev_out: cache [*, n] this segment's new values are compared with (NULL: none)
  const float *w_scale;    // non-NULL: w holds int8 values [n, K] and output column c is w_scale[c] times the sum over
                           // them; only where gemm_int8_in_kernel() says so, and for every matrix of a launch or none
};
struct GemmArgs {
  int dtype;
  const void *a;           // [*, K] row-major activations (storage type), pitch lda
  int lda;
  const int32_t *a_rows;   // gather: logical row r reads a[a_rows[r]] (NULL: r)
  int a_lo_off;            // bf16 EPI_SEG: > 0 = every row also holds the rounding remainders of its K values,
                           // a_lo_off elements further on; both parts are multiplied (float-accurate input)
  int M, K;
  int epi;
  int n_seg;               // EPI_SEG: 1..3 segments; EPI_SWIGLU: seg[0]=gate, seg[1]=up
  GemmSeg seg[3];          //   (dst/ld_dst of seg[0] receive silu(gate)*up);
                           // EPI_F32: seg[0] only (w, n)
  const float2 *rope_tab;  // EPI_SEG with rope
  int rope_half;           // rotary pairs (i, i + head_dim/2) instead of (2i, 2i+1); segments are whole heads
  const int32_t *row_pos;  // positions of the logical rows
  int head_dim;
  float *out_f32;          // EPI_F32: [M, n] float output, pitch n
  const float *resid;      // EPI_F32: added to the output; row r reads resid[resid_rows[r]]
  const int32_t *resid_rows;
  // EPI_F32: RMSNorm of the finished rows in the storage type (norm_gain NULL: none), pitch norm_ld;
  // norm_lo_off > 0: the rounding remainders are stored norm_lo_off elements after the values
  const void *norm_gain;
  void *norm_out;
  int norm_ld, norm_lo_off;
  float norm_eps;
  // EPI_SEG: dev_out[r] (r < n_dev) = squared distance of the row's stored new values from row
  // dev_row[r] of the segments' dev_cache arrays (NULL: no deviation)
  float *dev_out;
  int n_dev;
  const int32_t *dev_row;
  float *partial;          // scratch for parked sums (gemm_partial_floats); the K split is capped by it
  size_t partial_floats;
};
// Floats of scratch a problem of this shape parks its sums in when the scratch is not the limit
// (0 when the main kernel finishes the outputs itself); N is the total number of output columns
// (d_ff for EPI_SWIGLU); hl: (high, low) activation pairs; force_raw: a deviation is wanted; w8: int8
// weights (read by the kernel itself where it can).
// For workspace sizing.
// whether the projection kernels read int8 weights themselves for this storage type and K (else the caller
// expands them to the storage type first)
bool gemm_int8_in_kernel(int dtype, int K);
size_t gemm_partial_floats(int dtype, int epi, int M, int N, int K, int hl, int force_raw, int rope_half,
                           int head_dim, int w8 = 0);
// Main kernel.  EPI_F32 problems, problems with a deviation, and problems split along K
// (gemm_needs_finish) leave raw sums in g.partial and must be completed by launch_gemm_finish on
// the same stream.  EPI_F32 and deviation problems REQUIRE partial_floats >= M * N.
hipError_t launch_gemm(const GemmArgs &g, hipStream_t s);
bool gemm_needs_finish(const GemmArgs &g);
hipError_t launch_gemm_finish(const GemmArgs &g, hipStream_t s);

// ---- attention.hip ---------------------------------------------------------
// o[r, h, :] = softmax_{j <= q_pos[r]}(q[r,h,:] . K[j, h/g, :] / sqrt(dh)) V[j, h/g, :]
// o: [n_rows, Hq, dh] storage type; q: row r is read at q[q_rows[r]] (q_rows NULL: q[r]);
// caches [*, Hkv, dh]; q_pos in any order (ascending positions give the best key-range skipping).
// n_tokens: rows of the caches (upper bound of q_pos + 1).  partial: scratch for the KV split
// used when there are few query rows (attention_partial_floats floats; NULL or too small: no split).
size_t attention_partial_floats(int dtype, int n_rows, int n_q_heads, int n_kv_heads, int head_dim,
                                int n_tokens);
// upper bound of the above over every n_tokens (for workspace sizing)
size_t attention_partial_floats_bound(int dtype, int n_rows, int n_q_heads, int n_kv_heads, int head_dim);
// segs (device, NULL: one request): the table above with n_segs requests; q_rows / q_pos / o are then the
// stacked arrays of all requests, n_rows their total, n_tokens the longest cache, total_qwg the sum of
// attention_query_workgroups over the requests (bf16 only).
hipError_t launch_attention(int dtype, const void *q, const int32_t *q_rows, const int32_t *q_pos, int n_rows,
                            const void *k_cache, const void *v_cache, void *o, int n_q_heads,
                            int n_kv_heads, int head_dim, int n_tokens, float *partial,
                            size_t partial_floats, hipStream_t s, const int32_t *segs = nullptr, int n_segs = 0,
                            long total_qwg = 0);
// query workgroups (per kv head) a request with n_rows rows occupies in the bf16 kernel's grid
long attention_query_workgroups(int n_rows, int n_q_heads, int n_kv_heads);

// ---- head.hip ---------------------------------------------------------------
// logits[v] = T(rmsnorm(h_row) * gain) . w[v, :], v < vocab; w row-major [vocab, d]; d % 8 == 0,
// d <= 16384 (the normalised row is held in LDS).
hipError_t launch_lm_head(int dtype, const float *h_row, const void *gain, const void *w, int d, int vocab,
                          float eps, float *logits, hipStream_t s);
// token[0] = smallest index among the largest of logits[0..n).
hipError_t launch_argmax(const float *logits, int n, int32_t *token, hipStream_t s);

}  // namespace cb
