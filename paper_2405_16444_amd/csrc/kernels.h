// Host-side launchers of the gfx950 kernels (one .hip file per kernel family).
// dtype: 0 = float storage, 1 = bfloat16 storage (cb_dtype).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cb {

// ---- elementwise.hip -------------------------------------------------------
// In-place rotation of cached keys of chunks >= 1 by their offsets.
// rope_tab: float2 [max_tokens][head_dim/2] = (cos, sin)(p * theta_i).
// rope_half: rotary block i acts on channels (i, i + head_dim/2) of a head instead of (2i, 2i+1).
hipError_t launch_realign(int dtype, void *const *k_layers_host, int n_layers,
                          const int32_t *chunk_offsets_host, int n_chunks, int kv_dim,
                          int head_dim, int rope_half, const float2 *rope_tab, hipStream_t s);
hipError_t launch_to_f32(int dtype, const void *x, float *out, size_t n, hipStream_t s);
// out[r] = rmsnorm(h[r]) * gain, r < n_rows; out has storage type.
hipError_t launch_rmsnorm(int dtype, const float *h, const void *gain, void *out, int n_rows,
                          int d, float eps, hipStream_t s);
// dev[j] = |kvnew[j] - (K[pos_j] | V[pos_j])|^2; kvnew rows are [K(kv_dim) | V(kv_dim)].
hipError_t launch_deviation(int dtype, const void *kvnew, const int32_t *row_pos, int n_cand,
                            const void *k_cache, const void *v_cache, int kv_dim, float *dev,
                            hipStream_t s);
// K[pos_out[i]] = kvnew[sel_rows[i]][:kv_dim], V[...] = kvnew[...][kv_dim:], i < m.
hipError_t launch_scatter_kv(int dtype, const void *kvnew, const int32_t *sel_rows,
                             const int32_t *pos_out, int m, void *k_cache, void *v_cache,
                             int kv_dim, hipStream_t s);
// out[i] = in[first_row + i] for n_rows rows of width d (float).
hipError_t launch_copy_rows_f32(const float *in, float *out, size_t n, hipStream_t s);

// ---- select.hip ------------------------------------------------------------
// Keep the k largest of dev[0..n_cand) (ties -> lower index); sel_rows[0..k) = row_base + kept
// row indices ascending, then the n_suffix rows row_base + n_cand ..; pos_out[i] = row_pos of
// that row (row_pos indexed without row_base).  One workgroup.
hipError_t launch_topk(const float *dev, int n_cand, int k, int n_suffix, const int32_t *row_pos,
                       int32_t *sel_rows, int32_t *pos_out, int row_base, hipStream_t s);
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
};
struct GemmArgs {
  int dtype;
  const void *a;           // [*, K] row-major activations (storage type), pitch lda
  int lda;
  const int32_t *a_rows;   // gather: logical row r reads a[a_rows[r]] (NULL: r)
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
  float *partial;          // split-K scratch (gemm_partial_floats); too small or NULL: no split
  size_t partial_floats;
};
// Floats of split-K scratch a problem of this shape uses (0 when it is not split); N is the
// total number of output columns (d_ff for EPI_SWIGLU).  For workspace sizing.
size_t gemm_partial_floats(int dtype, int epi, int M, int N, int K, int rope_half = 0, int head_dim = 0);
// Main kernel.  A problem that was split along K (gemm_needs_reduce) leaves raw partial sums
// in g.partial and must be completed by launch_gemm_reduce on the same stream.
hipError_t launch_gemm(const GemmArgs &g, hipStream_t s);
bool gemm_needs_reduce(const GemmArgs &g);
hipError_t launch_gemm_reduce(const GemmArgs &g, hipStream_t s);

// ---- attention.hip ---------------------------------------------------------
// o[r, h, :] = softmax_{j <= q_pos[r]}(q[r,h,:] . K[j, h/g, :] / sqrt(dh)) V[j, h/g, :]
// o: [n_rows, Hq, dh] storage type; q: row r is read at q[q_rows[r]] (q_rows NULL: q[r]);
// caches [*, Hkv, dh]; q_pos ascending.
// n_tokens: rows of the caches (upper bound of q_pos + 1).  partial: scratch for the KV split
// used when there are few query rows (attention_partial_floats floats; NULL or too small: no split).
size_t attention_partial_floats(int dtype, int n_rows, int n_q_heads, int n_kv_heads, int head_dim,
                                int n_tokens);
hipError_t launch_attention(int dtype, const void *q, const int32_t *q_rows, const int32_t *q_pos, int n_rows,
                            const void *k_cache, const void *v_cache, void *o, int n_q_heads,
                            int n_kv_heads, int head_dim, int n_tokens, float *partial,
                            size_t partial_floats, hipStream_t s);

// ---- head.hip ---------------------------------------------------------------
// logits[v] = T(rmsnorm(h_row) * gain) . w[v, :], v < vocab; w row-major [vocab, d]; d % 8 == 0,
// d <= 16384 (the normalised row is held in LDS).
hipError_t launch_lm_head(int dtype, const float *h_row, const void *gain, const void *w, int d, int vocab,
                          float eps, float *logits, hipStream_t s);
// token[0] = smallest index among the largest of logits[0..n).
hipError_t launch_argmax(const float *logits, int n, int32_t *token, hipStream_t s);

}  // namespace cb
