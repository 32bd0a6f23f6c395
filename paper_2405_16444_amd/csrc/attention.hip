// Sparse-query causal attention of the recomputed rows over the whole fused KV
// cache (paper Sec. 4.2: "the attention matrix includes attention between selected
// tokens and all other tokens"); with every row selected it is plain causal
// attention (Sec. 2).  A query at global position p sees cache rows 0..p.
//
// bf16 kernel (MFMA 32x32x16).  One workgroup = one kv head x a block of
// "flattened queries" m = row * g + head_in_group, so the g query heads that share
// a kv head sit side by side in the MFMA N dimension and every K/V tile staged in
// LDS is used by all of them.  Each wavefront owns NQB blocks of 32 queries.
// Both products are computed transposed,
//     S^T[key, query] = K Q^T            O^T[channel, query] += V^T P^T
// so that a lane always holds values of ONE query (column = lane % 32): the running
// max / sum and the rescaling of O need no cross-lane traffic except one exchange
// between the two half-waves, and the exponentiated scores are already laid out as
// the B operand of the second product (they never leave registers).  The second
// product contracts over keys, so V is stored transposed in LDS ([channel][key]).
//
// float kernel: one wavefront per (row, query head), 64 keys per step, plain FMA.
#include "common.h"
#include "kernels.h"
#include <algorithm>

namespace cb {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;

// ---------------------------------------------------------------------------
constexpr int BKV = 64;                 // keys per tile
constexpr int VT_PITCH = BKV + 4;       // transposed V tile: [dh][BKV + 4] bf16

template <int DH, int NQB>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const bf16 *__restrict__ q,
                                                        const int32_t *__restrict__ q_pos, int n_rows,
                                                        const bf16 *__restrict__ kc,
                                                        const bf16 *__restrict__ vc, bf16 *__restrict__ o,
                                                        int n_q_heads, int n_kv_heads, float scale_log2e,
                                                        int split_tiles, float *__restrict__ part_o,
                                                        float *__restrict__ part_ml) {
  constexpr int KP = DH + 8;            // K tile pitch (elements)
  constexpr int KS = DH / 16;           // k-steps of the first product
  constexpr int DB = DH / 32;           // 32-channel blocks of the output
  constexpr int CH = DH / 8;            // 16-byte chunks per K/V row
  constexpr int K_CHUNKS = BKV * CH / 256;        // per thread
  constexpr int V_PAIRS = (BKV / 2) * CH / 256;   // per thread (two keys x 8 channels)
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16 *sK = reinterpret_cast<bf16 *>(smem_raw);   // [2][BKV * KP]
  bf16 *sVt = sK + 2 * BKV * KP;                    // [2][DH * VT_PITCH]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const int g = n_q_heads / n_kv_heads;
  const int kvh = blockIdx.y;
  const int n_flat = n_rows * g;
  const int m_wg = blockIdx.x * (128 * NQB);
  const int kv_dim = n_kv_heads * DH;

  // causal bound of the workgroup = position of its last valid row
  const int last_m = min(m_wg + 128 * NQB, n_flat) - 1;
  const int kv_len = q_pos[last_m / g] + 1;
  const int n_tiles_all = (kv_len + BKV - 1) / BKV;
  // KV split: workgroup z of gridDim.z handles tiles [t_begin, n_tiles) of the causal range and
  // leaves un-normalised partial results (flash-decoding style) for the merge kernel
  const int t_begin = blockIdx.z * split_tiles;
  if (t_begin >= n_tiles_all) return;
  const int n_tiles = min(n_tiles_all, t_begin + split_tiles);

  // this lane's queries
  int my_pos[NQB];
  long q_off[NQB];
  bool valid[NQB];
  bf16x8 qf[NQB][KS];
  int wave_max_pos = -1, wave_min_pos = 0x7fffffff;
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    const int m = m_wg + (wave * NQB + b) * 32 + ln;
    valid[b] = m < n_flat;
    const int mm = valid[b] ? m : n_flat - 1;
    const int r = mm / g, j = mm - r * g;
    my_pos[b] = valid[b] ? q_pos[r] : -1;
    q_off[b] = ((long)r * n_q_heads + kvh * g + j) * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[b][ks] = *reinterpret_cast<const bf16x8 *>(q + q_off[b] + ks * 16 + 8 * h);
    wave_max_pos = max(wave_max_pos, my_pos[b]);
    wave_min_pos = min(wave_min_pos, my_pos[b]);       // invalid queries (-1) force masking
  }
  wave_max_pos = (int)wave_max((float)wave_max_pos);  // positions < 2^24: exact in float
  wave_min_pos = -(int)wave_max((float)(-wave_min_pos));

  f32x16 oacc[NQB][DB];
  float row_max[NQB], row_sum[NQB];
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    row_max[b] = kNegBig;
    row_sum[b] = 0.f;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[b][d][i] = 0.f;
  }

  // global -> register -> LDS staging of one K/V tile
  bf16x8 rk[K_CHUNKS], rv[V_PAIRS][2];
  auto gload = [&](int t0) {
#pragma unroll
    for (int i = 0; i < K_CHUNKS; ++i) {
      const int id = tid + i * 256, key = id / CH, c = id % CH;
      const int row = min(t0 + key, kv_len - 1);
      rk[i] = *reinterpret_cast<const bf16x8 *>(kc + (size_t)row * kv_dim + kvh * DH + c * 8);
    }
#pragma unroll
    for (int i = 0; i < V_PAIRS; ++i) {
      const int id = tid + i * 256, kp = id % (BKV / 2), c = id / (BKV / 2);
      const int r0 = min(t0 + 2 * kp, kv_len - 1), r1 = min(t0 + 2 * kp + 1, kv_len - 1);
      rv[i][0] = *reinterpret_cast<const bf16x8 *>(vc + (size_t)r0 * kv_dim + kvh * DH + c * 8);
      rv[i][1] = *reinterpret_cast<const bf16x8 *>(vc + (size_t)r1 * kv_dim + kvh * DH + c * 8);
    }
  };
  auto sstore = [&](int st) {
#pragma unroll
    for (int i = 0; i < K_CHUNKS; ++i) {
      const int id = tid + i * 256, key = id / CH, c = id % CH;
      *reinterpret_cast<bf16x8 *>(sK + st * BKV * KP + key * KP + c * 8) = rk[i];
    }
#pragma unroll
    for (int i = 0; i < V_PAIRS; ++i) {
      const int id = tid + i * 256, kp = id % (BKV / 2), c = id / (BKV / 2);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        bf16x2 pr = {rv[i][0][e], rv[i][1][e]};
        *reinterpret_cast<bf16x2 *>(sVt + st * DH * VT_PITCH + (c * 8 + e) * VT_PITCH + 2 * kp) = pr;
      }
    }
  };

  gload(t_begin * BKV);
  sstore(t_begin & 1);
  __syncthreads();
  for (int t = t_begin; t < n_tiles; ++t) {
    const int t0 = t * BKV;
    if (t + 1 < n_tiles) gload(t0 + BKV);
    if (t0 <= wave_max_pos) {  // wave-uniform: tiles wholly in this wave's future are skipped
      const bf16 *ck = sK + (t & 1) * BKV * KP;
      const bf16 *cv = sVt + (t & 1) * DH * VT_PITCH;
      // ---- S^T = K Q^T ----
      f32x16 sacc[NQB][2];
#pragma unroll
      for (int b = 0; b < NQB; ++b)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[b][kb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ck + (kb * 32 + ln) * KP + ks * 16 + 8 * h);
#pragma unroll
          for (int b = 0; b < NQB; ++b)
            sacc[b][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[b][ks], sacc[b][kb], 0, 0, 0);
        }
      }
      // ---- online softmax (per lane = per query), in the raw score domain: p = 2^((s - m) c) ----
      bf16x8 pf[NQB][4];
      const bool diag = t0 + BKV - 1 > wave_min_pos;     // wave-uniform: some key of the tile is masked
#pragma unroll
      for (int b = 0; b < NQB; ++b) {
        float mx = kNegBig;
        if (diag) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = t0 + kb * 32 + (i >> 2) * 8 + h * 4 + (i & 3);
              sacc[b][kb][i] = key <= my_pos[b] ? sacc[b][kb][i] : kNegBig;
            }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[b][kb][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float new_max = fmaxf(row_max[b], mx);
        const float neg_mc = -new_max * scale_log2e;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][kb][i], scale_log2e, neg_mc));
            psum += pv;
            pf[b][kb * 2 + (i >> 3)][i & 7] = (bf16)pv;
          }
        // the accumulators only need rescaling when some query's running max moved, which
        // becomes rare after the first tiles
        if (__any(new_max > row_max[b])) {
          const float alpha = __builtin_amdgcn_exp2f((row_max[b] - new_max) * scale_log2e);
          row_sum[b] *= alpha;
#pragma unroll
          for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[b][d][i] *= alpha;
          row_max[b] = new_max;
        }
        row_sum[b] += psum;
      }
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const bf16 *vp = cv + (d * 32 + ln) * VT_PITCH + 16 * u + 4 * h;
          const bf16x4 v0 = *reinterpret_cast<const bf16x4 *>(vp);
          const bf16x4 v1 = *reinterpret_cast<const bf16x4 *>(vp + 8);
          const bf16x8 vf = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
#pragma unroll
          for (int b = 0; b < NQB; ++b)
            oacc[b][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[b][u], oacc[b][d], 0, 0, 0);
        }
      }
    }
    if (t + 1 < n_tiles) sstore((t + 1) & 1);
    __syncthreads();
  }
  if (gridDim.z > 1) {
    // ---- partial results: O (un-normalised), running max and sum per (kv head, query, split) ----
#pragma unroll
    for (int b = 0; b < NQB; ++b) {
      const float tot = row_sum[b] + __shfl_xor(row_sum[b], 32, 64);
      if (!valid[b]) continue;
      const int m = m_wg + (wave * NQB + b) * 32 + ln;
      const size_t slot = ((size_t)kvh * n_flat + m) * gridDim.z + blockIdx.z;
      if (h == 0) {
        part_ml[slot * 2] = row_max[b] * scale_log2e;
        part_ml[slot * 2 + 1] = tot;
      }
      float *dst = part_o + slot * DH;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int a = 0; a < 4; ++a)
          *reinterpret_cast<float4 *>(dst + d * 32 + a * 8 + h * 4) =
              make_float4(oacc[b][d][a * 4 + 0], oacc[b][d][a * 4 + 1], oacc[b][d][a * 4 + 2],
                          oacc[b][d][a * 4 + 3]);
    }
    return;
  }
  // ---- normalise and store ----
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    const float tot = row_sum[b] + __shfl_xor(row_sum[b], 32, 64);
    const float inv = 1.f / tot;
    if (!valid[b]) continue;
    bf16 *dst = o + q_off[b];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        bf16x4 w = {(bf16)(oacc[b][d][a * 4 + 0] * inv), (bf16)(oacc[b][d][a * 4 + 1] * inv),
                    (bf16)(oacc[b][d][a * 4 + 2] * inv), (bf16)(oacc[b][d][a * 4 + 3] * inv)};
        *reinterpret_cast<bf16x4 *>(dst + d * 32 + a * 8 + h * 4) = w;
      }
  }
}

// Merge of the KV-split partials: o = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s over the
// splits that ran for the query's workgroup (those below its causal bound).
template <int DH>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part_o,
                                                         const float *__restrict__ part_ml,
                                                         const int32_t *__restrict__ q_pos, int n_rows,
                                                         bf16 *__restrict__ o, int n_q_heads,
                                                         int n_kv_heads, int n_splits, int split_tiles,
                                                         int wg_queries) {
  constexpr int CG = DH / 4;                           // float4 channel groups per query
  const int g = n_q_heads / n_kv_heads, n_flat = n_rows * g;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)n_kv_heads * n_flat * CG) return;
  const int c = (int)(idx % CG);
  const long qh = idx / CG;                            // kvh * n_flat + m
  const int m = (int)(qh % n_flat), kvh = (int)(qh / n_flat);
  const int last_m = min((m / wg_queries + 1) * wg_queries, n_flat) - 1;
  const int n_tiles = (q_pos[last_m / g] + BKV) / BKV;
  const int ns = min(n_splits, (n_tiles + split_tiles - 1) / split_tiles);
  const float *ml = part_ml + qh * n_splits * 2;
  float mx = kNegBig;
  for (int s = 0; s < ns; ++s) mx = fmaxf(mx, ml[2 * s]);
  float den = 0.f;
  float4 acc = make_float4(0, 0, 0, 0);
  for (int s = 0; s < ns; ++s) {
    const float w = exp2f(ml[2 * s] - mx);
    den += w * ml[2 * s + 1];
    const float4 v = *reinterpret_cast<const float4 *>(part_o + (qh * n_splits + s) * DH + c * 4);
    acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
  }
  const float inv = 1.f / den;
  const int r = m / g, j = m - r * g;
  bf16x4 w4 = {(bf16)(acc.x * inv), (bf16)(acc.y * inv), (bf16)(acc.z * inv), (bf16)(acc.w * inv)};
  *reinterpret_cast<bf16x4 *>(o + ((size_t)r * n_q_heads + kvh * g + j) * DH + c * 4) = w4;
}

// ---------------------------------------------------------------------------
// float kernel.  Lane j of the wavefront scores key t0 + j; the 64 probabilities
// are then broadcast one by one while lane e accumulates output channels e, e+64.
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ q,
                                                       const int32_t *__restrict__ q_pos, int n_rows,
                                                       const float *__restrict__ kc,
                                                       const float *__restrict__ vc, float *__restrict__ o,
                                                       int n_q_heads, int n_kv_heads, float scale_log2e) {
  __shared__ float sq[4][DH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int idx = blockIdx.x * 4 + wave;
  const bool active = idx < n_rows * n_q_heads;
  const int r = active ? idx / n_q_heads : 0, hq = active ? idx % n_q_heads : 0;
  const int kvh = hq / (n_q_heads / n_kv_heads);
  const int kv_dim = n_kv_heads * DH;
  const float *qrow = q + ((size_t)r * n_q_heads + hq) * DH;
  for (int e = lane; e < DH; e += 64) sq[wave][e] = qrow[e];
  __syncthreads();
  if (!active) return;
  const int pos = q_pos[r];
  constexpr int EPL = DH / 64 > 0 ? DH / 64 : 1;  // channels per lane
  float acc[EPL] = {};
  float run_max = kNegBig, run_sum = 0.f;
  for (int t0 = 0; t0 <= pos; t0 += 64) {
    const int key = t0 + lane;
    float s = kNegBig;
    if (key <= pos) {
      const float *krow = kc + (size_t)key * kv_dim + kvh * DH;
      float dot = 0.f;
#pragma unroll 8
      for (int e = 0; e < DH; ++e) dot = fmaf(sq[wave][e], krow[e], dot);
      s = dot * scale_log2e;
    }
    const float new_max = fmaxf(run_max, wave_max(s));
    const float alpha = exp2f(run_max - new_max);
    const float pv = key <= pos ? exp2f(s - new_max) : 0.f;
    run_sum = run_sum * alpha + wave_sum(pv);
    run_max = new_max;
#pragma unroll
    for (int c = 0; c < EPL; ++c) acc[c] *= alpha;
    const int nk = min(64, pos + 1 - t0);
    for (int j = 0; j < nk; ++j) {
      const float pj = __shfl(pv, j, 64);
      const float *vrow = vc + (size_t)(t0 + j) * kv_dim + kvh * DH;
#pragma unroll
      for (int c = 0; c < EPL; ++c)
        if (lane + 64 * c < DH) acc[c] = fmaf(pj, vrow[lane + 64 * c], acc[c]);
    }
  }
  float *orow = o + ((size_t)r * n_q_heads + hq) * DH;
#pragma unroll
  for (int c = 0; c < EPL; ++c)
    if (lane + 64 * c < DH) orow[lane + 64 * c] = acc[c] / run_sum;
}

// Split plan of the bf16 kernel: few query workgroups (the selective layers) leave most CUs
// idle, so the key range is cut into n_splits pieces handled by separate workgroups.
static void attn_split_plan(int n_rows, int hq, int hkv, int n_tokens, int *nqb, int *n_splits,
                            int *split_tiles) {
  const long n_flat = (long)n_rows * (hq / hkv);
  const bool big = ((n_flat + 255) / 256) * hkv >= 512;
  *nqb = big ? 2 : 1;
  const long base = ((n_flat + 128 * *nqb - 1) / (128 * *nqb)) * hkv;
  const int max_tiles = (n_tokens + BKV - 1) / BKV;
  int ns = 1;
  if (base < 384) {
    ns = (int)((768 + base - 1) / base);
    ns = std::min(ns, std::max(1, max_tiles / 4));
    ns = std::min(ns, 32);
  }
  *split_tiles = (max_tiles + ns - 1) / ns;
  *n_splits = (max_tiles + *split_tiles - 1) / *split_tiles;
}

size_t attention_partial_floats(int dtype, int n_rows, int hq, int hkv, int dh, int n_tokens) {
  if (dtype == 0 || n_rows == 0) return 0;
  int nqb, ns, st;
  attn_split_plan(n_rows, hq, hkv, n_tokens, &nqb, &ns, &st);
  if (ns <= 1) return 0;
  return (size_t)n_rows * hq * ns * (dh + 2);
}

hipError_t launch_attention(int dtype, const void *q, const int32_t *q_pos, int n_rows,
                            const void *kc, const void *vc, void *o, int hq, int hkv, int dh,
                            int n_tokens, float *partial, size_t partial_floats, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  const float scale_log2e = kLog2e / sqrtf((float)dh);
  if (dtype == 0) {
    dim3 grid((n_rows * hq + 3) / 4);
    if (dh == 64)
      hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, (const float *)q, q_pos, n_rows,
                         (const float *)kc, (const float *)vc, (float *)o, hq, hkv, scale_log2e);
    else
      hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, (const float *)q, q_pos, n_rows,
                         (const float *)kc, (const float *)vc, (float *)o, hq, hkv, scale_log2e);
    return hipGetLastError();
  }
  const int g = hq / hkv;
  const long n_flat = (long)n_rows * g;
  int nqb, n_splits, split_tiles;
  attn_split_plan(n_rows, hq, hkv, n_tokens, &nqb, &n_splits, &split_tiles);
  if (n_splits > 1 && (!partial || partial_floats < (size_t)n_rows * hq * n_splits * (dh + 2))) {
    n_splits = 1;                                    // no scratch: one workgroup walks all keys
    split_tiles = (n_tokens + BKV - 1) / BKV;
  }
  float *part_o = partial;
  float *part_ml = partial ? partial + (size_t)n_rows * hq * n_splits * dh : nullptr;
#define CB_ATTN(DH_, NQB_)                                                                          \
  do {                                                                                              \
    constexpr int smem = 2 * (BKV * (DH_ + 8) + DH_ * VT_PITCH) * 2;                                \
    static bool attr_set = false;                                                                   \
    if (!attr_set) {                                                                                \
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<DH_, NQB_>),       \
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem);                  \
      attr_set = true;                                                                              \
    }                                                                                               \
    hipLaunchKernelGGL((attn_bf16_kernel<DH_, NQB_>),                                               \
                       dim3((unsigned)((n_flat + 128 * NQB_ - 1) / (128 * NQB_)), hkv, n_splits),   \
                       dim3(256), smem, s, (const bf16 *)q, q_pos, n_rows, (const bf16 *)kc,        \
                       (const bf16 *)vc, (bf16 *)o, hq, hkv, scale_log2e, split_tiles, part_o,      \
                       part_ml);                                                                    \
  } while (0)
  if (dh == 64) { if (nqb == 2) CB_ATTN(64, 2); else CB_ATTN(64, 1); }
  else          { if (nqb == 2) CB_ATTN(128, 2); else CB_ATTN(128, 1); }
#undef CB_ATTN
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1) return e;
  const long total = (long)hkv * n_flat * (dh / 4);
  const dim3 mgrid((unsigned)((total + 255) / 256));
  if (dh == 64)
    hipLaunchKernelGGL(attn_merge_kernel<64>, mgrid, dim3(256), 0, s, part_o, part_ml, q_pos, n_rows,
                       (bf16 *)o, hq, hkv, n_splits, split_tiles, 128 * nqb);
  else
    hipLaunchKernelGGL(attn_merge_kernel<128>, mgrid, dim3(256), 0, s, part_o, part_ml, q_pos, n_rows,
                       (bf16 *)o, hq, hkv, n_splits, split_tiles, 128 * nqb);
  return hipGetLastError();
}

}  // namespace cb
