// Sparse-query causal attention (paper Sec. 4.2): the recomputed rows are the queries,
// the keys and values are ALL rows of the fused cache, recomputed or reused; with every
// row selected it is plain causal attention (Sec. 2).  A query at global position p
// sees cache rows 0..p.
//
// bf16 kernel (MFMA 32x32x16).  One workgroup = one kv head x a block of
// "flattened queries" m = row * g + head_in_group, so the g query heads that share
// a kv head sit side by side in the MFMA N dimension and every K/V tile staged in
// LDS is used by all of them.  Each of the 8 wavefronts owns a block of 32 queries.
// Both products are computed transposed,
//     S^T[key, query] = K Q^T            O^T[channel, query] += V^T P^T
// so that a lane always holds values of ONE query (column = lane % 32): the running
// max / sum and the rescaling of O need no cross-lane traffic except one exchange
// between the two half-waves, and the exponentiated scores are already laid out as
// the B operand of the second product (they never leave registers).  The second
// product contracts over keys; V stays row-major in LDS and its operand is fetched with
// the transposing LDS read (ds_read_b64_tr_b16).  K/V tiles are streamed through a 3-stage
// LDS ring by direct global->LDS loads.
//
// float kernel: one wavefront per (row, query head), 64 keys per step, plain FMA.
#include "common.h"
#include "kernels.h"
#include <algorithm>
#include <mutex>

namespace cb {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;

// ---------------------------------------------------------------------------
constexpr int BKV = 64;                 // keys per tile
constexpr int ATT_S = 3;                // LDS ring stages (K tile + V tile each)

typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int DH, int NQB, int NW>
__global__ __launch_bounds__(64 * NW) void attn_bf16_kernel(const bf16 *__restrict__ q,
                                                        const int32_t *__restrict__ q_pos, int n_rows,
                                                        const bf16 *__restrict__ kc,
                                                        const bf16 *__restrict__ vc, bf16 *__restrict__ o,
                                                        int n_q_heads, int n_kv_heads, float scale_log2e,
                                                        int split_tiles, float *__restrict__ part_o,
                                                        float *__restrict__ part_ml,
                                                        const int32_t *__restrict__ q_rows,
                                                        int32_t *__restrict__ wg_tiles,
                                                        const int32_t *__restrict__ segs, int n_segs) {
  // K and V tiles sit row-major in LDS ([key][channel], no padding) and are filled by direct
  // global->LDS loads: one wavefront-wide 16-byte load writes 1 KB = RPI whole rows.  Instead of
  // padding, the 16-byte chunk c of row r is stored in slot c ^ f(r), which makes both the
  // 16-byte K operand reads and the transposing 8-byte V reads conflict-free.
  constexpr int ROWB = DH * 2;            // bytes per row
  constexpr int CH = DH / 8;              // 16-byte chunks per row
  constexpr int RPI = 1024 / ROWB;        // rows per wavefront-wide load
  constexpr int TILEB = BKV * ROWB;       // bytes of one K (or V) tile
  constexpr int STAGE = 2 * TILEB;
  constexpr int LPT = 2 * (BKV / RPI) / NW; // loads per lane per tile (K and V, NW wavefronts)
  constexpr int WGQ = 32 * NQB * NW;        // flattened queries per workgroup
  constexpr int KS = DH / 16;             // k-steps of the first product
  constexpr int DB = DH / 32;             // 32-channel blocks of the output
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const int g = n_q_heads / n_kv_heads;
  const int kvh = blockIdx.x;                          // kv head varies fastest in dispatch order
  const int kv_dim = n_kv_heads * DH;
  // workgroups with the longest key range (the last rows) are dispatched first, for every kv head
  const int qwg = (int)(gridDim.y - 1 - blockIdx.y);
  // Several requests in one launch: request s owns the query workgroups [segs[s].qwg, segs[s+1].qwg),
  // the rows [row0, row0 + rows) of q_pos / q_rows / o, and the cache rows from cache0 on.
  int seg_qwg0 = 0, row0 = 0;
  if (segs) {
    int lo = 0, hi = n_segs - 1;                       // last segment whose first workgroup is <= qwg
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (segs[mid * kSegInts + kSegQwg] <= qwg) lo = mid; else hi = mid - 1;
    }
    const int32_t *sg = segs + lo * kSegInts;
    seg_qwg0 = sg[kSegQwg];
    row0 = sg[kSegOutOff];
    n_rows = sg[kSegKeep] + sg[kSegSuffix];
    const size_t cache0 = (size_t)sg[kSegCacheRow] * kv_dim;
    kc += cache0;
    vc += cache0;
    q_pos += row0;
    if (q_rows) q_rows += row0;
  }
  const int n_flat = n_rows * g;
  const int m_wg = (qwg - seg_qwg0) * WGQ;             // first flattened query of the workgroup, within its request
  const int m_pad = qwg * WGQ;                         // the same in the launch-wide numbering of the scratch
  const int n_flat_pad = (int)gridDim.y * WGQ;

  // causal bound of the workgroup = largest position among its rows (they need not be sorted)
  __shared__ int s_max_pos;
  if (tid == 0) s_max_pos = -1;
  __syncthreads();
  {
    const int last_m = min(m_wg + WGQ, n_flat) - 1;
    int mp = -1;
    for (int r = m_wg / g + tid; r <= last_m / g; r += 64 * NW) mp = max(mp, q_pos[r]);
    mp = (int)wave_max((float)mp);                     // positions < 2^24: exact in float
    if (lane == 0 && mp >= 0) atomicMax(&s_max_pos, mp);
  }
  __syncthreads();
  const int kv_len = s_max_pos + 1;
  const int n_tiles_all = (kv_len + BKV - 1) / BKV;
  // the merge launch needs the same bound to know which pieces of the key range ran
  if (gridDim.z > 1 && kvh == 0 && blockIdx.z == 0 && tid == 0) wg_tiles[qwg] = n_tiles_all;
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
    q_off[b] = ((long)(row0 + r) * n_q_heads + kvh * g + j) * DH;
    const long q_src = ((long)(q_rows ? q_rows[r] : row0 + r) * n_q_heads + kvh * g + j) * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[b][ks] = *reinterpret_cast<const bf16x8 *>(q + q_src + ks * 16 + 8 * h);
    wave_max_pos = max(wave_max_pos, my_pos[b]);
    wave_min_pos = min(wave_min_pos, my_pos[b]);       // invalid queries (-1) force masking
  }
  wave_max_pos = (int)wave_max((float)wave_max_pos);  // positions < 2^24: exact in float
  wave_min_pos = -(int)wave_max((float)(-wave_min_pos));

  f32x16 oacc[NQB][DB];
  float row_max[NQB], row_sum[NQB];
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    row_max[b] = -INFINITY;
    row_sum[b] = 0.f;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[b][d][i] = 0.f;
  }

  // swizzle: DH = 128 rows start at bank 0 -> 16 slots, f(r) = r & 15; DH = 64 rows alternate
  // between the two bank halves -> 8 slots, f(r) = (r >> 1) & 7
  auto fswz = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };

  // ---- global -> LDS: this lane's share of the loads of one tile ----
  int ld_row[LPT], ld_col[LPT];           // tile row, element offset of the (de-swizzled) chunk
  bool ld_v[LPT];
#pragma unroll
  for (int i = 0; i < LPT; ++i) {
    const int gi = wave + NW * i;                      // load group: first K groups, then V groups
    ld_v[i] = gi >= BKV / RPI;
    const int gl = ld_v[i] ? gi - BKV / RPI : gi;
    ld_row[i] = gl * RPI + lane / CH;
    ld_col[i] = ((lane % CH) ^ fswz(ld_row[i])) * 8 + kvh * DH;
  }
  const bf16 *ld_base[LPT];
#pragma unroll
  for (int i = 0; i < LPT; ++i) ld_base[i] = (ld_v[i] ? vc : kc) + (size_t)ld_row[i] * kv_dim + ld_col[i];
  auto issue = [&](int t) {
    const int t0 = min(t, n_tiles_all - 1) * BKV;     // clamped: every call issues LPT loads
    char *stage = smem + (t % ATT_S) * STAGE;
    const bool whole = t0 + BKV <= kv_len;             // uniform: no row of the tile is past the bound
    const size_t adv = (size_t)t0 * kv_dim;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const bf16 *src = ld_base[i] + adv;
      if (!whole) {
        const int row = min(t0 + ld_row[i], kv_len - 1);
        src = (ld_v[i] ? vc : kc) + (size_t)row * kv_dim + ld_col[i];
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)(stage + (wave + NW * i) * 1024),
                                       16, 0, 0);
    }
  };
  // ---- LDS read offsets of this lane ----
  int k_off[KS];                                       // K operand: row ln (+32 kb), chunk 2 ks + h
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = ln * ROWB + (((2 * ks + h) ^ fswz(ln)) << 4);
  // V operand through the transposing read: lane s of a 16-lane block passes the address of
  // 4 channels (8 bytes) of key K0 + s/4 and receives, for channel C0 + s, the 4 keys K0..K0+3
  int v_off[DB][2];
  {
    const int s16 = lane & 15, qb = lane >> 4;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int key = 8 * a + 4 * (qb >> 1) + (s16 >> 2);               // + 16 u per MFMA
        const int ch = d * 32 + 16 * (qb & 1) + 4 * (s16 & 3);
        v_off[d][a] = TILEB + key * ROWB + (((ch >> 3) ^ fswz(key)) << 4) + (ch & 7) * 2;
      }
  }

#pragma unroll
  for (int sI = 0; sI < ATT_S - 1; ++sI) issue(t_begin + sI);
  for (int t = t_begin; t < n_tiles; ++t) {
    const int t0 = t * BKV;
    __builtin_amdgcn_s_waitcnt(((ATT_S - 2) * LPT) | (7 << 4) | (0 << 8));   // tile t landed; my LDS reads done
    asm volatile("s_barrier" ::: "memory");
    issue(t + ATT_S - 1);
    if (t0 <= wave_max_pos) {  // wave-uniform: tiles wholly in this wave's future are skipped
      const char *ck = smem + (t % ATT_S) * STAGE;
      // ---- S^T = K Q^T ----
      f32x16 sacc[NQB][2];
#pragma unroll
      for (int b = 0; b < NQB; ++b)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[b][kb][i] = 0.f;
      {
        // K operand reads run two steps ahead of the MFMAs that use them (step = (ks, kb))
        constexpr int NSTEP = 2 * KS;
        bf16x8 kf[3];
        kf[0] = *reinterpret_cast<const bf16x8 *>(ck + k_off[0]);
        kf[1] = *reinterpret_cast<const bf16x8 *>(ck + 32 * ROWB + k_off[0]);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
          if (st + 2 < NSTEP)
            kf[(st + 2) % 3] = *reinterpret_cast<const bf16x8 *>(ck + ((st + 2) & 1) * 32 * ROWB + k_off[(st + 2) >> 1]);
#pragma unroll
          for (int b = 0; b < NQB; ++b)
            sacc[b][st & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st % 3], qf[b][st >> 1], sacc[b][st & 1], 0, 0, 0);
        }
      }
      // ---- online softmax (per lane = per query), in the raw score domain: p = 2^((s - m) c) ----
      bf16x8 pf[NQB][4];
      const bool diag = t0 + BKV - 1 > wave_min_pos;     // wave-uniform: some key of the tile is masked
#pragma unroll
      for (int b = 0; b < NQB; ++b) {
        // masked scores are -inf; a query that has seen no key yet (possible inside a later piece of
        // the key range, or for the padding lanes) keeps max = -inf and gets p = 0 everywhere
        float mx = -INFINITY;
        if (diag) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = t0 + kb * 32 + (i >> 2) * 8 + h * 4 + (i & 3);
              sacc[b][kb][i] = key <= my_pos[b] ? sacc[b][kb][i] : -INFINITY;
            }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[b][kb][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float new_max = fmaxf(row_max[b], mx);
        const float neg_mc = new_max == -INFINITY ? 0.f : -new_max * scale_log2e;
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
          const float alpha = new_max > row_max[b] ? __builtin_amdgcn_exp2f((row_max[b] - new_max) * scale_log2e) : 1.f;
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
      {
        // V operand (two transposing reads) fetched one step ahead; step = (u, d)
        constexpr int NSTEP = 4 * DB;
        union VF { s16x4 s[2]; bf16x8 b; } vf[2];
        auto vread = [&](int st, VF &dst) {
          const int u = st / DB, d = st % DB;
          dst.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(ck + u * 16 * ROWB + v_off[d][0]));
          dst.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(ck + u * 16 * ROWB + v_off[d][1]));
        };
        vread(0, vf[0]);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
          if (st + 1 < NSTEP) vread(st + 1, vf[(st + 1) & 1]);
#pragma unroll
          for (int b = 0; b < NQB; ++b)
            oacc[b][st % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st & 1].b, pf[b][st / DB], oacc[b][st % DB], 0, 0, 0);
        }
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(7 << 4);      // drain the clamped tail loads before the workgroup ends
  if (gridDim.z > 1) {
    // ---- partial results: O (un-normalised), running max and sum per (kv head, query, split) ----
#pragma unroll
    for (int b = 0; b < NQB; ++b) {
      const float tot = row_sum[b] + __shfl_xor(row_sum[b], 32, 64);
      if (!valid[b]) continue;
      const int m = m_pad + (wave * NQB + b) * 32 + ln;
      const size_t slot = ((size_t)kvh * n_flat_pad + m) * gridDim.z + blockIdx.z;
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
                                                         int wg_queries, const int32_t *__restrict__ wg_tiles,
                                                         int n_flat_pad, const int32_t *__restrict__ segs,
                                                         int n_segs) {
  constexpr int CG = DH / 4;                           // float4 channel groups per query
  const int g = n_q_heads / n_kv_heads;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)n_kv_heads * n_flat_pad * CG) return;
  const int c = (int)(idx % CG);
  const long qh = idx / CG;                            // kvh * n_flat_pad + padded query number
  const int m_pad = (int)(qh % n_flat_pad), kvh = (int)(qh / n_flat_pad);
  const int qwg = m_pad / wg_queries;
  int seg_qwg0 = 0, row0 = 0;
  if (segs) {
    int lo = 0, hi = n_segs - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (segs[mid * kSegInts + kSegQwg] <= qwg) lo = mid; else hi = mid - 1;
    }
    const int32_t *sg = segs + lo * kSegInts;
    seg_qwg0 = sg[kSegQwg];
    row0 = sg[kSegOutOff];
    n_rows = sg[kSegKeep] + sg[kSegSuffix];
  }
  const int m = m_pad - seg_qwg0 * wg_queries;        // flattened query within its request
  if (m >= n_rows * g) return;                         // padding of the request's last workgroup
  const int n_tiles = wg_tiles[qwg];                 // key tiles of the query's workgroup
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
  *reinterpret_cast<bf16x4 *>(o + ((size_t)(row0 + r) * n_q_heads + kvh * g + j) * DH + c * 4) = w4;
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
                                                       int n_q_heads, int n_kv_heads, float scale_log2e,
                                                       const int32_t *__restrict__ q_rows) {
  __shared__ float sq[4][DH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int idx = blockIdx.x * 4 + wave;
  const bool active = idx < n_rows * n_q_heads;
  const int r = active ? idx / n_q_heads : 0, hq = active ? idx % n_q_heads : 0;
  const int kvh = hq / (n_q_heads / n_kv_heads);
  const int kv_dim = n_kv_heads * DH;
  const float *qrow = q + ((size_t)(q_rows ? q_rows[r] : r) * n_q_heads + hq) * DH;
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

// Workgroup = 8 wavefronts x 32 flattened queries (two wavefronts per SIMD: one runs its softmax
// on the VALU while the other feeds the matrix core, and neither needs more than 256 registers).
constexpr int ATT_NW = 8, ATT_WGQ = 32 * ATT_NW;

// Split plan of the bf16 kernel.  Few query workgroups (the selective layers) leave most CUs idle,
// so the key range is cut into pieces of split_tiles tiles handled by separate workgroups
// (workgroup z takes tiles [z*split_tiles, (z+1)*split_tiles) and exits when its own causal
// range ends before that).  Measured on 359..986-row layers: about one round of 256 workgroups
// in total is the optimum; more pieces cost more in partial results than they gain in balance.
// n_qwg: query workgroups per kv head.
static void attn_split_plan(long n_qwg, int hkv, int n_tokens, int *n_splits, int *split_tiles) {
  const long base = n_qwg * hkv;
  const int max_tiles = (n_tokens + BKV - 1) / BKV;
  int ns = 1;
  if (base < 128) {
    ns = (int)((256 + base - 1) / base);
    ns = std::min(ns, std::max(1, max_tiles / 4));
    ns = std::min(ns, 32);
  } else if (base < 256) {
    ns = std::min(2, std::max(1, max_tiles / 4));
  }
  *split_tiles = (max_tiles + ns - 1) / ns;
  *n_splits = (max_tiles + *split_tiles - 1) / *split_tiles;
}

static long query_workgroups(int n_rows, int hq, int hkv) {
  return ((long)n_rows * (hq / hkv) + ATT_WGQ - 1) / ATT_WGQ;
}

// scratch of a launch with n_qwg query workgroups per kv head and ns key-range pieces: partial O
// and (max, sum) pairs per (kv head, padded query, piece), and one key-tile count per query workgroup
static size_t attn_scratch_floats(long n_qwg, int hkv, int dh, int ns) {
  return (size_t)hkv * n_qwg * ATT_WGQ * ns * (dh + 2) + (size_t)n_qwg;
}

size_t attention_partial_floats(int dtype, int n_rows, int hq, int hkv, int dh, int n_tokens) {
  if (dtype == 0 || n_rows == 0) return 0;
  int ns, st;
  const long n_qwg = query_workgroups(n_rows, hq, hkv);
  attn_split_plan(n_qwg, hkv, n_tokens, &ns, &st);
  if (ns <= 1) return 0;
  return attn_scratch_floats(n_qwg, hkv, dh, ns);
}

// The same for ANY cache length: the piece count never exceeds what the row count alone allows.
size_t attention_partial_floats_bound(int dtype, int n_rows, int hq, int hkv, int dh) {
  if (dtype == 0 || n_rows == 0) return 0;
  const long n_qwg = query_workgroups(n_rows, hq, hkv);
  const long base = n_qwg * hkv;
  const int ns = base < 128 ? (int)std::min<long>(32, (256 + base - 1) / base) : (base < 256 ? 2 : 1);
  if (ns <= 1) return 0;
  return attn_scratch_floats(n_qwg, hkv, dh, ns);
}

long attention_query_workgroups(int n_rows, int hq, int hkv) { return query_workgroups(n_rows, hq, hkv); }

hipError_t launch_attention(int dtype, const void *q, const int32_t *q_rows, const int32_t *q_pos, int n_rows,
                            const void *kc, const void *vc, void *o, int hq, int hkv, int dh,
                            int n_tokens, float *partial, size_t partial_floats, hipStream_t s,
                            const int32_t *segs, int n_segs, long total_qwg) {
  if (n_rows == 0) return hipSuccess;
  const float scale_log2e = kLog2e / sqrtf((float)dh);
  if (dtype == 0) {
    if (segs) return hipErrorInvalidValue;           // the float kernel takes one request per launch
    dim3 grid((n_rows * hq + 3) / 4);
    if (dh == 64)
      hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, (const float *)q, q_pos, n_rows,
                         (const float *)kc, (const float *)vc, (float *)o, hq, hkv, scale_log2e, q_rows);
    else
      hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, (const float *)q, q_pos, n_rows,
                         (const float *)kc, (const float *)vc, (float *)o, hq, hkv, scale_log2e, q_rows);
    return hipGetLastError();
  }
  const long n_qwg = segs ? total_qwg : query_workgroups(n_rows, hq, hkv);
  int n_splits, split_tiles;
  attn_split_plan(n_qwg, hkv, n_tokens, &n_splits, &split_tiles);
  while (n_splits > 1 && (!partial || partial_floats < attn_scratch_floats(n_qwg, hkv, dh, n_splits))) {
    // scratch is short: fewer, longer pieces (down to one workgroup walking all keys)
    const int max_tiles = (n_tokens + BKV - 1) / BKV;
    const int ns = n_splits - 1;
    split_tiles = (max_tiles + ns - 1) / ns;
    n_splits = (max_tiles + split_tiles - 1) / split_tiles;
  }
  const int wgq = ATT_WGQ;
  const size_t slots = (size_t)hkv * n_qwg * ATT_WGQ * n_splits;
  float *part_o = partial;
  float *part_ml = partial ? partial + slots * dh : nullptr;
  int32_t *wg_tiles = partial ? reinterpret_cast<int32_t *>(part_ml + slots * 2) : nullptr;
#define CB_ATTN(DH_, NQB_, NW_)                                                                     \
  do {                                                                                              \
    constexpr int smem = ATT_S * 2 * BKV * DH_ * 2;                                                 \
    static std::once_flag once_;                                                                    \
    std::call_once(once_, [] {                                                                      \
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<DH_, NQB_, NW_>),  \
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem);                  \
    });                                                                                             \
    hipLaunchKernelGGL((attn_bf16_kernel<DH_, NQB_, NW_>), dim3(hkv, (unsigned)n_qwg, n_splits),    \
                       dim3(64 * NW_), smem, s, (const bf16 *)q, q_pos, n_rows, (const bf16 *)kc,   \
                       (const bf16 *)vc, (bf16 *)o, hq, hkv, scale_log2e, split_tiles, part_o,      \
                       part_ml, q_rows, wg_tiles, segs, n_segs);                                    \
  } while (0)
  if (dh == 64) CB_ATTN(64, 1, ATT_NW);
  else CB_ATTN(128, 1, ATT_NW);
#undef CB_ATTN
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1) return e;
  const int n_flat_pad = (int)n_qwg * ATT_WGQ;
  const long total = (long)hkv * n_flat_pad * (dh / 4);
  const dim3 mgrid((unsigned)((total + 255) / 256));
  if (dh == 64)
    hipLaunchKernelGGL(attn_merge_kernel<64>, mgrid, dim3(256), 0, s, part_o, part_ml, q_pos, n_rows,
                       (bf16 *)o, hq, hkv, n_splits, split_tiles, wgq, wg_tiles, n_flat_pad, segs, n_segs);
  else
    hipLaunchKernelGGL(attn_merge_kernel<128>, mgrid, dim3(256), 0, s, part_o, part_ml, q_pos, n_rows,
                       (bf16 *)o, hq, hkv, n_splits, split_tiles, wgq, wg_tiles, n_flat_pad, segs, n_segs);
  return hipGetLastError();
}

}  // namespace cb
