// Projections of the selectively recomputed rows (paper Sec. 4.2: Q/K/V of the
// selected tokens, then the ordinary attention and the rest of the layer).
// C[M, N] = A[M, K] * W[N, K]^T with both operands K-contiguous.
//
// bf16 storage: matrix-core MFMAs with float accumulation.  The main kernel
// (gemm_bf16_dma_kernel, v_mfma_f32_16x16x32_bf16) streams (32*I) x (64*NB) x 64 tiles through LDS
// rings filled by direct global->LDS loads, with an XCD-aware tile order; a simpler register-staged
// 128x128x64 kernel (v_mfma_f32_32x32x16_bf16) covers K that is not a multiple of 64.
// float storage: plain FMA tiles (parity mode, not tuned).
// The SwiGLU and float-output epilogues work straight from the accumulator registers (a lane
// holds four adjacent columns of a row); the segment epilogue parks the tile in LDS and walks it
// row-major, 4 adjacent columns per lane, which lets the two wavefront halves of an operand-pair
// tile be added and gives the half-split rotary order its partner column.  A problem with too few tiles to fill the chip is split along K: the main
// kernel then stores raw partial sums and a second kernel adds them in a fixed order
// (no atomics: bitwise reproducible) and applies the epilogue.
// Epilogues:
//   EPI_SEG    up to three column segments (Q | K | V), each with its own weight
//              matrix, destination, optional destination-row map (scatter into the
//              KV cache) and optional rotary embedding at the row's position
//   EPI_SWIGLU silu(x Wg^T) * (x Wu^T)
//   EPI_F32    float output (+ residual)
#include "common.h"
#include "kernels.h"
#include <algorithm>
#include <cstdint>
#include <mutex>

namespace cb {

struct GemmParams {
  const void *a;
  int lda;
  const int32_t *a_rows;
  int M, K, N;          // N: total output columns (EPI_SWIGLU: d_ff)
  int n_seg;
  const void *w[3];
  const float *w_scale[3];   // non-NULL (direct-to-LDS kernel only): w[i] holds int8 values and output column c of
                             // segment i is w_scale[i][c] times the sum over them
  int nb[4];            // column boundaries of the segments
  void *dst[3];
  int ld[3];
  const int32_t *row_map[3];
  int rope[3];
  const float2 *rope_tab;
  const int32_t *row_pos;
  int head_dim;
  int rope_half;        // rotary pairs (i, i + head_dim/2) instead of (2i, 2i+1)
  int raw_partial;      // the main kernel only parks its sums in `partial`; the finish launch applies the epilogue
  int a_lo_off;         // > 0: the activations are a (high, low) bf16 pair, the low parts a_lo_off elements after
                        // the high parts of the same row; both are multiplied and their products added
  float *out_f32;
  const float *resid;
  const int32_t *resid_rows;
  float *partial;
  // finish launch of EPI_SEG: squared distance of the stored new values of segment s from row
  // dev_row[r] of dev_cache[s] (pitch = the segment's width), summed over the segments, for rows < n_dev
  float *dev_out;
  int n_dev;
  const void *dev_cache[3];
  const int32_t *dev_row;
  // finish launch of EPI_F32: RMSNorm of the finished row (gain norm_gain, NULL: none) into norm_out
  // (pitch norm_ld); norm_lo_off > 0 also stores the rounding remainder norm_lo_off elements further on
  const void *norm_gain;
  void *norm_out;
  int norm_ld, norm_lo_off;
  float norm_eps;
  int splits, k_per_split;
  // EPI_SWIGLU: workgroup ids >= tail_first share the tiles of the last, partly filled round of
  // workgroups, tail_splits of them per tile, each over tail_k_per_split of K
  int tail_first, tail_splits, tail_k_per_split;
  // K split dealt to the XCDs (splits = 2, 4 or 8): XCD x computes split x % splits of the n-tiles
  // congruent to x / splits mod 8 / splits, so each L2 holds only its own K slice of the activations
  int xcd_split;
};

// weight row that feeds tile column gc (clamped into range)
// (es: elements of T per weight element, for byte-addressed callers)
template <typename T, int EPI>
__device__ __forceinline__ const T *weight_row(const GemmParams &p, int gc, int half_bn, int n0, int c, int es = 1) {
  if (EPI == EPI_SWIGLU) {
    // tile columns [0, half) come from the gate matrix, [half, 2*half) from the up matrix
    int which = c >= half_bn;
    int row = min(n0 + (which ? c - half_bn : c), p.N - 1);
    return reinterpret_cast<const T *>(p.w[which]) + (size_t)row * p.K * es;
  }
  gc = min(gc, p.N - 1);
  int s = 0;
  if (p.n_seg > 1 && gc >= p.nb[1]) s = 1;
  if (p.n_seg > 2 && gc >= p.nb[2]) s = 2;
  return reinterpret_cast<const T *>(p.w[s]) + (size_t)(gc - p.nb[s]) * p.K * es;
}

template <typename T> __device__ __forceinline__ float4 load4(const T *s);
template <> __device__ __forceinline__ float4 load4<float>(const float *s) { return *reinterpret_cast<const float4 *>(s); }
template <> __device__ __forceinline__ float4 load4<bf16>(const bf16 *s) {
  const bf16x4 v = *reinterpret_cast<const bf16x4 *>(s);
  return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}
// the value a float becomes when stored in the storage type
template <typename T> __device__ __forceinline__ float as_stored(float v) { return to_f32(from_f32<T>(v)); }
template <typename T> __device__ __forceinline__ void store4(T *d, float a, float b, float c, float e);
template <> __device__ __forceinline__ void store4<float>(float *d, float a, float b, float c, float e) {
  *reinterpret_cast<float4 *>(d) = make_float4(a, b, c, e);
}
template <> __device__ __forceinline__ void store4<bf16>(bf16 *d, float a, float b, float c, float e) {
  bf16x4 v = {(bf16)a, (bf16)b, (bf16)c, (bf16)e};
  *reinterpret_cast<bf16x4 *>(d) = v;
}

// Column offset from an output column to the channel it forms a rotary pair with when heads are in
// the (i, i + head_dim/2) order.  Segments are whole heads, so gc % head_dim is the channel.
__device__ __forceinline__ int rope_partner_offset(const GemmParams &p, int gc) {
  const int half = p.head_dim / 2;
  return gc % p.head_dim < half ? half : -half;
}

// EPI_SEG: the values of output columns gc .. gc+3 of logical row gr after the rotary embedding
// (a no-op for segments without it); *seg / *lcol receive the segment and the column inside it.
// u: with p.rope_half, the values of columns gc + rope_partner_offset .. + 3.
__device__ __forceinline__ float4 seg_rotate(float4 v, float4 u, int gr, int gc, const GemmParams &p, int *seg,
                                             int *lcol) {
  int s = 0;
  if (p.n_seg > 1 && gc >= p.nb[1]) s = 1;
  if (p.n_seg > 2 && gc >= p.nb[2]) s = 2;
  const int lc = gc - p.nb[s];
  *seg = s;
  *lcol = lc;
  if (!p.rope[s]) return v;
  const int half = p.head_dim / 2;
  float4 o;
  if (p.rope_half) {
    const int ch = lc % p.head_dim;
    const bool first = ch < half;
    const float2 *t = p.rope_tab + (size_t)p.row_pos[gr] * half + (first ? ch : ch - half);
    const float2 c0 = t[0], c1 = t[1], c2 = t[2], c3 = t[3];
    if (first) {          // x0' = x0 cos - x1 sin, the partner holds x1
      o.x = v.x * c0.x - u.x * c0.y;
      o.y = v.y * c1.x - u.y * c1.y;
      o.z = v.z * c2.x - u.z * c2.y;
      o.w = v.w * c3.x - u.w * c3.y;
    } else {              // x1' = x0 sin + x1 cos, the partner holds x0
      o.x = u.x * c0.y + v.x * c0.x;
      o.y = u.y * c1.y + v.y * c1.x;
      o.z = u.z * c2.y + v.z * c2.x;
      o.w = u.w * c3.y + v.w * c3.x;
    }
  } else {
    const float2 *t = p.rope_tab + (size_t)p.row_pos[gr] * half + (lc % p.head_dim) / 2;
    const float2 c0 = t[0], c1 = t[1];
    o.x = v.x * c0.x - v.y * c0.y;
    o.y = v.x * c0.y + v.y * c0.x;
    o.z = v.z * c1.x - v.w * c1.y;
    o.w = v.z * c1.y + v.w * c1.x;
  }
  return o;
}

// One group of 4 adjacent output columns (gc .. gc+3) of logical row gr.
// v: accumulated values; u: EPI_SWIGLU: the matching "up" values; EPI_SEG with p.rope_half: the
// values of columns gc + rope_partner_offset .. + 3.  (EPI_F32 sums always go through `partial`
// and are finished by resid_norm_finish_kernel.)
template <typename T, int EPI>
__device__ __forceinline__ void apply_epilogue(float4 v, float4 u, int gr, int gc, const GemmParams &p) {
  if (EPI == EPI_SEG) {
    int s, lc;
    v = seg_rotate(v, u, gr, gc, p, &s, &lc);
    const int dr = p.row_map[s] ? p.row_map[s][gr] : gr;
    store4<T>(reinterpret_cast<T *>(p.dst[s]) + (size_t)dr * p.ld[s] + lc, v.x, v.y, v.z, v.w);
  } else if (EPI == EPI_SWIGLU) {
    float4 o;
    o.x = v.x / (1.f + expf(-v.x)) * u.x;
    o.y = v.y / (1.f + expf(-v.y)) * u.y;
    o.z = v.z / (1.f + expf(-v.z)) * u.z;
    o.w = v.w / (1.f + expf(-v.w)) * u.w;
    store4<T>(reinterpret_cast<T *>(p.dst[0]) + (size_t)gr * p.ld[0] + gc, o.x, o.y, o.z, o.w);
  }
}

// Walks `rows` x BN floats parked in LDS (pitch `pitch`); m0/n0: first logical row /
// first output column of this block of rows; z: K-split index of the workgroup.
template <typename T, int EPI, int BN>
__device__ __forceinline__ void lds_epilogue(const float *sC, int pitch, int rows, int m0, int n0, int z,
                                             const GemmParams &p) {
  constexpr int OUT_COLS = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int GROUPS = OUT_COLS / 4;
  for (int g = threadIdx.x; g < rows * GROUPS; g += (int)blockDim.x) {
    const int r = g / GROUPS, c = (g % GROUPS) * 4;
    const int gr = m0 + r, gc = n0 + c;
    if (gr >= p.M || gc >= p.N) continue;
    const float4 v = *reinterpret_cast<const float4 *>(sC + r * pitch + c);
    if (EPI != EPI_SWIGLU && (p.splits > 1 || p.raw_partial)) {
      *reinterpret_cast<float4 *>(p.partial + ((size_t)z * p.M + gr) * p.N + gc) = v;
    } else {
      float4 u = v;
      if (EPI == EPI_SWIGLU) u = *reinterpret_cast<const float4 *>(sC + r * pitch + OUT_COLS + c);
      // the tile holds whole heads (its width is a multiple of head_dim), so the partner is parked too
      if (EPI == EPI_SEG && p.rope_half)
        u = *reinterpret_cast<const float4 *>(sC + r * pitch + c + rope_partner_offset(p, gc));
      apply_epilogue<T, EPI>(v, u, gr, gc, p);
    }
  }
}

// ---------------------------------------------------------------------------
// Main bf16 kernel.
//   tile        BM = 32*I rows (I = 2,4,6,8) x BN = 64*NB columns (NB = 4, or 2 when that
//               fills the CUs better) x 64 k per stage (128-byte
//               rows: every global request is a whole cache line)
//   wavefronts  NWV = 4 as 2 x 2 (128-column tiles; two such workgroups share a CU when the
//               rings fit twice) or NWV = 8 as 2 x 4 (256-column tiles: two wavefronts per
//               SIMD, each (BM/2) x 64).  A wavefront's sub-tile is cut into 16 x 16 blocks, one
//               v_mfma_f32_16x16x32_bf16 each per 32-deep k-step.  Operand reads are issued by
//               hand (inline ds_read_b128 + explicit s_waitcnt lgkmcnt) one half-step (half of
//               the wavefront's rows of one k-step) ahead of the MFMAs that use them, slotted
//               between those MFMAs.
//   LDS rings   activation tile (BM rows x 128 bytes): 2 stages; weight tile (256 rows x
//               128 bytes): the 3-4 stages that still fit in 160 KB -- weights stream
//               from HBM once and need the deeper queue, activations mostly hit L2.
//               Both are filled by global_load_lds_dwordx4 (no register staging).  A
//               wavefront-wide load writes 1 KB contiguously (lane l -> byte 16*l),
//               i.e. 8 rows x 8 chunks; lane l fetches global chunk (l%8) ^ f(row) of
//               row l/8, f(r) = (r&7) ^ ((r>>3)&1), so that the later 16-byte operand
//               reads of 8 (and of 16) consecutive rows hit distinct bank groups
//               (XOR swizzle instead of padding).
//   pipeline    one barrier per k-tile, placed before the LAST half-step of tile t: by
//               then every wavefront holds its last fragments of stage t in
//               registers, so after "tile t+1 landed" (s_waitcnt vmcnt) + barrier the
//               stage is refilled with tile t+S and the first fragments of tile t+1
//               are requested while the last MFMAs of tile t run.  The loads of a tile
//               are spread over four half-steps (no burst on the memory pipeline).  The
//               compiler does not order LDS reads against these loads, hence the
//               explicit waits; plain s_barrier is used because __syncthreads()
//               would drain every outstanding load.
//   tile order  1-D grid; workgroup id -> (xcd = id % 8, j = id / 8); an XCD walks
//               its own n-tiles (n % 8 == xcd) in groups of 8 m-tiles (xcd_tile), so the
//               workgroups that share a weight or activation tile run together on one L2.
//               With a K split of 2, 4 or 8 the XCDs are dealt one split each (GemmParams::xcd_split),
//               so an L2 only ever fetches its own K slice of the activations.
// Requires K % 64 == 0 and k_per_split % 64 == 0.
// ---------------------------------------------------------------------------
constexpr int DMA_BK = 64;
// Two rings: the activation tile (mostly L2 hits) is double-buffered, the weight tile (streamed
// from HBM, long latency) gets every remaining stage that fits in 160 KB, up to 4.
constexpr int DMA_SA = 2;
// w8: int8 weights, 64 bytes per weight row and stage instead of 128, so up to 6 stages fit.
constexpr int dma_w_stages(int I, int BN, bool w8 = false) {
  const int stage = BN * (w8 ? 64 : 128), cap = w8 ? 6 : 4;
  if (BN == 128 && I <= 4) {                           // <= 80 KB: two workgroups per CU
    const int n = (80 * 1024 - DMA_SA * 32 * I * 128) / stage;
    return w8 ? (n > cap ? cap : n) : 3;
  }
  const int left = 160 * 1024 - DMA_SA * 32 * I * 128;
  return left / stage > cap ? cap : left / stage;
}
constexpr int dma_smem_bytes(int I, int BN, bool w8 = false) {
  const int ring = DMA_SA * 32 * I * 128 + dma_w_stages(I, BN, w8) * BN * (w8 ? 64 : 128);
  const int park = (I < 4 ? 32 * I : 128) * (BN + 4) * 4;
  return ring > park ? ring : park;
}

#define CB_GLDS16(gptr, lptr)                                                              \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr), \
                                   (__attribute__((address_space(3))) void *)(lptr), 16, 0, 0)

// LDS operand read issued by hand: the result registers are valid only after a matching
// lds_wait<N>() (N = number of younger reads that may still be in flight).
template <int OFF> __device__ __forceinline__ void lds_read16(bf16x8 &dst, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
template <int OFF> __device__ __forceinline__ void lds_read8(u32x2 &dst, unsigned addr) {
  asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// eight int8 weights -> the bf16 MFMA fragment (exact: |value| <= 128 needs 8 significant bits)
__device__ __forceinline__ bf16x8 int8x8_to_bf16(u32x2 q) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)(float)(int)(signed char)(q[e >> 2] >> (8 * (e & 3)));
  return r;
}
template <int N> __device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N)); }
// ties a fragment to the preceding wait so that no use of it is scheduled before the wait
__device__ __forceinline__ void lds_pin(bf16x8 &f) { asm volatile("" : "+v"(f)); }
template <int N> __device__ __forceinline__ void vm_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Tile walked by the j-th workgroup of an XCD (j < nblk * tiles_m).  The XCD owns the n-tiles
// congruent to its index mod 8 (nblk of them); row tiles are taken in groups of 8 and, inside a
// group, the row tiles of one n-tile come first.  The ~32 workgroups resident on an XCD then
// cover about 4 n-tiles x 8 m-tiles, so every weight tile and every activation tile fetched into
// its L2 serves several of them (with all row tiles innermost, a problem with many row tiles
// would share no activation tile at all).
constexpr int kGroupM = 8;
__device__ __forceinline__ void xcd_tile(int j, int xcd, int tiles_m, int nblk, int *nt, int *mt, int stride = 8) {
  const int per_group = nblk * kGroupM, full = tiles_m / kGroupM;
  int g = j / per_group, r, gm;
  if (g >= full) { g = full; r = j - full * per_group; gm = tiles_m - full * kGroupM; }
  else { r = j - g * per_group; gm = kGroupM; }
  *nt = xcd + stride * (r / gm);
  *mt = g * kGroupM + r % gm;
}

// silu(gate) * up from one wavefront's accumulators (RB x CB blocks of 16 x 16): blocks
// 0..CB/2-1 of a lane hold gate columns, blocks CB/2..CB-1 the same columns of the up matrix;
// lane l holds row (l % 16) and columns 4*(l/16) .. +3 of each block.  row0 / col0: first output
// row / column of the wavefront.
template <int RB, int CB>
__device__ __forceinline__ void swiglu_from_registers(const f32x4 (&acc)[RB][CB], const GemmParams &p,
                                                      int row0, int col0, int lane) {
  const int l_row = lane & 15, l_col = (lane >> 4) * 4;
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int gr = row0 + i * 16 + l_row;
    if (gr >= p.M) continue;
    bf16 *orow = reinterpret_cast<bf16 *>(p.dst[0]) + (size_t)gr * p.ld[0];
#pragma unroll
    for (int jb = 0; jb < CB / 2; ++jb) {
      const int gc = col0 + jb * 16 + l_col;
      float o[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float gt = acc[i][jb][r], up = acc[i][jb + CB / 2][r];
        // silu(g) * u = g * u / (1 + 2^(-g log2 e))
        const float den = 1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt);
        o[r] = gt * up * __builtin_amdgcn_rcpf(den);
      }
      if (gc + 3 < p.N) {
        store4<bf16>(orow + gc, o[0], o[1], o[2], o[3]);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (gc + r < p.N) orow[gc + r] = (bf16)o[r];
      }
    }
  }
}

// Completes the tiles that several workgroups of the SwiGLU launch shared along K.  The partial
// sums lie in register order: [slot][split][wavefront][16-row block i][16-column block jb][lane][4].
// One wavefront here owns four (wavefront, i, gate block jb) units of a tile in turn: it adds the gate and
// the up block over the splits in ascending K order and applies the epilogue.
template <int I, int NB, int NWV>
__global__ __launch_bounds__(256) void swiglu_tail_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int IH = I / 2, BM = 32 * I, BN = 64 * NB, WN = NWV / 2, NBW = 2 * NB / WN;
  constexpr int RB = I, CB = 2 * NBW, HB = CB / 2;
  constexpr int UNITS = NWV * RB * HB;                    // per tile; a multiple of 16
  const int lane = threadIdx.x & 63;
  const int slot = blockIdx.x / (UNITS / 16);
  const int xcd = slot & 7, j = (p.tail_first >> 3) + (slot >> 3);
  int nt, mt;
  xcd_tile(j, xcd, tiles_m, (tiles_n + 7) >> 3, &nt, &mt);
  if (nt >= tiles_n) return;
  const int l_row = lane & 15, l_col = (lane >> 4) * 4;
  for (int q = 0; q < 4; ++q) {
    const int u = ((blockIdx.x % (UNITS / 16)) * 4 + (threadIdx.x >> 6)) * 4 + q;
    const int wave = u / (RB * HB), i = (u / HB) % RB, jb = u % HB;
    const float *pg = p.partial + (size_t)slot * p.tail_splits * (BM * BN) + (size_t)wave * (RB * CB * 4 * 64) +
                      (size_t)((i * CB + jb) * 64 + lane) * 4;
    f32x4 gate = {0.f, 0.f, 0.f, 0.f}, up = {0.f, 0.f, 0.f, 0.f};
    for (int zz = 0; zz < p.tail_splits; ++zz, pg += BM * BN) {
      gate += *reinterpret_cast<const f32x4 *>(pg);
      up += *reinterpret_cast<const f32x4 *>(pg + HB * 64 * 4);
    }
    const int wm = wave / WN, wn = wave % WN;
    const int gc = nt * (BN / 2) + wn * (BN / WN / 2) + jb * 16 + l_col;
    const int gr = mt * BM + wm * IH * 32 + i * 16 + l_row;
    if (gr >= p.M) continue;
    bf16 *orow = reinterpret_cast<bf16 *>(p.dst[0]) + (size_t)gr * p.ld[0];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (gc + r >= p.N) continue;
      const float den = 1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gate[r]);
      orow[gc + r] = (bf16)(gate[r] * up[r] * __builtin_amdgcn_rcpf(den));
    }
  }
}

// HL (EPI_SEG only): the activations are (high, low) bf16 pairs.  The activation tile then holds
// BM/2 logical rows twice -- their high parts in its first half, their low parts in its second --
// so the wavefronts with wm = 0 multiply the high parts and those with wm = 1 the low parts of the
// SAME output rows, and the two sets of sums are added in LDS before the epilogue.
// W8: the weights are int8 (one byte per element in memory and in LDS, half the traffic of both); a fragment
// is expanded to bf16 in registers right before its k-step and the per-column scales multiply the finished sums.
template <int I, int NB, int EPI, int NWV, bool HL = false, bool W8 = false>
__global__ __launch_bounds__(64 * NWV) void gemm_bf16_dma_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int BM = 32 * I, BN = 64 * NB, SW = dma_w_stages(I, BN, W8), DMA_CP = BN + 4;
  constexpr int WE = W8 ? 1 : 2;                         // bytes per weight element
  constexpr int BMO = HL ? BM / 2 : BM;                  // output rows per tile
  static_assert(!HL || EPI == EPI_SEG, "operand pairs are for the K/V projection only");
  constexpr int A_STAGE = BM * 128, W_STAGE = BN * 64 * WE, W_RING = DMA_SA * A_STAGE;
  constexpr int WN = NWV / 2;                            // wavefronts as 2 x WN
  constexpr int NBW = 2 * NB / WN;                       // 32-column groups per wavefront
  constexpr int LA = BM / (8 * NWV), LW = W_STAGE / (1024 * NWV);   // 16-byte loads per lane per tile (1 KB per wavefront each)
  static_assert(LW >= 2 && LW % 2 == 0, "the load schedule issues a weight tile in two halves");
  static_assert(SW >= 3, "the vmcnt bookkeeping below assumes at least 3 weight stages");
  constexpr int IH = I / 2;                              // 32-row groups per wavefront
  constexpr int RB = I, CB = 2 * NBW;                    // 16-row / 16-column MFMA blocks per wavefront
  constexpr int OUT_COLS = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  // scalar, so that the LDS targets of the loads are computed on the scalar unit: a vector instruction of one
  // wavefront does not overlap the MFMAs of the other wavefront on its SIMD, it costs matrix-core time
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;              // 2 x WN wavefronts, (BM/2) x (BN/WN) each

  // XCD-aware tile order
  int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, tail_z = -1;
  if (EPI == EPI_SWIGLU && (int)blockIdx.x >= p.tail_first) {
    const int v = ((int)blockIdx.x - p.tail_first) >> 3;
    tail_z = v % p.tail_splits;
    j = (p.tail_first >> 3) + v / p.tail_splits;
  }
  int z, nt, mt;
  if (EPI != EPI_SWIGLU && p.xcd_split) {
    const int groups = 8 / p.splits;                 // XCDs that share one split
    z = xcd % p.splits;
    xcd_tile(j, xcd / p.splits, tiles_m, (tiles_n + groups - 1) / groups, &nt, &mt, groups);
  } else {
    const int nblk = (tiles_n + 7) >> 3;
    const int per_z = nblk * tiles_m;
    z = j / per_z;
    xcd_tile(j - z * per_z, xcd, tiles_m, nblk, &nt, &mt);
  }
  if (nt >= tiles_n) return;
  const int m0 = mt * BMO, n0 = nt * OUT_COLS;
  const int kps = tail_z >= 0 ? p.tail_k_per_split : p.k_per_split;
  const int kb = (tail_z >= 0 ? tail_z : z) * kps;
  const int ke = min(p.K, kb + kps);
  const int nk = (ke - kb) / DMA_BK;

  // global source of each of this lane's loads per tile (row pointer + swizzled chunk)
  const bf16 *src_a[LA];
  const char *src_w[LW];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int r = (wave + NWV * i) * 8 + (lane >> 3);         // row of the activation tile
    const int chunk = (lane & 7) ^ ((r & 7) ^ ((r >> 3) & 1));
    int ar = min(m0 + (HL ? r % BMO : r), p.M - 1);
    if (p.a_rows) ar = p.a_rows[ar];
    src_a[i] = reinterpret_cast<const bf16 *>(p.a) + (size_t)ar * p.lda + chunk * 8 + kb +
               (HL && r >= BMO ? p.a_lo_off : 0);
  }
#pragma unroll
  for (int i = 0; i < LW; ++i) {
    // a wavefront-wide load brings 1 KB: 8 rows of 128 bytes, or 16 rows of 64 bytes of int8 weights, whose four
    // 16-byte chunks are swizzled by f8(r) = (r >> 2) & 3 (the 8-byte fragment reads of 16 rows then hit 64 banks)
    const int r = W8 ? (wave + NWV * i) * 16 + (lane >> 2) : (wave + NWV * i) * 8 + (lane >> 3);   // row of the weight tile
    const int chunk = W8 ? (lane & 3) ^ ((r >> 2) & 3) : (lane & 7) ^ ((r & 7) ^ ((r >> 3) & 1));
    const char *wrow;
    if (EPI == EPI_SWIGLU) {
      // each wavefront's half of the tile columns holds its gate columns followed by the SAME
      // up columns, so that a lane ends up with gate and up of one output element
      constexpr int WC = BN / WN, HC = WC / 2;         // columns per wavefront / per operand
      const int which = (r % WC) / HC, oc = min(n0 + (r / WC) * HC + (r % HC), p.N - 1);
      wrow = reinterpret_cast<const char *>(p.w[which]) + (size_t)oc * p.K * WE;
    } else {
      wrow = reinterpret_cast<const char *>(weight_row<char, EPI>(p, n0 + r, BN / 2, n0, r, WE));
    }
    src_w[i] = wrow + chunk * 16 + kb * WE;
  }
  // load number idx of tile t: idx < LA activation, else weight; tile indices are clamped so
  // that every tile issues the same number of loads
  auto issue_one = [&](int t, int idx) {
    if (idx < LA) {
      const int k0 = min(t, nk - 1) * DMA_BK;
      CB_GLDS16(src_a[idx] + k0, smem + (t % DMA_SA) * A_STAGE + (wave + NWV * idx) * 1024);
    } else {
      const int tw = t + SW - DMA_SA;                 // the weight ring runs SW - 2 tiles further ahead
      const int k0 = min(tw, nk - 1) * DMA_BK;
      CB_GLDS16(src_w[idx - LA] + k0 * WE, smem + W_RING + (tw % SW) * W_STAGE + (wave + NWV * (idx - LA)) * 1024);
    }
  };
  auto issue_w = [&](int t) {
    const int k0 = min(t, nk - 1) * DMA_BK;
#pragma unroll
    for (int i = 0; i < LW; ++i)
      CB_GLDS16(src_w[i] + k0 * WE, smem + W_RING + (t % SW) * W_STAGE + (wave + NWV * i) * 1024);
  };

  // v_mfma_f32_16x16x32_bf16 with the WEIGHT fragment as its first operand: block (i, jb) of a wavefront is
  // 16 output rows x 16 output columns, and lane l ends up with row (l % 16), columns 4*(l/16) .. +3 of it,
  // i.e. four adjacent output columns (one 16-byte store, one rotary pair twice over).  Of the two MFMA
  // shapes this one sustains the higher rate on this chip once the operands are real data: the chip is
  // power-limited then, and the 16x16 shape moves half the accumulator registers per flop.
  f32x4 acc[RB][CB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int jb = 0; jb < CB; ++jb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][jb][r] = 0.f;

  if (nk > 0) {
    // A fragment is 16 rows x 32 k: lane l reads the 16-byte chunk (l / 16) of the k-step's 64 bytes of row (l % 16)
    const int sw = (lane & 7) ^ ((lane >> 3) & 1);
    int rd[2];                                                    // k-step ks (32 deep) reads chunk 4*ks + l/16
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) rd[ks] = (lane & 15) * 128 + (((4 * ks + (lane >> 4)) ^ sw) << 4);
    const int a_off = (wm * IH * 32) * 128, b_off = (wn * (BN / WN)) * 128;
    int blk_ok = 0;                                    // bit i: 16-row block i of this wavefront holds a real row
#pragma unroll
    for (int i = 0; i < RB; ++i) blk_ok |= (m0 + (HL ? 0 : wm * IH * 32) + i * 16 < p.M) << i;
    blk_ok = __builtin_amdgcn_readfirstlane(blk_ok);
    // one scalar flag per block, re-read through an empty asm at every test: left alone the compiler hoists the
    // tests out of the loop as lane masks and rebuilds their complements with vector instructions inside it
    // (14 of the 48 vector instructions the loop had per k-tile; with these two changes it has 16)
    int row_ok[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) row_ok[i] = (blk_ok >> i) & 1;
    auto block_ok = [&](int i) {
      int v = row_ok[i];
      asm volatile("" : "+s"(v));
      return v != 0;
    };
    // A k-tile is walked in four HALF-STEPS hs = 2*ks + h: k-step ks (32 deep), row half h (IH of the wavefront's
    // 16-row blocks).  Activation fragments are double-buffered per half-step, weight fragments per k-step.
    // (int8 weights: the raw 8-byte fragments of the next k-step wait in fq and are expanded into fb[0] as the
    // k-step begins, each right before the first MFMA that uses it)
    bf16x8 fa[2][IH], fb[W8 ? 1 : 2][CB];
    u32x2 fq[W8 ? CB : 1];
    int rd8[2];                                        // int8 weights: 8 bytes of row (l % 16), k-step ks, k group l / 16
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      rd8[ks] = (lane & 15) * 64 + (((2 * ks + (lane >> 5)) ^ ((lane >> 2) & 3)) << 4) + ((lane >> 4) & 1) * 8;
    const int b_off8 = (wn * (BN / WN)) * 64;
    constexpr int NM = IH * CB;                        // MFMAs per half-step per wavefront
    constexpr int NL = LA + LW;                        // loads per tile per lane
    constexpr int NSLOT = NM > IH + CB ? NM : IH + CB;
    // fragment number n (16 rows each, 2 KB apart) of the operand whose first fragment this lane reads at `base`
    auto read_wq = [&](u32x2 &dst, unsigned base, int n) {     // int8 weight fragment n (16 rows, 1 KB apart)
      switch (n) {
        case 0: lds_read8<0>(dst, base); break;
        case 1: lds_read8<1024>(dst, base); break;
        case 2: lds_read8<2048>(dst, base); break;
        case 3: lds_read8<3072>(dst, base); break;
        case 4: lds_read8<4096>(dst, base); break;
        case 5: lds_read8<5120>(dst, base); break;
        case 6: lds_read8<6144>(dst, base); break;
        default: lds_read8<7168>(dst, base); break;
      }
    };
    auto read_frag = [&](bf16x8 &dst, unsigned base, int n) {
      switch (n) {
        case 0: lds_read16<0>(dst, base); break;
        case 1: lds_read16<2048>(dst, base); break;
        case 2: lds_read16<4096>(dst, base); break;
        case 3: lds_read16<6144>(dst, base); break;
        case 4: lds_read16<8192>(dst, base); break;
        case 5: lds_read16<10240>(dst, base); break;
        case 6: lds_read16<12288>(dst, base); break;
        default: lds_read16<14336>(dst, base); break;
      }
    };
    const unsigned lds0 = (unsigned)(size_t)smem;
    // One half-step hs of the current tile: its MFMAs, with the operand reads of the half-step that follows
    // (half-step hsn of tile tn: its activation fragments, and the weight fragments too when it opens a
    // k-step) and the global loads q0 .. q1-1 of tile tl slotted in between them.  A wavefront issues in
    // order, so anything not placed between two MFMAs would add to the MFMA time.
    auto step = [&](int hs, bool next_reads, int tn, int hsn, int q0, int q1, int tl) {
      const int ab = hs & 1, bb = W8 ? 0 : (hs >> 1) & 1, h = hs & 1;
      const int nab = hsn & 1, nbb = W8 ? 0 : (hsn >> 1) & 1;
      const bool with_w = (hsn & 1) == 0;
      const unsigned base_a = lds0 + (tn % DMA_SA) * A_STAGE + a_off + (hsn & 1) * (IH * 2048) + rd[hsn >> 1];
      const unsigned base_w = lds0 + W_RING + (tn % SW) * W_STAGE + (W8 ? b_off8 + rd8[hsn >> 1] : b_off + rd[hsn >> 1]);
      const int n_reads = next_reads ? IH + (with_w ? CB : 0) : 0;
      // what rides along in MFMA slot j: the global loads q0 .. q1-1 of tile tl, spread evenly over the slots of
      // this half-step, and one operand read of the next half-step
      auto slot_work = [&](int j) {
#pragma unroll
        for (int q = q0 + j * (q1 - q0) / NSLOT; q < q0 + (j + 1) * (q1 - q0) / NSLOT; ++q) issue_one(tl, q);
        if (j < n_reads) {
          if (j < IH) read_frag(fa[nab][j], base_a, j);
          else if (W8) read_wq(fq[j - IH], base_w, j - IH);
          else read_frag(fb[nbb][j - IH], base_w, j - IH);
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      if (W8 && h == 0) {
        // a k-step begins with int8 weights: its fragments are expanded one at a time, each while the MFMAs of
        // the fragment before it run, so this half-step walks the blocks column by column
#pragma unroll
        for (int jb = 0; jb < CB; ++jb) {
          fb[0][jb] = int8x8_to_bf16(fq[jb]);
#pragma unroll
          for (int ii = 0; ii < IH; ++ii) {
            if (block_ok(ii))
              acc[ii][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[0][jb], fa[ab][ii], acc[ii][jb], 0, 0, 0);
            slot_work(jb * IH + ii);
          }
        }
      } else {
#pragma unroll
      for (int ii = 0; ii < IH; ++ii) {
        // a 16-row block that lies wholly past the last row (only in the last row tile) is skipped: the
        // wavefront sharing the SIMD gets the matrix core instead.  One scalar branch per row block, not per
        // MFMA; the loads and reads of its slots follow outside the branch, so no register is written on two paths.
        if (block_ok(h * IH + ii)) {
#pragma unroll
          for (int jb = 0; jb < CB; ++jb)
            acc[h * IH + ii][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bb][jb], fa[ab][ii], acc[h * IH + ii][jb], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jb = 0; jb < CB; ++jb) slot_work(ii * CB + jb);
      }
      }
#pragma unroll
      for (int j = NM; j < NSLOT; ++j) slot_work(j);
      if (next_reads) {
        lds_wait<0>();
#pragma unroll
        for (int i = 0; i < IH; ++i) lds_pin(fa[nab][i]);
        if (with_w) {
#pragma unroll
          for (int jb = 0; jb < CB; ++jb) {
            if (W8) asm volatile("" : "+v"(fq[jb]));
            else lds_pin(fb[nbb][jb]);
          }
        }
      }
    };

    // Issue order: W(0..SW-2), A(0), A(1), W(SW-1) up front; from then on the loads of a tile are
    // spread over four half-steps so that the memory pipeline never sees a burst: after the barrier
    // of tile t (its stages are free) the first half of A(t+2); during the first three half-steps of
    // tile t+1 the second half of A(t+2), then W(t+SW) in two halves.  When tile t+1 is needed,
    // the only loads that may be younger than the last load of A(t+1) are the LW loads of
    // W(t+SW-1).
    constexpr int QA = LA / 2, QW = LA + LW / 2;
#pragma unroll
    for (int s = 0; s < SW - 1; ++s) issue_w(s);
#pragma unroll
    for (int q = 0; q < LA; ++q) issue_one(0, q);
    vm_wait<0>();
    wg_barrier();
#pragma unroll
    for (int q = 0; q < NL; ++q) issue_one(1, q);
#pragma unroll
    for (int q = 0; q < IH; ++q) read_frag(fa[0][q], lds0 + a_off + rd[0], q);
#pragma unroll
    for (int q = 0; q < CB; ++q) {
      if (W8) read_wq(fq[q], lds0 + W_RING + b_off8 + rd8[0], q);
      else read_frag(fb[0][q], lds0 + W_RING + b_off + rd[0], q);
    }
    lds_wait<0>();
#pragma unroll
    for (int q = 0; q < IH; ++q) lds_pin(fa[0][q]);
#pragma unroll
    for (int q = 0; q < CB; ++q) {
      if (W8) asm volatile("" : "+v"(fq[q]));
      else lds_pin(fb[0][q]);
    }
    if (nk > 1) {
      // tile 0: tile 1 is already on its way
      step(0, true, 0, 1, 0, 0, 0);
      step(1, true, 0, 2, 0, 0, 0);
      step(2, true, 0, 3, 0, 0, 0);
      vm_wait<LW>();
      wg_barrier();
      step(3, true, 1, 0, 0, QA, 2);
    }
    for (int t = 1; t + 1 < nk; ++t) {
      step(0, true, t, 1, QA, LA, t + 1);
      step(1, true, t, 2, LA, QW, t + 1);
      step(2, true, t, 3, QW, NL, t + 1);
      // last half-step: its fragments are in registers, so once tile t+1 has landed everywhere the
      // stages of tile t can be refilled while these MFMAs run
      vm_wait<LW>();
      wg_barrier();
      step(3, true, t + 1, 0, 0, QA, t + 2);
    }
    step(0, true, nk - 1, 1, 0, 0, 0);
    step(1, true, nk - 1, 2, 0, 0, 0);
    step(2, true, nk - 1, 3, 0, 0, 0);
    step(3, false, 0, 0, 0, 0, 0);
  }
  // Block (i, jb) of this wavefront, lane l: output row i*16 + l%16 and columns jb*16 + 4*(l/16) .. +3 of its sub-tile
  const int l_row = lane & 15, l_col = (lane >> 4) * 4;
  if (W8) {
    // the sums are over integer weights: scale every output column
#pragma unroll
    for (int jb = 0; jb < CB; ++jb) {
      f32x4 sc = {0.f, 0.f, 0.f, 0.f};
      if (EPI == EPI_SWIGLU) {
        const int gc = n0 + wn * (BN / WN / 2) + (jb % (CB / 2)) * 16 + l_col;
        const float *ps = p.w_scale[jb / (CB / 2)];
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (gc + r < p.N) sc[r] = ps[gc + r];
      } else {
        const int gc = n0 + wn * (BN / WN) + jb * 16 + l_col;
        int sg = 0;
        if (p.n_seg > 1 && gc >= p.nb[1]) sg = 1;
        if (p.n_seg > 2 && gc >= p.nb[2]) sg = 2;
        const float *ps = p.w_scale[sg] - p.nb[sg];
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (gc + r < p.N) sc[r] = ps[gc + r];
      }
#pragma unroll
      for (int i = 0; i < RB; ++i) acc[i][jb] *= sc;
    }
  }
  if (EPI == EPI_SWIGLU && tail_z >= 0) {
    // raw partial sums of a shared tile, in register order (each store is 1 KB contiguous)
    const int slot = (j - (p.tail_first >> 3)) * 8 + xcd;
    float *pb = p.partial + ((size_t)slot * p.tail_splits + tail_z) * (BM * BN) + (size_t)wave * (RB * CB * 4 * 64);
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int jb = 0; jb < CB; ++jb)
        *reinterpret_cast<f32x4 *>(pb + ((i * CB + jb) * 64 + lane) * 4) = acc[i][jb];
    return;
  }
  if (EPI == EPI_SWIGLU) {
    swiglu_from_registers<RB, CB>(acc, p, m0 + wm * IH * 32, n0 + wn * (BN / WN / 2), lane);
    return;
  }
  if (EPI != EPI_SEG) {
    // raw sums straight from the accumulator registers, four adjacent columns per lane
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      const int gr = m0 + wm * IH * 32 + i * 16 + l_row;
      if (gr >= p.M) continue;
      float *prow = p.partial + ((size_t)z * p.M + gr) * p.N;
#pragma unroll
      for (int jb = 0; jb < CB; ++jb) {
        const int gc = n0 + wn * (BN / WN) + jb * 16 + l_col;
        if (gc + 3 < p.N) {
          *reinterpret_cast<f32x4 *>(prow + gc) = acc[i][jb];
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (gc + r < p.N) prow[gc + r] = acc[i][jb][r];
        }
      }
    }
    return;
  }
  // EPI_SEG: drain the clamped tail loads, then reuse the rings as the parking area
  vm_wait<0>();
  __syncthreads();
  float *sC = reinterpret_cast<float *>(smem);
  if (HL) {
    // the sums over the high parts are parked first, the sums over the low parts added to them
#pragma unroll
    for (int part = 0; part < 2; ++part) {
      if (wm == part) {
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
          for (int jb = 0; jb < CB; ++jb) {
            f32x4 *dst = reinterpret_cast<f32x4 *>(sC + (i * 16 + l_row) * DMA_CP + wn * (BN / WN) + jb * 16 + l_col);
            if (part == 0) *dst = acc[i][jb];
            else *dst += acc[i][jb];
          }
      }
      __syncthreads();
    }
    lds_epilogue<bf16, EPI, BN>(sC, DMA_CP, BMO, m0, n0, z, p);
    return;
  }
  // park and walk the tile in passes of at most 128 rows (LDS holds 128 x 260 floats)
  constexpr int PASSES = (I + 3) / 4;
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    const int i0 = ps * 8;                                   // first 16-row block of the pass
    const int nb = (2 * I - i0) < 8 ? (2 * I - i0) : 8;
    if (ps > 0) __syncthreads();
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      const int ib = wm * RB + i;                            // this wavefront's 16-row block within the tile
      if (ib >= i0 && ib < i0 + 8) {
#pragma unroll
        for (int jb = 0; jb < CB; ++jb)
          *reinterpret_cast<f32x4 *>(sC + ((ib - i0) * 16 + l_row) * DMA_CP + wn * (BN / WN) + jb * 16 + l_col) = acc[i][jb];
      }
    }
    __syncthreads();
    lds_epilogue<bf16, EPI, BN>(sC, DMA_CP, nb * 16, m0 + i0 * 16, n0, z, p);
  }
}

// ---------------------------------------------------------------------------
// Register-staged bf16 kernel (any K % 8 == 0).  4 wavefronts as 2x2, each owning a
// 64x64 block = 2x2 MFMA tiles.  LDS rows are padded by 16 bytes so that the 16-byte
// operand reads of 8 consecutive lanes fall into 8 different bank groups.
// Operand layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (l % 32) and the
// 8 consecutive k values starting at 8 * (l / 32); the result lane l holds column
// (l % 32), rows 8*(i/4) + 4*(l/32) + i%4 for i = 0..15.
// ---------------------------------------------------------------------------
constexpr int BM16 = 128, BN16 = 128, BK16 = 64, PITCH16 = BK16 + 8;
constexpr int CPITCH16 = BN16 + 4;
constexpr size_t kSmemBf16 =
    (2 * (BM16 + BN16) * PITCH16 * 2 > BM16 * CPITCH16 * 4) ? 2 * (BM16 + BN16) * PITCH16 * 2
                                                             : BM16 * CPITCH16 * 4;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  bf16 *sA = reinterpret_cast<bf16 *>(smem);               // [2][BM][PITCH]
  bf16 *sB = sA + 2 * BM16 * PITCH16;                      // [2][BN][PITCH]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int OUT_COLS = (EPI == EPI_SWIGLU) ? BN16 / 2 : BN16;
  const int m0 = blockIdx.y * BM16, n0 = blockIdx.x * OUT_COLS;
  const int kb = blockIdx.z * p.k_per_split;
  const int ke = min(p.K, kb + p.k_per_split);
  const int nk = (ke - kb + BK16 - 1) / BK16;

  // each thread moves 4 A chunks and 4 B chunks (16 bytes each) per k-tile
  const bf16 *a_ptr[4], *b_ptr[4];
  int lds_off[4], kcol[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int id = tid + i * 256, row = id >> 3, kc = id & 7;
    int ar = min(m0 + row, p.M - 1);
    if (p.a_rows) ar = p.a_rows[ar];
    a_ptr[i] = reinterpret_cast<const bf16 *>(p.a) + (size_t)ar * p.lda + kc * 8;
    b_ptr[i] = weight_row<bf16, EPI>(p, n0 + row, BN16 / 2, n0, row) + kc * 8;
    lds_off[i] = row * PITCH16 + kc * 8;
    kcol[i] = kc * 8;
  }
  bf16x8 ra[4], rb[4];
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  // tile t of the k loop; with a (high, low) activation pair the K range is walked twice, the
  // second time over the low parts
  const int nt_all = p.a_lo_off > 0 ? 2 * nk : nk;
  auto gload = [&](int t) {
    const int lo = t >= nk;
    const int k0 = kb + (t - lo * nk) * BK16;
    const int a_adv = k0 + lo * p.a_lo_off;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = k0 + kcol[i] < ke;
      ra[i] = ok ? *reinterpret_cast<const bf16x8 *>(a_ptr[i] + a_adv) : zero;
      rb[i] = ok ? *reinterpret_cast<const bf16x8 *>(b_ptr[i] + k0) : zero;
    }
  };
  auto sstore = [&](int stage) {
    bf16 *da = sA + stage * BM16 * PITCH16, *db = sB + stage * BN16 * PITCH16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<bf16x8 *>(da + lds_off[i]) = ra[i];
      *reinterpret_cast<bf16x8 *>(db + lds_off[i]) = rb[i];
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (nk > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  const int frag_off = (lane & 31) * PITCH16 + 8 * (lane >> 5);
  for (int t = 0; t < nt_all; ++t) {
    if (t + 1 < nt_all) gload(t + 1);
    const bf16 *ca = sA + (t & 1) * BM16 * PITCH16 + (wm * 64) * PITCH16 + frag_off;
    const bf16 *cb_ = sB + (t & 1) * BN16 * PITCH16 + (wn * 64) * PITCH16 + frag_off;
#pragma unroll
    for (int ks = 0; ks < BK16 / 16; ++ks) {
      bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(ca + ks * 16);
      bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(ca + 32 * PITCH16 + ks * 16);
      bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(cb_ + ks * 16);
      bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(cb_ + 32 * PITCH16 + ks * 16);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (t + 1 < nt_all) sstore((t + 1) & 1);
    __syncthreads();
  }
  // park the accumulators in LDS (the operand stages are dead after the last barrier)
  float *sC = reinterpret_cast<float *>(smem);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wm * 64 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int col = wn * 64 + j * 32 + (lane & 31);
        sC[row * CPITCH16 + col] = acc[i][j][r];
      }
  __syncthreads();
  lds_epilogue<bf16, EPI, BN16>(sC, CPITCH16, BM16, m0, n0, blockIdx.z, p);
}

// ---------------------------------------------------------------------------
// float kernel: 64x64x16 tiles, 256 lanes, 4x4 outputs per lane, plain FMA.
// ---------------------------------------------------------------------------
constexpr int BM32 = 64, BN32 = 64, BK32 = 16, TP32 = BM32 + 4, CPITCH32 = BN32 + 4;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) float smem[BM32 * CPITCH32];  // >= 2*BK*TP32
  float *sA = smem;                 // [BK][TP32]  (k-major)
  float *sB = smem + BK32 * TP32;   // [BK][TP32]
  const int tid = threadIdx.x;
  constexpr int OUT_COLS = (EPI == EPI_SWIGLU) ? BN32 / 2 : BN32;
  const int m0 = blockIdx.y * BM32, n0 = blockIdx.x * OUT_COLS;
  const int kb = blockIdx.z * p.k_per_split;
  const int ke = min(p.K, kb + p.k_per_split);
  const int lrow = tid >> 2, lkc = (tid & 3) * 4;
  int ar = min(m0 + lrow, p.M - 1);
  if (p.a_rows) ar = p.a_rows[ar];
  const float *a_ptr = reinterpret_cast<const float *>(p.a) + (size_t)ar * p.lda + lkc;
  const float *b_ptr = weight_row<float, EPI>(p, n0 + lrow, BN32 / 2, n0, lrow) + lkc;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = kb; k0 < ke; k0 += BK32) {
    const bool ok = k0 + lkc < ke;
    float4 va = ok ? *reinterpret_cast<const float4 *>(a_ptr + k0) : make_float4(0, 0, 0, 0);
    float4 vb = ok ? *reinterpret_cast<const float4 *>(b_ptr + k0) : make_float4(0, 0, 0, 0);
    __syncthreads();
    sA[(lkc + 0) * TP32 + lrow] = va.x; sA[(lkc + 1) * TP32 + lrow] = va.y;
    sA[(lkc + 2) * TP32 + lrow] = va.z; sA[(lkc + 3) * TP32 + lrow] = va.w;
    sB[(lkc + 0) * TP32 + lrow] = vb.x; sB[(lkc + 1) * TP32 + lrow] = vb.y;
    sB[(lkc + 2) * TP32 + lrow] = vb.z; sB[(lkc + 3) * TP32 + lrow] = vb.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK32; ++k) {
      const float4 a4 = *reinterpret_cast<const float4 *>(sA + k * TP32 + ty * 4);
      const float4 b4 = *reinterpret_cast<const float4 *>(sB + k * TP32 + tx * 4);
      const float av[4] = {a4.x, a4.y, a4.z, a4.w}, bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
  }
  __syncthreads();
  float *sC = smem;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<float4 *>(sC + (ty * 4 + i) * CPITCH32 + tx * 4) =
        make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
  __syncthreads();
  lds_epilogue<float, EPI, BN32>(sC, CPITCH32, BM32, m0, n0, blockIdx.z, p);
}

// ---------------------------------------------------------------------------
// Finish launches: one workgroup per output row adds the parked partial sums in ascending split
// order (fixed order, no atomics: bitwise reproducible) and completes the row.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float4 sum_splits(const GemmParams &p, size_t e) {
  float4 acc = make_float4(0, 0, 0, 0);
  const size_t stride = (size_t)p.M * p.N;
  for (int z = 0; z < p.splits; ++z) {
    const float4 v = *reinterpret_cast<const float4 *>(p.partial + z * stride + e);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  return acc;
}

// EPI_SEG rows: rotary embedding, conversion to the storage type, store (optionally through the
// segment's row map) and -- for rows < n_dev -- the KV deviation of the row (Sec. 4.1, Sec. 6):
// the squared distance of the values as stored from the cached row, over the segments that name a cache.
template <typename T>
__global__ __launch_bounds__(256) void seg_finish_kernel(GemmParams p) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const bool want_dev = p.dev_out != nullptr && r < p.n_dev;
  const int crow = want_dev ? p.dev_row[r] : 0;
  float dsum = 0.f;
  for (int c = threadIdx.x * 4; c < p.N; c += 1024) {
    const size_t e = (size_t)r * p.N + c;
    const float4 acc = sum_splits(p, e);
    float4 partner = acc;
    if (p.rope_half) partner = sum_splits(p, (size_t)((long)e + rope_partner_offset(p, c)));
    int s, lc;
    const float4 v = seg_rotate(acc, partner, r, c, p, &s, &lc);
    const int dr = p.row_map[s] ? p.row_map[s][r] : r;
    store4<T>(reinterpret_cast<T *>(p.dst[s]) + (size_t)dr * p.ld[s] + lc, v.x, v.y, v.z, v.w);
    if (want_dev && p.dev_cache[s]) {
      const float4 old = load4<T>(reinterpret_cast<const T *>(p.dev_cache[s]) +
                                  (size_t)crow * (p.nb[s + 1] - p.nb[s]) + lc);
      const float d0 = as_stored<T>(v.x) - old.x, d1 = as_stored<T>(v.y) - old.y;
      const float d2 = as_stored<T>(v.z) - old.z, d3 = as_stored<T>(v.w) - old.w;
      dsum += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
    }
  }
  if (p.dev_out != nullptr) {              // uniform over the workgroup
    dsum = block_sum_256(dsum, red);
    if (want_dev && threadIdx.x == 0) p.dev_out[r] = dsum;
  }
}

// EPI_F32 rows: h = sum of the partial sums + residual, stored as float; then, when a gain is
// given, the RMSNorm of h in the storage type (the next projection's input), optionally as a
// (high, low) pair.  A lane re-reads only elements it wrote itself.
template <typename T>
__global__ __launch_bounds__(256) void resid_norm_finish_kernel(GemmParams p) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const int rr = p.resid_rows ? p.resid_rows[r] : r;
  float *orow = p.out_f32 + (size_t)r * p.N;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < p.N; c += 1024) {
    float4 v = sum_splits(p, (size_t)r * p.N + c);
    if (p.resid) {
      const float4 q = *reinterpret_cast<const float4 *>(p.resid + (size_t)rr * p.N + c);
      v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
    }
    *reinterpret_cast<float4 *>(orow + c) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  if (p.norm_gain == nullptr) return;      // uniform
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)p.N + p.norm_eps);
  const T *gain = reinterpret_cast<const T *>(p.norm_gain);
  T *nrow = reinterpret_cast<T *>(p.norm_out) + (size_t)r * p.norm_ld;
  for (int c = threadIdx.x * 4; c < p.N; c += 1024) {
    const float4 v = *reinterpret_cast<const float4 *>(orow + c);
    const float x[4] = {v.x * inv * to_f32(gain[c]), v.y * inv * to_f32(gain[c + 1]),
                        v.z * inv * to_f32(gain[c + 2]), v.w * inv * to_f32(gain[c + 3])};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const T hi = from_f32<T>(x[i]);
      nrow[c + i] = hi;
      if (p.norm_lo_off > 0) nrow[p.norm_lo_off + c + i] = from_f32<T>(x[i] - to_f32(hi));
    }
  }
}

// The same for rows of at most 1024 NC elements, with the row held in registers: a workgroup per row
// is little work in flight, so the loop above runs at the latency of one load after the other (its
// store may alias the next iteration's loads, which therefore wait for it).  Here every load of a
// split is issued before the first sum, two splits at a time, and the second pass reads no memory.
// Same order of additions per element as above.
template <typename T, int NC>
__global__ __launch_bounds__(256) void resid_norm_finish_row_kernel(GemmParams p) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const int rr = p.resid_rows ? p.resid_rows[r] : r;
  const size_t row = (size_t)r * p.N, stride = (size_t)p.M * p.N;
  const int c0 = threadIdx.x * 4;
  float4 q[NC], acc[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = c0 + i * 1024;
    acc[i] = make_float4(0, 0, 0, 0);
    q[i] = make_float4(0, 0, 0, 0);
    if (p.resid && c < p.N) q[i] = *reinterpret_cast<const float4 *>(p.resid + (size_t)rr * p.N + c);
  }
#pragma unroll 2
  for (int z = 0; z < p.splits; ++z) {
    float4 v[NC];
    const float *src = p.partial + z * stride + row;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = c0 + i * 1024;
      v[i] = c < p.N ? *reinterpret_cast<const float4 *>(src + c) : make_float4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      acc[i].x += v[i].x; acc[i].y += v[i].y; acc[i].z += v[i].z; acc[i].w += v[i].w;
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = c0 + i * 1024;
    if (p.resid) { acc[i].x += q[i].x; acc[i].y += q[i].y; acc[i].z += q[i].z; acc[i].w += q[i].w; }
    if (c < p.N) *reinterpret_cast<float4 *>(p.out_f32 + row + c) = acc[i];
    // the expression of the stand-alone norm kernel: a layer normalised there and one normalised here agree bitwise
    ss += acc[i].x * acc[i].x + acc[i].y * acc[i].y + acc[i].z * acc[i].z + acc[i].w * acc[i].w;
  }
  if (p.norm_gain == nullptr) return;      // uniform
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)p.N + p.norm_eps);
  const T *gain = reinterpret_cast<const T *>(p.norm_gain);
  T *nrow = reinterpret_cast<T *>(p.norm_out) + (size_t)r * p.norm_ld;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = c0 + i * 1024;
    if (c >= p.N) continue;
    const float4 gn = load4<T>(gain + c);
    const float x[4] = {acc[i].x * inv * gn.x, acc[i].y * inv * gn.y, acc[i].z * inv * gn.z, acc[i].w * inv * gn.w};
    float hi[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) hi[e] = to_f32(from_f32<T>(x[e]));
    store4<T>(nrow + c, x[0], x[1], x[2], x[3]);
    if (p.norm_lo_off > 0)
      store4<T>(nrow + p.norm_lo_off + c, x[0] - hi[0], x[1] - hi[1], x[2] - hi[2], x[3] - hi[3]);
  }
}

// ---------------------------------------------------------------------------
// Host side: choice of kernel, tile height and K split; launches.
// ---------------------------------------------------------------------------
struct GemmPlan {
  int kind;        // 0 float, 1 register-staged bf16, 2 direct-to-LDS bf16
  int I, NB;       // kind 2: the kernel's tile = 32I activation-tile rows x 64NB columns
  int nwv;         // kind 2: wavefronts per workgroup (4, or 8 = two per SIMD for the 256-column tiles)
  int hl;          // the activations are (high, low) pairs (bf16 EPI_SEG only)
  int bm, out_cols, bk;   // bm: OUTPUT rows per tile (half the activation-tile rows with hl, kind 2)
  int tiles_m, tiles_n, splits, k_per_split;
  int tail_first, tail_splits, tail_k_per_split;   // EPI_SWIGLU tail sharing (tail_splits <= 1: none)
  long grid_ids;                                   // kind 2: workgroups of the main launch
  int xcd_split;                                   // kind 2: splits dealt to XCDs (see GemmParams)
  int w8;                                          // kind 2: int8 weights read by the kernel itself
  int raw;                                         // sums are parked in `partial` and a finish launch completes them
  size_t partial_floats;
  bool bad;                                        // needs scratch the caller did not give
};

static int pick_row_blocks(int M) {
  // padded rows divided by a rough efficiency of the tile height
  const int cand[4] = {8, 6, 4, 2};
  const double eff[4] = {1.0, 0.97, 0.88, 0.62};
  int best = 8;
  double best_cost = 1e30;
  for (int i = 0; i < 4; ++i) {
    const int bm = 32 * cand[i];
    const double cost = (double)ceil_div(M, bm) * bm / eff[i];
    if (cost < best_cost - 1e-9) { best_cost = cost; best = cand[i]; }
  }
  return best;
}

// Tile shape and K split of the direct-to-LDS kernel for the Q/K/V, output and down projections,
// from a cost model in microseconds fitted to a sweep of every (tile, split) pair over the
// projection shapes of the 7B- and 70B-shaped workloads (row counts 295 .. 1264) on the chip:
//   main launch   = rounds x t_full x k-tiles per workgroup + 9.9 (launch, pipeline fill, epilogue)
//   t_full        = time of one 64-deep k-tile with every slot of the chip busy (a slot = one resident
//                   workgroup: two per CU for the tiles whose rings fit twice into LDS, else one)
//   partial round = runs faster per tile, because fewer workgroups share the chip's power and its
//                   L2 -> LDS paths: t_full x (1 - relief x (1 - fill))
//   finish launch = 2.3 + 0.258 us per MB of parked sums (splits x M x N floats)
// The model's choice is within 0 .. 5 % (mean 1 %) of the best measured pair on every shape of the sweep.
// max_splits caps the split (scratch the caller can spare); parked: a finish launch runs anyway.
struct DmaShape { int I, NB; double t_full; };
static const DmaShape kDmaShapes[] = {{2, 2, 0.80}, {4, 2, 1.23}, {6, 2, 1.02}, {8, 2, 1.28},
                                      {4, 4, 1.14}, {6, 4, 1.54}, {8, 4, 1.90}};

static void pick_dma_plan(int M, int N, int K, int max_splits, bool parked, size_t out_elems, bool w8, GemmPlan *pl) {
  const int k_tiles = K / DMA_BK;
  const double park_us = (double)out_elems * 4.0e-6 * 0.258;   // per split
  double best = 1e30;
  for (const DmaShape &c : kDmaShapes) {
    if (c.I == 2 && M > 64) continue;
    const int bm = 32 * c.I, bn = 64 * c.NB;
    const int slots = dma_smem_bytes(c.I, bn, w8) <= 80 * 1024 ? 512 : 256;
    const long tiles = (long)ceil_div(M, bm) * ceil_div(N, bn);
    for (int sp = 1; sp <= 16 && sp <= max_splits; ++sp) {
      if (sp > 1 && k_tiles / sp < 4) break;
      const long wgs = tiles * sp;
      const long full = wgs / slots;
      const double last = (double)(wgs - full * slots) / slots;          // fill of the last round
      const double relief = slots == 512 ? 0.69 : 0.45;
      const double per_tile = full * c.t_full + (last > 0 ? c.t_full * (1.0 - relief + relief * last) : 0.0);
      const double cost = per_tile * ceil_div(k_tiles, sp) + 9.9 + (sp > 1 || parked ? sp * park_us + 2.3 : 0.0);
      if (cost < best - 1e-9) { best = cost; pl->I = c.I; pl->NB = c.NB; pl->splits = sp; }
    }
  }
}

// The float kernel's 64-column tile does not hold a whole 128-channel head, so it cannot pair
// channel i with i + head_dim/2 itself: it parks its sums and the finish launch rotates them.
static bool needs_raw_partial(int dtype, int epi, int rope_half, int head_dim) {
  return dtype == 0 && epi == EPI_SEG && rope_half && head_dim > BN32;
}

bool gemm_int8_in_kernel(int dtype, int K) { return dtype == 1 && K % DMA_BK == 0; }

// Shape of one problem.  hl: (high, low) activation pairs; force_raw: the caller wants the finish
// launch (deviation, or the float output's residual + norm); scratch_floats: what `partial` holds
// (the K split is capped by it; SIZE_MAX when sizing).
static GemmPlan make_plan(int dtype, int epi, int M, int N, int K, int hl, int force_raw, int rope_half,
                          int head_dim, size_t scratch_floats, bool w8 = false) {
  GemmPlan pl = {};
  pl.w8 = w8;
  if (w8 && !gemm_int8_in_kernel(dtype, K)) pl.bad = true;
  pl.splits = 1;
  pl.hl = hl && dtype == 1 && epi == EPI_SEG;
  pl.raw = force_raw || epi == EPI_F32 || needs_raw_partial(dtype, epi, rope_half, head_dim);
  const size_t mn = (size_t)M * N;
  const int max_splits = (int)std::min<size_t>(16, std::max<size_t>(1, scratch_floats / std::max<size_t>(1, mn)));
  if (pl.raw && scratch_floats < mn) pl.bad = true;
  if (dtype == 0) {
    pl.kind = 0; pl.bm = BM32; pl.out_cols = epi == EPI_SWIGLU ? BN32 / 2 : BN32; pl.bk = BK32;
  } else if (K % DMA_BK != 0) {
    pl.kind = 1; pl.bm = BM16; pl.out_cols = epi == EPI_SWIGLU ? BN16 / 2 : BN16; pl.bk = BK16;
  } else if (epi == EPI_SWIGLU) {
    pl.kind = 2; pl.I = pick_row_blocks(M); pl.bk = DMA_BK;
    // 256-column tiles unless 128-column tiles (lower arithmetic intensity: measured ~1.4x
    // slower per flop) fill the rounds of 256 workgroups so much better that they still win,
    // which happens when there is a single row of tiles (M <= 256)
    pl.NB = 4;
    const long t4 = (long)ceil_div(M, 32 * pl.I) * ceil_div(N, 128), t2 = (long)ceil_div(M, 32 * pl.I) * ceil_div(N, 64);
    const double c4 = (double)((t4 + 255) / 256) * 2.0, c2 = (double)((t2 + 255) / 256) * 1.4;
    if (c2 < c4) pl.NB = 2;
  } else {
    pl.kind = 2; pl.bk = DMA_BK;
    // with operand pairs the activation tile holds every output row twice
    pick_dma_plan(pl.hl ? 2 * M : M, N, K, max_splits, pl.raw, mn, w8, &pl);
  }
  if (pl.kind == 2) {
    pl.nwv = (pl.NB == 4 && pl.I >= 4) ? 8 : 4;
    pl.bm = pl.hl ? 16 * pl.I : 32 * pl.I;
    pl.out_cols = (epi == EPI_SWIGLU ? 32 : 64) * pl.NB;
  }
  pl.tiles_m = ceil_div(M, pl.bm);
  pl.tiles_n = ceil_div(N, pl.out_cols);
  const int k_tiles = ceil_div(K, pl.bk);
  const long tiles = (long)pl.tiles_m * pl.tiles_n;
  if (pl.kind == 1 && epi != EPI_SWIGLU && tiles < 256) {
    // smallest split that fills >= 90 % of a whole number of 256-workgroup rounds
    double best_eff = 0;
    for (int sp = 1; sp <= 16 && sp <= max_splits; ++sp) {
      if (sp > 1 && k_tiles / sp < 4) break;
      const long wgs = tiles * sp;
      const double eff = (double)wgs / (double)((wgs + 255) / 256 * 256);
      if (eff > best_eff + 1e-9) { best_eff = eff; pl.splits = sp; }
      if (eff >= 0.9) break;
    }
  }
  pl.k_per_split = ceil_div(k_tiles, pl.splits) * pl.bk;
  pl.splits = ceil_div(K, pl.k_per_split);
  if (pl.splits > 1) pl.raw = 1;
  pl.partial_floats = pl.raw ? (size_t)pl.splits * mn : 0;
  pl.tail_splits = 1;
  if (pl.kind == 2) {
    const long ids = 8L * ceil_div(pl.tiles_n, 8) * pl.tiles_m;
    pl.grid_ids = ids * pl.splits;
    if (epi != EPI_SWIGLU && (pl.splits == 2 || pl.splits == 4 || pl.splits == 8)) {
      pl.xcd_split = 1;
      pl.grid_ids = 8L * ceil_div(pl.tiles_n, 8 / pl.splits) * pl.tiles_m;
    }
    pl.tail_first = (int)pl.grid_ids;
    if (epi == EPI_SWIGLU) {
      // The last round of 256 workgroups, when less than half full, is shared: ts workgroups per
      // tile, each over 1/ts of K, plus a fix-up launch.  Worth it when the time saved on the
      // round exceeds the round trip of the partial sums (~4 TB/s) and the extra launch.
      const long full = ids / 256 * 256, tail = ids - full;
      int ts = tail > 0 ? (int)std::min<long>(4, 256 / tail) : 1;
      while (ts > 1 && k_tiles / ts < 8) --ts;
      if (ts > 1) {
        const double t_tile = 0.3 * pl.I * (pl.NB == 4 ? 1.0 : 0.6);
        const double saved = (k_tiles - ceil_div(k_tiles, ts)) * t_tile;
        const double extra = (double)tail * ts * pl.bm * (64 * pl.NB) * 8.0 / 4.0e6 + 8.0;
        const size_t need = (size_t)tail * ceil_div(K, ceil_div(k_tiles, ts) * pl.bk) * pl.bm * (64 * pl.NB);
        if (saved > extra && need <= scratch_floats) {
          pl.tail_first = (int)full;
          pl.tail_k_per_split = ceil_div(k_tiles, ts) * pl.bk;
          pl.tail_splits = ceil_div(K, pl.tail_k_per_split);
          pl.grid_ids = full + tail * pl.tail_splits;
          pl.partial_floats = (size_t)tail * pl.tail_splits * pl.bm * (64 * pl.NB);
        }
      }
    }
  }
  return pl;
}

static int problem_n(const GemmArgs &g) {
  if (g.epi == EPI_SWIGLU) return g.seg[0].n;
  int n = 0;
  for (int i = 0; i < (g.epi == EPI_SEG ? g.n_seg : 1); ++i) n += g.seg[i].n;
  return n;
}

size_t gemm_partial_floats(int dtype, int epi, int M, int N, int K, int hl, int force_raw, int rope_half,
                           int head_dim, int w8) {
  if (M <= 0) return 0;
  return make_plan(dtype, epi, M, N, K, hl, force_raw, rope_half, head_dim, SIZE_MAX,
                   w8 && gemm_int8_in_kernel(dtype, K)).partial_floats;
}

static GemmPlan fill_params(const GemmArgs &g, GemmParams *pp) {
  GemmParams &p = *pp;
  p = GemmParams{};
  p.a = g.a; p.lda = g.lda; p.a_rows = g.a_rows; p.M = g.M; p.K = g.K;
  p.n_seg = g.epi == EPI_SEG ? g.n_seg : 1;
  p.nb[0] = 0;
  for (int i = 0; i < 3; ++i) {
    p.w[i] = g.seg[i].w; p.w_scale[i] = g.seg[i].w_scale; p.dst[i] = g.seg[i].dst; p.ld[i] = g.seg[i].ld_dst;
    p.row_map[i] = g.seg[i].row_map; p.rope[i] = g.seg[i].rope;
    p.nb[i + 1] = p.nb[i] + (i < p.n_seg ? g.seg[i].n : 0);
    p.dev_cache[i] = g.dev_out ? g.seg[i].dev_cache : nullptr;
  }
  p.N = problem_n(g);
  p.rope_tab = g.rope_tab; p.row_pos = g.row_pos; p.head_dim = g.head_dim;
  p.out_f32 = g.out_f32; p.resid = g.resid; p.resid_rows = g.resid_rows; p.partial = g.partial;
  p.rope_half = g.rope_half;
  p.dev_out = g.dev_out; p.n_dev = g.n_dev; p.dev_row = g.dev_row;
  p.norm_gain = g.norm_gain; p.norm_out = g.norm_out; p.norm_ld = g.norm_ld; p.norm_lo_off = g.norm_lo_off;
  p.norm_eps = g.norm_eps;
  GemmPlan pl = make_plan(g.dtype, g.epi, g.M, p.N, g.K, g.a_lo_off > 0, g.dev_out != nullptr, g.rope_half,
                          g.head_dim, g.partial ? g.partial_floats : 0, g.seg[0].w_scale != nullptr);
  // every matrix of a launch is in the same format
  const int n_w = g.epi == EPI_SEG ? g.n_seg : (g.epi == EPI_SWIGLU ? 2 : 1);
  for (int i = 1; i < n_w; ++i)
    if ((g.seg[i].w_scale != nullptr) != (g.seg[0].w_scale != nullptr)) pl.bad = true;
  p.a_lo_off = pl.hl ? g.a_lo_off : 0;
  p.raw_partial = pl.raw;
  p.splits = pl.splits;
  p.k_per_split = pl.k_per_split;
  p.tail_first = pl.tail_first; p.tail_splits = pl.tail_splits; p.tail_k_per_split = pl.tail_k_per_split;
  p.xcd_split = pl.xcd_split;
  return pl;
}

bool gemm_needs_finish(const GemmArgs &g) {
  if (g.M == 0) return false;
  GemmParams p;
  const GemmPlan pl = fill_params(g, &p);
  return pl.raw || pl.tail_splits > 1;
}

// sets a kernel's dynamic LDS limit once per process, whichever host thread launches it first
#define CB_LDS_LIMIT_ONCE(kernel_expr, bytes)                                                      \
  do {                                                                                             \
    static std::once_flag once_;                                                                   \
    std::call_once(once_, [] {                                                                     \
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel_expr),                       \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes));         \
    });                                                                                            \
  } while (0)

template <int I, int NB, int EPI, int NWV, bool HL = false>
static void launch_dma(const GemmPlan &pl, const GemmParams &p, hipStream_t s) {
  if (pl.w8) {
    constexpr int smem = dma_smem_bytes(I, 64 * NB, true);
    CB_LDS_LIMIT_ONCE((&gemm_bf16_dma_kernel<I, NB, EPI, NWV, HL, true>), smem);
    hipLaunchKernelGGL((gemm_bf16_dma_kernel<I, NB, EPI, NWV, HL, true>), dim3((unsigned)pl.grid_ids), dim3(64 * NWV),
                       smem, s, p, pl.tiles_m, pl.tiles_n);
    return;
  }
  constexpr int smem = dma_smem_bytes(I, 64 * NB);
  CB_LDS_LIMIT_ONCE((&gemm_bf16_dma_kernel<I, NB, EPI, NWV, HL>), smem);
  hipLaunchKernelGGL((gemm_bf16_dma_kernel<I, NB, EPI, NWV, HL>), dim3((unsigned)pl.grid_ids), dim3(64 * NWV), smem,
                     s, p, pl.tiles_m, pl.tiles_n);
}

template <int EPI, bool HL>
static void launch_dma_shape(const GemmPlan &pl, const GemmParams &p, hipStream_t s) {
  if (pl.NB == 2) {
    switch (pl.I) {
      case 2: launch_dma<2, 2, EPI, 4, HL>(pl, p, s); break;
      case 4: launch_dma<4, 2, EPI, 4, HL>(pl, p, s); break;
      case 6: launch_dma<6, 2, EPI, 4, HL>(pl, p, s); break;
      default: launch_dma<8, 2, EPI, 4, HL>(pl, p, s); break;
    }
  } else if (pl.nwv == 8) {
    switch (pl.I) {
      case 4: launch_dma<4, 4, EPI, 8, HL>(pl, p, s); break;
      case 6: launch_dma<6, 4, EPI, 8, HL>(pl, p, s); break;
      default: launch_dma<8, 4, EPI, 8, HL>(pl, p, s); break;
    }
  } else {
    launch_dma<2, 4, EPI, 4, HL>(pl, p, s);
  }
}

template <int EPI>
static void launch_typed(const GemmPlan &pl, const GemmParams &p, hipStream_t s) {
  const dim3 grid(pl.tiles_n, pl.tiles_m, pl.splits);
  if (pl.kind == 0) {
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, s, p);
  } else if (pl.kind == 1) {
    CB_LDS_LIMIT_ONCE((&gemm_bf16_kernel<EPI>), kSmemBf16);
    hipLaunchKernelGGL(gemm_bf16_kernel<EPI>, grid, dim3(256), kSmemBf16, s, p);
  } else if (EPI == EPI_SEG && pl.hl) {
    launch_dma_shape<EPI_SEG, true>(pl, p, s);
  } else {
    launch_dma_shape<EPI, false>(pl, p, s);
  }
}

hipError_t launch_gemm(const GemmArgs &g, hipStream_t s) {
  if (g.M == 0) return hipSuccess;
  GemmParams p;
  const GemmPlan pl = fill_params(g, &p);
  if (pl.bad) return hipErrorInvalidValue;
  if (g.epi == EPI_SEG) launch_typed<EPI_SEG>(pl, p, s);
  else if (g.epi == EPI_SWIGLU) launch_typed<EPI_SWIGLU>(pl, p, s);
  else launch_typed<EPI_F32>(pl, p, s);
  return hipGetLastError();
}

hipError_t launch_gemm_finish(const GemmArgs &g, hipStream_t s) {
  if (g.M == 0) return hipSuccess;
  GemmParams p;
  const GemmPlan pl = fill_params(g, &p);
  if (pl.bad) return hipErrorInvalidValue;
  if (pl.tail_splits > 1) {
    const dim3 tg((unsigned)((pl.grid_ids - pl.tail_first) / pl.tail_splits) * (pl.I / 2) * (pl.NB / 2));
#define CB_TAIL(I_, NB_, W_) hipLaunchKernelGGL((swiglu_tail_kernel<I_, NB_, W_>), tg, dim3(256), 0, s, p, pl.tiles_m, pl.tiles_n)
    if (pl.NB == 2) {
      switch (pl.I) { case 2: CB_TAIL(2, 2, 4); break; case 4: CB_TAIL(4, 2, 4); break; case 6: CB_TAIL(6, 2, 4); break; default: CB_TAIL(8, 2, 4); break; }
    } else if (pl.nwv == 8) {
      switch (pl.I) { case 4: CB_TAIL(4, 4, 8); break; case 6: CB_TAIL(6, 4, 8); break; default: CB_TAIL(8, 4, 8); break; }
    } else {
      CB_TAIL(2, 4, 4);
    }
#undef CB_TAIL
    return hipGetLastError();
  }
  if (!pl.raw) return hipSuccess;
  const dim3 grid((unsigned)g.M);
  if (g.epi == EPI_SEG) {
    if (g.dtype == 0) hipLaunchKernelGGL(seg_finish_kernel<float>, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(seg_finish_kernel<bf16>, grid, dim3(256), 0, s, p);
  } else {
#define CB_ROW(NC_)                                                                                        \
  do {                                                                                                     \
    if (g.dtype == 0) hipLaunchKernelGGL((resid_norm_finish_row_kernel<float, NC_>), grid, dim3(256), 0, s, p); \
    else hipLaunchKernelGGL((resid_norm_finish_row_kernel<bf16, NC_>), grid, dim3(256), 0, s, p);          \
  } while (0)
    if (p.N <= 2048) CB_ROW(2);
    else if (p.N <= 4096) CB_ROW(4);
    else if (p.N <= 8192) CB_ROW(8);
    else if (g.dtype == 0) hipLaunchKernelGGL(resid_norm_finish_kernel<float>, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(resid_norm_finish_kernel<bf16>, grid, dim3(256), 0, s, p);
#undef CB_ROW
  }
  return hipGetLastError();
}

}  // namespace cb
