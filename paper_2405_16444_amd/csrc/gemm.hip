// Projections of the selectively recomputed rows (paper Sec. 4.2: Q/K/V of the
// selected tokens, then "the same attention module" and the rest of the layer).
// C[M, N] = A[M, K] * W[N, K]^T with both operands K-contiguous.
//
// bf16 storage: v_mfma_f32_32x32x16_bf16, 128x128x64 tiles staged through LDS,
// float accumulation.  float storage: plain FMA tiles (parity mode, not tuned).
// Every kernel ends by parking its accumulator tile in LDS; one shared epilogue
// then walks it row-major, 4 adjacent columns per lane, which gives the rotary
// embedding its (2i, 2i+1) pair in one lane, SwiGLU its gate and up value in one
// lane, and coalesced stores.  Epilogues:
//   EPI_SEG    up to three column segments (Q | K | V), each with its own weight
//              matrix, destination, optional destination-row map (scatter into the
//              KV cache) and optional rotary embedding at the row's position
//   EPI_SWIGLU silu(x Wg^T) * (x Wu^T)
//   EPI_F32    float output (+ residual), or split-K partial sums reduced by a
//              second kernel in a fixed order (no atomics: bitwise reproducible)
#include "common.h"
#include "kernels.h"

namespace cb {

struct GemmParams {
  const void *a;
  int lda;
  const int32_t *a_rows;
  int M, K, N;          // N: total output columns (EPI_SWIGLU: d_ff)
  int n_seg;
  const void *w[3];
  int nb[4];            // column boundaries of the segments
  void *dst[3];
  int ld[3];
  const int32_t *row_map[3];
  int rope[3];
  const float2 *rope_tab;
  const int32_t *row_pos;
  int head_dim;
  float *out_f32;
  const float *resid;
  const int32_t *resid_rows;
  float *partial;
  int splits, k_per_split;
};

// weight row that feeds tile column gc (clamped into range)
template <typename T, int EPI>
__device__ __forceinline__ const T *weight_row(const GemmParams &p, int gc, int half_bn, int n0, int c) {
  if (EPI == EPI_SWIGLU) {
    // tile columns [0, half) come from the gate matrix, [half, 2*half) from the up matrix
    int which = c >= half_bn;
    int row = min(n0 + (which ? c - half_bn : c), p.N - 1);
    return reinterpret_cast<const T *>(p.w[which]) + (size_t)row * p.K;
  }
  gc = min(gc, p.N - 1);
  int s = 0;
  if (p.n_seg > 1 && gc >= p.nb[1]) s = 1;
  if (p.n_seg > 2 && gc >= p.nb[2]) s = 2;
  return reinterpret_cast<const T *>(p.w[s]) + (size_t)(gc - p.nb[s]) * p.K;
}

template <typename T> __device__ __forceinline__ void store4(T *d, float a, float b, float c, float e);
template <> __device__ __forceinline__ void store4<float>(float *d, float a, float b, float c, float e) {
  *reinterpret_cast<float4 *>(d) = make_float4(a, b, c, e);
}
template <> __device__ __forceinline__ void store4<bf16>(bf16 *d, float a, float b, float c, float e) {
  bf16x4 v = {(bf16)a, (bf16)b, (bf16)c, (bf16)e};
  *reinterpret_cast<bf16x4 *>(d) = v;
}

// sC: BM x (tile columns) floats, pitch `pitch`.  n0: first output column of the tile.
template <typename T, int EPI, int BM, int BN>
__device__ __forceinline__ void epilogue(const float *sC, int pitch, int m0, int n0, const GemmParams &p) {
  constexpr int OUT_COLS = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int GROUPS = OUT_COLS / 4;
  for (int g = threadIdx.x; g < BM * GROUPS; g += 256) {
    const int r = g / GROUPS, c = (g % GROUPS) * 4;
    const int gr = m0 + r, gc = n0 + c;
    if (gr >= p.M || gc >= p.N) continue;
    float4 v = *reinterpret_cast<const float4 *>(sC + r * pitch + c);
    if (EPI == EPI_SEG) {
      int s = 0;
      if (p.n_seg > 1 && gc >= p.nb[1]) s = 1;
      if (p.n_seg > 2 && gc >= p.nb[2]) s = 2;
      const int lc = gc - p.nb[s];
      if (p.rope[s]) {
        const int half = p.head_dim / 2;
        const float2 *t = p.rope_tab + (size_t)p.row_pos[gr] * half + (lc % p.head_dim) / 2;
        const float2 c0 = t[0], c1 = t[1];
        float4 o;
        o.x = v.x * c0.x - v.y * c0.y;
        o.y = v.x * c0.y + v.y * c0.x;
        o.z = v.z * c1.x - v.w * c1.y;
        o.w = v.z * c1.y + v.w * c1.x;
        v = o;
      }
      const int dr = p.row_map[s] ? p.row_map[s][gr] : gr;
      store4<T>(reinterpret_cast<T *>(p.dst[s]) + (size_t)dr * p.ld[s] + lc, v.x, v.y, v.z, v.w);
    } else if (EPI == EPI_SWIGLU) {
      const float4 u = *reinterpret_cast<const float4 *>(sC + r * pitch + OUT_COLS + c);
      float4 o;
      o.x = v.x / (1.f + expf(-v.x)) * u.x;
      o.y = v.y / (1.f + expf(-v.y)) * u.y;
      o.z = v.z / (1.f + expf(-v.z)) * u.z;
      o.w = v.w / (1.f + expf(-v.w)) * u.w;
      store4<T>(reinterpret_cast<T *>(p.dst[0]) + (size_t)gr * p.ld[0] + gc, o.x, o.y, o.z, o.w);
    } else {
      if (p.splits == 1) {
        if (p.resid) {
          const int rr = p.resid_rows ? p.resid_rows[gr] : gr;
          const float4 q = *reinterpret_cast<const float4 *>(p.resid + (size_t)rr * p.N + gc);
          v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
        }
        *reinterpret_cast<float4 *>(p.out_f32 + (size_t)gr * p.N + gc) = v;
      } else {
        *reinterpret_cast<float4 *>(p.partial + ((size_t)blockIdx.z * p.M + gr) * p.N + gc) = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.  4 wavefronts as 2x2, each owning a 64x64 block = 2x2 MFMA
// tiles of 32x32.  LDS rows are padded by 16 bytes so that the 16-byte operand
// reads of 8 consecutive lanes fall into 8 different bank groups.
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
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = k0 + kcol[i] < ke;
      ra[i] = ok ? *reinterpret_cast<const bf16x8 *>(a_ptr[i] + k0) : zero;
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
    gload(kb);
    sstore(0);
  }
  __syncthreads();
  const int frag_off = (lane & 31) * PITCH16 + 8 * (lane >> 5);
  for (int t = 0; t < nk; ++t) {
    if (t + 1 < nk) gload(kb + (t + 1) * BK16);
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
    if (t + 1 < nk) sstore((t + 1) & 1);
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
  epilogue<bf16, EPI, BM16, BN16>(sC, CPITCH16, m0, n0, p);
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
  epilogue<float, EPI, BM32, BN32>(sC, CPITCH32, m0, n0, p);
}

// out[r, c] = sum_z partial[z, r, c] (+ resid[resid_rows[r], c]), z ascending
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int splits,
                                                            int M, int N, const float *__restrict__ resid,
                                                            const int32_t *__restrict__ resid_rows,
                                                            float *__restrict__ out) {
  const size_t i4 = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total4 = (size_t)M * N / 4;
  if (i4 >= total4) return;
  const size_t e = i4 * 4;
  const int r = (int)(e / N), c = (int)(e % N);
  float4 acc = make_float4(0, 0, 0, 0);
  for (int z = 0; z < splits; ++z) {
    const float4 v = *reinterpret_cast<const float4 *>(partial + (size_t)z * M * N + e);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if (resid) {
    const int rr = resid_rows ? resid_rows[r] : r;
    const float4 q = *reinterpret_cast<const float4 *>(resid + (size_t)rr * N + c);
    acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
  }
  *reinterpret_cast<float4 *>(out + e) = acc;
}

// ---------------------------------------------------------------------------
static void tile_shape(int dtype, int epi, int *bm, int *out_cols, int *bk) {
  if (dtype == 0) { *bm = BM32; *out_cols = epi == EPI_SWIGLU ? BN32 / 2 : BN32; *bk = BK32; }
  else            { *bm = BM16; *out_cols = epi == EPI_SWIGLU ? BN16 / 2 : BN16; *bk = BK16; }
}

int gemm_splits(int dtype, int M, int N, int K) {
  int bm, oc, bk;
  tile_shape(dtype, EPI_F32, &bm, &oc, &bk);
  const long tiles = (long)ceil_div(M, bm) * ceil_div(N, oc);
  int want = (int)((512 + tiles - 1) / tiles);
  int max_by_k = K / (4 * bk);             // at least 4 k-tiles per split
  int s = want < 1 ? 1 : want;
  if (s > 8) s = 8;
  if (s > max_by_k) s = max_by_k < 1 ? 1 : max_by_k;
  int kper = ceil_div(ceil_div(K, s), bk) * bk;
  return ceil_div(K, kper);
}

template <int EPI>
static void launch_typed(int dtype, dim3 grid, const GemmParams &p, hipStream_t s) {
  if (dtype == 0) {
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, s, p);
  } else {
    static bool attr_set = false;
    if (!attr_set) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_kernel<EPI>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmemBf16);
      attr_set = true;
    }
    hipLaunchKernelGGL(gemm_bf16_kernel<EPI>, grid, dim3(256), kSmemBf16, s, p);
  }
}

// Fills the kernel parameters and the launch grid for a problem.
static void plan_gemm(const GemmArgs &g, GemmParams *pp, dim3 *grid) {
  GemmParams &p = *pp;
  p = GemmParams{};
  p.a = g.a; p.lda = g.lda; p.a_rows = g.a_rows; p.M = g.M; p.K = g.K;
  p.n_seg = g.epi == EPI_SEG ? g.n_seg : 1;
  p.nb[0] = 0;
  for (int i = 0; i < 3; ++i) {
    p.w[i] = g.seg[i].w; p.dst[i] = g.seg[i].dst; p.ld[i] = g.seg[i].ld_dst;
    p.row_map[i] = g.seg[i].row_map; p.rope[i] = g.seg[i].rope;
    p.nb[i + 1] = p.nb[i] + (i < p.n_seg ? g.seg[i].n : 0);
  }
  p.N = g.epi == EPI_SWIGLU ? g.seg[0].n : p.nb[p.n_seg];
  p.rope_tab = g.rope_tab; p.row_pos = g.row_pos; p.head_dim = g.head_dim;
  p.out_f32 = g.out_f32; p.resid = g.resid; p.resid_rows = g.resid_rows; p.partial = g.partial;
  int bm, oc, bk;
  tile_shape(g.dtype, g.epi, &bm, &oc, &bk);
  p.splits = 1;
  p.k_per_split = ceil_div(g.K, bk) * bk;
  if (g.epi == EPI_F32) {
    p.splits = gemm_splits(g.dtype, g.M, p.N, g.K);
    if (p.splits > 1) {
      if (!g.partial || g.partial_floats < (size_t)p.splits * g.M * p.N) p.splits = 1;
      else p.k_per_split = ceil_div(ceil_div(g.K, p.splits), bk) * bk;
    }
  }
  *grid = dim3(ceil_div(p.N, oc), ceil_div(g.M, bm), p.splits);
}

bool gemm_needs_reduce(const GemmArgs &g) {
  if (g.M == 0 || g.epi != EPI_F32) return false;
  GemmParams p;
  dim3 grid;
  plan_gemm(g, &p, &grid);
  return p.splits > 1;
}

hipError_t launch_gemm(const GemmArgs &g, hipStream_t s) {
  if (g.M == 0) return hipSuccess;
  GemmParams p;
  dim3 grid;
  plan_gemm(g, &p, &grid);
  if (g.epi == EPI_SEG) launch_typed<EPI_SEG>(g.dtype, grid, p, s);
  else if (g.epi == EPI_SWIGLU) launch_typed<EPI_SWIGLU>(g.dtype, grid, p, s);
  else launch_typed<EPI_F32>(g.dtype, grid, p, s);
  return hipGetLastError();
}

hipError_t launch_gemm_reduce(const GemmArgs &g, hipStream_t s) {
  if (!gemm_needs_reduce(g)) return hipSuccess;
  GemmParams p;
  dim3 grid;
  plan_gemm(g, &p, &grid);
  size_t total4 = (size_t)g.M * p.N / 4;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s,
                     g.partial, p.splits, g.M, p.N, g.resid, g.resid_rows, g.out_f32);
  return hipGetLastError();
}

}  // namespace cb
