// Bandwidth-bound kernels: positional re-alignment of cached keys (paper Sec. 4.3
// footnote / Appendix A), RMSNorm, the scatter of recomputed K/V rows into the fused
// cache for a given selection (Sec. 4.2) and copies.
#include "common.h"
#include "kernels.h"
#include <algorithm>

namespace cb {

// ---------------------------------------------------------------------------
// Re-alignment.  grid = (token tiles of the longest chunk, chunks >= 1 of this
// batch, layers of this batch).  All lanes of a block share one chunk, so the
// rotation (cos, sin) row of the table is the same for every token of the block.
// Each lane moves 16-byte vectors: several independent loads are issued before
// the first store to keep enough bytes in flight for HBM.
// ---------------------------------------------------------------------------
constexpr int kRealignLayers = 32;
constexpr int kRealignChunks = 64;
constexpr int kRealignTok = 8;
struct RealignArgs {
  void *layer[kRealignLayers];
  int32_t off[kRealignChunks + 1];  // off[i]..off[i+1] = rows of the i-th chunk of the batch
};

template <typename T>
__global__ __launch_bounds__(256) void realign_kernel(RealignArgs a, int kv_dim, int head_dim,
                                                      const float2 *__restrict__ rope_tab) {
  using V = Vec16<T>;
  const int c = blockIdx.y;
  const int begin = a.off[c], end = a.off[c + 1];
  const int tok0 = begin + blockIdx.x * kRealignTok;
  if (tok0 >= end) return;
  const int ntok = min(kRealignTok, end - tok0);
  const int vec_per_row = kv_dim / V::N;
  const int total = ntok * vec_per_row;
  V *base = reinterpret_cast<V *>(reinterpret_cast<T *>(a.layer[blockIdx.z]) + (size_t)tok0 * kv_dim);
  const float2 *tab = rope_tab + (size_t)begin * (head_dim / 2);  // rotation by the offset o_c
  constexpr int U = 4;
  for (int i0 = threadIdx.x; i0 < total; i0 += 256 * U) {
    V v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = i0 + u * 256;
      if (i < total) v[u] = base[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int i = i0 + u * 256;
      if (i < total) {
        int e0 = (i % vec_per_row) * V::N;       // first channel of this vector in the row
        int pair0 = (e0 % head_dim) / 2;
        V o;
#pragma unroll
        for (int j = 0; j < V::N / 2; ++j) {
          float2 cs = tab[pair0 + j];
          float x0 = v[u].get(2 * j), x1 = v[u].get(2 * j + 1);
          o.set(2 * j, x0 * cs.x - x1 * cs.y);
          o.set(2 * j + 1, x0 * cs.y + x1 * cs.x);
        }
        base[i] = o;
      }
    }
  }
}

// Same rotation for heads stored in the (i, i + head_dim/2) order: a work item is one 16-byte
// vector of the first half of a head together with the vector head_dim/2 channels further on.
template <typename T>
__global__ __launch_bounds__(256) void realign_half_kernel(RealignArgs a, int kv_dim, int head_dim,
                                                           const float2 *__restrict__ rope_tab) {
  using V = Vec16<T>;
  const int c = blockIdx.y;
  const int begin = a.off[c], end = a.off[c + 1];
  const int tok0 = begin + blockIdx.x * kRealignTok;
  if (tok0 >= end) return;
  const int ntok = min(kRealignTok, end - tok0);
  const int h = head_dim / 2;
  const int vec_per_row = kv_dim / V::N, vec_per_half = h / V::N;
  const int items_per_row = vec_per_row / 2;
  const int total = ntok * items_per_row;
  V *base = reinterpret_cast<V *>(reinterpret_cast<T *>(a.layer[blockIdx.z]) + (size_t)tok0 * kv_dim);
  const float2 *tab = rope_tab + (size_t)begin * h;
  constexpr int U = 2;
  for (int i0 = threadIdx.x; i0 < total; i0 += 256 * U) {
    V lo[U], hi[U];
    int at[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * 256;
      if (i < total) {
        const int row = i / items_per_row, j = i % items_per_row;
        at[u] = row * vec_per_row + (j / vec_per_half) * (2 * vec_per_half) + j % vec_per_half;
        lo[u] = base[at[u]];
        hi[u] = base[at[u] + vec_per_half];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * 256;
      if (i < total) {
        const int e0 = ((i % items_per_row) % vec_per_half) * V::N;   // first rotary block of this vector
        V olo, ohi;
#pragma unroll
        for (int j = 0; j < V::N; ++j) {
          const float2 cs = tab[e0 + j];
          const float x0 = lo[u].get(j), x1 = hi[u].get(j);
          olo.set(j, x0 * cs.x - x1 * cs.y);
          ohi.set(j, x0 * cs.y + x1 * cs.x);
        }
        base[at[u]] = olo;
        base[at[u] + vec_per_half] = ohi;
      }
    }
  }
}

hipError_t launch_realign(int dtype, void *const *k_layers, int n_layers, const int32_t *offs,
                          int n_chunks, int kv_dim, int head_dim, int rope_half, const float2 *rope_tab,
                          hipStream_t s) {
  for (int l0 = 0; l0 < n_layers; l0 += kRealignLayers) {
    int nl = std::min(kRealignLayers, n_layers - l0);
    for (int c0 = 1; c0 < n_chunks; c0 += kRealignChunks) {
      int nc = std::min(kRealignChunks, n_chunks - c0);
      RealignArgs a;
      for (int i = 0; i < kRealignLayers; ++i) a.layer[i] = k_layers[l0 + std::min(i, nl - 1)];
      int maxlen = 0;
      for (int i = 0; i <= kRealignChunks; ++i) a.off[i] = offs[c0 + std::min(i, nc)];
      for (int i = 0; i < nc; ++i) maxlen = std::max(maxlen, a.off[i + 1] - a.off[i]);
      if (maxlen <= 0) continue;
      dim3 grid((maxlen + kRealignTok - 1) / kRealignTok, nc, nl);
      if (rope_half) {
        if (dtype == 0)
          hipLaunchKernelGGL(realign_half_kernel<float>, grid, dim3(256), 0, s, a, kv_dim, head_dim, rope_tab);
        else
          hipLaunchKernelGGL(realign_half_kernel<bf16>, grid, dim3(256), 0, s, a, kv_dim, head_dim, rope_tab);
      } else if (dtype == 0) {
        hipLaunchKernelGGL(realign_kernel<float>, grid, dim3(256), 0, s, a, kv_dim, head_dim, rope_tab);
      } else {
        hipLaunchKernelGGL(realign_kernel<bf16>, grid, dim3(256), 0, s, a, kv_dim, head_dim, rope_tab);
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------
// 8-bit weights (the paper serves its larger models with 8-bit weights, Sec. 7.1): expands an int8
// matrix [rows, cols] with one float scale per row to bf16, out[r][c] = bf16(q[r][c] * scale[r]),
// 16 elements per lane (a 16-byte load, two 16-byte stores).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dequant_int8_kernel(const int8_t *__restrict__ q,
                                                           const float *__restrict__ scale,
                                                           bf16 *__restrict__ out, size_t n16, int cols16) {
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n16; i += stride) {
    const i32x4 w = reinterpret_cast<const i32x4 *>(q)[i];
    const float sc = scale[i / cols16];
    bf16x8 lo, hi;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int word = w[j];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float v = (float)((word << (24 - 8 * b)) >> 24) * sc;      // sign-extended byte b
        const int e = 4 * j + b;
        if (e < 8) lo[e] = (bf16)v; else hi[e - 8] = (bf16)v;
      }
    }
    reinterpret_cast<bf16x8 *>(out)[2 * i] = lo;
    reinterpret_cast<bf16x8 *>(out)[2 * i + 1] = hi;
  }
}
hipError_t launch_dequant_int8(const void *q, const float *scale, void *out, int rows, int cols, hipStream_t s) {
  if (rows == 0 || cols == 0) return hipSuccess;
  const size_t n16 = (size_t)rows * cols / 16;           // cols % 16 == 0 (checked by the caller)
  const int blocks = (int)std::min<size_t>((n16 + 255) / 256, 1 << 20);
  hipLaunchKernelGGL(dequant_int8_kernel, dim3(blocks), dim3(256), 0, s, (const int8_t *)q, scale, (bf16 *)out, n16,
                     cols / 16);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
template <typename T>
__global__ void to_f32_kernel(const T *__restrict__ x, float *__restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = to_f32(x[i]);
}
hipError_t launch_to_f32(int dtype, const void *x, float *out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  if (dtype == 0)
    hipLaunchKernelGGL(to_f32_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)x, out, n);
  else
    hipLaunchKernelGGL(to_f32_kernel<bf16>, dim3(blocks), dim3(256), 0, s, (const bf16 *)x, out, n);
  return hipGetLastError();
}

__global__ void copy_f32_kernel(const float4 *__restrict__ in, float4 *__restrict__ out, size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) out[i] = in[i];
}
hipError_t launch_copy_rows_f32(const float *in, float *out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t n4 = n / 4;  // callers pass multiples of 4 (d_model % 8 == 0)
  int blocks = (int)std::min<size_t>((n4 + 255) / 256, 65536);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks), dim3(256), 0, s, (const float4 *)in, (float4 *)out, n4);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// RMSNorm: one block per row; the row (float) is read twice (second read hits L2).
// With lo_off > 0 every value x is stored as the pair (hi, lo) = (T(x), T(x - hi)), lo lying
// lo_off elements after hi: the K/V projection multiplies both parts, which gives it an
// input accurate to float although the matrix cores take bf16 operands (the Q projection and
// the MLP read the high parts only).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *__restrict__ h,
                                                      const T *__restrict__ gain,
                                                      T *__restrict__ out, int ld_out, int lo_off, int d,
                                                      float eps) {
  __shared__ float red[4];
  const float4 *row = reinterpret_cast<const float4 *>(h + (size_t)blockIdx.x * d);
  const int n4 = d / 4;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 v = row[i];
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T *orow = out + (size_t)blockIdx.x * ld_out;
  for (int i = threadIdx.x; i < n4; i += 256) {
    const float4 v = row[i];
    const float x[4] = {v.x * inv * to_f32(gain[4 * i + 0]), v.y * inv * to_f32(gain[4 * i + 1]),
                        v.z * inv * to_f32(gain[4 * i + 2]), v.w * inv * to_f32(gain[4 * i + 3])};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const T hi = from_f32<T>(x[j]);
      orow[4 * i + j] = hi;
      if (lo_off > 0) orow[lo_off + 4 * i + j] = from_f32<T>(x[j] - to_f32(hi));
    }
  }
}
hipError_t launch_rmsnorm(int dtype, const float *h, const void *gain, void *out, int ld_out, int lo_off,
                          int n_rows, int d, float eps, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(n_rows), dim3(256), 0, s, h, (const float *)gain,
                       (float *)out, ld_out, lo_off, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<bf16>, dim3(n_rows), dim3(256), 0, s, h, (const bf16 *)gain,
                       (bf16 *)out, ld_out, lo_off, d, eps);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void scatter_kv_kernel(const T *__restrict__ kvnew,
                                                         const int32_t *__restrict__ sel_rows,
                                                         const int32_t *__restrict__ pos_out, int m,
                                                         T *__restrict__ kc, T *__restrict__ vc,
                                                         int kv_dim) {
  using V = Vec16<T>;
  const int nv = kv_dim / V::N;
  const size_t total = (size_t)m * 2 * nv;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int r = (int)(i / (2 * nv)), c = (int)(i % (2 * nv));
  const int src = sel_rows ? sel_rows[r] : r;
  const int p = pos_out[r];
  V v = reinterpret_cast<const V *>(kvnew + (size_t)src * 2 * kv_dim)[c];
  if (c < nv)
    reinterpret_cast<V *>(kc + (size_t)p * kv_dim)[c] = v;
  else
    reinterpret_cast<V *>(vc + (size_t)p * kv_dim)[c - nv] = v;
}
hipError_t launch_scatter_kv(int dtype, const void *kvnew, const int32_t *sel_rows,
                             const int32_t *pos_out, int m, void *kc, void *vc, int kv_dim,
                             hipStream_t s) {
  if (m == 0) return hipSuccess;
  const int vn = dtype == 0 ? 4 : 8;
  size_t total = (size_t)m * 2 * (kv_dim / vn);
  dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == 0)
    hipLaunchKernelGGL(scatter_kv_kernel<float>, grid, dim3(256), 0, s, (const float *)kvnew, sel_rows,
                       pos_out, m, (float *)kc, (float *)vc, kv_dim);
  else
    hipLaunchKernelGGL(scatter_kv_kernel<bf16>, grid, dim3(256), 0, s, (const bf16 *)kvnew, sel_rows,
                       pos_out, m, (bf16 *)kc, (bf16 *)vc, kv_dim);
  return hipGetLastError();
}

}  // namespace cb
