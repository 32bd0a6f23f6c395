// First-token head (paper Sec. 2: the prefill phase ends when the first token is
// generated): final RMSNorm of the last query token, vocabulary projection, greedy pick.
// A matrix-vector product: every weight is read once and used once, so the bound is HBM
// (vocab * d * sizeof(T) bytes), not the matrix cores.
#include "common.h"
#include "kernels.h"
#include <mutex>

namespace cb {

constexpr int kHeadRowsPerWave = 8;    // vocabulary rows per wavefront, two in flight at a time

// logits[v] = sum_e xn[e] * W[v, e], xn = T(h / sqrt(mean h^2 + eps) * gain) -- rounded to the
// storage type like every other projection input.  Each workgroup normalises the row again
// (16-32 KB of L2 hits) instead of a separate launch; its 4 wavefronts then take 8 rows each.
template <typename T>
__global__ __launch_bounds__(256) void lm_head_kernel(const float *__restrict__ h, const T *__restrict__ gain,
                                                      const T *__restrict__ w, int d, int vocab, float eps,
                                                      float *__restrict__ logits) {
  extern __shared__ __attribute__((aligned(16))) float xn[];
  __shared__ float red[4];
  float ss = 0.f;
  for (int e = threadIdx.x; e < d; e += 256) { const float v = h[e]; ss += v * v; }
  const float inv = rsqrtf(block_sum_256(ss, red) / (float)d + eps);
  for (int e = threadIdx.x; e < d; e += 256) xn[e] = to_f32(from_f32<T>(h[e] * inv * to_f32(gain[e])));
  __syncthreads();
  constexpr int N = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int v0 = (blockIdx.x * 4 + wave) * kHeadRowsPerWave;
  const int chunks = d / N;                        // 16-byte chunks per row
#pragma unroll 1
  for (int rr = 0; rr < kHeadRowsPerWave; rr += 2) {
    const int va = v0 + rr, vb = va + 1;
    if (va >= vocab) break;
    const T *ra = w + (size_t)va * d;
    const T *rb = w + (size_t)min(vb, vocab - 1) * d;
    float sa = 0.f, sb = 0.f;
    for (int c = lane; c < chunks; c += 64) {
      Vec16<T> a, b;
      a.raw = *reinterpret_cast<const decltype(a.raw) *>(ra + c * N);
      b.raw = *reinterpret_cast<const decltype(b.raw) *>(rb + c * N);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float x = xn[c * N + i];
        sa = fmaf(a.get(i), x, sa);
        sb = fmaf(b.get(i), x, sb);
      }
    }
    sa = wave_sum(sa);
    sb = wave_sum(sb);
    if (lane == 0) {
      logits[va] = sa;
      if (vb < vocab) logits[vb] = sb;
    }
  }
}

// token = smallest index among the largest logits.  One 1024-lane workgroup.
__global__ __launch_bounds__(1024) void argmax_kernel(const float *__restrict__ logits, int n,
                                                      int32_t *__restrict__ token) {
  __shared__ float s_val[16];
  __shared__ int s_idx[16];
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < n; i += 1024) {       // ascending i: strict > keeps the first
    const float v = logits[i];
    if (v > best || bi == 0x7fffffff) { best = v; bi = i; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { s_val[threadIdx.x >> 6] = best; s_idx[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 16; ++k)
      if (s_val[k] > best || (s_val[k] == best && s_idx[k] < bi)) { best = s_val[k]; bi = s_idx[k]; }
    token[0] = bi;
  }
}

hipError_t launch_lm_head(int dtype, const float *h_row, const void *gain, const void *w, int d, int vocab,
                          float eps, float *logits, hipStream_t s) {
  const int rows_per_wg = 4 * kHeadRowsPerWave;
  const dim3 grid((vocab + rows_per_wg - 1) / rows_per_wg);
  const size_t smem = (size_t)d * sizeof(float);
  // d = 16384 needs 64 KB of dynamic LDS on top of the static array: above the default limit
  static std::once_flag once;
  std::call_once(once, [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_kernel<float>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_kernel<bf16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
  });
  if (dtype == 0)
    hipLaunchKernelGGL(lm_head_kernel<float>, grid, dim3(256), smem, s, h_row, (const float *)gain,
                       (const float *)w, d, vocab, eps, logits);
  else
    hipLaunchKernelGGL(lm_head_kernel<bf16>, grid, dim3(256), smem, s, h_row, (const bf16 *)gain,
                       (const bf16 *)w, d, vocab, eps, logits);
  return hipGetLastError();
}

hipError_t launch_argmax(const float *logits, int n, int32_t *token, hipStream_t s) {
  hipLaunchKernelGGL(argmax_kernel, dim3(1), dim3(1024), 0, s, logits, n, token);
  return hipGetLastError();
}

}  // namespace cb
