// HKVD selection (paper Sec. 4.3): keep the k tokens with the largest KV deviation.
//
// One 1024-lane workgroup.  Deviations are sums of squares (>= +0, finite), so the
// unsigned order of their IEEE bit patterns is their numeric order.  Four 8-bit
// radix passes over LDS histograms find the bit pattern of the k-th largest value
// and how many entries equal to it must still be taken; one ordered compaction
// pass (wavefront ballots + per-wave totals in LDS) then emits, in ascending row
// order, every entry above the threshold plus the first `need` entries equal to
// it -- which is "ties go to the lower position".
#include "common.h"
#include "kernels.h"

namespace cb {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// exclusive prefix count of a 1-bit flag over the whole block, in thread order;
// returns this thread's exclusive count, *total = number of set flags in the block
__device__ __forceinline__ int block_excl_count(bool flag, int *wave_tot, int *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  unsigned long long m = __ballot(flag);
  int excl = __popcll(m & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[w] = __popcll(m);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) {
    int t = wave_tot[i];
    before += (i < w) ? t : 0;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return before + excl;
}

__global__ __launch_bounds__(kSelThreads) void topk_kernel(const float *__restrict__ dev, int n, int k,
                                                           int n_suffix,
                                                           const int32_t *__restrict__ row_pos,
                                                           int32_t *__restrict__ sel_rows,
                                                           int32_t *__restrict__ pos_out, int row_base) {
  __shared__ unsigned hist[256];
  __shared__ unsigned s_prefix, s_need;
  __shared__ int wave_tot[kSelWaves];
  const int tid = threadIdx.x;
  const unsigned *keys = reinterpret_cast<const unsigned *>(dev);

  unsigned prefix = 0, mask = 0, need = (unsigned)k;
  if (k > 0) {
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < n; i += kSelThreads) {
        unsigned key = keys[i];
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (tid < 64) {
        // digits are scanned from 255 downwards by one wavefront: lane l owns digits
        // 255-4l .. 252-4l; a wavefront prefix sum finds the lane, then the digit, at which
        // the running count reaches `need`
        unsigned hcnt[4], local = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { hcnt[q] = hist[255 - 4 * tid - q]; local += hcnt[q]; }
        unsigned incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          unsigned v = __shfl_up(incl, o, 64);
          if (tid >= o) incl += v;
        }
        const unsigned long long hit = __ballot(incl >= need);
        const int first = __ffsll((long long)hit) - 1;        // lowest lane whose inclusive sum reaches need
        if (tid == first) {
          unsigned cum = incl - local, digit = 0, nd = need;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (cum + hcnt[q] >= need) { digit = 255u - 4u * tid - q; nd = need - cum; break; }
            cum += hcnt[q];
          }
          s_prefix = prefix | (digit << shift);
          s_need = nd;
        }
      }
      __syncthreads();
      prefix = s_prefix;
      need = s_need;
      mask |= 0xFFu << shift;
      __syncthreads();
    }
  } else {
    prefix = 0xFFFFFFFFu;  // nothing is above or equal (no finite value has this pattern)
    need = 0;
  }
  // ordered compaction
  int eq_seen = 0, out_base = 0;
  for (int base = 0; base < n; base += kSelThreads) {
    const int i = base + tid;
    unsigned key = (i < n) ? keys[i] : 0u;
    const bool valid = i < n;
    const bool gt = valid && key > prefix;
    const bool eq = valid && key == prefix;
    int tot_eq, tot_take;
    int eq_rank = eq_seen + block_excl_count(eq, wave_tot, &tot_eq);
    const bool take = gt || (eq && (unsigned)eq_rank < need);
    int o = out_base + block_excl_count(take, wave_tot, &tot_take);
    if (take) {
      sel_rows[o] = row_base + i;
      pos_out[o] = row_pos[i];
    }
    eq_seen += tot_eq;
    out_base += tot_take;
  }
  for (int i = tid; i < n_suffix; i += kSelThreads) {
    sel_rows[k + i] = row_base + n + i;
    pos_out[k + i] = row_pos[n + i];
  }
}

hipError_t launch_topk(const float *dev, int n_cand, int k, int n_suffix, const int32_t *row_pos,
                       int32_t *sel_rows, int32_t *pos_out, int row_base, hipStream_t s) {
  if (k + n_suffix == 0) return hipSuccess;
  hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(kSelThreads), 0, s, dev, n_cand, k, n_suffix, row_pos,
                     sel_rows, pos_out, row_base);
  return hipGetLastError();
}

__global__ void forced_map_kernel(const int32_t *__restrict__ forced, int k,
                                  const int32_t *__restrict__ row_pos, int n_cand, int n_suffix,
                                  int32_t *__restrict__ sel_rows, int32_t *__restrict__ pos_out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < k) {
    const int p = forced[i];
    int lo = 0, hi = n_cand;  // lower bound of p in row_pos[0..n_cand)
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (row_pos[mid] < p) lo = mid + 1; else hi = mid;
    }
    lo = min(lo, n_cand - 1);
    sel_rows[i] = lo;
    pos_out[i] = row_pos[lo];
  } else if (i < k + n_suffix) {
    const int r = n_cand + (i - k);
    sel_rows[i] = r;
    pos_out[i] = row_pos[r];
  }
}

hipError_t launch_forced_map(const int32_t *forced, int k, const int32_t *row_pos, int n_cand,
                             int n_suffix, int32_t *sel_rows, int32_t *pos_out, hipStream_t s) {
  const int n = k + n_suffix;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(forced_map_kernel, dim3((n + 255) / 256), dim3(256), 0, s, forced, k, row_pos,
                     n_cand, n_suffix, sel_rows, pos_out);
  return hipGetLastError();
}

__global__ void gather_i32_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ idx, int n,
                                  int32_t *__restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = src[idx[i]];
}

hipError_t launch_gather_i32(const int32_t *src, const int32_t *idx, int n, int32_t *out, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, src, idx, n, out);
  return hipGetLastError();
}

}  // namespace cb
