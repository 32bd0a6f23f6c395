// HKVD selection (paper Sec. 4.3): keep the k tokens with the largest KV deviation.
//
// 1024-lane workgroups.  Deviations are sums of squares (>= +0, finite), so the
// unsigned order of their IEEE bit patterns is their numeric order.  Four 8-bit
// radix passes over LDS histograms find the bit pattern of the k-th largest value
// and how many entries equal to it must still be taken; one ordered compaction
// pass (wavefront ballots + per-wave totals in LDS) then emits, in ascending row
// order, every entry above the threshold plus the first `need` entries equal to
// it -- which is "ties go to the lower position".
#include "common.h"
#include "kernels.h"
#include <algorithm>

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

// Selection and cache update in one launch.  Every workgroup of the grid runs the same selection
// (the keys are few and sit in L2), workgroup 0 writes the index lists, and the new K/V of the
// kept rows (Sec. 6: only the kept tokens' KV is updated) are copied into the cache by workgroup
// o % gridDim.x, o being the row's rank in the output -- so the copies are spread over the chip
// without a second launch.  kvnew rows are [K | V] of vec_per_row 16-byte vectors each, indexed by
// row_base + candidate index; cache_row (NULL: row_pos) names each candidate's row in kc / vc.
constexpr int kSelList = 1024;          // kept rows one workgroup may have to copy
__global__ __launch_bounds__(kSelThreads) void topk_scatter_kernel(
    const float *__restrict__ dev, int n, int k, int n_suffix, const int32_t *__restrict__ row_pos,
    const int32_t *__restrict__ cache_row, int32_t *__restrict__ sel_rows, int32_t *__restrict__ pos_out,
    int32_t *__restrict__ cache_row_out, int row_base, const uint4 *__restrict__ kvnew, uint4 *__restrict__ kc,
    uint4 *__restrict__ vc, int vec_per_row, const int32_t *__restrict__ segs) {
  if (segs) {
    // several requests in one launch: blockIdx.y names the request, its share of every array
    // starts at its offsets in the table
    const int32_t *sg = segs + blockIdx.y * kSegInts;
    const int in_off = sg[kSegInOff], out_off = sg[kSegOutOff];
    n = sg[kSegCand]; k = sg[kSegKeep]; n_suffix = sg[kSegSuffix];
    dev += in_off; row_pos += in_off;
    if (cache_row) cache_row += in_off;
    sel_rows += out_off; pos_out += out_off;
    if (cache_row_out) cache_row_out += out_off;
    row_base = in_off;
  }
  __shared__ unsigned hist[256];
  __shared__ unsigned s_prefix, s_need;
  __shared__ int wave_tot[kSelWaves];
  __shared__ int2 list[kSelList];
  const int tid = threadIdx.x;
  const int G = gridDim.x, wg = blockIdx.x;
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
  auto emit = [&](int o, int i) {            // output rank o is candidate / suffix row i of this request
    const int cr = cache_row ? cache_row[i] : row_pos[i];
    if (wg == 0) {
      sel_rows[o] = row_base + i;
      pos_out[o] = row_pos[i];
      if (cache_row_out) cache_row_out[o] = cr;
    }
    if (o % G == wg) list[o / G] = make_int2(row_base + i, cr);
  };
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
    if (take) emit(o, i);
    eq_seen += tot_eq;
    out_base += tot_take;
  }
  for (int i = tid; i < n_suffix; i += kSelThreads) emit(k + i, n + i);
  if (kvnew == nullptr) return;              // uniform: selection only
  __syncthreads();
  const int n_out = k + n_suffix;
  const int mine = wg < n_out ? (n_out - wg + G - 1) / G : 0;
  const int per_row = 2 * vec_per_row;
  for (int idx = tid; idx < mine * per_row; idx += kSelThreads) {
    const int2 e = list[idx / per_row];
    const int c = idx % per_row;
    const uint4 v = kvnew[(size_t)e.x * per_row + c];
    if (c < vec_per_row) kc[(size_t)e.y * vec_per_row + c] = v;
    else vc[(size_t)e.y * vec_per_row + (c - vec_per_row)] = v;
  }
}

hipError_t launch_topk_scatter(const float *dev, int n_cand, int k, int n_suffix, const int32_t *row_pos,
                               const int32_t *cache_row, int32_t *sel_rows, int32_t *pos_out,
                               int32_t *cache_row_out, int row_base, const void *kvnew, void *kc, void *vc,
                               int kv_row_bytes, hipStream_t s, const int32_t *segs, int n_segs,
                               int max_out) {
  const int n_out = segs ? max_out : k + n_suffix;   // most kept + suffix rows of any request
  if (n_out == 0) return hipSuccess;
  int G = 1;
  if (kvnew) {
    G = std::min(segs ? std::max(1, 128 / n_segs) : 128, (n_out + 3) / 4);
    G = std::max(G, (n_out + kSelList - 1) / kSelList);
  }
  hipLaunchKernelGGL(topk_scatter_kernel, dim3(G, segs ? n_segs : 1), dim3(kSelThreads), 0, s, dev, n_cand, k,
                     n_suffix, row_pos, cache_row, sel_rows, pos_out, cache_row_out, row_base, (const uint4 *)kvnew,
                     (uint4 *)kc, (uint4 *)vc, kv_row_bytes / 16, segs);
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
