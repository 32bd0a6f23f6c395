// C ABI and host orchestration of the CacheBlend fusor (see include/cacheblend.h).
// Sequencing follows the paper's per-layer workflow (Sec. 4.2) with the check step
// of Sec. 6 placed right after the K/V projection: project K/V of the rows that
// reached the layer, measure their deviation from the cached K/V, keep the top-k,
// write only the kept rows into the cache, and run Q / attention / MLP on the kept
// rows alone.  Nothing here synchronises the device; row counts are known on the
// host because the keep counts are inputs.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/cacheblend.h"
#include "common.h"
#include "kernels.h"

using namespace cb;

struct ProfRec {
  int cls;
  hipEvent_t start, stop;
  double flops, bytes;
};

struct cb_ctx {
  cb_model_desc m;
  int max_tokens;
  int device;
  float2 *rope_tab;  // device [max_tokens][head_dim/2]
  int profiling;                         // 0 off, 1 every launch and the two phases, 2 the two phases only
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> free_events;
  std::vector<hipEvent_t> load_events;   // pipelined loading: [0] = entry fence, [1 + l] = layer l landed
  std::vector<int32_t> seg_tab_host;     // batched calls: host copy of the request tables being uploaded
  mutable std::vector<size_t> partial_memo;   // [rows] -> scratch floats layer calls with <= rows rows can use
  void *static_scratch;                  // this device's copy of the built-in scratch array (cb_fuse_layer_static)
};

// Built-in workspace of cb_fuse_layer_static, for callers that cannot allocate: one copy per GPU
// that loads the library, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress -- it is never passed to a kernel or a runtime call as if it were a
// device address; static_scratch_of() resolves the current device's copy once.
static __device__ __align__(256) unsigned char scratch[CB_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];            // per device: address of its copy of `scratch`

// Address of `scratch` on `device`, which must be the current device.  NULL on failure.
void *static_scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[device] = ptr;
  }
  return g_scratch_ptr[device];
}

size_t esize(const cb_ctx *c) { return c->m.dtype == CB_BF16 ? 2 : 4; }

hipEvent_t take_event(cb_ctx *c) {
  if (!c->free_events.empty()) {
    hipEvent_t e = c->free_events.back();
    c->free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

// brackets one launch (or launch group) with events when profiling is on
struct ProfScope {
  cb_ctx *c;
  hipStream_t s;
  ProfRec r;
  bool on;
  ProfScope(cb_ctx *ctx, hipStream_t st, int cls, double flops, double bytes) : c(ctx), s(st) {
    // the phase classes span many launches and are recorded in both modes
    on = ctx->profiling == 1 || (ctx->profiling == 2 && cls >= CB_PROF_PHASE_FIRST);
    if (!on) return;
    r.cls = cls; r.flops = flops; r.bytes = bytes;
    r.start = take_event(c);
    r.stop = take_event(c);
    (void)hipEventRecord(r.start, s);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(r.stop, s);
    c->recs.push_back(r);
  }
};

struct LayerWs {
  void *xn, *xn2, *kvnew, *qbuf, *obuf, *act;
  void *wstage;          // int8 weights: bf16 expansion of the projection that runs next
  float *hmid, *partial, *dev;
  int32_t *sel_rows;
  size_t partial_floats;
  size_t bytes;
};

// bf16 models feed the K/V projection a (high, low) pair per normalised activation, the low
// parts d_model elements after the high parts of the same row
int xn_lo_off(const cb_ctx *c) { return c->m.dtype == CB_BF16 ? c->m.d_model : 0; }
int xn_pitch(const cb_ctx *c) { return c->m.d_model + xn_lo_off(c); }

// Floats of scratch (parked projection sums, attention key-range pieces) that layer calls with up
// to max_rows rows can use: the maximum over EVERY row count, because neither the K split of a
// projection nor the number of key-range pieces is monotone in the row count.  Memoised per ctx.
size_t partial_floats_needed(const cb_ctx *c, int max_rows) {
  const cb_model_desc &m = c->m;
  const int d = m.d_model, q_dim = m.n_q_heads * m.head_dim, kv_dim = m.n_kv_heads * m.head_dim;
  const int rh = m.rope_layout == CB_ROPE_HALF, hl = xn_lo_off(c) > 0, w8 = m.weight_format == CB_W_INT8;
  std::vector<size_t> &memo = c->partial_memo;
  if (memo.empty()) memo.push_back(0);
  while ((int)memo.size() <= max_rows) {
    const int M = (int)memo.size();
    size_t need = memo.back();
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_SEG, M, 2 * kv_dim, d, hl, 1, rh, m.head_dim, w8));   // K|V, checked
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_SEG, M, 2 * kv_dim, d, hl, 0, rh, m.head_dim, w8));   // K|V, every row kept
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_SEG, M, q_dim, d, 0, 0, rh, m.head_dim, w8));         // Q
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_F32, M, d, q_dim, 0, 0, 0, 0, w8));
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_F32, M, d, m.d_ff, 0, 0, 0, 0, w8));
    need = std::max(need, gemm_partial_floats(m.dtype, EPI_SWIGLU, M, m.d_ff, d, 0, 0, 0, 0, w8));
    // the attention KV split borrows the same scratch (the two are never live together)
    need = std::max(need, attention_partial_floats_bound(m.dtype, M, m.n_q_heads, m.n_kv_heads, m.head_dim));
    memo.push_back(need);
  }
  return memo[max_rows];
}

// carve the per-layer workspace out of [base, base + avail); base may be NULL to size only
LayerWs carve_layer(const cb_ctx *c, char *base, int R) {
  const cb_model_desc &m = c->m;
  const size_t es = esize(c);
  const size_t q_dim = (size_t)m.n_q_heads * m.head_dim, kv_dim = (size_t)m.n_kv_heads * m.head_dim;
  LayerWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char *p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return (void *)p;
  };
  w.xn = take((size_t)R * xn_pitch(c) * es);
  w.xn2 = take((size_t)R * m.d_model * es);
  w.kvnew = take((size_t)R * 2 * kv_dim * es);
  w.qbuf = take((size_t)R * q_dim * es);
  w.obuf = take((size_t)R * q_dim * es);
  w.act = take((size_t)R * m.d_ff * es);
  w.hmid = (float *)take((size_t)R * m.d_model * 4);
  w.partial_floats = partial_floats_needed(c, R);
  w.partial = (float *)take(w.partial_floats * 4);
  w.dev = (float *)take((size_t)R * 4);
  w.sel_rows = (int32_t *)take((size_t)R * 4);
  // int8 weights that the projection kernels cannot read themselves: room for the widest such projection
  // (gate and up together, or K and V together) expanded to bf16
  size_t stage = 0;
  if (m.weight_format == CB_W_INT8) {
    const int dt = m.dtype == CB_BF16 ? 1 : 0;
    if (!gemm_int8_in_kernel(dt, m.d_model)) stage = std::max((size_t)2 * m.d_ff, q_dim + 2 * kv_dim) * m.d_model * 2;
    if (!gemm_int8_in_kernel(dt, (int)q_dim)) stage = std::max(stage, q_dim * m.d_model * 2);
    if (!gemm_int8_in_kernel(dt, m.d_ff)) stage = std::max(stage, (size_t)m.d_ff * m.d_model * 2);
  }
  w.wstage = take(stage);
  w.bytes = off;
  return w;
}

__global__ void iota_kernel(int32_t *p, int n, int base) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = base + i;
}

#define CB_HIP(expr)                     \
  do {                                   \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return CB_EHIP; \
  } while (0)

// The kernels move tensors in 16-byte vectors and index arrays in 4-byte words: a pointer that is
// not aligned accordingly would fault on the device, so it is refused on the host.  NULL passes
// (whether NULL is allowed is checked separately).
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
bool weights_aligned(const cb_layer_weights *w) {
  return aligned(w->attn_norm, 16) && aligned(w->wq, 16) && aligned(w->wk, 16) && aligned(w->wv, 16) &&
         aligned(w->wo, 16) && aligned(w->mlp_norm, 16) && aligned(w->w_gate, 16) && aligned(w->w_up, 16) &&
         aligned(w->w_down, 16);
}

// int8 weights: every matrix needs its scale array (float, 4-byte aligned)
int scales_ok_status(const cb_layer_weights *w) {
  const float *sc[7] = {w->wq_scale, w->wk_scale, w->wv_scale, w->wo_scale, w->w_gate_scale, w->w_up_scale,
                        w->w_down_scale};
  for (const float *p : sc) {
    if (!p) return CB_ENULL;
    if (!aligned(p, 4)) return CB_EINVAL;
  }
  return CB_OK;
}
bool scales_ok(const cb_layer_weights *w) { return scales_ok_status(w) == CB_OK; }

int check_layer_args(const cb_ctx *c, int layer, const cb_layer_weights *w, int n_rows, int n_suffix,
                     int n_tokens_total, int k_keep) {
  if (!c || !w) return CB_ENULL;
  if (!w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->mlp_norm || !w->w_gate || !w->w_up ||
      !w->w_down)
    return CB_ENULL;
  if (!weights_aligned(w)) return CB_EINVAL;
  if (c->m.weight_format == CB_W_INT8 && !scales_ok(w)) return scales_ok_status(w);
  if (layer < 0 || layer >= c->m.n_layers) return CB_EINVAL;
  if (n_rows < 0 || n_suffix < 0 || n_suffix > n_rows) return CB_EINVAL;
  if (k_keep < 0 || k_keep > n_rows - n_suffix) return CB_EINVAL;
  if (n_tokens_total < 1 || n_tokens_total > c->max_tokens || n_rows > n_tokens_total) return CB_EINVAL;
  return CB_OK;
}

// The matrices a projection launch reads.  Native weights: the caller's pointers.  int8 weights: the
// projection kernel reads them itself (scale non-NULL) wherever it can -- bf16 storage and an input width
// that is a multiple of 64 --; otherwise each matrix is expanded to the storage type into the staging area
// first (one after the other, so that the matrices of one launch lie side by side) and the launch reads
// the expansion.
struct WeightView { const void *w[3]; const float *scale[3]; };
int stage_weights(cb_ctx *c, hipStream_t s, const LayerWs &ws, int n, const void *const *w,
                  const float *const *scale, const int *rows, int cols, WeightView *out) {
  for (int i = 0; i < 3; ++i) out->scale[i] = nullptr;
  if (c->m.weight_format != CB_W_INT8) {
    for (int i = 0; i < n; ++i) out->w[i] = w[i];
    return CB_OK;
  }
  if (gemm_int8_in_kernel(c->m.dtype == CB_BF16 ? 1 : 0, cols)) {
    for (int i = 0; i < n; ++i) { out->w[i] = w[i]; out->scale[i] = scale[i]; }
    return CB_OK;
  }
  size_t off = 0, bytes = 0;
  for (int i = 0; i < n; ++i) bytes += (size_t)rows[i] * cols * 3;
  ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)bytes);
  for (int i = 0; i < n; ++i) {
    char *dst = (char *)ws.wstage + off;
    CB_HIP(launch_dequant_int8(w[i], scale[i], dst, rows[i], cols, s));
    out->w[i] = dst;
    off += align_up((size_t)rows[i] * cols * 2, 256);
  }
  return CB_OK;
}

// One request's share of the rows of a layer call: n rows enter (the last S of them its suffix),
// k context rows are kept, its caches hold T rows.
struct Seg { int n, S, k, T; };

// runs a projection: the main launch and, when its sums were parked, the finish launch
int run_gemm(cb_ctx *c, hipStream_t s, const GemmArgs &g, int finish_class, double flops, double bytes,
             double finish_bytes) {
  {
    ProfScope ps(c, s, CB_PROF_GEMM, flops, bytes);
    CB_HIP(launch_gemm(g, s));
  }
  if (gemm_needs_finish(g)) {
    ProfScope ps(c, s, finish_class, 0, finish_bytes);
    CB_HIP(launch_gemm_finish(g, s));
  }
  return CB_OK;
}
#define CB_TRY(expr)            \
  do {                          \
    const int st_ = (expr);     \
    if (st_ != CB_OK) return st_; \
  } while (0)

// The layer body; arguments already validated.  Rows of several requests may be stacked
// (request-major): the projections then run on all of them at once, selection and attention per
// request.  cache_row (NULL: row_pos) gives each row's row in the cache arrays, which hold the
// requests' slabs cache_stride rows apart; cache_row_out receives it for the kept rows.
// xn_ready: ws.xn already holds the normalised input rows (left there by the previous layer's
// call through next_gain).  next_gain (NULL: none): gain of the RMSNorm that will read h_out;
// the normalised rows are then left in ws.xn by the launch that finishes h_out.
int fuse_layer_impl(cb_ctx *c, const cb_layer_weights *w, const float *h_in, const int32_t *row_pos,
                    const int32_t *cache_row, const Seg *segs, int n_segs, size_t cache_stride, void *kc,
                    void *vc, const int32_t *forced, float *h_out, int32_t *pos_out, int32_t *cache_row_out,
                    float *dev_out, const LayerWs &ws, hipStream_t s, bool xn_ready, const void *next_gain,
                    const int32_t *seg_dev = nullptr) {
  const cb_model_desc &m = c->m;
  const int dt = m.dtype;
  const size_t es = esize(c);
  const int d = m.d_model, q_dim = m.n_q_heads * m.head_dim, kv_dim = m.n_kv_heads * m.head_dim;
  const int F = m.d_ff;
  const int lo_off = xn_lo_off(c), xld = xn_pitch(c);
  int n = 0, rows = 0;
  bool check = forced != nullptr;
  for (int b = 0; b < n_segs; ++b) {
    n += segs[b].n;
    rows += segs[b].k + segs[b].S;
    check = check || segs[b].k < segs[b].n - segs[b].S;
  }
  if (n == 0) return CB_OK;
  const int32_t *crow = cache_row ? cache_row : row_pos;

  if (!xn_ready) {
    ProfScope ps(c, s, CB_PROF_NORM, 0, (double)n * d * (4 + es * (lo_off ? 2 : 1)));
    CB_HIP(launch_rmsnorm(dt, h_in, w->attn_norm, ws.xn, xld, lo_off, n, d, m.rms_eps, s));
  }
  GemmArgs g = {};
  g.dtype = dt; g.rope_tab = c->rope_tab; g.head_dim = m.head_dim; g.rope_half = m.rope_layout == CB_ROPE_HALF;
  g.partial = ws.partial; g.partial_floats = ws.partial_floats;
  g.a = ws.xn; g.lda = xld; g.K = d; g.epi = EPI_SEG;
  const int32_t *sel_rows = nullptr;
  WeightView wv = {};
  // K and V of every row that reached this layer (Sec. 6: the KV computed anew on this layer), from the
  // (high, low) activation pairs: an error in a stored key is multiplied by the score it takes part in,
  // so the keys and values get a float-accurate input.  With a check they go to the workspace and the
  // launch that finishes them also measures every candidate's deviation from its cached K/V; without
  // one every row is kept and they are written straight into the cache.
  g.a_rows = nullptr; g.M = n; g.n_seg = 2; g.a_lo_off = lo_off;
  {
    const void *wm[2] = {w->wk, w->wv};
    const float *sc[2] = {w->wk_scale, w->wv_scale};
    const int wr[2] = {kv_dim, kv_dim};
    CB_TRY(stage_weights(c, s, ws, 2, wm, sc, wr, d, &wv));
  }
  g.row_pos = row_pos;
  const double kv_flops = 2.0 * n * d * 2 * kv_dim, kv_bytes = ((double)2 * kv_dim * d + (double)n * d + (double)n * 2 * kv_dim) * es;
  if (check) {
    g.seg[0] = {wv.w[0], kv_dim, ws.kvnew, 2 * kv_dim, nullptr, 1, kc, wv.scale[0]};
    g.seg[1] = {wv.w[1], kv_dim, (char *)ws.kvnew + (size_t)kv_dim * es, 2 * kv_dim, nullptr, 0, vc, wv.scale[1]};
    float *dev = dev_out ? dev_out : ws.dev;
    // one request: its candidates are the leading rows; several: every row gets a value (a
    // suffix row's is never looked at)
    const int n_dev = n_segs == 1 ? n - segs[0].S : n;
    g.dev_out = dev; g.n_dev = n_dev; g.dev_row = crow;
    CB_TRY(run_gemm(c, s, g, CB_PROF_DEV, kv_flops, kv_bytes, (double)n_dev * (4.0 * kv_dim * es + 4)));
    g.dev_out = nullptr;
    {
      ProfScope ps(c, s, CB_PROF_TOPK, 0, (double)n_dev * 4 + (double)rows * (8 + 4.0 * kv_dim * es));
      if (forced) {
        CB_HIP(launch_forced_map(forced, segs[0].k, row_pos, n - segs[0].S, segs[0].S, ws.sel_rows, pos_out, s));
        if (cache_row_out && rows > 0) CB_HIP(launch_gather_i32(crow, ws.sel_rows, rows, cache_row_out, s));
        // only the kept tokens' KV is updated (Sec. 6)
        CB_HIP(launch_scatter_kv(dt, ws.kvnew, ws.sel_rows, cache_row_out ? cache_row_out : pos_out, rows, kc, vc,
                                 kv_dim, s));
      } else {
        // selection and the update of the kept tokens' KV (Sec. 6) in one launch: one request, or all
        // requests of the call through the device table; without a table, a launch per request
        int in_off = 0, out_off = 0, max_out = 0;
        for (int b = 0; b < n_segs; ++b) max_out = std::max(max_out, segs[b].k + segs[b].S);
        if (seg_dev)
          CB_HIP(launch_topk_scatter(dev, 0, 0, 0, row_pos, cache_row, ws.sel_rows, pos_out, cache_row_out, 0,
                                     ws.kvnew, kc, vc, (int)(kv_dim * es), s, seg_dev, n_segs, max_out));
        for (int b = 0; b < n_segs && !seg_dev; ++b) {
          CB_HIP(launch_topk_scatter(dev + in_off, segs[b].n - segs[b].S, segs[b].k, segs[b].S, row_pos + in_off,
                                     cache_row ? cache_row + in_off : nullptr, ws.sel_rows + out_off,
                                     pos_out + out_off, cache_row_out ? cache_row_out + out_off : nullptr, in_off,
                                     ws.kvnew, kc, vc, (int)(kv_dim * es), s));
          in_off += segs[b].n;
          out_off += segs[b].k + segs[b].S;
        }
      }
    }
    if (rows == 0) return CB_OK;
    sel_rows = ws.sel_rows;
  } else {
    {
      ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)n * 8);
      CB_HIP(hipMemcpyAsync(pos_out, row_pos, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
      if (cache_row_out)
        CB_HIP(hipMemcpyAsync(cache_row_out, crow, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
    }
    g.seg[0] = {wv.w[0], kv_dim, kc, kv_dim, crow, 1, nullptr, wv.scale[0]};
    g.seg[1] = {wv.w[1], kv_dim, vc, kv_dim, crow, 0, nullptr, wv.scale[1]};
    CB_TRY(run_gemm(c, s, g, CB_PROF_REDUCE, kv_flops, kv_bytes, 0));
  }
  // Q of the rows that are kept (Sec. 4.2), gathered through the selection; plain bf16 operands
  g.a_rows = sel_rows; g.M = rows; g.n_seg = 1; g.a_lo_off = 0;
  {
    const void *wm[1] = {w->wq};
    const float *sc[1] = {w->wq_scale};
    const int wr[1] = {q_dim};
    CB_TRY(stage_weights(c, s, ws, 1, wm, sc, wr, d, &wv));
  }
  g.seg[0] = {wv.w[0], q_dim, ws.qbuf, q_dim, nullptr, 1, nullptr, wv.scale[0]};
  g.row_pos = pos_out;
  CB_TRY(run_gemm(c, s, g, CB_PROF_REDUCE, 2.0 * rows * d * q_dim,
                  ((double)q_dim * d + (double)rows * d + (double)rows * q_dim) * es, 0));
  {
    // attention is per request: its rows against its own cache slab -- all requests in one launch
    // through the device table (bf16), else a launch per request
    ProfScope ps(c, s, CB_PROF_ATTN, 0, 0);
    int out_off = 0;
    const bool varlen = seg_dev && dt == CB_BF16;
    if (varlen) {
      long total_qwg = 0;
      int max_t = 0;
      for (int b = 0; b < n_segs; ++b) {
        total_qwg += attention_query_workgroups(segs[b].k + segs[b].S, m.n_q_heads, m.n_kv_heads);
        max_t = std::max(max_t, segs[b].T);
      }
      CB_HIP(launch_attention(dt, ws.qbuf, nullptr, pos_out, rows, kc, vc, ws.obuf, m.n_q_heads,
                              m.n_kv_heads, m.head_dim, max_t, ws.partial, ws.partial_floats, s, seg_dev, n_segs,
                              total_qwg));
    }
    for (int b = 0; b < n_segs && !varlen; ++b) {
      const int rows_b = segs[b].k + segs[b].S;
      const char *q_b = (const char *)ws.qbuf + (size_t)out_off * q_dim * es;
      CB_HIP(launch_attention(dt, q_b, nullptr, pos_out + out_off, rows_b,
                              (char *)kc + (size_t)b * cache_stride * kv_dim * es,
                              (char *)vc + (size_t)b * cache_stride * kv_dim * es,
                              (char *)ws.obuf + (size_t)out_off * q_dim * es, m.n_q_heads, m.n_kv_heads,
                              m.head_dim, segs[b].T, ws.partial, ws.partial_floats, s));
      out_off += rows_b;
    }
  }
  // hmid = H + o Wo^T, and its RMSNorm (the MLP's input) from the launch that finishes it
  GemmArgs f = {};
  f.dtype = dt; f.a = ws.obuf; f.lda = q_dim; f.M = rows; f.K = q_dim; f.epi = EPI_F32; f.n_seg = 1;
  {
    const void *wm[1] = {w->wo};
    const float *sc[1] = {w->wo_scale};
    const int wr[1] = {d};
    CB_TRY(stage_weights(c, s, ws, 1, wm, sc, wr, q_dim, &wv));
  }
  f.seg[0].w = wv.w[0]; f.seg[0].w_scale = wv.scale[0]; f.seg[0].n = d;
  f.out_f32 = ws.hmid; f.resid = h_in; f.resid_rows = sel_rows;
  f.norm_gain = w->mlp_norm; f.norm_out = ws.xn2; f.norm_ld = d; f.norm_lo_off = 0; f.norm_eps = m.rms_eps;
  f.partial = ws.partial; f.partial_floats = ws.partial_floats;
  CB_TRY(run_gemm(c, s, f, CB_PROF_REDUCE, 2.0 * rows * q_dim * d, ((double)q_dim * d + (double)rows * q_dim) * es,
                  (double)rows * d * (12 + es)));
  GemmArgs u = {};
  u.dtype = dt; u.a = ws.xn2; u.lda = d; u.M = rows; u.K = d; u.epi = EPI_SWIGLU; u.n_seg = 2;
  {
    const void *wm[2] = {w->w_gate, w->w_up};
    const float *sc[2] = {w->w_gate_scale, w->w_up_scale};
    const int wr[2] = {F, F};
    CB_TRY(stage_weights(c, s, ws, 2, wm, sc, wr, d, &wv));
  }
  u.seg[0] = {wv.w[0], F, ws.act, F, nullptr, 0, nullptr, wv.scale[0]};
  u.seg[1] = {wv.w[1], F, nullptr, 0, nullptr, 0, nullptr, wv.scale[1]};
  u.partial = ws.partial; u.partial_floats = ws.partial_floats;
  CB_TRY(run_gemm(c, s, u, CB_PROF_REDUCE, 2.0 * rows * d * 2 * F,
                  ((double)2 * F * d + (double)rows * d + (double)rows * F) * es, 0));
  // h_out = hmid + act Wd^T; the next layer's normalised input comes from the same finish launch
  {
    const void *wm[1] = {w->w_down};
    const float *sc[1] = {w->w_down_scale};
    const int wr[1] = {d};
    CB_TRY(stage_weights(c, s, ws, 1, wm, sc, wr, F, &wv));
  }
  f.a = ws.act; f.lda = F; f.K = F; f.seg[0].w = wv.w[0]; f.seg[0].w_scale = wv.scale[0];
  f.out_f32 = h_out; f.resid = ws.hmid; f.resid_rows = nullptr;
  f.norm_gain = next_gain; f.norm_out = ws.xn; f.norm_ld = xld; f.norm_lo_off = lo_off;
  CB_TRY(run_gemm(c, s, f, CB_PROF_REDUCE, 2.0 * rows * F * d, ((double)F * d + (double)rows * F) * es,
                  (double)rows * d * (12 + (next_gain ? es * (lo_off ? 2 : 1) : 0))));
  return CB_OK;
}

}  // namespace

extern "C" {

const char *cb_strerror(int status) {
  switch (status) {
    case CB_OK: return "ok";
    case CB_EINVAL: return "invalid argument";
    case CB_ENULL: return "null pointer";
    case CB_EWORKSPACE: return "workspace too small";
    case CB_EUNSUPPORTED: return "unsupported model geometry";
    case CB_EHIP: return "HIP runtime error";
    case CB_ENOMEM: return "out of memory";
    default: return "unknown status";
  }
}

int cb_create(const cb_model_desc *desc, int32_t max_tokens, cb_ctx **out) {
  if (!desc || !out) return CB_ENULL;
  *out = nullptr;
  const cb_model_desc &m = *desc;
  if (m.n_layers < 1 || m.d_model < 8 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.d_ff < 8 ||
      max_tokens < 1 || max_tokens > (1 << 24) || !(m.rms_eps > 0.f) || !(m.rope_theta > 0.f))
    return CB_EINVAL;
  if (m.dtype != CB_F32 && m.dtype != CB_BF16) return CB_EINVAL;
  if (m.rope_layout != CB_ROPE_ADJACENT && m.rope_layout != CB_ROPE_HALF) return CB_EINVAL;
  if (m.weight_format != CB_W_NATIVE && m.weight_format != CB_W_INT8) return CB_EINVAL;
  // int8 weights are expanded 16 at a time into bf16
  if (m.weight_format == CB_W_INT8 && (m.dtype != CB_BF16 || m.d_model % 16 != 0 || m.d_ff % 16 != 0))
    return CB_EUNSUPPORTED;
  if (m.head_dim != 64 && m.head_dim != 128) return CB_EUNSUPPORTED;
  if (m.n_q_heads % m.n_kv_heads != 0) return CB_EUNSUPPORTED;
  if (m.d_model % 8 != 0 || m.d_ff % 8 != 0) return CB_EUNSUPPORTED;  // 16-byte operand vectors
  cb_ctx *c = new (std::nothrow) cb_ctx();
  if (!c) return CB_ENOMEM;
  c->m = m;
  c->max_tokens = max_tokens;
  c->profiling = 0;
  c->rope_tab = nullptr;
  if (hipGetDevice(&c->device) != hipSuccess) { delete c; return CB_EHIP; }
  c->static_scratch = static_scratch_of(c->device);
  if (!c->static_scratch) { delete c; return CB_EHIP; }
  // rotary table in double precision on the host: (cos, sin)(p * theta^(-2i/dh)) (Appendix A)
  const int half = m.head_dim / 2;
  std::vector<float2> tab;
  std::vector<double> freq;
  try {
    tab.resize((size_t)max_tokens * half);
    freq.resize(half);
  } catch (...) {                       // no exception may cross the C boundary
    delete c;
    return CB_ENOMEM;
  }
  for (int i = 0; i < half; ++i) freq[i] = std::pow((double)m.rope_theta, -2.0 * i / m.head_dim);
  for (int p = 0; p < max_tokens; ++p)
    for (int i = 0; i < half; ++i) {
      const double a = (double)p * freq[i];
      tab[(size_t)p * half + i] = make_float2((float)std::cos(a), (float)std::sin(a));
    }
  if (hipMalloc(&c->rope_tab, tab.size() * sizeof(float2)) != hipSuccess) { delete c; return CB_ENOMEM; }
  if (hipMemcpy(c->rope_tab, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(c->rope_tab);
    delete c;
    return CB_EHIP;
  }
  *out = c;
  return CB_OK;
}

void cb_destroy(cb_ctx *c) {
  if (!c) return;
  for (auto &r : c->recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  for (auto e : c->load_events) (void)hipEventDestroy(e);
  if (c->rope_tab) (void)hipFree(c->rope_tab);
  delete c;
}

size_t cb_layer_workspace_bytes(const cb_ctx *c, int32_t max_rows) {
  if (!c || max_rows < 1) return 0;
  return carve_layer(c, nullptr, max_rows).bytes;
}

size_t cb_prefill_workspace_bytes(const cb_ctx *c, int32_t n_tokens) {
  if (!c || n_tokens < 1) return 0;
  size_t h = align_up((size_t)n_tokens * c->m.d_model * 4, 256);
  size_t p = align_up((size_t)n_tokens * 4, 256);
  return 2 * h + 2 * p + carve_layer(c, nullptr, n_tokens).bytes;
}

int cb_default_schedule(int32_t n_layers, int32_t n_ctx, double r, double r1, int32_t flat,
                        int32_t *keep_counts) {
  if (!keep_counts) return CB_ENULL;
  if (n_layers < 1 || n_ctx < 0 || !(r >= 0.0) || r > 1.0) return CB_EINVAL;
  const double rd = r, r1d = (r1 > 0.0) ? r1 : 2.0 * rd;
  const double r_end = (3.0 * rd - r1d) / 2.0;
  keep_counts[0] = n_ctx;
  for (int l = 1; l < n_layers; ++l) {
    double rl = rd;
    if (!flat) {
      const double t = (double)(l - 1) / (double)std::max(1, n_layers - 2);
      rl = r_end + (r1d - r_end) * (1.0 - t) * (1.0 - t);
    }
    long k = (long)std::ceil(rl * n_ctx - 1e-9);
    if (k < 0) k = 0;
    if (k > keep_counts[l - 1]) k = keep_counts[l - 1];
    keep_counts[l] = (int32_t)k;
  }
  return CB_OK;
}

int cb_realign_rope(cb_ctx *c, void *const *k_cache_layers, int32_t layer_begin, int32_t layer_end,
                    const int32_t *chunk_offsets, int32_t n_chunks, void *stream) {
  if (!c || !k_cache_layers || !chunk_offsets) return CB_ENULL;
  if (layer_begin < 0 || layer_end > c->m.n_layers || layer_begin > layer_end || n_chunks < 1)
    return CB_EINVAL;
  if (chunk_offsets[0] != 0) return CB_EINVAL;
  for (int i = 0; i < n_chunks; ++i)
    if (chunk_offsets[i + 1] <= chunk_offsets[i]) return CB_EINVAL;
  if (chunk_offsets[n_chunks] > c->max_tokens) return CB_EINVAL;
  for (int l = layer_begin; l < layer_end; ++l) {
    if (!k_cache_layers[l]) return CB_ENULL;
    if (!aligned(k_cache_layers[l], 16)) return CB_EINVAL;
  }
  if (layer_begin == layer_end || n_chunks == 1) return CB_OK;
  hipStream_t s = (hipStream_t)stream;
  const int kv_dim = c->m.n_kv_heads * c->m.head_dim;
  const double moved = 2.0 * (layer_end - layer_begin) *
                       (double)(chunk_offsets[n_chunks] - chunk_offsets[1]) * kv_dim * esize(c);
  ProfScope ps(c, s, CB_PROF_REALIGN, 0, moved);
  CB_HIP(launch_realign(c->m.dtype, k_cache_layers + layer_begin, layer_end - layer_begin, chunk_offsets,
                        n_chunks, kv_dim, c->m.head_dim, c->m.rope_layout == CB_ROPE_HALF, c->rope_tab, s));
  return CB_OK;
}

int cb_fuse_layer(cb_ctx *c, int32_t layer, const cb_layer_weights *w, const float *h_in,
                  const int32_t *row_pos, int32_t n_rows, int32_t n_suffix, void *k_cache, void *v_cache,
                  int32_t n_tokens_total, int32_t k_keep, const int32_t *forced_sel, float *h_out,
                  int32_t *pos_out, float *dev_out, void *workspace, size_t workspace_bytes,
                  void *stream) {
  int st = check_layer_args(c, layer, w, n_rows, n_suffix, n_tokens_total, k_keep);
  if (st != CB_OK) return st;
  if (!h_in || !row_pos || !k_cache || !v_cache || !h_out || !pos_out || !workspace) return CB_ENULL;
  if (h_out == h_in || pos_out == row_pos) return CB_EINVAL;
  if (!aligned(h_in, 16) || !aligned(h_out, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
      !aligned(row_pos, 4) || !aligned(pos_out, 4) || !aligned(forced_sel, 4) || !aligned(dev_out, 4) ||
      !aligned(workspace, 256))
    return CB_EINVAL;
  if (n_rows == 0) return CB_OK;
  LayerWs ws = carve_layer(c, (char *)workspace, n_rows);
  if (ws.bytes > workspace_bytes) return CB_EWORKSPACE;
  const Seg seg = {n_rows, n_suffix, k_keep, n_tokens_total};
  return fuse_layer_impl(c, w, h_in, row_pos, nullptr, &seg, 1, 0, k_cache, v_cache, forced_sel, h_out, pos_out,
                         nullptr, dev_out, ws, (hipStream_t)stream, false, nullptr);
}

size_t cb_static_scratch_bytes(void) { return CB_STATIC_SCRATCH_BYTES; }

int cb_fuse_layer_static(cb_ctx *c, int32_t layer, const cb_layer_weights *w, const float *h_in,
                         const int32_t *row_pos, int32_t n_rows, int32_t n_suffix, void *k_cache,
                         void *v_cache, int32_t n_tokens_total, int32_t k_keep, const int32_t *forced_sel,
                         float *h_out, int32_t *pos_out, float *dev_out, void *stream) {
  if (!c) return CB_ENULL;
  if (n_rows > 0 && cb_layer_workspace_bytes(c, n_rows) > CB_STATIC_SCRATCH_BYTES) return CB_EWORKSPACE;
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return CB_EHIP;
  if (device != c->device) return CB_EINVAL;   // the ctx's device holds the scratch this call would use
  // per-launch timing creates events; this entry point creates nothing
  const int profiling = c->profiling;
  c->profiling = 0;
  const int st = cb_fuse_layer(c, layer, w, h_in, row_pos, n_rows, n_suffix, k_cache, v_cache, n_tokens_total,
                               k_keep, forced_sel, h_out, pos_out, dev_out, c->static_scratch,
                               CB_STATIC_SCRATCH_BYTES, stream);
  c->profiling = profiling;
  return st;
}

namespace {

// Body of cb_fuse_prefill and cb_fuse_prefill_pipelined.  k_host/v_host NULL: the caches are
// already on the device and all layers are re-aligned in one launch.  Otherwise layer l's rows
// are copied from host memory on copy_stream, and the compute stream waits for that copy,
// re-aligns the layer and fuses it (Sec. 5, pipelining of loading and recompute).
int prefill_impl(cb_ctx *c, const cb_layer_weights *layers, const void *x, const int32_t *chunk_lens,
                 int32_t n_chunks, int32_t n_suffix, const void *const *k_host, const void *const *v_host,
                 void *const *k_cache_layers, void *const *v_cache_layers, const int32_t *keep_counts,
                 const int32_t *const *forced_sel, float *final_hidden, int32_t *const *sel_dump,
                 float *const *dev_dump, void *workspace, size_t workspace_bytes, void *stream,
                 void *copy_stream) {
  if (!c || !layers || !x || !chunk_lens || !k_cache_layers || !v_cache_layers || !keep_counts ||
      !workspace)
    return CB_ENULL;
  if (n_chunks < 1 || n_suffix < 0) return CB_EINVAL;
  if (n_suffix > 0 && !final_hidden) return CB_ENULL;
  const int L = c->m.n_layers, d = c->m.d_model;
  std::vector<int32_t> off(n_chunks + 1, 0);
  for (int i = 0; i < n_chunks; ++i) {
    if (chunk_lens[i] < 1) return CB_EINVAL;
    if ((long)off[i] + chunk_lens[i] > c->max_tokens) return CB_EINVAL;
    off[i + 1] = off[i] + chunk_lens[i];
  }
  const int C = off[n_chunks];
  if ((long)C + n_suffix > c->max_tokens) return CB_EINVAL;
  const int T = C + n_suffix;
  if (keep_counts[0] != C) return CB_EINVAL;
  for (int l = 1; l < L; ++l)
    if (keep_counts[l] < 0 || keep_counts[l] > keep_counts[l - 1]) return CB_EINVAL;
  if (!aligned(x, 16) || !aligned(final_hidden, 16) || !aligned(workspace, 256)) return CB_EINVAL;
  for (int l = 0; l < L; ++l) {
    if (!k_cache_layers[l] || !v_cache_layers[l]) return CB_ENULL;
    if (k_host && (!k_host[l] || !v_host[l])) return CB_ENULL;
    if (!aligned(k_cache_layers[l], 16) || !aligned(v_cache_layers[l], 16)) return CB_EINVAL;
    if ((forced_sel && !aligned(forced_sel[l], 4)) || (sel_dump && !aligned(sel_dump[l], 4)) ||
        (dev_dump && !aligned(dev_dump[l], 4)))
      return CB_EINVAL;
    int st = check_layer_args(c, l, &layers[l], T, n_suffix, T, 0);
    if (st != CB_OK) return st;
  }
  if (cb_prefill_workspace_bytes(c, T) > workspace_bytes) return CB_EWORKSPACE;
  if (k_host) {
    // the copy stream first waits for whatever the compute stream still has in flight on the
    // destination buffers
    while ((int)c->load_events.size() < L + 1) {
      hipEvent_t e = nullptr;
      CB_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      c->load_events.push_back(e);
    }
    hipStream_t cs = (hipStream_t)copy_stream;
    CB_HIP(hipEventRecord(c->load_events[0], (hipStream_t)stream));
    CB_HIP(hipStreamWaitEvent(cs, c->load_events[0], 0));
  }
  // Copy of layer l's pre-computed K/V, queued on the copy stream.  Layer 0 recomputes every row
  // (keep_counts[0] == n_ctx) and never reads its cached K/V, so it has no copy.
  auto queue_load = [&](int l) -> hipError_t {
    if (!k_host || l < 1 || l >= L) return hipSuccess;
    hipStream_t cs = (hipStream_t)copy_stream;
    const size_t bytes = (size_t)C * c->m.n_kv_heads * c->m.head_dim * esize(c);
    hipError_t e = hipMemcpyAsync(k_cache_layers[l], k_host[l], bytes, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess) e = hipMemcpyAsync(v_cache_layers[l], v_host[l], bytes, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess) e = hipEventRecord(c->load_events[1 + l], cs);
    return e;
  };

  hipStream_t s = (hipStream_t)stream;
  char *base = (char *)workspace;
  const size_t hb = align_up((size_t)T * d * 4, 256), pb = align_up((size_t)T * 4, 256);
  float *h_cur = (float *)base, *h_nxt = (float *)(base + hb);
  int32_t *p_cur = (int32_t *)(base + 2 * hb), *p_nxt = (int32_t *)(base + 2 * hb + pb);
  LayerWs ws = carve_layer(c, base + 2 * hb + 2 * pb, T);

  // phase marks: everything up to the end of layer 0 (the full first layer), then the selective layers
  ProfScope *phase = new (std::nothrow) ProfScope(c, s, CB_PROF_PHASE_FIRST, 0, 0);
  struct PhaseGuard { ProfScope *&p; ~PhaseGuard() { delete p; } } phase_guard{phase};
  {
    ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)T * d * (4 + esize(c)));
    CB_HIP(launch_to_f32(c->m.dtype, x, h_cur, (size_t)T * d, s));
    hipLaunchKernelGGL(iota_kernel, dim3((T + 255) / 256), dim3(256), 0, s, p_cur, T, 0);
    CB_HIP(hipGetLastError());
  }
  int st = CB_OK;
  if (!k_host && L > 1) {      // layer 0 overwrites all of its rows: nothing of it to re-align
    st = cb_realign_rope(c, k_cache_layers, 1, L, off.data(), n_chunks, stream);
    if (st != CB_OK) return st;
  }

  // The host runs far ahead of the device, so queueing the copies two layers ahead of the layer
  // being launched keeps the copy stream busy from the start without holding back the first launch.
  CB_HIP(queue_load(1));
  CB_HIP(queue_load(2));
  int n = T;
  for (int l = 0; l < L; ++l) {
    const int k = keep_counts[l];
    CB_HIP(queue_load(l + 3));
    if (k_host && l > 0) {
      CB_HIP(hipStreamWaitEvent(s, c->load_events[1 + l], 0));
      st = cb_realign_rope(c, k_cache_layers, l, l + 1, off.data(), n_chunks, stream);
      if (st != CB_OK) return st;
    }
    const int32_t *forced = forced_sel ? forced_sel[l] : nullptr;
    float *dev_out = dev_dump ? dev_dump[l] : nullptr;
    const Seg seg = {n, n_suffix, k, T};
    // the launch that finishes a layer's output also normalises it for the next layer
    st = fuse_layer_impl(c, &layers[l], h_cur, p_cur, nullptr, &seg, 1, 0, k_cache_layers[l], v_cache_layers[l],
                         forced, h_nxt, p_nxt, nullptr, dev_out, ws, s, l > 0,
                         l + 1 < L ? layers[l + 1].attn_norm : nullptr);
    if (st != CB_OK) return st;
    if (sel_dump && sel_dump[l] && k > 0)
      CB_HIP(hipMemcpyAsync(sel_dump[l], p_nxt, (size_t)k * 4, hipMemcpyDeviceToDevice, s));
    std::swap(h_cur, h_nxt);
    std::swap(p_cur, p_nxt);
    n = k + n_suffix;
    if (l == 0) {
      delete phase;
      phase = L > 1 ? new (std::nothrow) ProfScope(c, s, CB_PROF_PHASE_SELECTIVE, 0, 0) : nullptr;
    }
  }
  if (n_suffix > 0) {
    ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)n_suffix * d * 8);
    CB_HIP(launch_copy_rows_f32(h_cur + (size_t)(n - n_suffix) * d, final_hidden, (size_t)n_suffix * d, s));
  }
  return CB_OK;
}

}  // namespace

int cb_fuse_prefill(cb_ctx *c, const cb_layer_weights *layers, const void *x, const int32_t *chunk_lens,
                    int32_t n_chunks, int32_t n_suffix, void *const *k_cache_layers,
                    void *const *v_cache_layers, const int32_t *keep_counts,
                    const int32_t *const *forced_sel, float *final_hidden, int32_t *const *sel_dump,
                    float *const *dev_dump, void *workspace, size_t workspace_bytes, void *stream) {
  try {
    return prefill_impl(c, layers, x, chunk_lens, n_chunks, n_suffix, nullptr, nullptr, k_cache_layers,
                        v_cache_layers, keep_counts, forced_sel, final_hidden, sel_dump, dev_dump, workspace,
                        workspace_bytes, stream, nullptr);
  } catch (...) {                       // host bookkeeping ran out of memory
    return CB_ENOMEM;
  }
}

int cb_fuse_prefill_pipelined(cb_ctx *c, const cb_layer_weights *layers, const void *x,
                              const int32_t *chunk_lens, int32_t n_chunks, int32_t n_suffix,
                              const void *const *k_host_layers, const void *const *v_host_layers,
                              void *const *k_cache_layers, void *const *v_cache_layers,
                              const int32_t *keep_counts, float *final_hidden, void *workspace,
                              size_t workspace_bytes, void *stream, void *copy_stream) {
  if (!k_host_layers || !v_host_layers) return CB_ENULL;
  if (stream == copy_stream) return CB_EINVAL;       // the copies must not queue behind the compute
  try {
    return prefill_impl(c, layers, x, chunk_lens, n_chunks, n_suffix, k_host_layers, v_host_layers,
                        k_cache_layers, v_cache_layers, keep_counts, nullptr, final_hidden, nullptr, nullptr,
                        workspace, workspace_bytes, stream, copy_stream);
  } catch (...) {
    return CB_ENOMEM;
  }
}

size_t cb_batched_workspace_bytes(const cb_ctx *c, int32_t total_tokens) {
  if (!c || total_tokens < 1) return 0;
  const size_t h = align_up((size_t)total_tokens * c->m.d_model * 4, 256);
  const size_t p = align_up((size_t)total_tokens * 4, 256);
  // + the per-layer request tables (at most one request per token)
  const size_t tab = align_up((size_t)c->m.n_layers * ((size_t)total_tokens + 1) * kSegInts * 4, 256);
  return 2 * h + 4 * p + tab + carve_layer(c, nullptr, total_tokens).bytes;
}

int cb_fuse_prefill_batched(cb_ctx *c, const cb_layer_weights *layers, int32_t n_requests, const void *x,
                            const int32_t *chunk_lens, const int32_t *n_chunks, const int32_t *n_suffix,
                            void *const *k_cache_layers, void *const *v_cache_layers, int32_t cache_stride,
                            const int32_t *keep_counts, float *final_hidden, int32_t *const *sel_dump,
                            float *const *dev_dump, void *workspace, size_t workspace_bytes, void *stream) try {
  if (!c || !layers || !x || !chunk_lens || !n_chunks || !n_suffix || !k_cache_layers || !v_cache_layers ||
      !keep_counts || !workspace)
    return CB_ENULL;
  if (n_requests < 1 || n_requests > 1024 || cache_stride < 1) return CB_EINVAL;
  const int B = n_requests, L = c->m.n_layers, d = c->m.d_model;
  const size_t es = esize(c), kv_row = (size_t)c->m.n_kv_heads * c->m.head_dim * es;
  std::vector<std::vector<int32_t>> off(B);
  std::vector<int> C(B), T(B);
  long total = 0, total_suffix = 0;
  int ci = 0;
  for (int b = 0; b < B; ++b) {
    if (n_chunks[b] < 1 || n_suffix[b] < 0) return CB_EINVAL;
    off[b].assign(n_chunks[b] + 1, 0);
    for (int i = 0; i < n_chunks[b]; ++i, ++ci) {
      if (chunk_lens[ci] < 1 || (long)off[b][i] + chunk_lens[ci] > c->max_tokens) return CB_EINVAL;
      off[b][i + 1] = off[b][i] + chunk_lens[ci];
    }
    C[b] = off[b][n_chunks[b]];
    T[b] = C[b] + n_suffix[b];
    if (T[b] > c->max_tokens || T[b] > cache_stride) return CB_EINVAL;
    if (keep_counts[(size_t)b * L] != C[b]) return CB_EINVAL;
    for (int l = 1; l < L; ++l)
      if (keep_counts[(size_t)b * L + l] < 0 || keep_counts[(size_t)b * L + l] > keep_counts[(size_t)b * L + l - 1])
        return CB_EINVAL;
    total += T[b];
    total_suffix += n_suffix[b];
  }
  if (total > (1 << 24) || (long)B * cache_stride > (1L << 30)) return CB_EINVAL;
  if (total_suffix > 0 && !final_hidden) return CB_ENULL;
  if (!aligned(x, 16) || !aligned(final_hidden, 16) || !aligned(workspace, 256)) return CB_EINVAL;
  for (int l = 0; l < L; ++l) {
    if (!k_cache_layers[l] || !v_cache_layers[l]) return CB_ENULL;
    const cb_layer_weights *w = &layers[l];
    if (!w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->mlp_norm || !w->w_gate || !w->w_up ||
        !w->w_down)
      return CB_ENULL;
    if (c->m.weight_format == CB_W_INT8 && !scales_ok(w)) return scales_ok_status(w);
    if (!weights_aligned(w) || !aligned(k_cache_layers[l], 16) || !aligned(v_cache_layers[l], 16) ||
        (dev_dump && !aligned(dev_dump[l], 4)))
      return CB_EINVAL;
  }
  if (sel_dump)
    for (size_t i = 0; i < (size_t)B * L; ++i)
      if (!aligned(sel_dump[i], 4)) return CB_EINVAL;
  const int N = (int)total;
  if (cb_batched_workspace_bytes(c, N) > workspace_bytes) return CB_EWORKSPACE;

  hipStream_t s = (hipStream_t)stream;
  char *base = (char *)workspace;
  const size_t hb = align_up((size_t)N * d * 4, 256), pb = align_up((size_t)N * 4, 256);
  float *h_cur = (float *)base, *h_nxt = (float *)(base + hb);
  int32_t *p_cur = (int32_t *)(base + 2 * hb), *p_nxt = (int32_t *)(base + 2 * hb + pb);
  int32_t *r_cur = (int32_t *)(base + 2 * hb + 2 * pb), *r_nxt = (int32_t *)(base + 2 * hb + 3 * pb);
  int32_t *seg_tab = (int32_t *)(base + 2 * hb + 4 * pb);
  const size_t tab_bytes = align_up((size_t)L * ((size_t)N + 1) * kSegInts * 4, 256);
  LayerWs ws = carve_layer(c, base + 2 * hb + 4 * pb + tab_bytes, N);

  // Request tables of every layer (the keep counts are inputs, so all of them are known now), built
  // on the host and uploaded once: selection and attention then take all requests in one launch each.
  std::vector<int32_t> &tab = c->seg_tab_host;       // outlives the call: the upload below may read it later
  tab.assign((size_t)L * (B + 1) * kSegInts, 0);
  {
    std::vector<int> n_in(B);
    for (int b = 0; b < B; ++b) n_in[b] = T[b];
    for (int l = 0; l < L; ++l) {
      int in_off = 0, out_off = 0;
      long qwg = 0;
      for (int b = 0; b <= B; ++b) {
        int32_t *e = &tab[((size_t)l * (B + 1) + b) * kSegInts];
        e[kSegInOff] = in_off; e[kSegOutOff] = out_off; e[kSegQwg] = (int32_t)qwg;
        if (b == B) break;
        const int S = n_suffix[b], k = keep_counts[(size_t)b * L + l];
        e[kSegCand] = n_in[b] - S; e[kSegKeep] = k; e[kSegSuffix] = S; e[kSegCacheRow] = b * cache_stride;
        in_off += n_in[b];
        out_off += k + S;
        qwg += attention_query_workgroups(k + S, c->m.n_q_heads, c->m.n_kv_heads);
        n_in[b] = k + S;
      }
    }
  }
  if (B > 1) CB_HIP(hipMemcpyAsync(seg_tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, s));

  {
    ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)N * d * (4 + es));
    CB_HIP(launch_to_f32(c->m.dtype, x, h_cur, (size_t)N * d, s));
    int o = 0;
    for (int b = 0; b < B; ++b) {
      hipLaunchKernelGGL(iota_kernel, dim3((T[b] + 255) / 256), dim3(256), 0, s, p_cur + o, T[b], 0);
      hipLaunchKernelGGL(iota_kernel, dim3((T[b] + 255) / 256), dim3(256), 0, s, r_cur + o, T[b], b * cache_stride);
      o += T[b];
    }
    CB_HIP(hipGetLastError());
  }
  std::vector<void *> kptr(L);
  for (int b = 0; b < B && L > 1; ++b) {     // layer 0 overwrites all of its rows: nothing of it to re-align
    for (int l = 0; l < L; ++l) kptr[l] = (char *)k_cache_layers[l] + (size_t)b * cache_stride * kv_row;
    int st = cb_realign_rope(c, kptr.data(), 1, L, off[b].data(), n_chunks[b], stream);
    if (st != CB_OK) return st;
  }

  std::vector<Seg> segs(B);
  for (int b = 0; b < B; ++b) segs[b] = {T[b], n_suffix[b], 0, T[b]};
  // phase marks as in the one-request call: the full first layer, then the selective layers
  ProfScope *phase = new (std::nothrow) ProfScope(c, s, CB_PROF_PHASE_FIRST, 0, 0);
  struct PhaseGuard { ProfScope *&p; ~PhaseGuard() { delete p; } } phase_guard{phase};
  for (int l = 0; l < L; ++l) {
    for (int b = 0; b < B; ++b) segs[b].k = keep_counts[(size_t)b * L + l];
    int st = fuse_layer_impl(c, &layers[l], h_cur, p_cur, r_cur, segs.data(), B, (size_t)cache_stride,
                             k_cache_layers[l], v_cache_layers[l], nullptr, h_nxt, p_nxt, r_nxt,
                             dev_dump ? dev_dump[l] : nullptr, ws, s, l > 0,
                             l + 1 < L ? layers[l + 1].attn_norm : nullptr,
                             B > 1 ? seg_tab + (size_t)l * (B + 1) * kSegInts : nullptr);
    if (st != CB_OK) return st;
    int o = 0;
    for (int b = 0; b < B; ++b) {
      int32_t *dst = sel_dump ? sel_dump[(size_t)b * L + l] : nullptr;
      if (dst && segs[b].k > 0)
        CB_HIP(hipMemcpyAsync(dst, p_nxt + o, (size_t)segs[b].k * 4, hipMemcpyDeviceToDevice, s));
      o += segs[b].k + segs[b].S;
      segs[b].n = segs[b].k + segs[b].S;
    }
    std::swap(h_cur, h_nxt);
    std::swap(p_cur, p_nxt);
    std::swap(r_cur, r_nxt);
    if (l == 0) {
      delete phase;
      phase = L > 1 ? new (std::nothrow) ProfScope(c, s, CB_PROF_PHASE_SELECTIVE, 0, 0) : nullptr;
    }
  }
  {
    ProfScope ps(c, s, CB_PROF_OTHER, 0, (double)total_suffix * d * 8);
    int o = 0, fo = 0;
    for (int b = 0; b < B; ++b) {
      if (segs[b].S > 0)
        CB_HIP(launch_copy_rows_f32(h_cur + (size_t)(o + segs[b].n - segs[b].S) * d, final_hidden + (size_t)fo * d,
                                    (size_t)segs[b].S * d, s));
      o += segs[b].n;
      fo += segs[b].S;
    }
  }
  return CB_OK;
} catch (...) {                 // host bookkeeping ran out of memory
  return CB_ENOMEM;
}

int cb_first_token(cb_ctx *c, const float *final_hidden, int32_t n_suffix, const void *final_norm,
                   const void *lm_head, int32_t vocab, float *logits, int32_t *token, void *stream) {
  if (!c || !final_hidden || !final_norm || !lm_head || !logits || !token) return CB_ENULL;
  if (n_suffix < 1 || vocab < 1) return CB_EINVAL;
  if (!aligned(final_hidden, 16) || !aligned(final_norm, 16) || !aligned(lm_head, 16) || !aligned(logits, 16) ||
      !aligned(token, 4))
    return CB_EINVAL;
  const int d = c->m.d_model;
  if (d % 8 != 0 || d > 16384) return CB_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  const size_t es = esize(c);
  {
    ProfScope ps(c, s, CB_PROF_HEAD, 2.0 * vocab * d, (double)vocab * d * es + (double)vocab * 4);
    CB_HIP(launch_lm_head(c->m.dtype, final_hidden + (size_t)(n_suffix - 1) * d, final_norm, lm_head, d, vocab,
                          c->m.rms_eps, logits, s));
  }
  {
    ProfScope ps(c, s, CB_PROF_HEAD, 0, (double)vocab * 4);
    CB_HIP(launch_argmax(logits, vocab, token, s));
  }
  return CB_OK;
}

double cb_recompute_delay(double ratio, double prefill_delay) { return ratio * prefill_delay; }

double cb_load_delay(double per_token_kv_bytes, double n_tokens, double throughput_bytes_per_s) {
  if (!(throughput_bytes_per_s > 0.0)) return HUGE_VAL;
  return per_token_kv_bytes * n_tokens / throughput_bytes_per_s;
}

double cb_pick_recompute_ratio(double prefill_delay, double load_delay, double min_ratio) {
  double r = prefill_delay > 0.0 ? load_delay / prefill_delay : 1.0;
  if (r < min_ratio) r = min_ratio;
  if (r > 1.0) r = 1.0;
  return r;
}

int32_t cb_pick_storage_device(double recompute_delay, const double *load_delays, const double *costs,
                               int32_t n) {
  if (!load_delays || !costs) return -1;
  int32_t best = -1;
  for (int32_t i = 0; i < n; ++i)
    if (load_delays[i] <= recompute_delay && (best < 0 || costs[i] < costs[best])) best = i;
  return best;
}

int cb_profile_enable(cb_ctx *c, int32_t enable) {
  if (!c) return CB_ENULL;
  if (enable < 0 || enable > 2) return CB_EINVAL;
  c->profiling = enable;
  return CB_OK;
}

int cb_profile_read(cb_ctx *c, double *ms, int64_t *launches, double *flops, double *bytes) {
  if (!c || !ms || !launches || !flops || !bytes) return CB_ENULL;
  for (int i = 0; i < CB_PROF_NCLASS; ++i) { ms[i] = 0; launches[i] = 0; flops[i] = 0; bytes[i] = 0; }
  if (!c->recs.empty()) CB_HIP(hipEventSynchronize(c->recs.back().stop));
  for (auto &r : c->recs) {
    float t = 0.f;
    CB_HIP(hipEventElapsedTime(&t, r.start, r.stop));
    ms[r.cls] += t;
    launches[r.cls] += 1;
    flops[r.cls] += r.flops;
    bytes[r.cls] += r.bytes;
    c->free_events.push_back(r.start);
    c->free_events.push_back(r.stop);
  }
  c->recs.clear();
  return CB_OK;
}

}  // extern "C"
