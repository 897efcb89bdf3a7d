// C ABI of libprsgd: host-side driver of Algorithm 1 (and the epochs of Algorithms 2 and 3).
// Only argument checking, buffer carving and kernel sequencing live here; every arithmetic
// step of the method runs in the kernels.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "prsgd_aux.h"
#include "prsgd_internal.h"

using namespace prsgd;

namespace prsgd {
const char* kernel_kind_name(int kind) {
  static const char* names[KK_COUNT] = {"gather",  "gemm_fwd", "softmax_xent", "gemm_dx",   "gemm_dw",
                                        "sgd_update", "average", "mean",       "broadcast", "lsq_steps",
                                        "mlp2_epoch", "gemm_bwd", "restart_mean", "step_mean", "gemm_bwd_first", "refresh_shadow"};
  return (kind >= 0 && kind < KK_COUNT) ? names[kind] : "?";
}
}  // namespace prsgd

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

thread_local char g_init_error[256] = "";

struct Carve {
  size_t xb = 0, yb = 0, idx = 0, xb2 = 0, yb2 = 0, idx2 = 0, logits = 0, losses = 0, row_loss = 0, part = 0, sync = 0, shadow = 0, grads = 0, mean = 0, mean_shadow = 0, steps = 0, vel = 0;
  size_t h[PRSGD_MAX_DIMS] = {0}, delta[PRSGD_MAX_DIMS] = {0};
  size_t total = 0;
};

bool build_layout(const prsgd_config* c, Layout* lo, char* err, size_t errn) {
  auto fail = [&](const char* msg) { snprintf(err, errn, "%s", msg); return false; };
  if (c == nullptr) return fail("config is null");
  if (c->n_workers < 1 || c->n_workers > 65535) return fail("n_workers out of range");
  if (c->batch < 1 || c->batch > kMaxBatch) return fail("batch out of range (1..4096)");
  if (c->rows_per_worker < 1 || c->rows_per_worker > (1LL << 31) ||
      (c->rows_per_worker & (c->rows_per_worker - 1)) != 0)
    return fail("rows_per_worker must be a power of two");
  if (!(c->lr == c->lr)) return fail("lr is NaN");
  if (!(c->momentum >= 0.0f && c->momentum < 1.0f)) return fail("momentum must be in [0, 1)");
  if (c->momentum_restart < PRSGD_MOM_KEEP || c->momentum_restart > PRSGD_MOM_RESET)
    return fail("unknown momentum_restart");
  memset(lo, 0, sizeof(*lo));
  if (c->model == PRSGD_LSQ) {
    if (c->n_dims != 1) return fail("least squares takes n_dims == 1");
    if (c->dims[0] < 1 || c->dims[0] > kMaxLsqDim) return fail("least-squares dimension out of range");
    lo->n_layers = 0;
    lo->d[0] = c->dims[0];
    lo->ld[0] = c->dims[0];
    lo->m = c->dims[0];
    lo->m_pad = (long)align_up((size_t)c->dims[0], 64);
    return true;
  }
  if (c->model != PRSGD_MLP) return fail("unknown model");
  if (c->n_dims < 2 || c->n_dims > PRSGD_MAX_DIMS) return fail("an MLP takes 2..16 dims");
  if (c->activation != PRSGD_TANH && c->activation != PRSGD_RELU) return fail("unknown activation");
  if (c->gemm_dtype != PRSGD_F32 && c->gemm_dtype != PRSGD_BF16) return fail("unknown gemm_dtype");
  lo->n_layers = c->n_dims - 1;
  long off = 0, m = 0;
  for (int l = 0; l < c->n_dims; ++l) {
    if (c->dims[l] < 1 || c->dims[l] > (1 << 20)) return fail("layer width out of range");
    lo->d[l] = c->dims[l];
    // rows of 8 elements; wide layers (>= 512) are padded to whole 64-column tiles so that the
    // whole-tile kernels apply to them (the padding columns hold zeros and stay zero)
    lo->ld[l] = (int)align_up((size_t)c->dims[l], (l > 0 && c->dims[l] >= 512) ? 64 : 8);
  }
  for (int l = 1; l < c->n_dims; ++l) {
    lo->w_off[l - 1] = off;
    off = (long)align_up((size_t)off + (size_t)lo->d[l - 1] * lo->ld[l], 64);
    lo->b_off[l - 1] = off;
    off = (long)align_up((size_t)off + (size_t)lo->ld[l], 64);
    m += (long)lo->d[l - 1] * lo->d[l] + lo->d[l];
  }
  lo->m = m;
  lo->m_pad = off;
  return true;
}

// Momentum (v <- mu v + G, x <- x - gamma v) is fused into the one-pass backward kernel of the
// bf16 configurations and into the epoch kernel of the one-hidden-layer fp32 MLPs; elsewhere the
// gradients go to HBM and an elementwise kernel applies it.
bool bwd_fused_config(const prsgd_config& c) {
  return c.model == PRSGD_MLP && c.gemm_dtype == PRSGD_BF16 && c.fused_update &&
         prsgd::bwd_fused_supported(c.batch);
}
// shapes the epoch kernel may take (whether it does is decided at init, on the device)
bool epoch_candidate(const prsgd_config& c) {
  return c.model == PRSGD_MLP && c.gemm_dtype == PRSGD_F32 && c.n_dims == 3 && c.fused_update &&
         (c.dims[1] % 16) == 0 && c.dims[2] <= 64 && c.batch <= 64;
}
prsgd_config effective_config(const prsgd_config* c) {
  prsgd_config e = *c;
  if (e.momentum != 0.0f && !bwd_fused_config(e) && !epoch_candidate(e)) e.fused_update = 0;
  return e;
}

void build_carve(const prsgd_config* c_in, const Layout& lo, Carve* cv) {
  const prsgd_config eff = effective_config(c_in);
  const prsgd_config* c = &eff;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, kAlign); return o; };
  const size_t n = (size_t)c->n_workers, b = (size_t)c->batch;
  const bool bf16 = c->model == PRSGD_MLP && c->gemm_dtype == PRSGD_BF16;
  const size_t es = bf16 ? 2 : 4;
  cv->idx = take(n * b * 4);
  cv->losses = take(n * 4);
  cv->steps = take(n * 4);
  cv->mean = take((size_t)lo.m_pad * 4);
  if (c->momentum != 0.0f) cv->vel = take(n * (size_t)lo.m_pad * 4);
  if (c->model == PRSGD_MLP) {
    const int L = lo.n_layers;
    cv->yb = take(n * b * 4);
    cv->row_loss = take(n * b * 4);
    cv->xb = take(n * b * lo.ld[0] * es);
    // second set: the next iteration's minibatch is gathered while the current one is in use
    cv->xb2 = take(n * b * lo.ld[0] * es);
    cv->yb2 = take(n * b * 4);
    cv->idx2 = take(n * b * 4);
    for (int l = 1; l < L; ++l) {
      cv->h[l] = take(n * b * lo.ld[l] * es);
      cv->delta[l] = take(n * b * lo.ld[l] * es);
    }
    cv->delta[L] = take(n * b * lo.ld[L] * es);
    cv->logits = take((size_t)kMaxLogitSplits * n * b * lo.ld[L] * 4);   // room for split partial sums
    if (bf16) {
      cv->shadow = take(n * (size_t)lo.m_pad * 2);
      cv->mean_shadow = take((size_t)lo.m_pad * 2);
    }
    if (epoch_candidate(*c)) {
      // epoch kernel: partial logits for the finest team split, arrival counters, abort flag
      // batch tiles come in 1, 2 or 4 blocks of 16 rows
      const size_t mr = c->batch <= 16 ? 16 : c->batch <= 32 ? 32 : 64;
      const size_t d2p = ((size_t)lo.d[2] + 15) / 16 * 16;
      cv->part = take(2 * n * (size_t)(lo.d[1] / 16) * mr * d2p * 4);
      cv->sync = take((n + 1) * 128);
    }
    // un-fused update; also the fallback of a momentum run whose epoch kernel does not fit the device
    if (!c->fused_update || (c->momentum != 0.0f && !bwd_fused_config(*c)))
      cv->grads = take(n * (size_t)lo.m_pad * 4);
  }
  cv->total = off;
}

struct EventPair { hipEvent_t a, b; int kind; };

}  // namespace

struct prsgd_ctx {
  prsgd_config cfg;
  Layout lo;
  Carve cv;
  bool bf16;
  bool use_fused2;      // one-hidden-layer fp32 MLP: whole epochs in one launch
  Fused2Plan f2;
  bool streaming;       // replica set >= 1 GiB: weight traffic bypasses the last-level cache
  bool lazy_restart;    // a restart only writes the node average; the next local iteration
                        // reads it as every worker's starting point (no broadcast)
  bool at_mean;         // the replicas are stale: every worker's current point is the vector `mean`
  bool poisoned;        // the epoch kernel gave up a team barrier: the replicas are inconsistent
                        // until the caller restores them (prsgd_write_params)
  unsigned char restored[65536 / 8];   // bit i: worker i written since the abort
  size_t n_restored;
  unsigned int spin_limit;      // polls of the epoch kernel's team barrier before it gives up
  hipStream_t stream;
  const float* features;
  const void* targets;
  float* params;
  char* ws;
  int64_t t;
  // two minibatch buffer sets (layer-wise MLP path): batch_t[k] is the iteration whose draw set k
  // holds for ALL workers (-1: none), batch_cur the set of the last local iteration
  int64_t batch_t[2];
  int batch_cur;
  // first hidden activation computed ahead by the first layer's backward kernel: valid for
  // iteration h1_t on batch set h1_batch while the replicas are untouched (-1: none)
  int64_t h1_t;
  int h1_batch;
  bool restart_fusion;  // prsgd_run: take an epoch's last iteration and the restart as one pass
  bool first_fusion;    // let the first layer's backward kernel run the next forward product
  bool shadow1_stale;   // that kernel skipped the bf16 shadow of W_1 (nothing reads it while the
                        // chain of ahead-computed activations holds): refresh before any other reader
  float lr;
  char err[256];
  // profiling
  bool profiling;
  std::vector<EventPair> pool;
  size_t pool_used;
  double prof_ms[KK_COUNT];
  int64_t prof_n[KK_COUNT];
  // scratch host buffer for padded <-> dense parameter conversion
  float* host_pad;                    // [m_pad]
  std::vector<float> host_pad_heap;   // owns it, unless the context lives in static storage
  int static_slot;                    // >= 0: context, workspace and host_pad are the per-device
                                      // static ones of prsgd_init_static

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  void* xb(int k) const { return at<void>(k ? cv.xb2 : cv.xb); }
  int32_t* yb(int k) const { return at<int32_t>(k ? cv.yb2 : cv.yb); }
  int32_t* idx(int k) const { return at<int32_t>(k ? cv.idx2 : cv.idx); }
  uint16_t* shadow() const { return bf16 ? at<uint16_t>(cv.shadow) : nullptr; }
  float* mean() const { return at<float>(cv.mean); }
  float* velocity() const { return cfg.momentum != 0.0f ? at<float>(cv.vel) : nullptr; }
  uint16_t* mean_shadow() const { return bf16 ? at<uint16_t>(cv.mean_shadow) : nullptr; }
  // where a worker's current point is read from, and the stride between workers
  const float* src() const { return at_mean ? mean() : params; }
  long src_stride() const { return at_mean ? 0 : lo.m_pad; }
  // configurations whose first local iteration can start from the shared node average
  bool can_start_from_mean() const {
    return cfg.model == PRSGD_LSQ || use_fused2 ||
           (bf16 && cfg.fused_update && prsgd::bwd_fused_supported(cfg.batch));
  }
  float* grads() const { return cfg.fused_update ? nullptr : at<float>(cv.grads); }
};

namespace {

int set_err(prsgd_ctx* ctx, int code, const char* fmt, const char* detail = "") {
  if (ctx != nullptr) snprintf(ctx->err, sizeof(ctx->err), fmt, detail);
  else snprintf(g_init_error, sizeof(g_init_error), fmt, detail);
  return code;
}
int hip_fail(prsgd_ctx* ctx, hipError_t e, const char* what) {
  char buf[200];
  snprintf(buf, sizeof(buf), "%s: %s", what, hipGetErrorString(e));
  return set_err(ctx, PRSGD_EHIP, "%s", buf);
}

// Drains finished event pairs into the per-kind totals.
int profile_flush(prsgd_ctx* ctx) {
  if (ctx->pool_used == 0) return PRSGD_OK;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "hipStreamSynchronize");
  for (size_t i = 0; i < ctx->pool_used; ++i) {
    float ms = 0.0f;
    e = hipEventElapsedTime(&ms, ctx->pool[i].a, ctx->pool[i].b);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipEventElapsedTime");
    ctx->prof_ms[ctx->pool[i].kind] += ms;
    ctx->prof_n[ctx->pool[i].kind] += 1;
  }
  ctx->pool_used = 0;
  return PRSGD_OK;
}

// Brackets one kernel launch with an event pair while profiling is on.
struct Timed {
  prsgd_ctx* ctx;
  EventPair* ep = nullptr;
  Timed(prsgd_ctx* c, int kind) : ctx(c) {
    if (!c->profiling) return;
    if (c->pool_used == c->pool.size() && profile_flush(c) != PRSGD_OK) return;
    ep = &c->pool[c->pool_used++];
    ep->kind = kind;
    (void)hipEventRecord(ep->a, c->stream);
  }
  ~Timed() {
    if (ep != nullptr) (void)hipEventRecord(ep->b, ctx->stream);
  }
};

#define LAUNCH(ctx, kind, call)                                        \
  do {                                                                 \
    hipError_t e_;                                                     \
    {                                                                  \
      Timed timed_(ctx, kind);                                         \
      e_ = (call);                                                     \
    }                                                                  \
    if (e_ != hipSuccess) return hip_fail(ctx, e_, kernel_kind_name(kind)); \
  } while (0)

int materialize(prsgd_ctx* ctx);

// bf16 shadow of W_1 of every replica from its fp32 master (after first-layer kernels that skipped it)
int refresh_first_shadow(prsgd_ctx* ctx) {
  const Layout& lo = ctx->lo;
  const long count = (long)lo.d[0] * lo.ld[1];
  for (int i = 0; i < ctx->cfg.n_workers; ++i) {
    const size_t off = (size_t)i * lo.m_pad + lo.w_off[0];
    LAUNCH(ctx, KK_REFRESH, launch_refresh_shadow(ctx->params + off, ctx->shadow() + off, count, ctx->stream));
  }
  ctx->shadow1_stale = false;
  return PRSGD_OK;
}

// One local iteration of every (active) MLP worker: gradient observation + eq. (3).
// fuse_average: this iteration is followed by a restart, and both are taken together,
//   (1/N) sum_i (x_i - gamma G_i) = ybar - (gamma / N) sum_i G_i,   ybar = (1/N) sum_i x_i   (eq. 2-3).
// The backward pass contracts over the stacked minibatches of all workers and writes only the new
// ybar; the replicas are not rewritten and the context ends "at the mean".  With every worker
// already at ybar (I = 1) it is one mini-batch SGD step with the N B samples of all workers (first
// footnote of Section 1).
int mlp_step(prsgd_ctx* ctx, int64_t t, const int* worker_steps, int step, bool fuse_average = false) {
  const prsgd_config& c = ctx->cfg;
  const Layout& lo = ctx->lo;
  const Carve& cv = ctx->cv;
  const int N = c.n_workers, B = c.batch, L = lo.n_layers;
  const bool bf16 = ctx->bf16;
  hipStream_t s = ctx->stream;

  // The minibatch of iteration t: already there when the previous iteration's loss-head launch
  // drew it (below); otherwise gathered now.  A masked draw (Algorithm 3) is never reused.
  auto batch_args = [&](int k, int64_t tt) {
    return gather_args(ctx->features, reinterpret_cast<const int32_t*>(ctx->targets), ctx->xb(k), ctx->yb(k),
                       ctx->idx(k), B, lo.d[0], lo.ld[0], (long)c.rows_per_worker, c.seed, tt);
  };
  int bk = -1;
  if (worker_steps == nullptr) bk = ctx->batch_t[0] == t ? 0 : ctx->batch_t[1] == t ? 1 : -1;
  if (bk < 0) {
    bk = ctx->batch_cur;
    ctx->batch_t[bk] = -1;
    LAUNCH(ctx, KK_GATHER, launch_gather(batch_args(bk, t), N, bf16, worker_steps, step, s));
    if (worker_steps == nullptr) ctx->batch_t[bk] = t;
  }
  ctx->batch_cur = bk;

  GemmArgs base;
  memset(&base, 0, sizeof(base));
  base.act = c.activation;
  base.lr = ctx->lr;
  base.params = ctx->params;
  base.grads = ctx->grads();
  base.shadow = ctx->shadow();
  base.p_gs = lo.m_pad;
  base.worker_steps = worker_steps;
  base.streaming = ctx->streaming ? 1 : 0;
  base.step = step;

  auto act_in = [&](int l) -> const void* {   // H_l as stored (l = 0: the gathered batch)
    return l == 0 ? ctx->xb(bk) : ctx->at<void>(cv.h[l]);
  };
  const bool fused_bwd = bf16 && c.fused_update && bwd_fused_supported(B);
  // Right after a restart every worker starts from the shared node average (stride 0); only
  // the fused backward kernel writes complete replicas from it, so every other path first
  // broadcasts the average.  A masked worker (Algorithm 3) would keep a stale replica.
  if (ctx->at_mean && (!fused_bwd || worker_steps != nullptr)) {
    const int rc = materialize(ctx);
    if (rc != PRSGD_OK) return rc;
  }
  const bool from_mean = ctx->at_mean;
  const long w_gs = from_mean ? 0 : lo.m_pad;
  // The matrix products read weights from the bf16 shadow (bf16 mode) or the fp32 master.
  const void* wsrc = bf16 ? (const void*)(from_mean ? ctx->mean_shadow() : ctx->shadow())
                          : (const void*)ctx->params;
  base.bias_src = ctx->src();
  base.bias_gs = ctx->src_stride();

  // forward.  H_1 may already be there: the previous iteration's first-layer backward kernel computes
  // it from the weights it writes, for this iteration's minibatch
  const bool h1_ready = fused_bwd && !from_mean && worker_steps == nullptr && L >= 2 &&
                        ctx->h1_t == t && ctx->h1_batch == bk;
  ctx->h1_t = -1;
  if (!h1_ready && ctx->shadow1_stale && !from_mean) {
    const int rc = refresh_first_shadow(ctx);
    if (rc != PRSGD_OK) return rc;
  }
  int logit_parts = 1;
  const long logit_part_stride = (long)N * B * lo.ld[L];
  // a narrow logits layer (bf16 operands, at most 16 classes) is multiplied inside the loss-head launch
  const bool narrow_head = softmax_narrow_applies(lo.d[L], lo.ld[L], bf16);
  for (int l = 1; l <= L; ++l) {
    if (l == 1 && h1_ready) continue;
    if (l == L && narrow_head) continue;
    GemmArgs p = base;
    p.a = act_in(l - 1); p.a_gs = (long)B * lo.ld[l - 1]; p.lda = lo.ld[l - 1];
    p.b = bf16 ? (const void*)(reinterpret_cast<const uint16_t*>(wsrc) + lo.w_off[l - 1])
               : (const void*)(reinterpret_cast<const float*>(wsrc) + lo.w_off[l - 1]);
    p.b_gs = w_gs; p.ldb = lo.ld[l];
    p.M = B; p.N = lo.d[l]; p.Kc = lo.d[l - 1];
    p.b_off = lo.b_off[l - 1];
    p.out_gs = (long)B * lo.ld[l]; p.ldo = lo.ld[l]; p.out_cols = lo.ld[l];
    if (l < L) { p.epi = EPI_FWD_HIDDEN; p.out = ctx->at<void>(cv.h[l]); }
    else {
      p.epi = EPI_FWD_LOGITS; p.out = ctx->at<void>(cv.logits);
      logit_parts = gemm_logit_splits(p, N, bf16);
      p.k_splits = logit_parts; p.split_stride = logit_part_stride;
    }
    LAUNCH(ctx, KK_FWD, launch_gemm_fwd(p, N, bf16, s));
  }

  // the loss-head launch also draws the minibatch of iteration t + 1 into the other buffer set
  const bool prefetch = worker_steps == nullptr;
  GatherArgs next_batch = batch_args(bk ^ 1, t + 1);
  if (prefetch) ctx->batch_t[bk ^ 1] = -1;
  if (narrow_head)
    LAUNCH(ctx, KK_LOSS,
           launch_softmax_xent_narrow(reinterpret_cast<const uint16_t*>(act_in(L - 1)), (long)B * lo.ld[L - 1],
                                      lo.ld[L - 1], lo.d[L - 1],
                                      reinterpret_cast<const uint16_t*>(wsrc) + lo.w_off[L - 1], w_gs,
                                      ctx->src() + lo.b_off[L - 1], ctx->src_stride(), ctx->yb(bk),
                                      ctx->at<uint16_t>(cv.delta[L]), ctx->at<float>(cv.row_loss), N, B, lo.d[L],
                                      lo.ld[L], worker_steps, step, prefetch ? &next_batch : nullptr, s));
  else
  LAUNCH(ctx, KK_LOSS,
         launch_softmax_xent(ctx->at<float>(cv.logits), logit_parts, logit_part_stride,
                             logit_parts > 1 ? ctx->src() + lo.b_off[L - 1] : nullptr, ctx->src_stride(),
                             ctx->yb(bk),
                             ctx->at<void>(cv.delta[L]), ctx->at<float>(cv.row_loss), N, B, lo.d[L],
                             lo.ld[L], bf16, worker_steps, step, prefetch ? &next_batch : nullptr, s));
  if (prefetch) ctx->batch_t[bk ^ 1] = t + 1;

  if (fuse_average) {
    // The workers' points differ (the last iteration of an epoch with I >= 2, or the first
    // iteration of a run): ybar is first taken from the points as they are (the restart kernel),
    // then moved by the averaged gradient; the points themselves are not rewritten.
    if (!from_mean)
      LAUNCH(ctx, KK_RESTART_MEAN,
             launch_mean(ctx->params, ctx->mean(), ctx->mean_shadow(), lo.m_pad, N, ctx->streaming, s));
    // eq. (3) and eq. (2) in one pass over ybar, layer by layer from the top: D_{l-1} needs the
    // weights the forward pass used (the bf16 image of ybar, or of every worker's own point), and
    // when that is ybar it runs before layer l's pass changes it
    for (int l = L; l >= 1; --l) {
      if (l > 1) {
        GemmArgs p = base;
        p.a = ctx->at<void>(cv.delta[l]); p.a_gs = (long)B * lo.ld[l]; p.lda = lo.ld[l];
        p.b = (const void*)((from_mean ? ctx->mean_shadow() : ctx->shadow()) + lo.w_off[l - 1]);
        p.b_gs = from_mean ? 0 : lo.m_pad; p.ldb = lo.ld[l];
        p.M = B; p.N = lo.d[l - 1]; p.Kc = lo.d[l];
        p.epi = EPI_DX;
        p.out = ctx->at<void>(cv.delta[l - 1]); p.out_gs = (long)B * lo.ld[l - 1];
        p.ldo = lo.ld[l - 1]; p.out_cols = lo.ld[l - 1];
        p.aux = act_in(l - 1); p.aux_gs = (long)B * lo.ld[l - 1]; p.ldaux = lo.ld[l - 1];
        LAUNCH(ctx, KK_DX, launch_gemm_dx(p, N, true, s));
      }
      // all minibatches stacked: sum_i dW_i = [H_1; ..; H_N]^T [D_1; ..; D_N], one contraction of N B
      // rows, and ybar <- ybar - (gamma / N) sum_i dW_i (likewise the bias from the column sums)
      GemmArgs p = base;
      p.a = act_in(l - 1); p.a_gs = 0; p.lda = lo.ld[l - 1];
      p.b = ctx->at<void>(cv.delta[l]); p.b_gs = 0; p.ldb = lo.ld[l];
      p.M = lo.d[l - 1]; p.N = lo.d[l]; p.Kc = N * B;
      p.epi = EPI_DW_FUSED;
      p.lr = ctx->lr / (float)N;
      p.params = ctx->mean(); p.shadow = ctx->mean_shadow(); p.p_gs = 0;
      p.w_off = lo.w_off[l - 1]; p.b_off = lo.b_off[l - 1]; p.ldw = lo.ld[l];
      LAUNCH(ctx, KK_STEP_MEAN, launch_gemm_dw_stacked(p, s));
    }
    ctx->at_mean = true;             // every worker's point is the new ybar; the replicas are stale
    return PRSGD_OK;
  }

  // backward.  bf16 operands with the fused update: one kernel per layer does the weight
  // gradient, eq. (3) and the delta of the layer below in a single pass over W_l.
  for (int l = L; fused_bwd && l >= 1; --l) {
    BwdArgs q;
    memset(&q, 0, sizeof(q));
    q.h = reinterpret_cast<const uint16_t*>(act_in(l - 1)); q.h_gs = (long)B * lo.ld[l - 1]; q.ldh = lo.ld[l - 1];
    q.d = ctx->at<uint16_t>(cv.delta[l]); q.d_gs = (long)B * lo.ld[l]; q.ldd = lo.ld[l];
    q.params = ctx->params; q.shadow = ctx->shadow(); q.p_gs = lo.m_pad;
    q.src = ctx->src(); q.src_gs = ctx->src_stride();
    q.w_off = lo.w_off[l - 1]; q.b_off = lo.b_off[l - 1]; q.ldw = lo.ld[l];
    if (l > 1) { q.dx = ctx->at<uint16_t>(cv.delta[l - 1]); q.dx_gs = (long)B * lo.ld[l - 1]; q.lddx = lo.ld[l - 1]; }
    q.B = B; q.K = lo.d[l - 1]; q.Nn = lo.d[l];
    q.n_groups = N; q.act = c.activation; q.streaming = ctx->streaming ? 1 : 0;
    q.lr = ctx->lr;
    q.vel = ctx->velocity(); q.mu = c.momentum;
    q.worker_steps = worker_steps; q.step = step;
    if (l == 1 && L >= 2 && ctx->first_fusion && prefetch && ctx->batch_t[bk ^ 1] == t + 1) {
      q.x_next = reinterpret_cast<const uint16_t*>(ctx->xb(bk ^ 1)); q.x_gs = (long)B * lo.ld[0]; q.ldx = lo.ld[0];
      q.h_next = ctx->at<uint16_t>(cv.h[1]); q.hn_gs = (long)B * lo.ld[1]; q.ldhn = lo.ld[1];
      if (bwd_first_fwd_applies(q)) {
        q.shadow = nullptr;                 // replica shadows of W_1 have no reader while H_1 comes from here
        LAUNCH(ctx, KK_BWD_FIRST, launch_bwd_first_fwd(q, s));
        ctx->shadow1_stale = true;
        ctx->h1_t = t + 1;
        ctx->h1_batch = bk ^ 1;
        continue;
      }
    }
    LAUNCH(ctx, KK_BWD, launch_bwd_fused(q, s));
  }
  // otherwise: D_{l-1} needs the pre-update W_l, so it runs before layer l's weight kernel
  for (int l = L; !fused_bwd && l >= 1; --l) {
    if (l > 1) {
      GemmArgs p = base;
      p.a = ctx->at<void>(cv.delta[l]); p.a_gs = (long)B * lo.ld[l]; p.lda = lo.ld[l];
      p.b = bf16 ? (const void*)(reinterpret_cast<const uint16_t*>(wsrc) + lo.w_off[l - 1])
                 : (const void*)(reinterpret_cast<const float*>(wsrc) + lo.w_off[l - 1]);
      p.b_gs = lo.m_pad; p.ldb = lo.ld[l];
      p.M = B; p.N = lo.d[l - 1]; p.Kc = lo.d[l];
      p.epi = EPI_DX;
      p.out = ctx->at<void>(cv.delta[l - 1]); p.out_gs = (long)B * lo.ld[l - 1];
      p.ldo = lo.ld[l - 1]; p.out_cols = lo.ld[l - 1];
      p.aux = act_in(l - 1); p.aux_gs = (long)B * lo.ld[l - 1]; p.ldaux = lo.ld[l - 1];
      LAUNCH(ctx, KK_DX, launch_gemm_dx(p, N, bf16, s));
    }
    GemmArgs p = base;
    p.a = act_in(l - 1); p.a_gs = (long)B * lo.ld[l - 1]; p.lda = lo.ld[l - 1];
    p.b = ctx->at<void>(cv.delta[l]); p.b_gs = (long)B * lo.ld[l]; p.ldb = lo.ld[l];
    p.M = lo.d[l - 1]; p.N = lo.d[l]; p.Kc = B;
    p.epi = c.fused_update ? EPI_DW_FUSED : EPI_DW_GRAD;
    p.w_off = lo.w_off[l - 1]; p.b_off = lo.b_off[l - 1]; p.ldw = lo.ld[l];
    LAUNCH(ctx, KK_DW, launch_gemm_dw(p, N, bf16, s));
  }

  if (!c.fused_update) {
    if (ctx->velocity() != nullptr)
      LAUNCH(ctx, KK_UPDATE, launch_momentum_update(ctx->params, ctx->velocity(), ctx->grads(), ctx->shadow(),
                                                    (size_t)N * lo.m_pad, ctx->lr, c.momentum, s));
    else if (worker_steps == nullptr)
      LAUNCH(ctx, KK_UPDATE, launch_update(ctx->params, ctx->grads(), ctx->shadow(),
                                           (size_t)N * lo.m_pad, ctx->lr, s));
    else
      LAUNCH(ctx, KK_UPDATE, launch_update_masked(ctx->params, ctx->grads(), ctx->shadow(), lo.m_pad,
                                                  N, ctx->lr, worker_steps, step, s));
  }
  ctx->at_mean = false;            // every parameter of every replica has been rewritten
  return PRSGD_OK;
}

Fused2Args fused2_args(prsgd_ctx* ctx, int k, const int* worker_steps) {
  const prsgd_config& c = ctx->cfg;
  const Layout& lo = ctx->lo;
  Fused2Args a;
  memset(&a, 0, sizeof(a));
  a.features = ctx->features;
  a.labels = reinterpret_cast<const int32_t*>(ctx->targets);
  a.params = ctx->params;
  a.src = ctx->src();
  a.src_stride = ctx->src_stride();
  a.m_pad = lo.m_pad;
  a.w1_off = lo.w_off[0]; a.b1_off = lo.b_off[0]; a.w2_off = lo.w_off[1]; a.b2_off = lo.b_off[1];
  a.ld1 = lo.ld[1]; a.ld2 = lo.ld[2];
  a.n_workers = c.n_workers;
  a.d0 = lo.d[0]; a.d1 = lo.d[1]; a.d2 = lo.d[2];
  a.batch = c.batch;
  a.rows = (long)c.rows_per_worker;
  a.log2n = 0;
  while ((1LL << a.log2n) < c.rows_per_worker) ++a.log2n;
  a.act = c.activation;
  a.lr = ctx->lr;
  a.seed = c.seed;
  a.t0 = (uint64_t)ctx->t;
  a.k = k;
  a.worker_steps = worker_steps;
  a.part = ctx->at<float>(ctx->cv.part);
  a.sync = ctx->at<unsigned int>(ctx->cv.sync);
  a.spin_limit = ctx->spin_limit;
  a.row_loss = ctx->at<float>(ctx->cv.row_loss);
  a.idx = ctx->at<int32_t>(ctx->cv.idx);
  a.vel = ctx->velocity();
  a.mu = c.momentum;
  return a;
}

constexpr const char* kPoisonedMsg =
    "the epoch kernel gave up waiting for a team member (was other work running on the device?); "
    "the replicas are inconsistent: restore them with prsgd_write_params (and prsgd_set_iteration)";

// Calls that enqueue work refuse to run on replicas an aborted epoch launch left inconsistent.
int check_poisoned(prsgd_ctx* ctx) {
  return ctx->poisoned ? set_err(ctx, PRSGD_ESTATE, "%s", kPoisonedMsg) : PRSGD_OK;
}

// The epoch kernel's bounded team barrier raises a flag instead of hanging.  Called wherever the
// stream is synchronised anyway: reads the flag (4 bytes); if it is set, clears it, marks the
// context poisoned and switches every later local step to the per-layer kernel chain, which needs
// no co-resident workgroups.
int check_fused2_abort(prsgd_ctx* ctx) {
  if (ctx->poisoned) return set_err(ctx, PRSGD_ESTATE, "%s", kPoisonedMsg);
  if (!ctx->use_fused2) return PRSGD_OK;
  unsigned int* flag_dev = ctx->at<unsigned int>(ctx->cv.sync) + (size_t)ctx->cfg.n_workers * 32;
  unsigned int flag = 0;
  hipError_t e = hipMemcpyAsync(&flag, flag_dev, sizeof(flag), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "abort-flag read");
  if (flag == 0) return PRSGD_OK;
  const unsigned int zero = 0;
  e = hipMemcpyAsync(flag_dev, &zero, sizeof(zero), hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "abort-flag reset");
  ctx->use_fused2 = false;
  if (ctx->cfg.momentum != 0.0f) ctx->cfg.fused_update = 0;   // the chain applies momentum elementwise
  ctx->poisoned = true;
  ctx->at_mean = false;
  ctx->n_restored = 0;
  memset(ctx->restored, 0, sizeof(ctx->restored));
  return set_err(ctx, PRSGD_ESTATE, "%s", kPoisonedMsg);
}

// Writes the node average into every replica (and the bf16 shadow) if the last restart left the
// replicas stale.
int materialize(prsgd_ctx* ctx) {
  ctx->h1_t = -1;
  if (!ctx->at_mean) return PRSGD_OK;
  ctx->shadow1_stale = false;               // the broadcast rewrites every shadow
  LAUNCH(ctx, KK_BROADCAST, launch_broadcast(ctx->mean(), ctx->params, ctx->shadow(), ctx->lo.m_pad,
                                             ctx->cfg.n_workers, ctx->stream));
  ctx->at_mean = false;
  return PRSGD_OK;
}

int pad_from_dense(const prsgd_ctx* ctx, const float* dense, float* padded) {
  const Layout& lo = ctx->lo;
  memset(padded, 0, sizeof(float) * (size_t)lo.m_pad);
  if (lo.n_layers == 0) { memcpy(padded, dense, sizeof(float) * (size_t)lo.m); return 0; }
  size_t src = 0;
  for (int l = 1; l <= lo.n_layers; ++l) {
    for (int r = 0; r < lo.d[l - 1]; ++r) {
      memcpy(padded + lo.w_off[l - 1] + (size_t)r * lo.ld[l], dense + src, sizeof(float) * lo.d[l]);
      src += lo.d[l];
    }
    memcpy(padded + lo.b_off[l - 1], dense + src, sizeof(float) * lo.d[l]);
    src += lo.d[l];
  }
  return 0;
}
void dense_from_pad(const prsgd_ctx* ctx, const float* padded, float* dense) {
  const Layout& lo = ctx->lo;
  if (lo.n_layers == 0) { memcpy(dense, padded, sizeof(float) * (size_t)lo.m); return; }
  size_t dst = 0;
  for (int l = 1; l <= lo.n_layers; ++l) {
    for (int r = 0; r < lo.d[l - 1]; ++r) {
      memcpy(dense + dst, padded + lo.w_off[l - 1] + (size_t)r * lo.ld[l], sizeof(float) * lo.d[l]);
      dst += lo.d[l];
    }
    memcpy(dense + dst, padded + lo.b_off[l - 1], sizeof(float) * lo.d[l]);
    dst += lo.d[l];
  }
}

}  // namespace

extern "C" {

size_t prsgd_param_count(const prsgd_config* cfg) {
  Layout lo;
  char err[128];
  return build_layout(cfg, &lo, err, sizeof(err)) ? (size_t)lo.m : 0;
}
size_t prsgd_param_stride(const prsgd_config* cfg) {
  Layout lo;
  char err[128];
  return build_layout(cfg, &lo, err, sizeof(err)) ? (size_t)lo.m_pad : 0;
}
size_t prsgd_workspace_bytes(const prsgd_config* cfg) {
  Layout lo;
  char err[128];
  if (!build_layout(cfg, &lo, err, sizeof(err))) return 0;
  Carve cv;
  build_carve(cfg, lo, &cv);
  return cv.total;
}

}  // extern "C"

namespace {

// Workspace of prsgd_init_static: one array per device, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels and memsets get the
// device address resolved once per device below.
constexpr size_t kStaticBytes = PRSGD_STATIC_WORKSPACE_BYTES;
constexpr int kMaxStaticDevices = 8;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

struct StaticSlot {
  void* ws_dev = nullptr;             // device address of `scratch` on this device
  bool in_use = false;
  alignas(prsgd_ctx) unsigned char ctx_mem[sizeof(prsgd_ctx)];
};
StaticSlot g_static[kMaxStaticDevices];
float g_static_pad[kMaxStaticDevices][kStaticBytes / sizeof(float)];   // host staging, per device
std::mutex g_static_mutex;

void release_ctx(prsgd_ctx* ctx) {
  if (ctx->static_slot < 0) { delete ctx; return; }
  const int slot = ctx->static_slot;
  ctx->~prsgd_ctx();
  std::lock_guard<std::mutex> lock(g_static_mutex);
  g_static[slot].in_use = false;
}

// Shared body of prsgd_init and prsgd_init_static.  static_slot < 0: the context goes on the heap
// and `workspace_dev` is the caller's; otherwise context, staging buffer and workspace are the
// slot's static ones and nothing is allocated.
int init_common(const prsgd_config* cfg, const float* x0_host, const void* features_dev,
                const void* targets_dev, void* params_dev, void* workspace_dev, void* hip_stream,
                int static_slot, prsgd_ctx** out_ctx) {
  Layout lo;
  char err[128];
  if (!build_layout(cfg, &lo, err, sizeof(err))) return set_err(nullptr, PRSGD_EINVAL, "%s", err);
  if (x0_host == nullptr || features_dev == nullptr || targets_dev == nullptr || params_dev == nullptr ||
      workspace_dev == nullptr)
    return set_err(nullptr, PRSGD_EINVAL, "null buffer");
  if (((uintptr_t)params_dev % kAlign) != 0 || ((uintptr_t)workspace_dev % kAlign) != 0)
    return set_err(nullptr, PRSGD_EINVAL, "params_dev and workspace_dev must be 256-byte aligned");
  if (((uintptr_t)features_dev % 16) != 0 || ((uintptr_t)targets_dev % 4) != 0)
    return set_err(nullptr, PRSGD_EINVAL, "features_dev must be 16-byte and targets_dev 4-byte aligned");

  prsgd_ctx* ctx;
  if (static_slot < 0) {
    ctx = new (std::nothrow) prsgd_ctx();
    if (ctx == nullptr) return set_err(nullptr, PRSGD_ENOMEM, "out of host memory");
  } else {
    // claim the device's slot; from here on every failure path gives it back (release_ctx)
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static[static_slot].in_use)
      return set_err(nullptr, PRSGD_ESTATE, "prsgd_init_static: the device's static workspace already "
                                            "serves a live context; destroy it first");
    g_static[static_slot].in_use = true;
    ctx = new (g_static[static_slot].ctx_mem) prsgd_ctx();
  }
  ctx->static_slot = static_slot;
  ctx->cfg = effective_config(cfg);
  ctx->lo = lo;
  build_carve(cfg, lo, &ctx->cv);
  ctx->bf16 = cfg->model == PRSGD_MLP && cfg->gemm_dtype == PRSGD_BF16;
  ctx->streaming = (size_t)cfg->n_workers * (size_t)lo.m_pad * sizeof(float) >= ((size_t)1 << 30);
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  ctx->use_fused2 = ctx->cv.part != 0 && ctx->cv.sync != 0 &&
                    fused2_plan(cfg->n_workers, lo.d[0], lo.d[1], lo.d[2], cfg->batch,
                                cfg->momentum != 0.0f, &ctx->f2);
  if (cfg->momentum != 0.0f && !bwd_fused_config(ctx->cfg) && !ctx->use_fused2) ctx->cfg.fused_update = 0;
  ctx->features = reinterpret_cast<const float*>(features_dev);
  ctx->targets = targets_dev;
  ctx->params = reinterpret_cast<float*>(params_dev);
  ctx->ws = reinterpret_cast<char*>(workspace_dev);
  ctx->t = 0;
  ctx->batch_t[0] = ctx->batch_t[1] = -1;
  ctx->batch_cur = 0;
  ctx->h1_t = -1;
  ctx->h1_batch = 0;
  ctx->first_fusion = true;
  ctx->restart_fusion = true;
  ctx->shadow1_stale = false;
  ctx->lazy_restart = true;
  ctx->at_mean = false;
  ctx->poisoned = false;
  ctx->n_restored = 0;
  memset(ctx->restored, 0, sizeof(ctx->restored));
  ctx->spin_limit = kFused2SpinLimit;
  ctx->lr = cfg->lr;
  ctx->err[0] = 0;
  ctx->profiling = false;
  ctx->pool_used = 0;
  memset(ctx->prof_ms, 0, sizeof(ctx->prof_ms));
  memset(ctx->prof_n, 0, sizeof(ctx->prof_n));
  if (static_slot >= 0) {
    ctx->host_pad = g_static_pad[static_slot];       // m_pad floats fit: the workspace holds as many
  } else {
    try {
      ctx->host_pad_heap.resize((size_t)lo.m_pad);
    } catch (...) {
      release_ctx(ctx);
      return set_err(nullptr, PRSGD_ENOMEM, "out of host memory");
    }
    ctx->host_pad = ctx->host_pad_heap.data();
  }

  // Zero the workspace once: padding columns of every activation buffer must read as zero, and
  // the epoch kernel's arrival counters and abort flag start at zero (the static workspace keeps
  // what the previous context left in it).
  hipError_t e = hipMemsetAsync(ctx->ws, 0, ctx->cv.total, ctx->stream);
  if (e == hipSuccess) {
    pad_from_dense(ctx, x0_host, ctx->host_pad);
    e = hipMemcpyAsync(ctx->at<float>(ctx->cv.mean), ctx->host_pad, sizeof(float) * (size_t)lo.m_pad,
                       hipMemcpyHostToDevice, ctx->stream);
  }
  if (e == hipSuccess)
    e = launch_broadcast(ctx->at<float>(ctx->cv.mean), ctx->params, ctx->shadow(), lo.m_pad,
                         cfg->n_workers, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) {
    hip_fail(nullptr, e, "prsgd_init");
    release_ctx(ctx);
    return PRSGD_EHIP;
  }
  *out_ctx = ctx;
  return PRSGD_OK;
}

}  // namespace

extern "C" {

int prsgd_init(const prsgd_config* cfg, const float* x0_host, const void* features_dev,
               const void* targets_dev, void* params_dev, void* workspace_dev, void* hip_stream,
               prsgd_ctx** out_ctx) {
  if (out_ctx == nullptr) return set_err(nullptr, PRSGD_EINVAL, "out_ctx is null");
  *out_ctx = nullptr;
  return init_common(cfg, x0_host, features_dev, targets_dev, params_dev, workspace_dev, hip_stream, -1,
                     out_ctx);
}

int prsgd_init_static(const prsgd_config* cfg, const float* x0_host, const void* features_dev,
                      const void* targets_dev, void* params_dev, void* hip_stream, prsgd_ctx** out_ctx) {
  if (out_ctx == nullptr) return set_err(nullptr, PRSGD_EINVAL, "out_ctx is null");
  *out_ctx = nullptr;
  Layout lo;
  char err[128];
  if (!build_layout(cfg, &lo, err, sizeof(err))) return set_err(nullptr, PRSGD_EINVAL, "%s", err);
  Carve cv;
  build_carve(cfg, lo, &cv);
  if (cv.total > kStaticBytes) {
    char msg[200];
    snprintf(msg, sizeof(msg), "prsgd_init_static: this configuration needs %zu bytes of workspace, the "
             "static workspace holds %zu; use prsgd_init", cv.total, kStaticBytes);
    return set_err(nullptr, PRSGD_EINVAL, "%s", msg);
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxStaticDevices)
    return set_err(nullptr, PRSGD_EINVAL, "prsgd_init_static: device index beyond the static slots");
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticSlot& slot = g_static[dev];
    if (slot.ws_dev == nullptr) {                  // once per device, with that device current
      void* ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess || ptr == nullptr)
        return hip_fail(nullptr, e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress");
      slot.ws_dev = ptr;
    }
    ws = slot.ws_dev;
  }
  return init_common(cfg, x0_host, features_dev, targets_dev, params_dev, ws, hip_stream, dev, out_ctx);
}

int prsgd_local_steps(prsgd_ctx* ctx, int32_t k) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (k < 0) return set_err(ctx, PRSGD_EINVAL, "k must be >= 0");
  if (check_poisoned(ctx) != PRSGD_OK) return PRSGD_ESTATE;
  const prsgd_config& c = ctx->cfg;
  if (c.model == PRSGD_LSQ) {
    if (k == 0) return PRSGD_OK;
    LAUNCH(ctx, KK_LSQ,
           launch_lsq_steps(ctx->features, reinterpret_cast<const float*>(ctx->targets), ctx->src(),
                            ctx->src_stride(), ctx->params, ctx->velocity(), c.momentum,
                            ctx->at<float>(ctx->cv.losses), ctx->at<int32_t>(ctx->cv.idx), c.n_workers,
                            ctx->lo.d[0], ctx->lo.m_pad, (long)c.rows_per_worker, c.batch, ctx->lr, c.seed,
                            ctx->t, k, nullptr, ctx->stream));
    ctx->at_mean = false;
    ctx->t += k;
    return PRSGD_OK;
  }
  if (ctx->use_fused2) {
    if (k > 0) {
      LAUNCH(ctx, KK_FUSED2, launch_fused2(ctx->f2, fused2_args(ctx, k, nullptr), ctx->stream));
      ctx->at_mean = false;
    }
    ctx->t += k;
    return PRSGD_OK;
  }
  for (int32_t s = 0; s < k; ++s) {
    const int rc = mlp_step(ctx, ctx->t + 1, nullptr, 0);
    if (rc != PRSGD_OK) return rc;
    ctx->t += 1;
  }
  return PRSGD_OK;
}

int prsgd_local_steps_hetero(prsgd_ctx* ctx, const int32_t* steps_host) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (steps_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "steps_host is null");
  if (ctx->cfg.momentum != 0.0f)
    return set_err(ctx, PRSGD_EINVAL, "heterogeneous epochs are not defined with momentum");
  if (check_poisoned(ctx) != PRSGD_OK) return PRSGD_ESTATE;
  const prsgd_config& c = ctx->cfg;
  int32_t k_max = 0;
  for (int i = 0; i < c.n_workers; ++i) {
    if (steps_host[i] < 0) return set_err(ctx, PRSGD_EINVAL, "worker step counts must be >= 0");
    if (steps_host[i] > k_max) k_max = steps_host[i];
  }
  // a worker that takes no step must still hold the restart point: broadcast it first
  const int mrc = materialize(ctx);
  if (mrc != PRSGD_OK) return mrc;
  int* steps_dev = ctx->at<int>(ctx->cv.steps);
  // The pageable source may be reused by the caller right after return: wait for the copy.
  hipError_t e = hipMemcpyAsync(steps_dev, steps_host, sizeof(int32_t) * c.n_workers,
                                hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "copy of worker step counts");
  if (c.model == PRSGD_LSQ) {
    LAUNCH(ctx, KK_LSQ,
           launch_lsq_steps(ctx->features, reinterpret_cast<const float*>(ctx->targets), ctx->params,
                            ctx->lo.m_pad, ctx->params, nullptr, 0.0f,
                            ctx->at<float>(ctx->cv.losses), ctx->at<int32_t>(ctx->cv.idx), c.n_workers,
                            ctx->lo.d[0], ctx->lo.m_pad, (long)c.rows_per_worker, c.batch, ctx->lr, c.seed,
                            ctx->t, k_max, steps_dev, ctx->stream));
    ctx->t += k_max;
    return PRSGD_OK;
  }
  if (ctx->use_fused2) {
    if (k_max > 0)
      LAUNCH(ctx, KK_FUSED2, launch_fused2(ctx->f2, fused2_args(ctx, k_max, steps_dev), ctx->stream));
    ctx->t += k_max;
    return PRSGD_OK;
  }
  for (int32_t s = 0; s < k_max; ++s) {
    const int rc = mlp_step(ctx, ctx->t + 1, steps_dev, s);
    if (rc != PRSGD_OK) return rc;
    ctx->t += 1;
  }
  return PRSGD_OK;
}

int prsgd_average(prsgd_ctx* ctx) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (check_poisoned(ctx) != PRSGD_OK) return PRSGD_ESTATE;
  if (ctx->at_mean) return PRSGD_OK;        // all workers already sit at their node average
  ctx->h1_t = -1;                           // an activation computed ahead belongs to the old points
  if (ctx->velocity() != nullptr && ctx->cfg.momentum_restart != PRSGD_MOM_KEEP) {
    // the paper leaves the momentum buffers at a restart open: average them like the points,
    // or start every epoch without momentum
    if (ctx->cfg.momentum_restart == PRSGD_MOM_AVERAGE)
      LAUNCH(ctx, KK_AVERAGE, launch_average(ctx->velocity(), nullptr, ctx->lo.m_pad, ctx->cfg.n_workers,
                                             ctx->streaming, ctx->stream));
    else
      LAUNCH(ctx, KK_UPDATE, launch_fill_zero(ctx->velocity(), (size_t)ctx->cfg.n_workers * ctx->lo.m_pad,
                                              ctx->stream));
  }
  if (ctx->lazy_restart && ctx->can_start_from_mean()) {
    // eq. (2) without the broadcast: ybar is written once; the next local iteration reads it as
    // every worker's starting point and writes the replicas  x_i = ybar - gamma G_i  itself
    LAUNCH(ctx, KK_RESTART_MEAN,
           launch_mean(ctx->params, ctx->mean(), ctx->mean_shadow(), ctx->lo.m_pad, ctx->cfg.n_workers,
                       ctx->streaming, ctx->stream));
    ctx->at_mean = true;
    return PRSGD_OK;
  }
  LAUNCH(ctx, KK_AVERAGE,
         launch_average(ctx->params, ctx->shadow(), ctx->lo.m_pad, ctx->cfg.n_workers, ctx->streaming,
                        ctx->stream));
  ctx->shadow1_stale = false;               // the averaging kernel rewrites every shadow
  return PRSGD_OK;
}

int prsgd_set_lazy_restart(prsgd_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (!on) {
    const int rc = materialize(ctx);
    if (rc != PRSGD_OK) return rc;
  }
  ctx->lazy_restart = on != 0;
  return PRSGD_OK;
}

int prsgd_run(prsgd_ctx* ctx, int64_t iterations, int32_t interval) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (iterations < 0 || interval < 1) return set_err(ctx, PRSGD_EINVAL, "iterations >= 0, interval >= 1");
  int64_t left = iterations;
  // Plain SGD on bf16 operands with the deferred broadcast: the iteration that completes an epoch
  // and the restart after it are one pass that writes only ybar (with I = 1: every iteration)
  const bool can_fuse = ctx->cfg.model == PRSGD_MLP && ctx->bf16 && ctx->cfg.fused_update &&
                        ctx->cfg.momentum == 0.0f && ctx->lazy_restart && !ctx->use_fused2 &&
                        ctx->restart_fusion && bwd_fused_supported(ctx->cfg.batch);
  while (left > 0) {
    if (can_fuse && interval - (ctx->t % interval) <= left) {
      const int64_t k_epoch = interval - (ctx->t % interval);
      if (k_epoch > 1) {
        const int rc = prsgd_local_steps(ctx, (int32_t)(k_epoch - 1));
        if (rc != PRSGD_OK) return rc;
      }
      if (check_poisoned(ctx) != PRSGD_OK) return PRSGD_ESTATE;
      const int rc = mlp_step(ctx, ctx->t + 1, nullptr, 0, true);
      if (rc != PRSGD_OK) return rc;
      ctx->t += 1;
      left -= k_epoch;
      continue;
    }
    int64_t k = interval - (ctx->t % interval);      // steps until the next multiple of I
    if (k > left) k = left;
    int rc = prsgd_local_steps(ctx, (int32_t)k);
    if (rc != PRSGD_OK) return rc;
    left -= k;
    if (ctx->t % interval == 0) {
      rc = prsgd_average(ctx);
      if (rc != PRSGD_OK) return rc;
    }
  }
  return PRSGD_OK;
}

int prsgd_read_params(prsgd_ctx* ctx, int32_t worker, float* out_host, size_t m) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (out_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "out_host is null");
  if (m != (size_t)ctx->lo.m) return set_err(ctx, PRSGD_EINVAL, "m does not match the parameter count");
  if (worker < -1 || worker >= ctx->cfg.n_workers) return set_err(ctx, PRSGD_EINVAL, "worker out of range");
  const int arc = check_fused2_abort(ctx);
  if (arc != PRSGD_OK) return arc;
  const float* src;
  if (ctx->at_mean) {
    src = ctx->mean();                      // every worker's point, and their average
  } else if (worker < 0) {
    LAUNCH(ctx, KK_MEAN, launch_mean(ctx->params, ctx->mean(), nullptr, ctx->lo.m_pad,
                                     ctx->cfg.n_workers, true, ctx->stream));
    src = ctx->mean();
  } else {
    src = ctx->params + (size_t)worker * ctx->lo.m_pad;
  }
  hipError_t e = hipMemcpyAsync(ctx->host_pad, src, sizeof(float) * (size_t)ctx->lo.m_pad,
                                hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_read_params");
  dense_from_pad(ctx, ctx->host_pad, out_host);
  return PRSGD_OK;
}

int prsgd_write_params(prsgd_ctx* ctx, int32_t worker, const float* in_host, size_t m) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (in_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "in_host is null");
  if (m != (size_t)ctx->lo.m) return set_err(ctx, PRSGD_EINVAL, "m does not match the parameter count");
  if (worker < -1 || worker >= ctx->cfg.n_workers) return set_err(ctx, PRSGD_EINVAL, "worker out of range");
  if (worker >= 0) {                        // the other replicas must hold their restart point
    const int mrc = materialize(ctx);
    if (mrc != PRSGD_OK) return mrc;
  }
  if (ctx->poisoned) {                      // an aborted epoch launch: usable again once every
    if (worker < 0) {                       // replica has been rewritten
      ctx->poisoned = false;
    } else if (!((ctx->restored[worker >> 3] >> (worker & 7)) & 1)) {
      ctx->restored[worker >> 3] |= (unsigned char)(1u << (worker & 7));
      if (++ctx->n_restored == (size_t)ctx->cfg.n_workers) ctx->poisoned = false;
    }
  }
  ctx->at_mean = false;
  ctx->h1_t = -1;
  pad_from_dense(ctx, in_host, ctx->host_pad);
  const size_t bytes = sizeof(float) * (size_t)ctx->lo.m_pad;
  hipError_t e;
  if (worker < 0) {
    e = hipMemcpyAsync(ctx->at<float>(ctx->cv.mean), ctx->host_pad, bytes, hipMemcpyHostToDevice,
                       ctx->stream);
    if (e == hipSuccess)
      e = launch_broadcast(ctx->at<float>(ctx->cv.mean), ctx->params, ctx->shadow(), ctx->lo.m_pad,
                           ctx->cfg.n_workers, ctx->stream);
    ctx->shadow1_stale = false;
  } else {
    float* dst = ctx->params + (size_t)worker * ctx->lo.m_pad;
    e = hipMemcpyAsync(dst, ctx->host_pad, bytes, hipMemcpyHostToDevice, ctx->stream);
    if (e == hipSuccess && ctx->bf16)
      e = launch_refresh_shadow(dst, ctx->shadow() + (size_t)worker * ctx->lo.m_pad, ctx->lo.m_pad,
                                ctx->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_write_params");
  return PRSGD_OK;
}

int prsgd_read_velocity(prsgd_ctx* ctx, int32_t worker, float* out_host, size_t m) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (out_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "out_host is null");
  if (m != (size_t)ctx->lo.m) return set_err(ctx, PRSGD_EINVAL, "m does not match the parameter count");
  if (worker < 0 || worker >= ctx->cfg.n_workers) return set_err(ctx, PRSGD_EINVAL, "worker out of range");
  if (ctx->velocity() == nullptr) return set_err(ctx, PRSGD_ESTATE, "the context has no momentum buffers");
  const int arc = check_fused2_abort(ctx);
  if (arc != PRSGD_OK) return arc;
  hipError_t e = hipMemcpyAsync(ctx->host_pad, ctx->velocity() + (size_t)worker * ctx->lo.m_pad,
                                sizeof(float) * (size_t)ctx->lo.m_pad, hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_read_velocity");
  dense_from_pad(ctx, ctx->host_pad, out_host);
  return PRSGD_OK;
}

int prsgd_write_velocity(prsgd_ctx* ctx, int32_t worker, const float* in_host, size_t m) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (in_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "in_host is null");
  if (m != (size_t)ctx->lo.m) return set_err(ctx, PRSGD_EINVAL, "m does not match the parameter count");
  if (worker < 0 || worker >= ctx->cfg.n_workers) return set_err(ctx, PRSGD_EINVAL, "worker out of range");
  if (ctx->velocity() == nullptr) return set_err(ctx, PRSGD_ESTATE, "the context has no momentum buffers");
  pad_from_dense(ctx, in_host, ctx->host_pad);
  hipError_t e = hipMemcpyAsync(ctx->velocity() + (size_t)worker * ctx->lo.m_pad, ctx->host_pad,
                                sizeof(float) * (size_t)ctx->lo.m_pad, hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_write_velocity");
  return PRSGD_OK;
}

int prsgd_read_loss(prsgd_ctx* ctx, float* out_host) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (out_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "out_host is null");
  const int arc = check_fused2_abort(ctx);
  if (arc != PRSGD_OK) return arc;
  hipError_t e = hipSuccess;
  if (ctx->cfg.model == PRSGD_MLP)
    e = launch_loss_mean(ctx->at<float>(ctx->cv.row_loss), ctx->at<float>(ctx->cv.losses),
                         ctx->cfg.n_workers, ctx->cfg.batch, ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(out_host, ctx->at<float>(ctx->cv.losses), sizeof(float) * ctx->cfg.n_workers,
                                hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_read_loss");
  return PRSGD_OK;
}

int prsgd_read_indices(prsgd_ctx* ctx, int32_t* out_host) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (out_host == nullptr) return set_err(ctx, PRSGD_EINVAL, "out_host is null");
  const int arc = check_fused2_abort(ctx);
  if (arc != PRSGD_OK) return arc;
  const size_t bytes = sizeof(int32_t) * (size_t)ctx->cfg.n_workers * ctx->cfg.batch;
  // the layer-wise MLP path alternates between two buffer sets; the others only use the first
  hipError_t e = hipMemcpyAsync(out_host, ctx->idx(ctx->batch_cur), bytes, hipMemcpyDeviceToHost,
                                ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_read_indices");
  return PRSGD_OK;
}

int prsgd_sample_indices(uint64_t seed, int32_t n_workers, int32_t batch, int64_t rows_per_worker,
                         int64_t t_first, int32_t n_steps, int32_t* out_dev, void* hip_stream) {
  if (out_dev == nullptr || n_workers < 1 || batch < 1 || n_steps < 0 || t_first < 0 ||
      rows_per_worker < 1 || rows_per_worker > (1LL << 31) ||
      (rows_per_worker & (rows_per_worker - 1)) != 0)
    return set_err(nullptr, PRSGD_EINVAL, "prsgd_sample_indices: bad argument");
  hipError_t e = launch_sample_indices(seed, n_workers, batch, (long)rows_per_worker, t_first, n_steps,
                                       out_dev, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(nullptr, e, "prsgd_sample_indices");
  return PRSGD_OK;
}

int prsgd_sgd_update(float* x_dev, const float* g_dev, uint16_t* shadow_dev, size_t count, float lr,
                     void* hip_stream) {
  if (x_dev == nullptr || g_dev == nullptr) return set_err(nullptr, PRSGD_EINVAL, "null buffer");
  if (((uintptr_t)x_dev % 16) != 0 || ((uintptr_t)g_dev % 16) != 0 || ((uintptr_t)shadow_dev % 8) != 0)
    return set_err(nullptr, PRSGD_EINVAL, "prsgd_sgd_update: misaligned buffer");
  hipError_t e = launch_update(x_dev, g_dev, shadow_dev, count, lr, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(nullptr, e, "prsgd_sgd_update");
  return PRSGD_OK;
}

int prsgd_copy_bytes(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (dst_dev == nullptr || src_dev == nullptr || (bytes % 16) != 0 || ((uintptr_t)dst_dev % 16) != 0 ||
      ((uintptr_t)src_dev % 16) != 0)
    return set_err(nullptr, PRSGD_EINVAL, "prsgd_copy_bytes: bad argument");
  hipError_t e = launch_copy(dst_dev, src_dev, bytes, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(nullptr, e, "prsgd_copy_bytes");
  return PRSGD_OK;
}

int prsgd_status(prsgd_ctx* ctx) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  const int arc = check_fused2_abort(ctx);
  if (arc != PRSGD_OK) return arc;
  const hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e, "prsgd_status");
  return PRSGD_OK;
}

int prsgd_set_restart_fusion(prsgd_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  ctx->restart_fusion = on != 0;
  return PRSGD_OK;
}

int prsgd_set_first_layer_fusion(prsgd_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  ctx->first_fusion = on != 0;
  ctx->h1_t = -1;
  return PRSGD_OK;
}

int prsgd_set_epoch_wait_limit(prsgd_ctx* ctx, uint32_t polls) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  ctx->spin_limit = polls;
  return PRSGD_OK;
}

int prsgd_time_varying_schedule(int32_t n_epochs, int32_t n_workers, int32_t* lengths_host,
                                float* rates_host) {
  if (n_epochs < 0 || n_workers < 1 || (n_epochs > 0 && (lengths_host == nullptr || rates_host == nullptr)))
    return set_err(nullptr, PRSGD_EINVAL, "prsgd_time_varying_schedule: bad argument");
  // K^s = ceil(s^(1/3) / N) is the smallest integer k with (k N)^3 >= s: integer arithmetic, so
  // that perfect cubes land exactly.  k N only ever grows with s.
  unsigned __int128 kn = (unsigned __int128)n_workers;      // current k N
  int32_t k = 1;
  for (int32_t s = 1; s <= n_epochs; ++s) {
    while (kn * kn * kn < (unsigned __int128)s) { kn += (unsigned __int128)n_workers; ++k; }
    lengths_host[s - 1] = k;
    const double c = cbrt((double)s);
    rates_host[s - 1] = (float)((double)n_workers / (c * c));
  }
  return PRSGD_OK;
}

int prsgd_set_lr(prsgd_ctx* ctx, float lr) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (!(lr == lr)) return set_err(ctx, PRSGD_EINVAL, "lr is NaN");
  ctx->lr = lr;
  return PRSGD_OK;
}
int prsgd_set_iteration(prsgd_ctx* ctx, int64_t t) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (t < 0) return set_err(ctx, PRSGD_EINVAL, "t must be >= 0");
  ctx->t = t;
  return PRSGD_OK;
}
int64_t prsgd_iteration(const prsgd_ctx* ctx) { return ctx == nullptr ? -1 : ctx->t; }

int prsgd_profile_enable(prsgd_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (on && ctx->pool.empty()) {
    constexpr size_t kPairs = 2048;
    try {
      ctx->pool.reserve(kPairs);
    } catch (...) {
      return set_err(ctx, PRSGD_ENOMEM, "out of host memory");
    }
    for (size_t i = 0; i < kPairs; ++i) {
      EventPair ep;
      hipError_t e = hipEventCreate(&ep.a);
      if (e == hipSuccess) {
        e = hipEventCreate(&ep.b);
        if (e != hipSuccess) (void)hipEventDestroy(ep.a);
      }
      if (e != hipSuccess) return hip_fail(ctx, e, "hipEventCreate");
      ep.kind = 0;
      ctx->pool.push_back(ep);
    }
  }
  if (!on) {
    const int rc = profile_flush(ctx);
    if (rc != PRSGD_OK) return rc;
  }
  ctx->profiling = on != 0;
  return PRSGD_OK;
}

int prsgd_profile_read(prsgd_ctx* ctx, prsgd_kernel_stat* out, int32_t max) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  if (out == nullptr || max < 0) return set_err(ctx, PRSGD_EINVAL, "bad output buffer");
  const int rc = profile_flush(ctx);
  if (rc != PRSGD_OK) return rc;
  int n = 0;
  for (int k = 0; k < KK_COUNT; ++k) {
    if (ctx->prof_n[k] == 0) continue;
    if (n < max) {
      memset(&out[n], 0, sizeof(out[n]));
      snprintf(out[n].name, sizeof(out[n].name), "%s", kernel_kind_name(k));
      out[n].launches = ctx->prof_n[k];
      out[n].total_ms = ctx->prof_ms[k];
    }
    ++n;
  }
  memset(ctx->prof_ms, 0, sizeof(ctx->prof_ms));
  memset(ctx->prof_n, 0, sizeof(ctx->prof_n));
  return n;
}

int prsgd_destroy(prsgd_ctx* ctx) {
  if (ctx == nullptr) return PRSGD_EINVAL;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  for (auto& ep : ctx->pool) {
    (void)hipEventDestroy(ep.a);
    (void)hipEventDestroy(ep.b);
  }
  release_ctx(ctx);
  return e == hipSuccess ? PRSGD_OK : PRSGD_EHIP;
}

const char* prsgd_last_error(const prsgd_ctx* ctx) { return ctx != nullptr ? ctx->err : g_init_error; }

}  // extern "C"
