/*
 * prsgd.h -- C ABI of the MI355X (gfx950) Parallel Restarted SGD hot path.
 *
 * The library simulates the N workers of the paper's problem statement
 * (Section 1, eq. 1:  min_x f(x) = (1/N) sum_i f_i(x),  f_i = E_{zeta ~ D_i} F_i(x; zeta))
 * on ONE GPU.  Every worker owns a model replica x_i in HBM and a private data
 * shard (its distribution D_i).  Algorithm 1 is driven through three calls:
 *
 *   prsgd_local_steps(k)  k iterations of  x_i <- x_i - gamma * G_i  on every worker
 *                         (Algorithm 1, eq. 3), G_i the minibatch gradient of F_i at the
 *                         worker's own current point; no exchange between workers.
 *   prsgd_average()       the restart: ybar = (1/N) sum_i x_i overwrites every replica
 *                         (Algorithm 1, eq. 2 and the paragraph below the algorithm).
 *   prsgd_read_params()   copies one replica, or the node average xbar of eq. (4), to the host.
 *
 * Interval I = 1 (one local step, then an average) is parallel mini-batch SGD
 * (Section 1, first footnote).
 *
 * Conventions
 *   - Every function returns a status (PRSGD_OK == 0, negative on error) unless stated
 *     otherwise, never throws and never aborts.  prsgd_last_error() gives the text of the
 *     last failure of a context (or of the last failed prsgd_init when ctx == NULL).
 *   - "_dev" pointers are device (HBM) addresses, "_host" pointers are host addresses.
 *   - All device buffers are CALLER-OWNED.  The library borrows them between prsgd_init and
 *     prsgd_destroy, allocates no device memory itself and enqueues work only on the HIP
 *     stream given to prsgd_init.  Calls are asynchronous with respect to the host except
 *     the prsgd_read_* / prsgd_write_* calls, which synchronise that stream.
 *   - A context is not thread-safe; use it from one host thread at a time.
 */
#ifndef PRSGD_H
#define PRSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct prsgd_ctx prsgd_ctx;

enum { PRSGD_OK = 0, PRSGD_EINVAL = -1, PRSGD_ESTATE = -2, PRSGD_EHIP = -3, PRSGD_ENOMEM = -4 };
enum { PRSGD_LSQ = 0, PRSGD_MLP = 1 };          /* objective F_i                          */
enum { PRSGD_TANH = 0, PRSGD_RELU = 1 };        /* hidden activation of the MLP           */
enum { PRSGD_F32 = 0, PRSGD_BF16 = 1 };         /* operand type of the matrix products    */
/* what a restart does to the workers' momentum buffers (the paper does not say) */
enum { PRSGD_MOM_KEEP = 0, PRSGD_MOM_AVERAGE = 1, PRSGD_MOM_RESET = 2 };
#define PRSGD_MAX_DIMS 16

/*
 * Problem description.  The paper leaves F_i abstract; two objectives are provided:
 *   PRSGD_LSQ  dims = {d}.        F = 1/(2B) sum_j (a_j . x - y_j)^2,   m = d.
 *   PRSGD_MLP  dims = {d_0..d_L}. h_l = phi(h_{l-1} W_l + b_l), last layer linear,
 *              F = mean softmax cross-entropy over the B rows;  m = sum_l (d_{l-1} + 1) d_l.
 * With PRSGD_BF16 the operands of every matrix product (weights, activations, back-propagated
 * deltas) are rounded to bfloat16 (nearest, ties to even) and accumulated in fp32; the master
 * parameters, bias add, activation, softmax, loss, update and average stay fp32.
 */
typedef struct {
  int32_t  n_workers;              /* N >= 1                                                   */
  int32_t  model;                  /* PRSGD_LSQ | PRSGD_MLP                                    */
  int32_t  n_dims;                 /* 1 for LSQ, L+1 >= 2 for an MLP                           */
  int32_t  dims[PRSGD_MAX_DIMS];
  int32_t  activation;             /* PRSGD_TANH | PRSGD_RELU (MLP only)                       */
  int32_t  gemm_dtype;             /* PRSGD_F32 | PRSGD_BF16 (MLP only)                        */
  int32_t  batch;                  /* B rows per worker per iteration, 1..4096                 */
  int32_t  fused_update;           /* MLP: 1 = eq. (3) applied inside the weight-gradient
                                      kernel; 0 = gradients written to HBM, then a separate
                                      elementwise update kernel                               */
  int64_t  rows_per_worker;        /* n, a power of two: rows in each worker's shard           */
  float    lr;                     /* gamma                                                    */
  uint64_t seed;                   /* seed of the minibatch index stream                       */
  float    momentum;               /* mu in [0, 1).  0: the plain local step of eq. (3).  Otherwise the
                                      momentum-SGD local step of the paper's experiment (Section 4,
                                      momentum 0.9), in the form  v_i <- mu v_i + G_i,
                                      x_i <- x_i - gamma v_i  with v_i = 0 at the start.  With
                                      fused_update = 1 it is applied inside the one-pass backward
                                      kernel (bf16 operands, B <= 128) or the epoch kernel (fp32,
                                      one hidden layer); otherwise the gradients go to HBM and an
                                      elementwise kernel applies it.                                */
  int32_t  momentum_restart;       /* PRSGD_MOM_KEEP (buffers stay local, default) | _AVERAGE (node
                                      average of the buffers overwrites them) | _RESET (zeroed)    */
} prsgd_config;

/* m, the dimension of x in eq. (1): scalar parameters of one replica (0 if the config is invalid). */
size_t prsgd_param_count(const prsgd_config* cfg);
/* Floats per replica in the device layout (m rounded up with alignment padding). */
size_t prsgd_param_stride(const prsgd_config* cfg);
/* Bytes of device workspace prsgd_init needs (0 if the config is invalid). */
size_t prsgd_workspace_bytes(const prsgd_config* cfg);

/*
 * Creates a context.  Every replica starts from the same point (Algorithm 1, input line).
 *   x0_host       [m] fp32, host.  MLP layout: W_1 (d_0 x d_1 row-major), b_1, W_2, b_2, ...
 *   features_dev  [N][n][d_0] fp32, device, dense; worker i samples only its own [n][d_0] slab.
 *   targets_dev   [N][n] device: fp32 targets (LSQ) or int32 class labels in [0, d_L) (MLP).
 *   params_dev    [N][prsgd_param_stride] fp32, device, 256-byte aligned: the replicas.
 *   workspace_dev prsgd_workspace_bytes bytes, device, 256-byte aligned.
 *   hip_stream    a hipStream_t (NULL = the default stream).
 * The iteration counter starts at 0.  Errors: PRSGD_EINVAL for a null pointer, a size out of
 * range, n not a power of two or misaligned buffers; PRSGD_EHIP if a HIP call fails.
 */
int prsgd_init(const prsgd_config* cfg, const float* x0_host, const void* features_dev,
               const void* targets_dev, void* params_dev, void* workspace_dev, void* hip_stream,
               prsgd_ctx** out_ctx);

/*
 * prsgd_init for callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops, harnesses that forbid it): the same context, but its workspace is a static
 * array inside the library, PRSGD_STATIC_WORKSPACE_BYTES per device, held by every device the
 * library runs on until the process ends.  The call itself allocates nothing, neither on the
 * device nor on the host (the context and its staging buffer live in static storage too); the
 * caller still passes the shards and the replica buffer.  A configuration whose
 * prsgd_workspace_bytes exceeds the limit is refused with PRSGD_EINVAL (the limit covers the
 * small, latency-bound configurations: c1, c2, c4); device indices 0..7.  All static contexts of a
 * device share the one array, so only one may be live per device at a time: a second call before
 * prsgd_destroy returns PRSGD_ESTATE.  The array keeps what the previous context left in it;
 * the call clears what the new one needs.  Everything else (errors, stream, ownership) as
 * prsgd_init.
 */
#define PRSGD_STATIC_WORKSPACE_BYTES (16u << 20)
int prsgd_init_static(const prsgd_config* cfg, const float* x0_host, const void* features_dev,
                      const void* targets_dev, void* params_dev, void* hip_stream,
                      prsgd_ctx** out_ctx);

/*
 * k >= 0 iterations of eq. (3) on every worker.  At iteration t (counted from 1) worker i
 * draws B rows of its shard uniformly with replacement: slot j uses word (j mod 4) of
 * Philox4x32-10 with counter (j / 4, t mod 2^32, t >> 32, i) and key (seed mod 2^32,
 * seed >> 32), reduced to a row by taking its top log2(n) bits -- an unbiased, independent
 * sample of D_i as Section 1 requires.  Advances the iteration counter by k.
 */
int prsgd_local_steps(prsgd_ctx* ctx, int32_t k);

/*
 * One epoch of the heterogeneous variant (Algorithm 3): worker i takes steps_host[i] >= 0
 * local iterations; a worker that has finished keeps its point (the paper's imagined
 * zero-gradient steps).  The iteration counter advances by max_i steps_host[i].
 * Not defined with momentum (a zero-gradient step would still move the point): PRSGD_EINVAL.
 */
int prsgd_local_steps_hetero(prsgd_ctx* ctx, const int32_t* steps_host /* [N] */);

/*
 * Restart: x_i <- (1/N) sum_j x_j for every i (eq. 2), in fp32, in a fixed order: workers are
 * summed in ascending order, then one division by N.  Small replica sets (N >= 8 and fewer than
 * 262144 floats per replica) split the workers into four consecutive quarters that are summed in
 * ascending order each and then added quarter by quarter, ((q0 + q1) + q2) + q3.  Either way the
 * result is the same from run to run.
 * After the call every worker's point (as seen by prsgd_read_params and by the next local
 * iteration) is the node average.  By default the broadcast is deferred where the kernels
 * support it: the average is written once and the next local iteration, which rewrites every
 * replica anyway (x_i = ybar - gamma G_i, the form of eq. 2), reads it as the common starting
 * point -- what the first footnote of Section 1 describes for I = 1.  Calling it again before
 * any local step is a no-op.
 */
int prsgd_average(prsgd_ctx* ctx);
/*
 * on = 0: every prsgd_average overwrites all replicas at once (one read and one write of the
 * whole replica set: the stand-alone averaging kernel).  on = 1 (default): deferred broadcast.
 * Results are identical either way, except that prsgd_run takes an epoch's last iteration and the
 * restart as one pass (see there; equal up to fp32 rounding) only with the deferred broadcast.
 */
int prsgd_set_lazy_restart(prsgd_ctx* ctx, int32_t on);

/*
 * Algorithm 1 for `iterations` iterations from the current counter t: local steps, and an
 * average after every iteration whose number is a multiple of `interval` (so a run whose
 * length is not a multiple of the interval ends un-averaged).
 * For MLPs with bf16 operands, plain SGD, the fused update and the deferred broadcast (the defaults)
 * the iteration that completes an epoch and the restart after it are taken as one pass,
 *   ybar' = (1/N) sum_i (x_i - gamma G_i(x_i)) = ybar - (gamma / N) sum_i G_i(x_i),  ybar = (1/N) sum_i x_i:
 * ybar is averaged from the points as they are, the weight gradients of all N minibatches are
 * contracted as one product of N B rows and applied to it; the replicas are not rewritten (every
 * worker's point reads as ybar').  Equal to eq. (2)-(3) taken one after the other up to fp32
 * rounding (gamma / N is rounded to fp32; fewer roundings per parameter).  With interval = 1 every
 * iteration after the first starts at ybar and is exactly one mini-batch SGD step with the N B
 * samples of all workers (first footnote of Section 1).  prsgd_local_steps followed by
 * prsgd_average always runs the two kernels separately.
 */
int prsgd_run(prsgd_ctx* ctx, int64_t iterations, int32_t interval);

/*
 * Copies replica `worker` (0..N-1) -- or, with worker == -1, the node average xbar of
 * eq. (4), computed without modifying any replica -- to out_host[m] in the x0 layout.
 * m must equal prsgd_param_count.  Synchronises the stream.
 */
int prsgd_read_params(prsgd_ctx* ctx, int32_t worker, float* out_host, size_t m);
/* Overwrites replica `worker`, or every replica with worker == -1 (checkpoint restore). */
int prsgd_write_params(prsgd_ctx* ctx, int32_t worker, const float* in_host, size_t m);
/*
 * Momentum buffer v_i of worker `worker` (0..N-1) in the x0 layout, for checkpoints.
 * PRSGD_ESTATE if the context was created with momentum == 0.  Synchronise the stream.
 */
int prsgd_read_velocity(prsgd_ctx* ctx, int32_t worker, float* out_host, size_t m);
int prsgd_write_velocity(prsgd_ctx* ctx, int32_t worker, const float* in_host, size_t m);

/*
 * Minibatch loss F_i(x_i^{t-1}; zeta_i^t) (the stochastic objective of eq. 1, evaluated where
 * Algorithm 1 observes the gradient) of each worker at its most recent local iteration,
 * out_host[N].  Synchronises the stream.
 */
int prsgd_read_loss(prsgd_ctx* ctx, float* out_host);
/* Row indices each worker used at its most recent local iteration, out_host[N][B]. */
int prsgd_read_indices(prsgd_ctx* ctx, int32_t* out_host);

/*
 * Stateless view of the index stream: fills out_dev[n_steps][N][B] (int32, device) with the
 * rows of iterations t_first .. t_first + n_steps - 1, exactly as prsgd_local_steps draws them.
 */
int prsgd_sample_indices(uint64_t seed, int32_t n_workers, int32_t batch, int64_t rows_per_worker,
                         int64_t t_first, int32_t n_steps, int32_t* out_dev, void* hip_stream);

/*
 * Stand-alone form of eq. (3) on flat device vectors: x <- x - lr * g for `count` fp32
 * elements; if shadow_dev is non-null it also receives bfloat16(x).  x_dev, g_dev 16-byte and
 * shadow_dev 8-byte aligned.  This is the kernel the fused_update = 0 path runs.
 */
int prsgd_sgd_update(float* x_dev, const float* g_dev, uint16_t* shadow_dev, size_t count,
                     float lr, void* hip_stream);

/*
 * Epoch lengths and learning rates of Algorithm 2 as Theorem 2 chooses them:
 *   lengths_host[s-1] = K^s = ceil(s^(1/3) / N),   rates_host[s-1] = gamma^s = N / s^(2/3),
 * s = 1..n_epochs (host arrays of n_epochs elements).  K^s is computed in integer arithmetic
 * (the smallest k with (k N)^3 >= s).  Algorithm 2 is then: for every epoch prsgd_average,
 * prsgd_set_lr(gamma^s), prsgd_local_steps(K^s).  PRSGD_EINVAL for a null array or N < 1.
 */
int prsgd_time_varying_schedule(int32_t n_epochs, int32_t n_workers, int32_t* lengths_host,
                                float* rates_host);

/*
 * Learning rate of the iterations that follow: gamma of Algorithm 1, or gamma^s of epoch s of
 * Algorithm 2 (time-varying rates, Theorem 2) when called between epochs.
 */
int     prsgd_set_lr(prsgd_ctx* ctx, float lr);
/* t of Algorithm 1: iterations done so far (the index stream and the restart phase follow it). */
int     prsgd_set_iteration(prsgd_ctx* ctx, int64_t t);   /* resume from a checkpoint            */
int64_t prsgd_iteration(const prsgd_ctx* ctx);            /* < 0 on a null context               */

/*
 * Synchronises the stream and reports whether every launch so far ran to completion.
 * One-hidden-layer fp32 MLPs run whole epochs in one launch whose workgroups wait for each other
 * inside the kernel; that needs all of them resident at once, which holds on a device that runs
 * nothing else (checked at prsgd_init) -- keep the device otherwise idle while such a context is
 * stepping.  If other work did hold compute units, the kernel's bounded wait gives up instead of
 * hanging: this call (like every prsgd_read_* call) then returns PRSGD_ESTATE, the replicas are
 * inconsistent, and prsgd_local_steps / prsgd_average / prsgd_run keep returning PRSGD_ESTATE
 * until every replica has been rewritten with prsgd_write_params (worker -1, or each worker
 * once).  From then on the context runs its local steps as a chain of per-layer kernels, which
 * needs no co-resident workgroups.
 */
int prsgd_status(prsgd_ctx* ctx);

/*
 * Per-kernel timing with HIP events on the context's stream.  While enabled every kernel
 * launch is bracketed by an event pair (this serialises launches; leave it off when timing
 * whole runs).  prsgd_profile_read synchronises, then fills up to `max` records, returns the
 * number of kernel kinds (or a negative status) and resets the counters.
 */
typedef struct {
  char     name[48];
  int64_t  launches;
  double   total_ms;
} prsgd_kernel_stat;
int prsgd_profile_enable(prsgd_ctx* ctx, int32_t on);
int prsgd_profile_read(prsgd_ctx* ctx, prsgd_kernel_stat* out, int32_t max);

/* Releases the context (not the caller's buffers).  Synchronises the stream. */
int prsgd_destroy(prsgd_ctx* ctx);
const char* prsgd_last_error(const prsgd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PRSGD_H */
