// Internal declarations shared by the HIP translation units of libprsgd (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "prsgd.h"

namespace prsgd {

constexpr int kThreads = 256;        // 4 wavefronts of 64 lanes per workgroup
constexpr int kWave = 64;
constexpr int kMaxBatch = 4096;
constexpr int kMaxLsqDim = 8192;

// Device layout of one replica x_i (floats).  An MLP replica is
//   [W_1][b_1][W_2][b_2]...   W_l stored row-major as [d_{l-1}][ld_l], ld_l = d_l rounded up
// to a multiple of 8 so that every row starts 32-byte aligned; each segment starts on a
// 64-float boundary.  All padding holds zeros and stays zero under update and average.
struct Layout {
  int  n_layers;                     // L (0 for least squares)
  int  d[PRSGD_MAX_DIMS];            // logical widths d_0..d_L
  int  ld[PRSGD_MAX_DIMS];           // padded widths
  long w_off[PRSGD_MAX_DIMS];        // offset of W_l, index l-1
  long b_off[PRSGD_MAX_DIMS];        // offset of b_l, index l-1
  long m;                            // logical parameter count
  long m_pad;                        // replica stride in floats
};

enum GemmEpilogue {
  EPI_FWD_HIDDEN = 0,   // out = T(phi(acc + bias))
  EPI_FWD_LOGITS = 1,   // out = float(acc + bias)
  EPI_DX = 2,           // out = T(acc * phi'(aux))
  EPI_DW_FUSED = 3,     // W <- W - lr * acc (and bf16 shadow), b likewise from column sums
  EPI_DW_GRAD = 4,      // G_W = acc, G_b = column sums
};

// One grouped matrix product: for every group (replica) g
//   C_g[m][n] = sum_c A_g(m, c) * B_g(n, c),   m < M, n < N, c < Kc
// followed by an epilogue.  Operand element (r, c) sits at base + g*gs + r*ld + c when the
// operand is contraction-contiguous, or at base + g*gs + c*ld + r when it is transposed.
struct GemmArgs {
  const void* a; long a_gs; int lda;
  const void* b; long b_gs; int ldb;
  int M, N, Kc;
  int n_groups;                       // filled in by the launcher
  int epi;
  int streaming;                      // weights far exceed the caches: non-temporal accesses
  int act;                            // PRSGD_TANH | PRSGD_RELU
  float lr;
  // parameters / gradients (fp32, replica stride m_pad), bf16 shadow of the parameters
  float* params; float* grads; uint16_t* shadow; long p_gs;
  // where the forward products read the bias from: the replicas, or (right after a restart
  // whose broadcast was skipped) the shared node average with stride 0
  const float* bias_src; long bias_gs;
  long w_off, b_off; int ldw;
  // activation-like output (element type T, or float for logits) and auxiliary input
  void* out; long out_gs; int ldo; int out_cols;
  const void* aux; long aux_gs; int ldaux;
  // Algorithm 3: group g is skipped once step >= worker_steps[g] (nullptr = all active)
  const int* worker_steps; int step;
  // logits product of a narrow last layer: the contraction is cut into k_splits ranges, split s
  // writes its partial sums (no bias) at out + s * split_stride; the loss head adds them up
  int k_splits; long split_stride;
};
// contraction splits the forward launcher wants for the logits product described by p
int gemm_logit_splits(const GemmArgs& p, int n_groups, bool bf16);
constexpr int kMaxLogitSplits = 4;

enum KernelKind {
  KK_GATHER = 0, KK_FWD, KK_LOSS, KK_DX, KK_DW, KK_UPDATE, KK_AVERAGE, KK_MEAN, KK_BROADCAST,
  KK_LSQ, KK_FUSED2, KK_BWD, KK_RESTART_MEAN, KK_STEP_MEAN, KK_BWD_FIRST, KK_REFRESH, KK_COUNT
};

// Fused backward step of one layer with bf16 operands (kernels_bwd.hip): weight gradient, local
// update of W_l and b_l, and the delta of the layer below, in one pass over W_l.
struct BwdArgs {
  const uint16_t* h; long h_gs; int ldh;        // H_{l-1} [N][B][ldh]
  const uint16_t* d; long d_gs; int ldd;        // D_l     [N][B][ldd]
  float* params; uint16_t* shadow; long p_gs;   // fp32 master and bf16 shadow, replica stride
  const float* src; long src_gs;                // where the old parameters are read from: the
                                                // replicas (src_gs = p_gs) or the shared node
                                                // average right after a restart (src_gs = 0)
  long w_off, b_off; int ldw;
  uint16_t* dx; long dx_gs; int lddx;           // D_{l-1} [N][B][lddx]; nullptr for the first layer
  int B, K, Nn;                                 // minibatch rows, d_{l-1}, d_l
  int n_groups, act, streaming;
  float lr;
  float* vel; float mu;                         // momentum buffers [N][p_gs] (nullptr = plain SGD)
  const int* worker_steps; int step;            // Algorithm 3 mask (nullptr = all active)
  // first layer only (kernels_bwd_first.hip): minibatch of the next iteration [N][B][ldx] and
  // where its first hidden activation goes [N][B][ldhn]
  const uint16_t* x_next; long x_gs; int ldx;
  uint16_t* h_next; long hn_gs; int ldhn;
};
bool bwd_fused_supported(int batch);
hipError_t launch_bwd_fused(const BwdArgs& p, hipStream_t s);
// Layer 1: backward step fused with the next iteration's forward product of that layer.
bool bwd_first_fwd_applies(const BwdArgs& p);
hipError_t launch_bwd_first_fwd(const BwdArgs& p, hipStream_t s);

// Epoch kernel for fp32 MLPs with one hidden layer (kernels_fused2.hip).
struct Fused2Plan {
  int KBI, NT, MT;     // template shape: W_1 row blocks per wavefront, hidden tiles, batch tiles
  int P;               // workgroups per worker
  int d2p, ldx;        // padded class count, LDS row stride of the gathered batch
  int momentum;        // 1: the variant that carries velocities
};
struct Fused2Args {
  const float* features; const int32_t* labels;
  float* params; long m_pad; long w1_off, b1_off, w2_off, b2_off; int ld1, ld2;
  const float* src; long src_stride;   // starting point of every worker: its replica, or the shared
                                       // node average (stride 0) right after a restart
  int n_workers, P, d0, d1, d2, d2p, ldx, batch; long rows; int log2n;
  int act; float lr; uint64_t seed; uint64_t t0; int k;
  const int* worker_steps;       // Algorithm 3 step counts (nullptr: every worker takes k steps)
  float* part;                   // [2][N][P][MT*16][d2p] partial logits
  unsigned int* sync;            // [N][32] arrival counters (+ launch base), then the abort flag
  unsigned int spin_limit;       // polls of the team barrier before a member gives up
  float* row_loss; int32_t* idx;
  float* vel; float mu;          // momentum buffers [N][m_pad] (nullptr = plain SGD)
};
constexpr unsigned int kFused2SpinLimit = 1u << 22;   // default bound of the team barrier's wait
size_t fused2_lds_bytes(const Fused2Plan& pl);
bool fused2_plan(int n_workers, int d0, int d1, int d2, int batch, bool momentum, Fused2Plan* pl);
hipError_t launch_fused2(const Fused2Plan& pl, Fused2Args args, hipStream_t s);
const char* kernel_kind_name(int kind);

// ---- launchers (each returns the hipError_t of the launch) --------------------------------
hipError_t launch_gemm_fwd(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s);
hipError_t launch_gemm_dx(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s);
hipError_t launch_gemm_dw_stacked(const GemmArgs& p, hipStream_t s);   // bf16 operands, one group
hipError_t launch_gemm_dw(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s);

// Minibatch draw of iteration t: rows of the workers' shards copied into the batch buffer.
struct GatherArgs {
  const float* features; const int32_t* labels;
  void* xb; int32_t* yb; int32_t* idx;        // batch rows [N][B][ld0], labels and row indices [N][B]
  int batch, d0, ld0; long rows; int log2n;
  uint64_t seed, t;
};
GatherArgs gather_args(const float* features, const int32_t* labels, void* xb, int32_t* yb, int32_t* idx,
                       int batch, int d0, int ld0, long rows, uint64_t seed, int64_t t);
hipError_t launch_gather(const GatherArgs& a, int n_workers, bool bf16, const int* worker_steps, int step,
                         hipStream_t s);
hipError_t launch_sample_indices(uint64_t seed, int n_workers, int batch, long rows, int64_t t_first,
                                 int n_steps, int32_t* out, hipStream_t s);
// next != nullptr: the launch also gathers that minibatch (all workers, no step mask)
hipError_t launch_softmax_xent(const float* logits, int n_parts, long part_stride, const float* bias,
                               long bias_gs, const int32_t* yb, void* delta, float* row_loss,
                               int n_workers, int batch, int n_classes, int ldc, bool bf16,
                               const int* worker_steps, int step, const GatherArgs* next, hipStream_t s);
// Narrow head (<= 16 classes, bf16 operands): logits product, softmax and delta in one launch
bool softmax_narrow_applies(int n_classes, int ldc, bool bf16);
hipError_t launch_softmax_xent_narrow(const uint16_t* h, long h_gs, int ldh, int k_dim, const uint16_t* w_sh,
                                      long w_gs, const float* bias, long bias_gs, const int32_t* yb,
                                      uint16_t* delta, float* row_loss, int n_workers, int batch, int n_classes,
                                      int ldc, const int* worker_steps, int step, const GatherArgs* next,
                                      hipStream_t s);
hipError_t launch_loss_mean(const float* row_loss, float* losses, int n_workers, int batch,
                            hipStream_t s);

hipError_t launch_average(float* params, uint16_t* shadow, long m_pad, int n_workers, bool streaming,
                          hipStream_t s);
hipError_t launch_mean(const float* params, float* out, uint16_t* out_shadow, long m_pad, int n_workers,
                       bool streaming, hipStream_t s);
hipError_t launch_broadcast(const float* src, float* params, uint16_t* shadow, long m_pad,
                            int n_workers, hipStream_t s);
hipError_t launch_refresh_shadow(const float* params, uint16_t* shadow, long count, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_update(float* x, const float* g, uint16_t* shadow, size_t count, float lr,
                         hipStream_t s);
hipError_t launch_momentum_update(float* x, float* v, const float* g, uint16_t* shadow, size_t count,
                                  float lr, float mu, hipStream_t s);
hipError_t launch_fill_zero(float* x, size_t count, hipStream_t s);
hipError_t launch_update_masked(float* x, const float* g, uint16_t* shadow, long m_pad, int n_workers,
                                float lr, const int* worker_steps, int step, hipStream_t s);

hipError_t launch_lsq_steps(const float* features, const float* targets, const float* src,
                            long src_stride, float* params, float* velocity, float mu, float* losses,
                            int32_t* idx, int n_workers, int d, long m_pad, long rows, int batch,
                            float lr, uint64_t seed, int64_t t0, int k, const int* worker_steps,
                            hipStream_t s);

// ---- small device helpers ------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  // a NaN stays a NaN (quiet bit set): adding the rounding bias would carry some NaN patterns
  // into the exponent and turn them into infinity or zero
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);          // round to nearest, ties to even
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}

// ---- bf16 MFMA operand fragments out of LDS ----------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// Fragment of lane (r = lane % 32, kb = lane / 32) for the kk-th 16-deep contraction slice of a
// tile stored [row][c] (contraction index contiguous): one 16-byte read.
__device__ __forceinline__ bf16x8_t frag_contig(const uint16_t* lds, int stride, int row_block, int kk,
                                                int lane) {
  const u16x8_t u = *reinterpret_cast<const u16x8_t*>(lds + (row_block + (lane & 31)) * stride + kk * 16 +
                                                      (lane >> 5) * 8);
  return __builtin_bit_cast(bf16x8_t, u);
}
// The same fragment of a tile stored [c][row] (contraction index is the LDS row), read with the
// LDS transpose load (ds_read_b64_tr_b16): inside each group of 16 lanes, lane r supplies the
// address of a 4-element row M[r] and lane i receives M[4j + i/4][i%4], j = 0..3.  Addressing
// lane r at (c = c0 + r/4, rows 4*(r%4)..+3) therefore hands lane i the four consecutive c of
// row i: a 4(c) x 16(row) block transposed in flight.  Two such loads give the eight contraction
// elements of the fragment.
__device__ __forceinline__ bf16x8_t frag_trans(const uint16_t* lds, int stride, int row_block, int kk,
                                               int lane) {
  typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
  typedef __attribute__((address_space(3))) bf16x4_t* lds_bf16x4_ptr;
  const int g = lane >> 4, r = lane & 15;
  const int c = kk * 16 + 8 * (g >> 1) + (r >> 2);
  const int row = row_block + 16 * (g & 1) + 4 * (r & 3);
  const uint16_t* p = lds + c * stride + row;
  const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p));
  const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + 4 * stride));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies
// with the key advanced by the Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Row drawn by worker `worker` at iteration t for minibatch slot j (top log2(n) bits).
__device__ __forceinline__ int32_t sample_row(uint64_t seed, uint32_t worker, uint64_t t, uint32_t j,
                                              int log2n) {
  uint32_t w[4];
  philox4x32_10(j >> 2, (uint32_t)t, (uint32_t)(t >> 32), worker, (uint32_t)seed,
                (uint32_t)(seed >> 32), w);
  const uint32_t sel = j & 3u;
  const uint32_t word = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
  return log2n == 0 ? 0 : (int32_t)(word >> (32 - log2n));
}

}  // namespace prsgd
