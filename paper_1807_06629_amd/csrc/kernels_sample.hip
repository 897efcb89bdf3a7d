// Minibatch draw zeta_i^t and the loss head of the MLP.
//
// Section 1 of the paper only requires unbiased stochastic gradients that are independent
// across workers and iterations.  Here worker i draws B rows of its own shard uniformly with
// replacement; slot j of iteration t is a pure function of (seed, i, t, j) through
// Philox4x32-10, so the stream needs no state and can be replayed from any t.
#include <cstring>

#include "prsgd_internal.h"

namespace prsgd {

static int ilog2(long n) {
  int l = 0;
  while ((1L << l) < n) ++l;
  return l;
}

// One workgroup per (slot j, worker i): draw the row, copy it into the batch buffer.
template <bool BF16>
__device__ __forceinline__ void gather_row(const GatherArgs& a, int j, int i) {
  const int32_t row = sample_row(a.seed, (uint32_t)i, a.t, (uint32_t)j, a.log2n);
  const size_t slot = (size_t)i * a.batch + j;
  if (threadIdx.x == 0) {
    a.idx[slot] = row;
    a.yb[slot] = a.labels[(size_t)i * a.rows + row];
  }
  const int d0 = a.d0, ld0 = a.ld0;
  const float* src = a.features + ((size_t)i * a.rows + row) * d0;
  if ((d0 & 3) == 0) {
    const float4* src4 = reinterpret_cast<const float4*>(src);
    for (int c = threadIdx.x; c < d0 / 4; c += kThreads) {
      const float4 v = src4[c];
      if (BF16) {
        uint2 h;
        h.x = (uint32_t)f32_to_bf16_rne(v.x) | ((uint32_t)f32_to_bf16_rne(v.y) << 16);
        h.y = (uint32_t)f32_to_bf16_rne(v.z) | ((uint32_t)f32_to_bf16_rne(v.w) << 16);
        reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.xb) + slot * ld0)[c] = h;
      } else {
        reinterpret_cast<float4*>(reinterpret_cast<float*>(a.xb) + slot * ld0)[c] = v;
      }
    }
  } else {
    for (int c = threadIdx.x; c < d0; c += kThreads) {
      if (BF16) reinterpret_cast<uint16_t*>(a.xb)[slot * ld0 + c] = f32_to_bf16_rne(src[c]);
      else reinterpret_cast<float*>(a.xb)[slot * ld0 + c] = src[c];
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void gather_kernel(GatherArgs a, const int* __restrict__ worker_steps,
                                                          int step) {
  const int j = blockIdx.x, i = blockIdx.y;
  if (worker_steps != nullptr && step >= worker_steps[i]) return;
  gather_row<BF16>(a, j, i);
}

__global__ __launch_bounds__(kThreads) void sample_indices_kernel(int32_t* __restrict__ out,
                                                                  int n_workers, int batch, int log2n,
                                                                  uint64_t seed, uint64_t t_first,
                                                                  size_t total) {
  for (size_t k = (size_t)blockIdx.x * kThreads + threadIdx.x; k < total;
       k += (size_t)gridDim.x * kThreads) {
    const uint32_t j = (uint32_t)(k % batch);
    const uint32_t i = (uint32_t)((k / batch) % n_workers);
    const uint64_t s = k / ((size_t)batch * n_workers);
    out[k] = sample_row(seed, i, t_first + s, j, log2n);
  }
}

// Softmax cross-entropy head: one wavefront per minibatch row (4 rows per workgroup).  The same
// launch can carry the row gather of the next iteration in extra workgroups.
//   row_loss[b] = -log softmax(z_b)[c_b],   delta = (softmax(z) - onehot(c)) / B
template <bool BF16>
__global__ __launch_bounds__(kThreads) void softmax_xent_kernel(
    const float* __restrict__ logits, int n_parts, long part_stride, const float* __restrict__ bias,
    long bias_gs, const int32_t* __restrict__ yb, void* __restrict__ delta,
    float* __restrict__ row_loss, int batch, int n_classes, int ldc,
    const int* __restrict__ worker_steps, int step, int head_blocks, GatherArgs next) {
  const int g = blockIdx.y;
  // workgroups beyond the loss head's own: the minibatch draw of the NEXT iteration, which depends
  // on nothing this iteration computes (zeta_i^t is a function of seed, i, t and the slot alone)
  if ((int)blockIdx.x >= head_blocks) {
    gather_row<BF16>(next, (int)blockIdx.x - head_blocks, g);
    return;
  }
  if (worker_steps != nullptr && step >= worker_steps[g]) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.x * (kThreads / kWave) + wave;
  if (b >= batch) return;
  const float inv_b = 1.0f / (float)batch;
  const size_t r = (size_t)g * batch + b;
  // logit of class c: the product's output, or (split contraction) the bias plus the partial
  // sums in split order
  const float* bias_g = bias != nullptr ? bias + (size_t)g * bias_gs : nullptr;
  auto logit = [&](int c) {
    float z = bias_g != nullptr ? bias_g[c] : 0.0f;
    for (int s = 0; s < n_parts; ++s) z += logits[(size_t)s * part_stride + r * ldc + c];
    return z;
  };
  const int label = yb[r];
  constexpr int ZR = 16;                             // classes per lane held in registers
  if (n_classes <= ZR * kWave) {
    float z[ZR];
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < ZR; ++q) {
      const int c = lane + kWave * q;
      z[q] = (kWave * q < n_classes && c < n_classes) ? logit(c) : -INFINITY;
      mx = fmaxf(mx, z[q]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float zl = 0.0f, se = 0.0f;                      // the label's logit lives in one lane
#pragma unroll
    for (int q = 0; q < ZR; ++q) {
      const int c = lane + kWave * q;
      if (c == label && c < n_classes) zl = z[q];
      z[q] = (kWave * q < n_classes && c < n_classes) ? expf(z[q] - mx) : 0.0f;
      se += z[q];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      se += __shfl_xor(se, o);
      zl += __shfl_xor(zl, o);
    }
#pragma unroll
    for (int q = 0; q < ZR; ++q) {
      const int c = lane + kWave * q;
      if (kWave * q < ldc && c < ldc) {
        const float d = c < n_classes ? (z[q] / se - (c == label ? 1.0f : 0.0f)) * inv_b : 0.0f;
        if (BF16) reinterpret_cast<uint16_t*>(delta)[r * ldc + c] = f32_to_bf16_rne(d);
        else reinterpret_cast<float*>(delta)[r * ldc + c] = d;
      }
    }
    // an out-of-range label selects nothing (zl stays 0)
    if (lane == 0) row_loss[r] = (mx + logf(se)) - zl;
    return;
  }
  float mx = -INFINITY;
  for (int c = lane; c < n_classes; c += kWave) mx = fmaxf(mx, logit(c));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  float se = 0.0f;
  for (int c = lane; c < n_classes; c += kWave) se += expf(logit(c) - mx);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o);
  for (int c = lane; c < ldc; c += kWave) {
    float d = 0.0f;
    if (c < n_classes) d = (expf(logit(c) - mx) / se - (c == label ? 1.0f : 0.0f)) * inv_b;
    if (BF16) reinterpret_cast<uint16_t*>(delta)[r * ldc + c] = f32_to_bf16_rne(d);
    else reinterpret_cast<float*>(delta)[r * ldc + c] = d;
  }
  // an out-of-range label must not index outside the row
  const float z_label = (label >= 0 && label < n_classes) ? logit(label) : 0.0f;
  if (lane == 0) row_loss[r] = (mx + logf(se)) - z_label;
}

// The same head for wide class counts (257 .. 1024): one workgroup per minibatch row, at most four
// classes per thread, so that a row's loads are spread over four wavefronts instead of queueing in
// one (1000 classes, four partial sums per logit: 20 loads per lane instead of 80).
template <bool BF16>
__global__ __launch_bounds__(kThreads) void softmax_xent_row_kernel(
    const float* __restrict__ logits, int n_parts, long part_stride, const float* __restrict__ bias,
    long bias_gs, const int32_t* __restrict__ yb, void* __restrict__ delta,
    float* __restrict__ row_loss, int batch, int n_classes, int ldc,
    const int* __restrict__ worker_steps, int step, int head_blocks, GatherArgs next) {
  const int g = blockIdx.y;
  if ((int)blockIdx.x >= head_blocks) {                 // the minibatch draw of the next iteration
    gather_row<BF16>(next, (int)blockIdx.x - head_blocks, g);
    return;
  }
  if (worker_steps != nullptr && step >= worker_steps[g]) return;
  __shared__ float red[3][kThreads / kWave];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t r = (size_t)g * batch + blockIdx.x;
  const float inv_b = 1.0f / (float)batch;
  const float* bias_g = bias != nullptr ? bias + (size_t)g * bias_gs : nullptr;
  const int label = yb[r];
  constexpr int ZT = 4;                                 // classes per thread
  float z[ZT];
  float mx = -INFINITY;
#pragma unroll
  for (int q = 0; q < ZT; ++q) {
    const int c = tid + kThreads * q;
    float v = -INFINITY;
    if (c < n_classes) {                                // bias plus the partial sums in split order
      v = bias_g != nullptr ? bias_g[c] : 0.0f;
      for (int s = 0; s < n_parts; ++s) v += logits[(size_t)s * part_stride + r * ldc + c];
    }
    z[q] = v;
    mx = fmaxf(mx, v);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (lane == 0) red[0][wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
  float se = 0.0f, zl = 0.0f;                           // the label's logit lives in one thread
#pragma unroll
  for (int q = 0; q < ZT; ++q) {
    const int c = tid + kThreads * q;
    if (c == label && c < n_classes) zl = z[q];
    z[q] = c < n_classes ? expf(z[q] - mx) : 0.0f;
    se += z[q];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    se += __shfl_xor(se, o);
    zl += __shfl_xor(zl, o);
  }
  if (lane == 0) { red[1][wave] = se; red[2][wave] = zl; }
  __syncthreads();
  se = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];     // fixed order
  zl = ((red[2][0] + red[2][1]) + red[2][2]) + red[2][3];
#pragma unroll
  for (int q = 0; q < ZT; ++q) {
    const int c = tid + kThreads * q;
    if (c < ldc) {
      const float d = c < n_classes ? (z[q] / se - (c == label ? 1.0f : 0.0f)) * inv_b : 0.0f;
      if (BF16) reinterpret_cast<uint16_t*>(delta)[r * ldc + c] = f32_to_bf16_rne(d);
      else reinterpret_cast<float*>(delta)[r * ldc + c] = d;
    }
  }
  if (tid == 0) row_loss[r] = (mx + logf(se)) - zl;     // an out-of-range label selects nothing
}

// Narrow head (at most 16 classes, bf16 operands): the logits product is taken here as well,
//   z_b = H_{L-1}[b, :] bf16(W_L) + b_L,
// one wavefront per minibatch row with the contraction spread over its lanes -- a product of a few
// thousand multiply-adds per row does not pay for a launch of its own (and its split contraction).
__global__ __launch_bounds__(kThreads) void softmax_xent_narrow_kernel(
    const uint16_t* __restrict__ h, long h_gs, int ldh, int k_dim, const uint16_t* __restrict__ w_sh,
    long w_gs, const float* __restrict__ bias, long bias_gs, const int32_t* __restrict__ yb,
    uint16_t* __restrict__ delta, float* __restrict__ row_loss, int batch, int n_classes, int ldc,
    const int* __restrict__ worker_steps, int step, int head_blocks, GatherArgs next) {
  const int g = blockIdx.y;
  if ((int)blockIdx.x >= head_blocks) {                 // the minibatch draw of the next iteration
    gather_row<true>(next, (int)blockIdx.x - head_blocks, g);
    return;
  }
  if (worker_steps != nullptr && step >= worker_steps[g]) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.x * (kThreads / kWave) + wave;
  if (b >= batch) return;
  const size_t r = (size_t)g * batch + b;
  const uint16_t* h_r = h + (size_t)g * h_gs + (size_t)b * ldh;
  const uint16_t* w_g = w_sh + (size_t)g * w_gs;        // [k_dim][ldc], ldc = 8 or 16
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  float acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = 0.0f;
#pragma unroll 8
  for (int k = lane; k < k_dim; k += kWave) {
    const float hv = bf16_to_f32(h_r[k]);
    const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(w_g + (size_t)k * ldc);
    u32x4_t hi = {0u, 0u, 0u, 0u};
    if (ldc > 8) hi = *reinterpret_cast<const u32x4_t*>(w_g + (size_t)k * ldc + 8);   // uniform
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] = fmaf(hv, __uint_as_float(lo[j] << 16), acc[2 * j]);
      acc[2 * j + 1] = fmaf(hv, __uint_as_float(lo[j] & 0xFFFF0000u), acc[2 * j + 1]);
      acc[8 + 2 * j] = fmaf(hv, __uint_as_float(hi[j] << 16), acc[8 + 2 * j]);
      acc[8 + 2 * j + 1] = fmaf(hv, __uint_as_float(hi[j] & 0xFFFF0000u), acc[8 + 2 * j + 1]);
    }
  }
#pragma unroll
  for (int c = 0; c < 16; ++c)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc[c] += __shfl_xor(acc[c], o);
  // lane c keeps class c
  float z = -INFINITY;
#pragma unroll
  for (int c = 0; c < 16; ++c)
    if (lane == c && c < n_classes) z = acc[c] + bias[(size_t)g * bias_gs + c];
  float mx = z;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  const int label = yb[r];
  const float e = lane < n_classes ? expf(z - mx) : 0.0f;
  float se = e, zl = (lane == label && lane < n_classes) ? z : 0.0f;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    se += __shfl_xor(se, o);
    zl += __shfl_xor(zl, o);
  }
  if (lane < ldc) {
    const float d = lane < n_classes ? (e / se - (lane == label ? 1.0f : 0.0f)) * (1.0f / (float)batch) : 0.0f;
    delta[r * ldc + lane] = f32_to_bf16_rne(d);
  }
  if (lane == 0) row_loss[r] = (mx + logf(se)) - zl;    // an out-of-range label selects nothing
}

// Minibatch loss of each worker: mean of its row losses, rows summed in slot order.
__global__ void loss_mean_kernel(const float* __restrict__ row_loss, float* __restrict__ losses,
                                 int n_workers, int batch) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_workers) return;
  float s = 0.0f;
  for (int b = 0; b < batch; ++b) s += row_loss[(size_t)g * batch + b];
  losses[g] = s / (float)batch;
}

hipError_t launch_gather(const GatherArgs& a, int n_workers, bool bf16, const int* worker_steps, int step,
                         hipStream_t s) {
  dim3 grid(a.batch, n_workers);
  if (bf16) hipLaunchKernelGGL(gather_kernel<true>, grid, dim3(kThreads), 0, s, a, worker_steps, step);
  else hipLaunchKernelGGL(gather_kernel<false>, grid, dim3(kThreads), 0, s, a, worker_steps, step);
  return hipGetLastError();
}

GatherArgs gather_args(const float* features, const int32_t* labels, void* xb, int32_t* yb, int32_t* idx,
                       int batch, int d0, int ld0, long rows, uint64_t seed, int64_t t) {
  GatherArgs a;
  a.features = features; a.labels = labels; a.xb = xb; a.yb = yb; a.idx = idx;
  a.batch = batch; a.d0 = d0; a.ld0 = ld0; a.rows = rows; a.log2n = ilog2(rows);
  a.seed = seed; a.t = (uint64_t)t;
  return a;
}

hipError_t launch_sample_indices(uint64_t seed, int n_workers, int batch, long rows, int64_t t_first,
                                 int n_steps, int32_t* out, hipStream_t s) {
  const size_t total = (size_t)n_steps * n_workers * batch;
  if (total == 0) return hipSuccess;
  size_t blocks = (total + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(sample_indices_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, out,
                     n_workers, batch, ilog2(rows), seed, (uint64_t)t_first, total);
  return hipGetLastError();
}

hipError_t launch_softmax_xent(const float* logits, int n_parts, long part_stride, const float* bias,
                               long bias_gs, const int32_t* yb, void* delta, float* row_loss,
                               int n_workers, int batch, int n_classes, int ldc, bool bf16,
                               const int* worker_steps, int step, const GatherArgs* next, hipStream_t s) {
  GatherArgs ga;
  memset(&ga, 0, sizeof(ga));
  if (next != nullptr) ga = *next;
  if (n_classes > 256 && n_classes <= 4 * kThreads && ldc <= 4 * kThreads) {   // one workgroup per row
    dim3 grid(batch + (next != nullptr ? next->batch : 0), n_workers);
    if (bf16)
      hipLaunchKernelGGL(softmax_xent_row_kernel<true>, grid, dim3(kThreads), 0, s, logits, n_parts, part_stride,
                         bias, bias_gs, yb, delta, row_loss, batch, n_classes, ldc, worker_steps, step, batch, ga);
    else
      hipLaunchKernelGGL(softmax_xent_row_kernel<false>, grid, dim3(kThreads), 0, s, logits, n_parts, part_stride,
                         bias, bias_gs, yb, delta, row_loss, batch, n_classes, ldc, worker_steps, step, batch, ga);
    return hipGetLastError();
  }
  const int head_blocks = (batch + kThreads / kWave - 1) / (kThreads / kWave);
  dim3 grid(head_blocks + (next != nullptr ? next->batch : 0), n_workers);
  if (bf16)
    hipLaunchKernelGGL(softmax_xent_kernel<true>, grid, dim3(kThreads), 0, s, logits, n_parts, part_stride,
                       bias, bias_gs, yb, delta, row_loss, batch, n_classes, ldc, worker_steps, step,
                       head_blocks, ga);
  else
    hipLaunchKernelGGL(softmax_xent_kernel<false>, grid, dim3(kThreads), 0, s, logits, n_parts, part_stride,
                       bias, bias_gs, yb, delta, row_loss, batch, n_classes, ldc, worker_steps, step,
                       head_blocks, ga);
  return hipGetLastError();
}

bool softmax_narrow_applies(int n_classes, int ldc, bool bf16) {
  return bf16 && n_classes >= 1 && n_classes <= 16 && (ldc == 8 || ldc == 16);
}

hipError_t launch_softmax_xent_narrow(const uint16_t* h, long h_gs, int ldh, int k_dim, const uint16_t* w_sh,
                                      long w_gs, const float* bias, long bias_gs, const int32_t* yb,
                                      uint16_t* delta, float* row_loss, int n_workers, int batch, int n_classes,
                                      int ldc, const int* worker_steps, int step, const GatherArgs* next,
                                      hipStream_t s) {
  if (!softmax_narrow_applies(n_classes, ldc, true) || (ldh % 2) != 0) return hipErrorInvalidValue;
  const int head_blocks = (batch + kThreads / kWave - 1) / (kThreads / kWave);
  GatherArgs ga;
  memset(&ga, 0, sizeof(ga));
  if (next != nullptr) ga = *next;
  dim3 grid(head_blocks + (next != nullptr ? next->batch : 0), n_workers);
  hipLaunchKernelGGL(softmax_xent_narrow_kernel, grid, dim3(kThreads), 0, s, h, h_gs, ldh, k_dim, w_sh, w_gs, bias,
                     bias_gs, yb, delta, row_loss, batch, n_classes, ldc, worker_steps, step, head_blocks, ga);
  return hipGetLastError();
}

hipError_t launch_loss_mean(const float* row_loss, float* losses, int n_workers, int batch,
                            hipStream_t s) {
  hipLaunchKernelGGL(loss_mean_kernel, dim3((n_workers + 63) / 64), dim3(64), 0, s, row_loss, losses,
                     n_workers, batch);
  return hipGetLastError();
}

}  // namespace prsgd
