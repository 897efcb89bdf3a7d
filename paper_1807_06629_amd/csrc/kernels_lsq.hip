// Least-squares workers: k consecutive local iterations of
//   x_i <- x_i - gamma * (1/B) A_b^T (A_b x_i - y_b)             (Algorithm 1, eq. 3)
// in ONE launch.  Workers never exchange anything inside an epoch (paragraph below
// Algorithm 1), so one workgroup per worker keeps x_i in LDS for the whole call and only the
// sampled rows travel from HBM.
#include "prsgd_internal.h"

namespace prsgd {

static int ilog2_rows(long n) {
  int l = 0;
  while ((1L << l) < n) ++l;
  return l;
}

__global__ __launch_bounds__(kThreads) void lsq_steps_kernel(
    const float* __restrict__ features, const float* __restrict__ targets, const float* src,
    long src_stride, float* params, float* velocity, float mu, float* __restrict__ losses, int32_t* __restrict__ idx, int d, long m_pad, long rows, int log2n,
    int batch, float lr, uint64_t seed, uint64_t t0, int k, const int* __restrict__ worker_steps) {
  extern __shared__ float lds[];
  float* x = lds;                                   // [d]
  float* vel = lds + d;                             // [d] momentum buffer (unused when mu == 0)
  float* res = vel + d;                             // [batch] residuals a_j . x - y_j
  int32_t* row = reinterpret_cast<int32_t*>(res + batch);   // [batch]

  const int i = blockIdx.x;
  const int my_k = worker_steps != nullptr ? min(worker_steps[i], k) : k;
  if (my_k <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* feat_i = features + (size_t)i * rows * d;
  const float* targ_i = targets + (size_t)i * rows;
  float* x_glob = params + (size_t)i * m_pad;
  const float inv_b = 1.0f / (float)batch;

  const float* x_start = src + (size_t)i * src_stride;     // the replica, or the shared node average
  float* v_glob = velocity != nullptr ? velocity + (size_t)i * m_pad : nullptr;
  for (int c = tid; c < d; c += kThreads) {
    x[c] = x_start[c];
    vel[c] = v_glob != nullptr ? v_glob[c] : 0.0f;
  }
  float loss = 0.0f;

  for (int s = 1; s <= my_k; ++s) {
    const uint64_t t = t0 + (uint64_t)s;
    for (int j = tid; j < batch; j += kThreads) row[j] = sample_row(seed, (uint32_t)i, t, (uint32_t)j, log2n);
    __syncthreads();
    // residuals: one wavefront per sampled row, lanes stride over the features
    for (int j = wave; j < batch; j += kThreads / kWave) {
      const float* a = feat_i + (size_t)row[j] * d;
      float dot = 0.0f;
      for (int c = lane; c < d; c += kWave) dot = fmaf(a[c], x[c], dot);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
      if (lane == 0) res[j] = dot - targ_i[row[j]];
    }
    __syncthreads();
    // gradient column c and update; rows summed in slot order
    for (int c = tid; c < d; c += kThreads) {
      float gc = 0.0f;
      for (int j = 0; j < batch; ++j) gc = fmaf(feat_i[(size_t)row[j] * d + c], res[j], gc);
      if (v_glob != nullptr) {                      // v <- mu v + G,  x <- x - gamma v
        const float vc = fmaf(mu, vel[c], gc * inv_b);
        vel[c] = vc;
        x[c] = fmaf(-lr, vc, x[c]);
      } else {
        x[c] = fmaf(-lr, gc * inv_b, x[c]);
      }
    }
    if (s == my_k && tid == 0) {
      float sq = 0.0f;
      for (int j = 0; j < batch; ++j) sq = fmaf(res[j], res[j], sq);
      loss = 0.5f * sq * inv_b;
    }
    if (s == my_k)
      for (int j = tid; j < batch; j += kThreads) idx[(size_t)i * batch + j] = row[j];
    __syncthreads();
  }
  for (int c = tid; c < d; c += kThreads) {
    x_glob[c] = x[c];
    if (v_glob != nullptr) v_glob[c] = vel[c];
  }
  if (tid == 0) losses[i] = loss;
}

hipError_t launch_lsq_steps(const float* features, const float* targets, const float* src,
                            long src_stride, float* params, float* velocity, float mu, float* losses,
                            int32_t* idx, int n_workers, int d, long m_pad, long rows, int batch,
                            float lr, uint64_t seed, int64_t t0, int k, const int* worker_steps,
                            hipStream_t s) {
  if (k <= 0) return hipSuccess;
  const size_t lds_bytes = (2 * (size_t)d + 2 * (size_t)batch) * sizeof(float);
  hipLaunchKernelGGL(lsq_steps_kernel, dim3(n_workers), dim3(kThreads), lds_bytes, s, features, targets,
                     src, src_stride, params, velocity, mu, losses, idx, d, m_pad, rows, ilog2_rows(rows), batch, lr, seed,
                     (uint64_t)t0, k, worker_steps);
  return hipGetLastError();
}

}  // namespace prsgd
