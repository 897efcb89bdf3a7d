// Least-squares workers: k consecutive local iterations of
//   x_i <- x_i - gamma * (1/B) A_b^T (A_b x_i - y_b)             (Algorithm 1, eq. 3)
// in ONE launch.  Workers never exchange anything inside an epoch (paragraph below
// Algorithm 1), so one workgroup per worker keeps x_i in LDS for the whole call and only the
// sampled rows travel from HBM.
#include <type_traits>

#include "prsgd_internal.h"

namespace prsgd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMaxStagedFloats = 8192;   // minibatch floats the staged kernel keeps in LDS
constexpr int kMaxStagedBatch = 512;     // its targets travel in two registers per thread and stage

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

// Sum over the 64 lanes of a wavefront, returned in every lane: butterflies inside each row of
// 16 lanes on the data-parallel-primitive path (no LDS round trips), then the four row sums.
__device__ inline float wave_sum(float v) {
  auto dpp = [](float f, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(f), decltype(ctrl)::value, 0xF, 0xF, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>());    // quad_perm [1,0,3,2]
  v += dpp(v, std::integral_constant<int, 0x4E>());    // quad_perm [2,3,0,1]
  v += dpp(v, std::integral_constant<int, 0x141>());   // row_half_mirror
  v += dpp(v, std::integral_constant<int, 0x140>());   // row_mirror
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

// Staged variant for minibatches of at most kMaxStagedFloats floats (d a multiple of 4): the
// sampled rows pass through LDS (two buffers, so an iteration costs two workgroup barriers),
// and because the index stream is a pure function of (seed, worker, t, slot) the rows of
// iteration s + D are requested D iterations early and wait in registers: no iteration stalls
// on HBM latency.  The rows themselves are drawn D iterations at a time, two blocks ahead.
// PFV = 16-byte vectors per thread and minibatch, D = prefetch depth in iterations.
template <int PFV, int D>
__global__ __launch_bounds__(kThreads) void lsq_steps_staged_kernel(
    const float* __restrict__ features, const float* __restrict__ targets, const float* src,
    long src_stride, float* params, float* velocity, float mu, float* __restrict__ losses,
    int32_t* __restrict__ idx, int d, long m_pad, long rows, int log2n, int batch, float lr,
    uint64_t seed, uint64_t t0, int k, const int* __restrict__ worker_steps) {
  constexpr int YV = (kMaxStagedBatch + kThreads - 1) / kThreads;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int bd = batch * d;
  float* A = lds;                                   // [2][batch][d] rows of the current / next iteration
  float* x = A + 2 * (size_t)bd;                    // [d]
  float* vel = x + d;                               // [d]
  float* res = vel + d;                             // [batch]
  float* ys = res + batch;                          // [2][batch] targets
  int32_t* row = reinterpret_cast<int32_t*>(ys + 2 * batch);   // [3][D][batch]: block b of D iterations at slot b % 3

  const int i = blockIdx.x;
  const int my_k = worker_steps != nullptr ? min(worker_steps[i], k) : k;
  if (my_k <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* feat_i = features + (size_t)i * rows * d;
  const float* targ_i = targets + (size_t)i * rows;
  float* x_glob = params + (size_t)i * m_pad;
  const float inv_b = 1.0f / (float)batch;
  const int d4 = d >> 2, nvec = batch * d4;

  const float* x_start = src + (size_t)i * src_stride;
  float* v_glob = velocity != nullptr ? velocity + (size_t)i * m_pad : nullptr;
  for (int c = tid; c < d; c += kThreads) {
    x[c] = x_start[c];
    vel[c] = v_glob != nullptr ? v_glob[c] : 0.0f;
  }
  // rows of block b: iterations b*D + 1 ... b*D + D of this call
  auto draw_block = [&](int b) {
    int32_t* r = row + (size_t)(b % 3) * D * batch;
    for (int e = tid; e < D * batch; e += kThreads) {
      const int u = e / batch, j = e - u * batch;
      r[e] = sample_row(seed, (uint32_t)i, t0 + (uint64_t)(b * D + 1 + u), (uint32_t)j, log2n);
    }
  };
  f32x4_t pre[D][PFV];
  float ypre[D][YV];
  auto issue = [&](int b, int u) {                  // request the minibatch of iteration b*D + 1 + u
    const int32_t* r = row + ((size_t)(b % 3) * D + u) * batch;
#pragma unroll
    for (int v = 0; v < PFV; ++v) {
      const int e = tid + kThreads * v;
      const int ec = e < nvec ? e : 0;
      const int j = ec / d4, c4 = ec - j * d4;
      pre[u][v] = *reinterpret_cast<const f32x4_t*>(feat_i + (size_t)r[j] * d + 4 * c4);
    }
#pragma unroll
    for (int v = 0; v < YV; ++v) {
      const int j = tid + kThreads * v;
      ypre[u][v] = targ_i[r[j < batch ? j : 0]];
    }
  };
  auto land = [&](int u, float* Ab, float* yb) {    // registers -> LDS
#pragma unroll
    for (int v = 0; v < PFV; ++v) {
      const int e = tid + kThreads * v;
      if (e < nvec) *reinterpret_cast<f32x4_t*>(Ab + 4 * (size_t)e) = pre[u][v];
    }
#pragma unroll
    for (int v = 0; v < YV; ++v) {
      const int j = tid + kThreads * v;
      if (j < batch) yb[j] = ypre[u][v];
    }
  };

  draw_block(0);
  draw_block(1);
  __syncthreads();
#pragma unroll
  for (int u = 0; u < D; ++u)
    if (1 + u <= my_k) issue(0, u);
  constexpr int RW = 4;                             // rows in flight per wavefront

  for (int b = 0; b * D < my_k; ++b) {
    draw_block(b + 2);                              // read from the next block on: barriers in between
#pragma unroll
    for (int u = 0; u < D; ++u) {
      const int s = b * D + 1 + u;
      if (s <= my_k) {                              // uniform over the workgroup
        float* Ab = A + (size_t)(s & 1) * bd;
        float* yb = ys + (size_t)(s & 1) * batch;
        land(u, Ab, yb);
        if (s + D <= my_k) issue(b + 1, u);         // nothing is requested past the last iteration
        __syncthreads();
        // residuals: RW rows per wavefront at a time, lanes stride over the features
        for (int j0 = wave * RW; j0 < batch; j0 += (kThreads / kWave) * RW) {
          float dot[RW];
#pragma unroll
          for (int q = 0; q < RW; ++q) dot[q] = 0.0f;
          for (int c = lane; c < d; c += kWave) {
            const float xc = x[c];
#pragma unroll
            for (int q = 0; q < RW; ++q)
              dot[q] = fmaf(Ab[(size_t)min(j0 + q, batch - 1) * d + c], xc, dot[q]);
          }
#pragma unroll
          for (int q = 0; q < RW; ++q) {
            const float t = wave_sum(dot[q]);
            if (lane == q && j0 + q < batch) res[j0 + q] = t - yb[j0 + q];
          }
        }
        __syncthreads();
        // gradient column c and update; rows summed in slot order
        for (int c = tid; c < d; c += kThreads) {
          float gc = 0.0f;
#pragma unroll 8
          for (int j = 0; j < batch; ++j) gc = fmaf(Ab[(size_t)j * d + c], res[j], gc);
          if (v_glob != nullptr) {
            const float vc = fmaf(mu, vel[c], gc * inv_b);
            vel[c] = vc;
            x[c] = fmaf(-lr, vc, x[c]);
          } else {
            x[c] = fmaf(-lr, gc * inv_b, x[c]);
          }
        }
        if (s == my_k && tid == kThreads - 1) {     // a lane of the last wavefront: idle when d is small
          float sq = 0.0f;
          for (int j = 0; j < batch; ++j) sq = fmaf(res[j], res[j], sq);
          losses[i] = 0.5f * sq * inv_b;
        }
      }
    }
  }
  __syncthreads();
  for (int c = tid; c < d; c += kThreads) {
    x_glob[c] = x[c];
    if (v_glob != nullptr) v_glob[c] = vel[c];
  }
  for (int j = tid; j < batch; j += kThreads)
    idx[(size_t)i * batch + j] = sample_row(seed, (uint32_t)i, t0 + (uint64_t)my_k, (uint32_t)j, log2n);
}

hipError_t launch_lsq_steps(const float* features, const float* targets, const float* src,
                            long src_stride, float* params, float* velocity, float mu, float* losses,
                            int32_t* idx, int n_workers, int d, long m_pad, long rows, int batch,
                            float lr, uint64_t seed, int64_t t0, int k, const int* worker_steps,
                            hipStream_t s) {
  if (k <= 0) return hipSuccess;
  const long floats = (long)batch * d;
  if ((d & 3) == 0 && floats <= kMaxStagedFloats && batch <= kMaxStagedBatch) {
    const int pfv = (int)((floats / 4 + kThreads - 1) / kThreads);
#define STAGED(PFV, D)                                                                                  \
  do {                                                                                                  \
    const size_t lds_b = (2 * (size_t)floats + 2 * (size_t)d + 3 * (size_t)batch + 3 * (size_t)D * batch) * \
                         sizeof(float);                                                                 \
    if (lds_b > 48 * 1024) {                                                                            \
      const hipError_t ea = hipFuncSetAttribute(                                                        \
          reinterpret_cast<const void*>(lsq_steps_staged_kernel<PFV, D>),                               \
          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_b);                                      \
      if (ea != hipSuccess) return ea;                                                                  \
    }                                                                                                   \
    hipLaunchKernelGGL((lsq_steps_staged_kernel<PFV, D>), dim3(n_workers), dim3(kThreads), lds_b, s,    \
                       features, targets, src, src_stride, params, velocity, mu, losses, idx, d, m_pad, \
                       rows, ilog2_rows(rows), batch, lr, seed, (uint64_t)t0, k, worker_steps);         \
    return hipGetLastError();                                                                           \
  } while (0)
    if (pfv <= 1) STAGED(1, 8);
    if (pfv <= 2) STAGED(2, 4);
    if (pfv <= 4) STAGED(4, 2);
    STAGED(8, 1);
#undef STAGED
  }
  // at most (2 * 8192 + 2 * 4096) floats = 96 KiB: inside the 160 KiB of a compute unit, but
  // above the default limit of a launch
  const size_t lds_bytes = (2 * (size_t)d + 2 * (size_t)batch) * sizeof(float);
  if (lds_bytes > 48 * 1024) {
    const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(lsq_steps_kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (ea != hipSuccess) return ea;
  }
  hipLaunchKernelGGL(lsq_steps_kernel, dim3(n_workers), dim3(kThreads), lds_bytes, s, features, targets,
                     src, src_stride, params, velocity, mu, losses, idx, d, m_pad, rows, ilog2_rows(rows), batch, lr, seed,
                     (uint64_t)t0, k, worker_steps);
  return hipGetLastError();
}

}  // namespace prsgd
