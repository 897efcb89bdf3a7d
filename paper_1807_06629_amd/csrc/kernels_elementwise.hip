// Bandwidth-bound kernels over the replica-batched parameter buffer [N][m_pad]:
//   restart average   ybar = (1/N) sum_i x_i, then x_i <- ybar for every i   (Algorithm 1, eq. 2)
//   node average      xbar of eq. (4) into a separate vector (read-out, replicas untouched)
//   local update      x <- x - gamma g                                       (Algorithm 1, eq. 3)
// The reduction runs across replicas, not across lanes: a thread owns one 16-byte column of the
// buffer, streams the N replica values through registers in ascending worker order (a fixed,
// run-to-run deterministic summation order) and writes the mean back N times.  Every global
// access is a fully coalesced 16-byte vector, so the kernels need neither LDS nor cross-lane
// traffic and are limited by HBM alone.
#include "prsgd_internal.h"

namespace prsgd {

constexpr int kChunk = 8;   // replica loads kept in flight per thread

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

// Streaming accesses: the replica buffer is far larger than any cache level and every element
// is touched once per pass, so loads and stores carry the non-temporal hint.
template <bool NT> __device__ __forceinline__ f32x4_t ld4(const f32x4_t* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT> __device__ __forceinline__ void st4(f32x4_t* p, f32x4_t v) {
  if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}
template <bool NT> __device__ __forceinline__ void st2(u32x2_t* p, u32x2_t v) {
  if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}

__device__ __forceinline__ uint2 pack_bf16x4(float4 v) {
  uint2 r;
  r.x = (uint32_t)f32_to_bf16_rne(v.x) | ((uint32_t)f32_to_bf16_rne(v.y) << 16);
  r.y = (uint32_t)f32_to_bf16_rne(v.z) | ((uint32_t)f32_to_bf16_rne(v.w) << 16);
  return r;
}
__device__ __forceinline__ u32x2_t pack_bf16x4(f32x4_t v) {
  u32x2_t r;
  r.x = (uint32_t)f32_to_bf16_rne(v.x) | ((uint32_t)f32_to_bf16_rne(v.y) << 16);
  r.y = (uint32_t)f32_to_bf16_rne(v.z) | ((uint32_t)f32_to_bf16_rne(v.w) << 16);
  return r;
}

// Sums of U columns (16-byte indices col[u]) over the replicas, ascending i, kChunk x U loads in
// flight.
template <bool NT, int U>
__device__ __forceinline__ void replica_sums(const f32x4_t* __restrict__ p, size_t stride4,
                                             const size_t (&col)[U], int n, f32x4_t (&s)[U]) {
#pragma unroll
  for (int u = 0; u < U; ++u) s[u] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
  int i = 0;
  for (; i + kChunk <= n; i += kChunk) {
    f32x4_t v[kChunk][U];
#pragma unroll
    for (int c = 0; c < kChunk; ++c)
#pragma unroll
      for (int u = 0; u < U; ++u) v[c][u] = ld4<NT>(p + (size_t)(i + c) * stride4 + col[u]);
#pragma unroll
    for (int c = 0; c < kChunk; ++c)
#pragma unroll
      for (int u = 0; u < U; ++u) s[u] += v[c][u];
  }
  if (i < n) {
    // last, partial chunk without branches between the loads: a replica index past the end
    // re-reads the last replica and contributes nothing
    f32x4_t v[kChunk][U];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      const int r = i + c < n ? i + c : n - 1;
#pragma unroll
      for (int u = 0; u < U; ++u) v[c][u] = ld4<NT>(p + (size_t)r * stride4 + col[u]);
    }
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
#pragma unroll
      for (int u = 0; u < U; ++u) s[u] += (i + c < n) ? v[c][u] : (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
    }
  }
}

// Columns per thread: a workgroup takes contiguous chunks of U x 256 columns.  Two columns keep
// more loads in flight on replica sets that fill the machine; small ones need every workgroup
// they can get and take one.
constexpr size_t kTwoColumnsFrom = (size_t)2 * 256 * 2048;   // columns: >= 2048 workgroups at U = 2

// Columns of this thread in the chunk that starts at `base`; a column beyond the end is replaced
// by column 0 (its loads stay in bounds, its result is dropped).
template <int U>
__device__ __forceinline__ void chunk_columns(size_t base, size_t stride4, size_t (&col)[U], bool (&ok)[U]) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t c = base + (size_t)u * kThreads + threadIdx.x;
    ok[u] = c < stride4;
    col[u] = ok[u] ? c : 0;
  }
}

template <bool SHADOW, bool NT, int U>
__global__ __launch_bounds__(kThreads) void average_kernel(f32x4_t* __restrict__ params,
                                                           u32x2_t* __restrict__ shadow, size_t stride4,
                                                           int n, float n_f) {
  constexpr size_t kPer = (size_t)U * kThreads;
  for (size_t base = (size_t)blockIdx.x * kPer; base < stride4; base += (size_t)gridDim.x * kPer) {
    size_t col[U];
    bool ok[U];
    f32x4_t sum[U];
    chunk_columns<U>(base, stride4, col, ok);
    replica_sums<NT, U>(params, stride4, col, n, sum);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!ok[u]) continue;
      const f32x4_t mean = sum[u] / n_f;
      for (int i = 0; i < n; ++i) st4<NT>(params + (size_t)i * stride4 + col[u], mean);
      if (SHADOW) {
        const u32x2_t h = pack_bf16x4(mean);
        for (int i = 0; i < n; ++i) st2<NT>(shadow + (size_t)i * stride4 + col[u], h);
      }
    }
  }
}

// Node average into a separate vector (and its bf16 image): the replicas are only read.
template <bool SHADOW, bool NT, int U>
__global__ __launch_bounds__(kThreads) void mean_kernel(const f32x4_t* __restrict__ params,
                                                        f32x4_t* __restrict__ out,
                                                        u32x2_t* __restrict__ out_shadow, size_t stride4,
                                                        int n, float n_f) {
  constexpr size_t kPer = (size_t)U * kThreads;
  for (size_t base = (size_t)blockIdx.x * kPer; base < stride4; base += (size_t)gridDim.x * kPer) {
    size_t col[U];
    bool ok[U];
    f32x4_t sum[U];
    chunk_columns<U>(base, stride4, col, ok);
    replica_sums<NT, U>(params, stride4, col, n, sum);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!ok[u]) continue;
      const f32x4_t mean = sum[u] / n_f;
      out[col[u]] = mean;
      if (SHADOW) out_shadow[col[u]] = pack_bf16x4(mean);
    }
  }
}

__global__ __launch_bounds__(kThreads) void broadcast_kernel(const float4* __restrict__ src,
                                                             float4* __restrict__ params,
                                                             uint2* __restrict__ shadow, size_t stride4,
                                                             int n) {
  for (size_t col = (size_t)blockIdx.x * kThreads + threadIdx.x; col < stride4;
       col += (size_t)gridDim.x * kThreads) {
    const float4 v = src[col];
    for (int i = 0; i < n; ++i) params[(size_t)i * stride4 + col] = v;
    if (shadow != nullptr) {
      const uint2 h = pack_bf16x4(v);
      for (int i = 0; i < n; ++i) shadow[(size_t)i * stride4 + col] = h;
    }
  }
}

__global__ __launch_bounds__(kThreads) void refresh_shadow_kernel(const float4* __restrict__ params,
                                                                  uint2* __restrict__ shadow,
                                                                  size_t count4) {
  for (size_t k = (size_t)blockIdx.x * kThreads + threadIdx.x; k < count4;
       k += (size_t)gridDim.x * kThreads)
    shadow[k] = pack_bf16x4(params[k]);
}

// x <- x - lr * g on 16-byte vectors; `tail` scalars at the end when count % 4 != 0.  A workgroup
// takes contiguous chunks of U x 256 vectors and issues all its loads before the first store.
template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void update_kernel(float* __restrict__ x,
                                                          const float* __restrict__ g,
                                                          uint16_t* __restrict__ shadow, size_t count,
                                                          float lr) {
  const size_t count4 = count / 4;
  f32x4_t* x4 = reinterpret_cast<f32x4_t*>(x);
  const f32x4_t* g4 = reinterpret_cast<const f32x4_t*>(g);
  u32x2_t* s4 = reinterpret_cast<u32x2_t*>(shadow);
  constexpr size_t kPer = (size_t)U * kThreads;
  for (size_t b = (size_t)blockIdx.x * kPer; b < count4; b += (size_t)gridDim.x * kPer) {
    f32x4_t xv[U], gv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = b + (size_t)u * kThreads + threadIdx.x;
      if (k < count4) { xv[u] = ld4<NT>(x4 + k); gv[u] = ld4<NT>(g4 + k); }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = b + (size_t)u * kThreads + threadIdx.x;
      if (k < count4) {
        f32x4_t w = xv[u];
        w.x = fmaf(-lr, gv[u].x, w.x);
        w.y = fmaf(-lr, gv[u].y, w.y);
        w.z = fmaf(-lr, gv[u].z, w.z);
        w.w = fmaf(-lr, gv[u].w, w.w);
        st4<NT>(x4 + k, w);
        if (shadow != nullptr) st2<NT>(s4 + k, pack_bf16x4(w));
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < (count & 3)) {
    const size_t k = count4 * 4 + threadIdx.x;
    const float xv = fmaf(-lr, g[k], x[k]);
    x[k] = xv;
    if (shadow != nullptr) shadow[k] = f32_to_bf16_rne(xv);
  }
}

// Momentum form of the local step:  v <- mu v + g,  x <- x - lr v  (one rounding each).
template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void momentum_update_kernel(f32x4_t* __restrict__ x4,
                                                                   f32x4_t* __restrict__ v4,
                                                                   const f32x4_t* __restrict__ g4,
                                                                   u32x2_t* __restrict__ s4, size_t count4,
                                                                   float lr, float mu) {
  constexpr size_t kPer = (size_t)U * kThreads;
  for (size_t b = (size_t)blockIdx.x * kPer; b < count4; b += (size_t)gridDim.x * kPer) {
    f32x4_t xv[U], vv[U], gv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = b + (size_t)u * kThreads + threadIdx.x;
      if (k < count4) { xv[u] = ld4<NT>(x4 + k); vv[u] = ld4<NT>(v4 + k); gv[u] = ld4<NT>(g4 + k); }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = b + (size_t)u * kThreads + threadIdx.x;
      if (k < count4) {
        f32x4_t v = vv[u], w = xv[u];
        v.x = fmaf(mu, v.x, gv[u].x); v.y = fmaf(mu, v.y, gv[u].y);
        v.z = fmaf(mu, v.z, gv[u].z); v.w = fmaf(mu, v.w, gv[u].w);
        w.x = fmaf(-lr, v.x, w.x); w.y = fmaf(-lr, v.y, w.y);
        w.z = fmaf(-lr, v.z, w.z); w.w = fmaf(-lr, v.w, w.w);
        st4<NT>(v4 + k, v);
        st4<NT>(x4 + k, w);
        if (s4 != nullptr) st2<NT>(s4 + k, pack_bf16x4(w));
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(f32x4_t* __restrict__ x4, size_t count4) {
  for (size_t k = (size_t)blockIdx.x * kThreads + threadIdx.x; k < count4;
       k += (size_t)gridDim.x * kThreads)
    x4[k] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
}

// Same update over [N][m_pad] with finished workers (Algorithm 3) left untouched.
__global__ __launch_bounds__(kThreads) void update_masked_kernel(float4* __restrict__ x,
                                                                 const float4* __restrict__ g,
                                                                 uint2* __restrict__ shadow,
                                                                 size_t stride4, float lr,
                                                                 const int* __restrict__ worker_steps,
                                                                 int step) {
  const int i = blockIdx.y;
  if (worker_steps != nullptr && step >= worker_steps[i]) return;
  for (size_t col = (size_t)blockIdx.x * kThreads + threadIdx.x; col < stride4;
       col += (size_t)gridDim.x * kThreads) {
    const size_t k = (size_t)i * stride4 + col;
    float4 xv = x[k];
    const float4 gv = g[k];
    xv.x = fmaf(-lr, gv.x, xv.x);
    xv.y = fmaf(-lr, gv.y, xv.y);
    xv.z = fmaf(-lr, gv.z, xv.z);
    xv.w = fmaf(-lr, gv.w, xv.w);
    x[k] = xv;
    if (shadow != nullptr) shadow[k] = pack_bf16x4(xv);
  }
}

// Plain streaming copy with exactly known traffic (bandwidth / counter calibration).
__global__ __launch_bounds__(kThreads) void copy_kernel(float4* __restrict__ dst,
                                                        const float4* __restrict__ src, size_t count4) {
  for (size_t k = (size_t)blockIdx.x * kThreads + threadIdx.x; k < count4;
       k += (size_t)gridDim.x * kThreads)
    dst[k] = src[k];
}

static int grid_for(size_t items, int max_blocks) {
  size_t b = (items + kThreads - 1) / kThreads;
  if (b < 1) b = 1;
  if (b > (size_t)max_blocks) b = max_blocks;
  return (int)b;
}

// 256 CUs x 8 resident workgroups: enough waves to cover HBM latency without a long tail.
constexpr int kStreamBlocks = 256 * 8;

// Small replica sets (fewer than a workgroup per compute unit at 256 columns each): a workgroup
// takes 64 columns and its four wavefronts each sum a quarter of the replicas, so that four times
// as many workgroups run and the chain of dependent loads per thread is four times shorter.  The
// quarters are added in order through LDS; the broadcast form writes each quarter's replicas.
template <bool SHADOW, bool BCAST>
__global__ __launch_bounds__(kThreads) void restart_small_kernel(f32x4_t* __restrict__ params,
                                                                 u32x2_t* __restrict__ shadow,
                                                                 f32x4_t* __restrict__ out, size_t stride4,
                                                                 int n, float n_f) {
  __shared__ f32x4_t part[4][64];
  const int lane = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const size_t c = (size_t)blockIdx.x * 64 + lane;
  const bool ok = c < stride4;
  const size_t col[1] = {ok ? c : 0};
  const int n_per = (n + 3) / 4;
  const int i0 = min(n, rg * n_per), i1 = min(n, i0 + n_per);
  f32x4_t sum[1] = {(f32x4_t){0.0f, 0.0f, 0.0f, 0.0f}};
  if (i1 > i0) replica_sums<false, 1>(params + (size_t)i0 * stride4, stride4, col, i1 - i0, sum);
  part[rg][lane] = sum[0];
  __syncthreads();
  if (!ok) return;
  const f32x4_t mean = (((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]) / n_f;
  if (BCAST) {
    for (int i = i0; i < i1; ++i) params[(size_t)i * stride4 + c] = mean;
    if (SHADOW) {
      const u32x2_t h = pack_bf16x4(mean);
      for (int i = i0; i < i1; ++i) shadow[(size_t)i * stride4 + c] = h;
    }
  } else if (rg == 0) {
    out[c] = mean;
    if (SHADOW) shadow[c] = pack_bf16x4(mean);
  }
}
// Which decomposition a shape gets (the same for both restart kernels, so that they sum in the
// same order and stay bit-identical to each other).
static bool restart_is_small(size_t stride4, int n) { return n >= 8 && stride4 < (size_t)256 * 256; }

template <bool SHADOW, bool NT, int U>
static void launch_average_u(f32x4_t* p4, u32x2_t* s2, size_t stride4, int n, hipStream_t s) {
  const int grid = grid_for((stride4 + U - 1) / U, 65536);
  hipLaunchKernelGGL((average_kernel<SHADOW, NT, U>), dim3(grid), dim3(kThreads), 0, s, p4, s2, stride4, n,
                     (float)n);
}
template <bool SHADOW, bool NT, int U>
static void launch_mean_u(const f32x4_t* p4, f32x4_t* o4, u32x2_t* s2, size_t stride4, int n, hipStream_t s) {
  const int grid = grid_for((stride4 + U - 1) / U, 65536);
  hipLaunchKernelGGL((mean_kernel<SHADOW, NT, U>), dim3(grid), dim3(kThreads), 0, s, p4, o4, s2, stride4, n,
                     (float)n);
}

hipError_t launch_average(float* params, uint16_t* shadow, long m_pad, int n_workers, bool streaming,
                          hipStream_t s) {
  const size_t stride4 = (size_t)m_pad / 4;
  // the non-temporal variants are for replica sets far beyond the 256 MB last-level cache
  f32x4_t* p4 = reinterpret_cast<f32x4_t*>(params);
  u32x2_t* s2 = reinterpret_cast<u32x2_t*>(shadow);
  if (restart_is_small(stride4, n_workers)) {
    const int grid = (int)((stride4 + 63) / 64);
    if (shadow != nullptr)
      hipLaunchKernelGGL((restart_small_kernel<true, true>), dim3(grid), dim3(kThreads), 0, s, p4, s2,
                         (f32x4_t*)nullptr, stride4, n_workers, (float)n_workers);
    else
      hipLaunchKernelGGL((restart_small_kernel<false, true>), dim3(grid), dim3(kThreads), 0, s, p4, s2,
                         (f32x4_t*)nullptr, stride4, n_workers, (float)n_workers);
    return hipGetLastError();
  }
  const bool two = stride4 >= kTwoColumnsFrom;
#define PRSGD_AVG(SH, NTV) \
  do { if (two) launch_average_u<SH, NTV, 2>(p4, s2, stride4, n_workers, s); \
       else launch_average_u<SH, NTV, 1>(p4, s2, stride4, n_workers, s); } while (0)
  if (shadow != nullptr) { if (streaming) PRSGD_AVG(true, true); else PRSGD_AVG(true, false); }
  else { if (streaming) PRSGD_AVG(false, true); else PRSGD_AVG(false, false); }
#undef PRSGD_AVG
  return hipGetLastError();
}

hipError_t launch_mean(const float* params, float* out, uint16_t* out_shadow, long m_pad, int n_workers,
                       bool streaming, hipStream_t s) {
  const size_t stride4 = (size_t)m_pad / 4;
  const f32x4_t* p4 = reinterpret_cast<const f32x4_t*>(params);
  f32x4_t* o4 = reinterpret_cast<f32x4_t*>(out);
  u32x2_t* s2 = reinterpret_cast<u32x2_t*>(out_shadow);
  if (restart_is_small(stride4, n_workers)) {
    const int grid = (int)((stride4 + 63) / 64);
    f32x4_t* pm = const_cast<f32x4_t*>(p4);              // read only in this form
    if (out_shadow != nullptr)
      hipLaunchKernelGGL((restart_small_kernel<true, false>), dim3(grid), dim3(kThreads), 0, s, pm, s2, o4,
                         stride4, n_workers, (float)n_workers);
    else
      hipLaunchKernelGGL((restart_small_kernel<false, false>), dim3(grid), dim3(kThreads), 0, s, pm, s2, o4,
                         stride4, n_workers, (float)n_workers);
    return hipGetLastError();
  }
  const bool two = stride4 >= kTwoColumnsFrom;
#define PRSGD_MEAN(SH, NTV) \
  do { if (two) launch_mean_u<SH, NTV, 2>(p4, o4, s2, stride4, n_workers, s); \
       else launch_mean_u<SH, NTV, 1>(p4, o4, s2, stride4, n_workers, s); } while (0)
  if (out_shadow != nullptr) { if (streaming) PRSGD_MEAN(true, true); else PRSGD_MEAN(true, false); }
  else { if (streaming) PRSGD_MEAN(false, true); else PRSGD_MEAN(false, false); }
#undef PRSGD_MEAN
  return hipGetLastError();
}

hipError_t launch_broadcast(const float* src, float* params, uint16_t* shadow, long m_pad,
                            int n_workers, hipStream_t s) {
  const size_t stride4 = (size_t)m_pad / 4;
  hipLaunchKernelGGL(broadcast_kernel, dim3(grid_for(stride4, kStreamBlocks)), dim3(kThreads), 0, s,
                     reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(params),
                     reinterpret_cast<uint2*>(shadow), stride4, n_workers);
  return hipGetLastError();
}

hipError_t launch_refresh_shadow(const float* params, uint16_t* shadow, long count, hipStream_t s) {
  const size_t count4 = (size_t)count / 4;
  hipLaunchKernelGGL(refresh_shadow_kernel, dim3(grid_for(count4, kStreamBlocks)), dim3(kThreads), 0,
                     s, reinterpret_cast<const float4*>(params), reinterpret_cast<uint2*>(shadow),
                     count4);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t count4 = bytes / 16;
  if (count4 == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3(grid_for(count4, kStreamBlocks)), dim3(kThreads), 0, s,
                     reinterpret_cast<float4*>(dst), reinterpret_cast<const float4*>(src), count4);
  return hipGetLastError();
}

hipError_t launch_update(float* x, const float* g, uint16_t* shadow, size_t count, float lr,
                         hipStream_t s) {
  if (count == 0) return hipSuccess;
  // vectors far beyond the 256 MB last-level cache are streamed with non-temporal accesses
  const bool nt = count * sizeof(float) >= ((size_t)1 << 28);
  constexpr int U = 4;
  const int grid = grid_for((count / 4 + U - 1) / U + 1, 65536);
  if (nt) hipLaunchKernelGGL((update_kernel<U, true>), dim3(grid), dim3(kThreads), 0, s, x, g, shadow, count, lr);
  else hipLaunchKernelGGL((update_kernel<U, false>), dim3(grid), dim3(kThreads), 0, s, x, g, shadow, count, lr);
  return hipGetLastError();
}

// count is a multiple of 4 (whole padded replica buffers).
hipError_t launch_momentum_update(float* x, float* v, const float* g, uint16_t* shadow, size_t count,
                                  float lr, float mu, hipStream_t s) {
  if (count == 0) return hipSuccess;
  const bool nt = count * sizeof(float) >= ((size_t)1 << 28);
  constexpr int U = 2;
  const size_t count4 = count / 4;
  const int grid = grid_for((count4 + U - 1) / U, 65536);
  f32x4_t* x4 = reinterpret_cast<f32x4_t*>(x);
  f32x4_t* v4 = reinterpret_cast<f32x4_t*>(v);
  const f32x4_t* g4 = reinterpret_cast<const f32x4_t*>(g);
  u32x2_t* s4 = reinterpret_cast<u32x2_t*>(shadow);
  if (nt) hipLaunchKernelGGL((momentum_update_kernel<U, true>), dim3(grid), dim3(kThreads), 0, s, x4, v4, g4, s4, count4, lr, mu);
  else hipLaunchKernelGGL((momentum_update_kernel<U, false>), dim3(grid), dim3(kThreads), 0, s, x4, v4, g4, s4, count4, lr, mu);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float* x, size_t count, hipStream_t s) {
  const size_t count4 = count / 4;
  if (count4 == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(count4, kStreamBlocks)), dim3(kThreads), 0, s,
                     reinterpret_cast<f32x4_t*>(x), count4);
  return hipGetLastError();
}

hipError_t launch_update_masked(float* x, const float* g, uint16_t* shadow, long m_pad, int n_workers,
                                float lr, const int* worker_steps, int step, hipStream_t s) {
  const size_t stride4 = (size_t)m_pad / 4;
  int gx = grid_for(stride4, kStreamBlocks / (n_workers < 8 ? n_workers : 8));
  hipLaunchKernelGGL(update_masked_kernel, dim3(gx, n_workers), dim3(kThreads), 0, s,
                     reinterpret_cast<float4*>(x), reinterpret_cast<const float4*>(g),
                     reinterpret_cast<uint2*>(shadow), stride4, lr, worker_steps, step);
  return hipGetLastError();
}

}  // namespace prsgd
