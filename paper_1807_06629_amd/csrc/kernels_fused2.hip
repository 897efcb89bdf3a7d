// One launch = a whole epoch of local iterations (Algorithm 1, eq. 3) for small fp32 MLPs with
// one hidden layer, the latency-bound regime where a chain of per-layer kernels is dominated
// by launch gaps and by re-reading weights that would fit on chip.
//
// Workers never exchange anything inside an epoch (paragraph below Algorithm 1), so the only
// coupling is inside one worker's own forward/backward pass.  Worker i is served by a TEAM of P
// workgroups; workgroup j of the team owns W = d_1 / P hidden units:
//   - its [d_0][W] slice of W_1 lives in REGISTERS for the whole launch, laid out so that the
//     MFMA B-operand registers of the forward product are, element for element, the accumulator
//     registers of the weight-gradient product: eq. (3) for W_1 is a register-to-register fma;
//   - its slices of b_1 and W_2 (and a private copy of b_2) live in LDS;
//   - per iteration it draws the minibatch rows, gathers them into LDS, computes its slice of the
//     hidden layer, and contributes a partial logit block.  One team-wide barrier per iteration
//     (a counter in HBM, bounded spin) lets every member sum the P partials in fixed order;
//     everything after that (softmax, both delta blocks, dW_2, db, dW_1) is local to the slice.
// Teams of different workers never synchronise.  Summation orders are fixed, so a run is
// bit-reproducible.
#include "prsgd_internal.h"

namespace prsgd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr unsigned kSpinLimit = 1u << 22;     // bounded wait: a lost team member aborts the launch

__device__ __forceinline__ f32x4_t mfma16(float a, float b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float act2_fwd(float z, int act) {
  return act == PRSGD_TANH ? tanhf(z) : fmaxf(z, 0.0f);
}
__device__ __forceinline__ float act2_bwd(float h, int act) {
  return act == PRSGD_TANH ? (1.0f - h * h) : (h > 0.0f ? 1.0f : 0.0f);
}

// KBI: 16-row blocks of W_1 per wavefront (register budget); NT: 16-column tiles of the hidden
// slice; MT: 16-row tiles of the minibatch.
template <int KBI, int NT, int MT>
__global__ __launch_bounds__(kThreads) void mlp2_epoch_kernel(Fused2Args p) {
  constexpr int W = NT * 16, MR = MT * 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;

  // team mapping: consecutive workgroups go round-robin to the 8 XCDs; keep a team on one XCD
  // (its partial logits then stay in that XCD's L2) when the worker count allows it
  int i, j;
  if ((p.n_workers & 7) == 0) {
    const int slot = blockIdx.x >> 3;
    i = (blockIdx.x & 7) + 8 * (slot / p.P);
    j = slot % p.P;
  } else {
    i = blockIdx.x / p.P;
    j = blockIdx.x % p.P;
  }
  const int my_k = p.worker_steps != nullptr ? min(p.worker_steps[i], p.k) : p.k;
  if (my_k <= 0) return;                                   // uniform over the team
  unsigned int* cnt = p.sync + (size_t)i * 32;             // one 128-byte line per team
  unsigned int* abort_flag = p.sync + (size_t)p.n_workers * 32;
  unsigned int* base_slot = cnt + 1;
  if (__hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
  const unsigned base = *base_slot;                        // arrivals counted before this launch

  const int d0 = p.d0, d2 = p.d2, B = p.batch, D2P = p.d2p, ldx = p.ldx;
  const int KB = (d0 + 15) / 16;

  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* X = lds;                                          // [MR][ldx]   gathered rows
  float* red = X + (size_t)MR * ldx;                       // [4][MR][W]  per-wavefront partial z_1
  float* h = red + 4 * MR * W;                             // [MR][W]
  float* dl1 = h + MR * W;                                 // [MR][W]
  float* lg = dl1 + MR * W;                                // [MR][D2P]   logits, then delta_2
  float* w2 = lg + MR * D2P;                               // [W][D2P]
  float* b1 = w2 + W * D2P;                                // [W]
  float* b2 = b1 + W;                                      // [D2P]
  int* rows = reinterpret_cast<int*>(b2 + D2P);            // [MR]
  int* ylab = rows + MR;                                   // [MR]
  int* flag = ylab + MR;                                   // [1] abort broadcast

  float* prm = p.params + (size_t)i * p.m_pad;
  const float* feat = p.features + (size_t)i * p.rows * d0;
  const int32_t* lab = p.labels + (size_t)i * p.rows;

  // ---- load the slice: W_1 to registers, W_2 / b_1 / b_2 to LDS -------------------------------
  float w1[KBI][NT][4];
#pragma unroll
  for (int kbi = 0; kbi < KBI; ++kbi) {
    const int kb = wave + 4 * kbi;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int k = 16 * kb + 4 * q4 + s;
        const bool ok = kb < KB && k < d0;
        const float v = prm[p.w1_off + (ok ? (size_t)k * p.ld1 + j * W + nt * 16 + n16 : (size_t)0)];
        w1[kbi][nt][s] = ok ? v : 0.0f;
      }
  }
  for (int e = tid; e < W * D2P; e += kThreads) {
    const int n = e / D2P, c = e % D2P;
    w2[e] = c < d2 ? prm[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] : 0.0f;
  }
  if (tid < W) b1[tid] = prm[p.b1_off + j * W + tid];
  if (tid < D2P) b2[tid] = tid < d2 ? prm[p.b2_off + tid] : 0.0f;
  for (int e = tid; e < MR * ldx; e += kThreads) X[e] = 0.0f;     // pad rows / columns stay zero
  if (tid == 0) flag[0] = 0;
  __syncthreads();

  const float inv_b = 1.0f / (float)B;
  const size_t part_team = (size_t)MR * D2P;                      // floats per (team member)
  bool aborted = false;

  for (int s = 1; s <= my_k; ++s) {
    const uint64_t t = p.t0 + (uint64_t)s;
    // (a) minibatch rows of this iteration
    if (tid < B) {
      const int r = sample_row(p.seed, (uint32_t)i, t, (uint32_t)tid, p.log2n);
      rows[tid] = r;
      ylab[tid] = lab[r];
    }
    __syncthreads();
    // (b) gather the rows into LDS (16-byte vectors; d0 is a multiple of 4).  Eight loads per
    // thread are issued before the first is consumed so that their HBM latencies overlap.
    {
      constexpr int G = 8;
      const int v4 = d0 >> 2, total = B * v4;
      for (int e0 = 0; e0 < total; e0 += G * kThreads) {
        f32x4_t v[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
          const int e = e0 + u * kThreads + tid;
          const int ec = e < total ? e : 0;
          const int r = ec / v4, c = ec - r * v4;
          v[u] = *reinterpret_cast<const f32x4_t*>(feat + (size_t)rows[r] * d0 + 4 * c);
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
          const int e = e0 + u * kThreads + tid;
          if (e < total) {
            const int r = e / v4, c = e - r * v4;
            *reinterpret_cast<f32x4_t*>(X + (size_t)r * ldx + 4 * c) = v[u];
          }
        }
      }
    }
    __syncthreads();
    // (c) forward slice: contraction index of MFMA step s is k = 16 kb + 4 q4 + s
    {
      f32x4_t acc[MT][NT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int kbi = 0; kbi < KBI; ++kbi) {
        const int kb = wave + 4 * kbi;
        if (kb < KB) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const f32x4_t a4 =
                *reinterpret_cast<const f32x4_t*>(X + (size_t)(mt * 16 + n16) * ldx + 16 * kb + 4 * q4);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
              for (int q = 0; q < 4; ++q) acc[mt][nt] = mfma16(a4[q], w1[kbi][nt][q], acc[mt][nt]);
          }
        }
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            red[((size_t)wave * MR + mt * 16 + 4 * q4 + v) * W + nt * 16 + n16] = acc[mt][nt][v];
    }
    __syncthreads();
    for (int e = tid; e < MR * W; e += kThreads) {
      const int b = e / W, n = e % W;
      const float z = b1[n] + red[e] + red[MR * W + e] + red[2 * MR * W + e] + red[3 * MR * W + e];
      h[e] = b < B ? act2_fwd(z, p.act) : 0.0f;
    }
    __syncthreads();
    // (d) this slice's contribution to the logits
    float* my_part = p.part + (((size_t)(s & 1) * p.n_workers + i) * p.P + j) * part_team;
    for (int e = tid; e < MR * D2P; e += kThreads) {
      const int b = e / D2P, c = e % D2P;
      float sum = 0.0f;
#pragma unroll 8
      for (int n = 0; n < W; ++n) sum = fmaf(h[b * W + n], w2[n * D2P + c], sum);
      // agent-scope store: visible to the other compute units without flushing whole caches
      __hip_atomic_store(my_part + e, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // (e) team barrier: arrivals are counted in HBM; the wait is bounded.  The partials were
    // written with agent-scope stores; draining this wavefront's stores before the workgroup
    // barrier orders them before the arrival count without a cache-wide release fence.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned target = base + (unsigned)p.P * (unsigned)s;
      unsigned spins = 0;
      int bad = 0;
      while ((int)(__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
        if (++spins > kSpinLimit ||
            __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
          __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          bad = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      flag[0] = bad;
    }
    __syncthreads();
    if (flag[0] != 0) { aborted = true; break; }
    // (f) logits = b_2 + sum of the P partials in member order; softmax cross-entropy head
    {
      const float* team_part = p.part + (((size_t)(s & 1) * p.n_workers + i) * p.P) * part_team;
      for (int e = tid; e < MR * D2P; e += kThreads) {
        float sum = b2[e % D2P];
        // agent-scope loads (never a stale cached copy), eight in flight at a time; the sum
        // itself runs in member order
        for (int j0 = 0; j0 < p.P; j0 += 8) {
          float v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int jj = j0 + u < p.P ? j0 + u : 0;
            v[u] = __hip_atomic_load(team_part + (size_t)jj * part_team + e, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (j0 + u < p.P) sum += v[u];
        }
        lg[e] = sum;
      }
    }
    __syncthreads();
    if (tid < MR) {
      float* row = lg + tid * D2P;
      if (tid < B) {
        float mx = -INFINITY;
        for (int c = 0; c < d2; ++c) mx = fmaxf(mx, row[c]);
        float se = 0.0f;
        for (int c = 0; c < d2; ++c) se += expf(row[c] - mx);
        const int y = ylab[tid];
        const float zy = (y >= 0 && y < d2) ? row[y] : 0.0f;
        if (j == 0) p.row_loss[(size_t)i * B + tid] = (mx + logf(se)) - zy;
        for (int c = 0; c < D2P; ++c)
          row[c] = c < d2 ? (expf(row[c] - mx) / se - (c == y ? 1.0f : 0.0f)) * inv_b : 0.0f;
      } else {
        for (int c = 0; c < D2P; ++c) row[c] = 0.0f;
      }
    }
    __syncthreads();
    // (g) delta_1 slice (needs the pre-update W_2), then the small updates
    for (int e = tid; e < MR * W; e += kThreads) {
      const int b = e / W, n = e % W;
      float sum = 0.0f;
      for (int c = 0; c < D2P; ++c) sum = fmaf(lg[b * D2P + c], w2[n * D2P + c], sum);
      dl1[e] = sum * act2_bwd(h[e], p.act);
    }
    __syncthreads();
    for (int e = tid; e < W * D2P; e += kThreads) {
      const int n = e / D2P, c = e % D2P;
      float sum = 0.0f;
      for (int b = 0; b < B; ++b) sum = fmaf(h[b * W + n], lg[b * D2P + c], sum);
      w2[e] = fmaf(-p.lr, sum, w2[e]);
    }
    if (tid < D2P) {
      float sum = 0.0f;
      for (int b = 0; b < B; ++b) sum += lg[b * D2P + tid];
      b2[tid] = fmaf(-p.lr, sum, b2[tid]);
    }
    if (tid >= 64 && tid < 64 + W) {
      const int n = tid - 64;
      float sum = 0.0f;
      for (int b = 0; b < B; ++b) sum += dl1[b * W + n];
      b1[n] = fmaf(-p.lr, sum, b1[n]);
    }
    // (h) dW_1 slice and eq. (3) in registers: contraction index of MFMA step u is b = 4u + q4
    {
      float dfr[MT * 4][NT];
#pragma unroll
      for (int u = 0; u < MT * 4; ++u)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) dfr[u][nt] = dl1[(4 * u + q4) * W + nt * 16 + n16];
#pragma unroll
      for (int kbi = 0; kbi < KBI; ++kbi) {
        const int kb = wave + 4 * kbi;
        if (kb < KB) {
          f32x4_t g[NT];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) g[nt] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int u = 0; u < MT * 4; ++u) {
            const float a = X[(size_t)(4 * u + q4) * ldx + 16 * kb + n16];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) g[nt] = mfma16(a, dfr[u][nt], g[nt]);
          }
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) w1[kbi][nt][v] = fmaf(-p.lr, g[nt][v], w1[kbi][nt][v]);
        }
      }
    }
    __syncthreads();                                     // X and the small buffers are reused
  }

  if (aborted) return;
  // ---- write the slice back ------------------------------------------------------------------
#pragma unroll
  for (int kbi = 0; kbi < KBI; ++kbi) {
    const int kb = wave + 4 * kbi;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = 16 * kb + 4 * q4 + q;
        if (kb < KB && k < d0) prm[p.w1_off + (size_t)k * p.ld1 + j * W + nt * 16 + n16] = w1[kbi][nt][q];
      }
  }
  for (int e = tid; e < W * D2P; e += kThreads) {
    const int n = e / D2P, c = e % D2P;
    if (c < d2) prm[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] = w2[e];
  }
  if (tid < W) prm[p.b1_off + j * W + tid] = b1[tid];
  if (j == 0) {
    if (tid < d2) prm[p.b2_off + tid] = b2[tid];
    if (tid < B) p.idx[(size_t)i * B + tid] = rows[tid];
    if (tid == 0) *base_slot = base + (unsigned)p.P * (unsigned)my_k;   // all arrivals are in
  }
}

// ---- host side --------------------------------------------------------------------------------
size_t fused2_lds_bytes(const Fused2Plan& pl) {
  const size_t MR = (size_t)pl.MT * 16, W = (size_t)pl.NT * 16;
  const size_t floats = MR * pl.ldx + 4 * MR * W + 2 * MR * W + MR * pl.d2p + W * pl.d2p + W + pl.d2p +
                        2 * MR + 4;
  return floats * sizeof(float);
}

template <int KBI, int NT, int MT> static const void* fused2_symbol() {
  return reinterpret_cast<const void*>(mlp2_epoch_kernel<KBI, NT, MT>);
}

static const void* fused2_pick(int kbi, int nt, int mt) {
#define PICK(K, N, M) if (kbi == K && nt == N && mt == M) return fused2_symbol<K, N, M>();
  PICK(4, 1, 1) PICK(4, 1, 2) PICK(4, 1, 4) PICK(4, 2, 1) PICK(4, 2, 2) PICK(4, 2, 4)
  PICK(8, 1, 1) PICK(8, 1, 2) PICK(8, 1, 4) PICK(8, 2, 1) PICK(8, 2, 2) PICK(8, 2, 4)
  PICK(16, 1, 1) PICK(16, 1, 2) PICK(16, 1, 4) PICK(16, 2, 1) PICK(16, 2, 2) PICK(16, 2, 4)
#undef PICK
  return nullptr;
}

// Decides whether the epoch kernel applies and how the team is shaped.  It needs every
// workgroup of the grid resident at once (checked against the occupancy the runtime reports).
bool fused2_plan(int n_workers, int d0, int d1, int d2, int batch, Fused2Plan* pl) {
  if (d0 < 4 || (d0 & 3) != 0 || d0 > 1024 || (d1 & 15) != 0 || d2 > 64 || batch > 64) return false;
  pl->MT = batch <= 16 ? 1 : batch <= 32 ? 2 : 4;
  const int kb = (d0 + 15) / 16, kbi_need = (kb + 3) / 4;
  pl->KBI = kbi_need <= 4 ? 4 : kbi_need <= 8 ? 8 : 16;
  pl->d2p = (d2 + 15) / 16 * 16;
  int ldx = (d0 + 15) / 16 * 16 + 4;                        // (ldx / 4) odd: conflict-free 16-byte rows
  if (((ldx / 4) & 1) == 0) ldx += 4;
  pl->ldx = ldx;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return false;
  for (int nt = 1; nt <= 2; ++nt) {
    if (d1 % (16 * nt) != 0) continue;
    pl->NT = nt;
    pl->P = d1 / (16 * nt);
    const size_t lds_bytes = fused2_lds_bytes(*pl);
    if (lds_bytes > 160 * 1024) continue;
    const void* sym = fused2_pick(pl->KBI, pl->NT, pl->MT);
    if (sym == nullptr) return false;
    if (hipFuncSetAttribute(sym, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return false;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sym, kThreads, lds_bytes) != hipSuccess)
      return false;
    if ((long)n_workers * pl->P <= (long)per_cu * cus) return true;
  }
  return false;
}

hipError_t launch_fused2(const Fused2Plan& pl, Fused2Args args, hipStream_t s) {
  const void* sym = fused2_pick(pl.KBI, pl.NT, pl.MT);
  if (sym == nullptr) return hipErrorInvalidValue;
  args.P = pl.P;
  args.d2p = pl.d2p;
  args.ldx = pl.ldx;
  void* kargs[] = {&args};
  // Plain launch: fused2_plan has checked that the whole grid fits on the device at once, and a
  // team member that never shows up ends in the kernel's bounded wait, not in a hang.
  return hipLaunchKernel(sym, dim3((unsigned)(args.n_workers * pl.P)), dim3(kThreads), kargs,
                         fused2_lds_bytes(pl), s);
}

}  // namespace prsgd
