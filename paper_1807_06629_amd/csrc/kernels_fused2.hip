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
//   - per iteration it computes its slice of the hidden layer on the minibatch held in LDS and
//     contributes a partial logit block; the next iteration's rows are drawn meanwhile and, for
//     shapes with registers to spare, gathered (HBM -> registers) meanwhile as well -- otherwise
//     at the end of the iteration, with loads that write LDS directly.  One team-wide barrier per iteration
//     (a counter in HBM, bounded spin) lets every member sum the P partials in fixed order;
//     everything after that (softmax, both delta blocks, dW_2, db, dW_1) is local to the slice.
// Teams of different workers never synchronise.  Summation orders are fixed, so a run is
// bit-reproducible.
#include "prsgd_internal.h"

namespace prsgd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kTT = 512;                      // threads per team member: two wavefronts per SIMD, so
constexpr int kTW = kTT / kWave;              // that the latency-bound phases of one overlap the other's
constexpr int kAgentScope = 16;               // buffer-load cache policy: the sc1 bit (agent scope)

__device__ __forceinline__ f32x4_t mfma16(float a, float b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float act2_fwd(float z, int act) {
  return act == PRSGD_TANH ? tanhf(z) : fmaxf(z, 0.0f);
}
__device__ __forceinline__ float act2_bwd(float h, int act) {
  return act == PRSGD_TANH ? (1.0f - h * h) : (h > 0.0f ? 1.0f : 0.0f);
}

// Butterfly over each aligned group of 16 lanes on the data-parallel-primitive path (no LDS round
// trips): every lane of the group ends with the same max / sum.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));      // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_move<0x4E>(v));      // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_move<0x141>(v));     // row_half_mirror
  return fmaxf(v, dpp_move<0x140>(v));  // row_mirror
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  return v + dpp_move<0x140>(v);
}

// KBI: 16-row blocks of W_1 per wavefront (register budget); NT: 16-column tiles of the hidden
// slice; MT: 16-row tiles of the minibatch.  MOM: momentum form of the local update
// (v <- mu v + G, x <- x - gamma v) with the velocity of the slice held next to the slice.
template <int KBI, int NT, int MT, bool MOM>
__global__ __launch_bounds__(kTT) void mlp2_epoch_kernel(Fused2Args p) {
  constexpr int W = NT * 16, MR = MT * 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n16 = lane & 15, q4 = lane >> 4;

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
  float* red = X + (size_t)MR * ldx;                       // [kTW][MR][W] per-wavefront partial z_1
  float* h = red + kTW * MR * W;                           // [MR][W]
  float* dl1 = h + MR * W;                                 // [MR][W]
  float* lg = dl1 + MR * W;                                // [MR][D2P]   logits, then delta_2
  float* w2 = lg + MR * D2P;                               // [W][D2P]
  float* b1 = w2 + W * D2P;                                // [W]
  float* b2 = b1 + W;                                      // [D2P]
  int* rows = reinterpret_cast<int*>(b2 + D2P);            // [MR] rows of this iteration
  int* ylab = rows + MR;                                   // [MR] their labels
  int* rows_ahead = ylab + MR;                             // [2][MR] rows of iteration t at [t & 1], drawn early
  int* flag = rows_ahead + 2 * MR;                         // [4] abort broadcast
  float* vw2 = reinterpret_cast<float*>(flag + 4);         // [W][D2P] velocities (MOM only)
  float* vb1 = vw2 + W * D2P;                              // [W]
  float* vb2 = vb1 + W;                                    // [D2P]

  float* prm = p.params + (size_t)i * p.m_pad;
  const float* prm0 = p.src + (size_t)i * p.src_stride;      // this worker's starting point
  const float* feat = p.features + (size_t)i * p.rows * d0;
  const int32_t* lab = p.labels + (size_t)i * p.rows;

  // Rows of the first iteration first: their features, their labels and the parameter slice are
  // then requested together, so that the launch pays one memory latency instead of three.
  int row_first = 0;
  if (tid < B) {
    row_first = sample_row(p.seed, (uint32_t)i, p.t0 + 1, (uint32_t)tid, p.log2n);
    rows[tid] = row_first;
  }
  for (int e = tid; e < MR * ldx; e += kTT) X[e] = 0.0f;     // pad rows / columns stay zero
  if (tid == 0) flag[0] = 0;
  __syncthreads();

  const float inv_b = 1.0f / (float)B;
  const size_t part_team = (size_t)MR * D2P;                      // floats per (team member)
  bool aborted = false;

  // ---- minibatch pipeline ----------------------------------------------------------------------
  // The index stream is a pure function of (seed, worker, iteration, slot): the rows of iteration
  // s+1 are drawn at the start of iteration s and their features travel HBM -> registers while
  // iteration s computes; they are written to LDS once X is no longer read.  A thread owns the
  // 16-byte column pc of rows rg, rg + ng, rg + 2 ng, ... (a row is at most 256 vectors wide).
  // Rows B .. MR-1 of X receive a copy of the first drawn row: finite values that only ever meet
  // zero deltas.
  // PF vectors per thread make up a minibatch and are requested an iteration early; 0 = no
  // prefetch, for the shapes whose W_1 slice leaves no registers for it (measured on 784-256-10,
  // seven row blocks per wavefront: 200 us per 16-iteration launch without, 219 us with)
  constexpr int PF = (MT > 2 || KBI * NT > 4) ? 0 : 8 * MT;
  const int v4 = d0 >> 2, total4 = B * v4;
  int cw_log = 5;                                          // ng <= 16 divides MR
  while ((1 << cw_log) < v4) ++cw_log;
  const int pc = tid & ((1 << cw_log) - 1), ng = kTT >> cw_log;
  const bool pc_ok = pc < v4;
  int rg = tid >> cw_log;
  f32x4_t pre[PF > 0 ? PF : 1];
  auto gather_issue = [&](const int* rws) {
    // opaque copy: keeps the per-vector addresses and predicates from being hoisted out of the
    // iteration loop into (spilled) registers
    asm volatile("" : "+v"(rg));
    const float* src = feat + (pc_ok ? 4 * pc : 0);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      if (ng * u < B) {                                    // uniform over the workgroup
        const int r = rg + ng * u;
        pre[u] = *reinterpret_cast<const f32x4_t*>(src + (size_t)rws[r < B ? r : 0] * d0);
      }
    }
  };
  auto gather_store = [&]() {
    asm volatile("" : "+v"(rg));
    if (pc_ok) {
      float* dst = X + (size_t)rg * ldx + 4 * pc;
      const int step = ng * ldx;
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        if (ng * u < B) *reinterpret_cast<f32x4_t*>(dst) = pre[u];
        dst += step;
      }
    }
  };
  // Gather without the register stage (shapes whose minibatch does not fit the register budget):
  // loads that write LDS directly, one instruction per 64 consecutive 16-byte vectors of a row
  // (the lanes' data lands at consecutive LDS addresses from a wavefront-uniform base), so the
  // whole minibatch is in flight at once at no register cost.
  auto gather_direct = [&]() {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int cpr = (v4 + 63) >> 6;                        // 64-vector chunks per row
    for (int t = wave; t < B * cpr; t += kTW) {
      const int r = t / cpr, ch = t - r * cpr;
      const int c = 64 * ch + lane;
      const int lds_off = __builtin_amdgcn_readfirstlane(r * ldx + 256 * ch);
      if (c < v4)
        __builtin_amdgcn_global_load_lds((gptr_t)(feat + (size_t)rows[r] * d0 + 4 * c), (lptr_t)(X + lds_off),
                                         16, 0, 0);
    }
  };
  auto gather_direct_wait = [&]() {                        // the data is in LDS before the next barrier
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  // labels and features of the first iteration, requested before the parameter slice
  int lab_first = 0;
  if (tid < B) lab_first = lab[row_first];
  if constexpr (PF > 0) gather_issue(rows); else gather_direct();
  // ---- load the slice: W_1 to registers, W_2 / b_1 / b_2 to LDS -------------------------------
  float w1[KBI][NT][4];
#pragma unroll
  for (int kbi = 0; kbi < KBI; ++kbi) {
    const int kb = wave + kTW * kbi;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int k = 16 * kb + 4 * q4 + s;
        const bool ok = kb < KB && k < d0;
        const float v = prm0[p.w1_off + (ok ? (size_t)k * p.ld1 + j * W + nt * 16 + n16 : (size_t)0)];
        w1[kbi][nt][s] = ok ? v : 0.0f;
      }
  }
  for (int e = tid; e < W * D2P; e += kTT) {
    const int n = e / D2P, c = e % D2P;
    w2[e] = c < d2 ? prm0[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] : 0.0f;
  }
  if (tid < W) b1[tid] = prm0[p.b1_off + j * W + tid];
  if (tid < D2P) b2[tid] = tid < d2 ? prm0[p.b2_off + tid] : 0.0f;
  // velocity of the slice, same places
  float* vel = MOM ? p.vel + (size_t)i * p.m_pad : nullptr;
  float vw1[MOM ? KBI : 1][NT][4];
  if constexpr (MOM) {
#pragma unroll
    for (int kbi = 0; kbi < KBI; ++kbi) {
      const int kb = wave + kTW * kbi;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int k = 16 * kb + 4 * q4 + q;
          const bool ok = kb < KB && k < d0;
          const float v = vel[p.w1_off + (ok ? (size_t)k * p.ld1 + j * W + nt * 16 + n16 : (size_t)0)];
          vw1[kbi][nt][q] = ok ? v : 0.0f;
        }
    }
    for (int e = tid; e < W * D2P; e += kTT) {
      const int n = e / D2P, c = e % D2P;
      vw2[e] = c < d2 ? vel[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] : 0.0f;
    }
    if (tid < W) vb1[tid] = vel[p.b1_off + j * W + tid];
    if (tid < D2P) vb2[tid] = tid < d2 ? vel[p.b2_off + tid] : 0.0f;
  }
  if (tid < B) ylab[tid] = lab_first;
  if constexpr (PF > 0) gather_store(); else gather_direct_wait();
  // rows and labels of the second iteration (the pipeline runs one iteration ahead)
  int lab_next = 0;
  if (PF > 0 && my_k > 1 && tid < B) {
    const int r = sample_row(p.seed, (uint32_t)i, p.t0 + 2, (uint32_t)tid, p.log2n);
    rows_ahead[tid] = r;                                   // iteration 2 of this call: slot 0
    lab_next = lab[r];
  }
  __syncthreads();

  // partial-logit exchange: Q 16-byte vectors per member; G groups of members are summed in
  // parallel (group g = members [g * PG, (g+1) * PG) in order), then the groups in order
  const int Q = MR * D2P / 4;
  const int G = Q < kTT ? kTT / Q : 1;
  const int PG = (p.P + G - 1) / G;

  for (int s = 1; s <= my_k; ++s) {
    // opaque copies: LDS addresses built from the lane indices are recomputed every iteration
    // instead of being hoisted out of the loop into dozens of registers.  Measured: a gain for
    // the shapes with few row blocks per wavefront; with many row blocks the matrix-instruction
    // loops are issue-bound and run faster on hoisted addresses.
    if constexpr (KBI <= 4) asm volatile("" : "+v"(n16), "+v"(q4));
    // (a) start the features of iteration s+1 (rows drawn one iteration ago) towards the
    // registers: their issue stalls once the memory pipeline is full, and the matrix products
    // of the forward slice below do not need that pipeline
    if constexpr (PF > 0) {
      if (s < my_k) gather_issue(rows_ahead + ((s + 1) & 1) * MR);
    }
    // (c) forward slice: contraction index of MFMA step q is k = 16 kb + 4 q4 + q.  Row blocks
    // past the last one hold zero weights and re-read the last block, so the loop is branch-free.
    {
      f32x4_t acc[MT][NT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
      // the A fragments of row block kbi+1 are read from LDS while block kbi is multiplied; the
      // scheduling fence keeps the compiler from hoisting every block's reads (and their
      // registers) to the top
      auto load_a = [&](int kbi, f32x4_t (&a)[MT]) {
        const int kb = min(wave + kTW * kbi, KB - 1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          a[mt] = *reinterpret_cast<const f32x4_t*>(X + (size_t)(mt * 16 + n16) * ldx + 16 * kb + 4 * q4);
      };
      f32x4_t a_cur[MT], a_nxt[MT];
      load_a(0, a_cur);
#pragma unroll
      for (int kbi = 0; kbi < KBI; ++kbi) {
        if (kbi + 1 < KBI) load_a(kbi + 1, a_nxt);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[mt][nt] = mfma16(a_cur[mt][q], w1[kbi][nt][q], acc[mt][nt]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a_cur[mt] = a_nxt[mt];
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
    for (int e = tid; e < MR * W; e += kTT) {
      const int b = e / W, n = e % W;
      float z = b1[n];
#pragma unroll
      for (int w = 0; w < kTW; ++w) z += red[w * MR * W + e];          // wavefronts in order
      h[e] = b < B ? act2_fwd(z, p.act) : 0.0f;
    }
    __syncthreads();
    // (d) this slice's contribution to the logits, one 16 x 16 block per wavefront on the matrix
    // cores: part[b][c] = sum_n h[b][n] W_2[n][c]  (rows b >= B of h are zero)
    float* my_part = p.part + (((size_t)(s & 1) * p.n_workers + i) * p.P + j) * part_team;
    {
      const int ctiles = D2P >> 4;
      for (int tile = wave; tile < MT * ctiles; tile += kTW) {
        const int mt = tile / ctiles, ct = tile - mt * ctiles;
        f32x4_t g = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int u = 0; u < NT * 4; ++u)
          g = mfma16(h[(mt * 16 + n16) * W + 4 * u + q4], w2[(4 * u + q4) * D2P + ct * 16 + n16], g);
        // agent-scope stores: visible to the other compute units without flushing whole caches
#pragma unroll
        for (int v = 0; v < 4; ++v)
          __hip_atomic_store(my_part + (mt * 16 + 4 * q4 + v) * D2P + ct * 16 + n16, g[v], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
      }
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
        if (++spins > p.spin_limit ||
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
    // (f) sum the P partial blocks.  The other members wrote them through to the coherence
    // point; reading them with agent-scope (sc1) 16-byte buffer loads never returns a copy
    // cached before the arrivals just observed, and needs no cache-wide invalidate.
    {
      const float* team_part = p.part + (((size_t)(s & 1) * p.n_workers + i) * p.P) * part_team;
      const __amdgpu_buffer_rsrc_t team_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<float*>(team_part), 0, (int)(p.P * part_team * sizeof(float)), 0x00020000);
      float* lgp = red;                                    // [G][MR * D2P] group sums
      for (int w0 = tid; w0 < G * Q; w0 += kTT) {          // one pass when Q <= 512
        const int g = w0 / Q, q = w0 - g * Q;
        const int j_lo = g * PG, j_hi = min(p.P, j_lo + PG);
        f32x4_t sum = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
        for (int j0 = j_lo; j0 < j_hi; j0 += 8) {
          u32x4_t v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int jj = j0 + u < j_hi ? j0 + u : j_lo;
            v[u] = __builtin_amdgcn_raw_buffer_load_b128(
                team_rsrc, (int)((jj * part_team + 4 * q) * sizeof(float)), 0, kAgentScope);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (j0 + u < j_hi) sum += __builtin_bit_cast(f32x4_t, v[u]);
        }
        *reinterpret_cast<f32x4_t*>(lgp + (size_t)g * MR * D2P + 4 * q) = sum;
      }
    }
    __syncthreads();
    // logits = b_2 + group sums in order; softmax cross-entropy head, 16 lanes per minibatch
    // row, lane l holding classes l, l + 16, l + 32, l + 48 (d_2 <= 64)
    {
      const float* lgp = red;
      const int l16 = tid & 15;
      for (int b = tid >> 4; b < MR; b += kTT / 16) {
        float* row = lg + b * D2P;
        if (b < B) {
          float z[4];
          float mx = -INFINITY;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int c = l16 + 16 * q;
            z[q] = -INFINITY;
            if (c < d2) {
              float sum = b2[c];
              for (int g = 0; g < G; ++g) sum += lgp[(size_t)g * MR * D2P + b * D2P + c];
              z[q] = sum;
              mx = fmaxf(mx, sum);
            }
          }
          mx = row16_max(mx);
          float ex[4];
          float se = 0.0f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            ex[q] = (l16 + 16 * q < d2) ? expf(z[q] - mx) : 0.0f;
            se += ex[q];
          }
          se = row16_sum(se);
          const float inv_se = __builtin_amdgcn_rcpf(se);    // 1 <= se <= 64; one ulp
          const int y = ylab[b];
          const bool y_ok = y >= 0 && y < d2;               // an out-of-range label selects nothing
          if (j == 0 && l16 == (y_ok ? (y & 15) : 0)) {
            const int yq = y_ok ? (y >> 4) : 0;
            const float zy = !y_ok ? 0.0f : yq == 0 ? z[0] : yq == 1 ? z[1] : yq == 2 ? z[2] : z[3];
            p.row_loss[(size_t)i * B + b] = (mx + logf(se)) - zy;
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int c = l16 + 16 * q;
            if (c < D2P) row[c] = c < d2 ? (ex[q] * inv_se - (c == y ? 1.0f : 0.0f)) * inv_b : 0.0f;
          }
        } else {
          for (int c = l16; c < D2P; c += 16) row[c] = 0.0f;
        }
      }
    }
    __syncthreads();
    // (g) delta_1 slice (needs the pre-update W_2), then the small updates
    for (int e = tid; e < MR * W; e += kTT) {
      const int b = e / W, n = e % W;
      float sum = 0.0f;
      for (int c = 0; c < D2P; c += 4) {
        const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(lg + b * D2P + c);
        const f32x4_t w4 = *reinterpret_cast<const f32x4_t*>(w2 + n * D2P + c);
        sum = fmaf(d4.x, w4.x, sum); sum = fmaf(d4.y, w4.y, sum);
        sum = fmaf(d4.z, w4.z, sum); sum = fmaf(d4.w, w4.w, sum);
      }
      dl1[e] = sum * act2_bwd(h[e], p.act);
    }
    // dW_2 = h^T delta_2 (one 16 x 16 block per wavefront) and db_2 = column sums of delta_2 (a
    // product with a matrix of ones) on the matrix cores, kept in registers until every read of
    // the old W_2 above is done.  Rows b >= B of delta_2 are zero.
    const int ctiles2 = D2P >> 4;
    const bool has_w = wave < NT * ctiles2;                       // NT * ctiles2 <= 8 wavefronts
    const int nt_w = wave / ctiles2, ct_w = wave - nt_w * ctiles2;
    const int ct_b = kTW - 1 - wave;                              // db_2 blocks go to the last wavefronts
    const bool has_b2 = ct_b < ctiles2;
    f32x4_t gw = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f}, gb2 = gw;
    if (has_w) {
#pragma unroll
      for (int u = 0; u < MT * 4; ++u)
        gw = mfma16(h[(4 * u + q4) * W + nt_w * 16 + n16], lg[(4 * u + q4) * D2P + ct_w * 16 + n16], gw);
    }
    if (has_b2) {
#pragma unroll
      for (int u = 0; u < MT * 4; ++u) gb2 = mfma16(1.0f, lg[(4 * u + q4) * D2P + ct_b * 16 + n16], gb2);
    }
    __syncthreads();
    if (has_w) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int e = (nt_w * 16 + 4 * q4 + v) * D2P + ct_w * 16 + n16;
        float g = gw[v];
        if constexpr (MOM) { g = fmaf(p.mu, vw2[e], g); vw2[e] = g; }
        w2[e] = fmaf(-p.lr, g, w2[e]);
      }
    }
    if (has_b2 && q4 == 0) {
      float g = gb2[0];
      if constexpr (MOM) { g = fmaf(p.mu, vb2[ct_b * 16 + n16], g); vb2[ct_b * 16 + n16] = g; }
      b2[ct_b * 16 + n16] = fmaf(-p.lr, g, b2[ct_b * 16 + n16]);
    }
    if (wave >= 2 && wave < 2 + NT) {                             // db_1 = column sums of delta_1
      const int nt_b = wave - 2;
      f32x4_t gb1 = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int u = 0; u < MT * 4; ++u) gb1 = mfma16(1.0f, dl1[(4 * u + q4) * W + nt_b * 16 + n16], gb1);
      if (q4 == 0) {
        float g = gb1[0];
        if constexpr (MOM) { g = fmaf(p.mu, vb1[nt_b * 16 + n16], g); vb1[nt_b * 16 + n16] = g; }
        b1[nt_b * 16 + n16] = fmaf(-p.lr, g, b1[nt_b * 16 + n16]);
      }
    }
    // (h) dW_1 slice and eq. (3) in registers: contraction index of MFMA step u is b = 4u + q4
    {
      float dfr[MT * 4][NT];
#pragma unroll
      for (int u = 0; u < MT * 4; ++u)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) dfr[u][nt] = dl1[(4 * u + q4) * W + nt * 16 + n16];
      auto load_x = [&](int kbi, float (&a)[MT * 4]) {
        const int kb = min(wave + kTW * kbi, KB - 1);
#pragma unroll
        for (int u = 0; u < MT * 4; ++u) a[u] = X[(size_t)(4 * u + q4) * ldx + 16 * kb + n16];
      };
      float x_cur[MT * 4], x_nxt[MT * 4];
      load_x(0, x_cur);
#pragma unroll
      for (int kbi = 0; kbi < KBI; ++kbi) {
        if (kbi + 1 < KBI) load_x(kbi + 1, x_nxt);
        f32x4_t g[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) g[nt] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int u = 0; u < MT * 4; ++u)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) g[nt] = mfma16(x_cur[u], dfr[u][nt], g[nt]);
        const bool live = wave + kTW * kbi < KB;           // blocks past the end keep zero weights
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float gv = g[nt][v];
            if constexpr (MOM) {
              gv = live ? fmaf(p.mu, vw1[kbi][nt][v], gv) : 0.0f;
              vw1[kbi][nt][v] = gv;
            }
            w1[kbi][nt][v] = live ? fmaf(-p.lr, gv, w1[kbi][nt][v]) : 0.0f;
          }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < MT * 4; ++u) x_cur[u] = x_nxt[u];
      }
    }
    __syncthreads();                                     // X and the small buffers are free
    // (i) the next minibatch takes its place
    if (s < my_k) {
      if constexpr (PF > 0) {
        const int* rows_next = rows_ahead + ((s + 1) & 1) * MR;
        gather_store();
        if (tid < B) {
          rows[tid] = rows_next[tid];
          ylab[tid] = lab_next;
          if (s + 1 < my_k) {                            // rows and labels of iteration s+2 (other slot)
            const int r = sample_row(p.seed, (uint32_t)i, p.t0 + (uint64_t)s + 2, (uint32_t)tid, p.log2n);
            rows_ahead[(s & 1) * MR + tid] = r;
            lab_next = lab[r];
          }
        }
      } else {
        if (tid < B) {
          const int r = sample_row(p.seed, (uint32_t)i, p.t0 + (uint64_t)s + 1, (uint32_t)tid, p.log2n);
          rows[tid] = r;
          ylab[tid] = lab[r];
        }
        __syncthreads();
        gather_direct();
        gather_direct_wait();
      }
      __syncthreads();
    }
  }

  if (aborted) return;
  // ---- write the slice back ------------------------------------------------------------------
#pragma unroll
  for (int kbi = 0; kbi < KBI; ++kbi) {
    const int kb = wave + kTW * kbi;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = 16 * kb + 4 * q4 + q;
        if (kb < KB && k < d0) prm[p.w1_off + (size_t)k * p.ld1 + j * W + nt * 16 + n16] = w1[kbi][nt][q];
      }
  }
  for (int e = tid; e < W * D2P; e += kTT) {
    const int n = e / D2P, c = e % D2P;
    if (c < d2) prm[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] = w2[e];
  }
  if (tid < W) prm[p.b1_off + j * W + tid] = b1[tid];
  if constexpr (MOM) {
#pragma unroll
    for (int kbi = 0; kbi < KBI; ++kbi) {
      const int kb = wave + kTW * kbi;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int k = 16 * kb + 4 * q4 + q;
          if (kb < KB && k < d0) vel[p.w1_off + (size_t)k * p.ld1 + j * W + nt * 16 + n16] = vw1[kbi][nt][q];
        }
    }
    for (int e = tid; e < W * D2P; e += kTT) {
      const int n = e / D2P, c = e % D2P;
      if (c < d2) vel[p.w2_off + (size_t)(j * W + n) * p.ld2 + c] = vw2[e];
    }
    if (tid < W) vel[p.b1_off + j * W + tid] = vb1[tid];
    if (j == 0 && tid < d2) vel[p.b2_off + tid] = vb2[tid];
  }
  if (j == 0) {
    if (tid < d2) prm[p.b2_off + tid] = b2[tid];
    if (tid < B) p.idx[(size_t)i * B + tid] = rows[tid];
    if (tid == 0) *base_slot = base + (unsigned)p.P * (unsigned)my_k;   // all arrivals are in
  }
}

// ---- host side --------------------------------------------------------------------------------
size_t fused2_lds_bytes(const Fused2Plan& pl) {
  const size_t MR = (size_t)pl.MT * 16, W = (size_t)pl.NT * 16;
  size_t floats = MR * pl.ldx + kTW * MR * W + 2 * MR * W + MR * pl.d2p + W * pl.d2p + W + pl.d2p +
                  4 * MR + 4;
  if (pl.momentum) floats += W * pl.d2p + W + pl.d2p;
  return floats * sizeof(float);
}

template <int KBI, int NT, int MT> static const void* fused2_symbol(bool mom) {
  return mom ? reinterpret_cast<const void*>(mlp2_epoch_kernel<KBI, NT, MT, true>)
             : reinterpret_cast<const void*>(mlp2_epoch_kernel<KBI, NT, MT, false>);
}

static const void* fused2_pick(int kbi, int nt, int mt, bool mom) {
#define PICK(K, N, M) if (kbi == K && nt == N && mt == M) return fused2_symbol<K, N, M>(mom);
  PICK(2, 1, 1) PICK(2, 1, 2) PICK(2, 1, 4) PICK(2, 2, 1) PICK(2, 2, 2) PICK(2, 2, 4)
  PICK(4, 1, 1) PICK(4, 1, 2) PICK(4, 1, 4) PICK(4, 2, 1) PICK(4, 2, 2) PICK(4, 2, 4)
  PICK(7, 1, 1) PICK(7, 1, 2) PICK(7, 1, 4) PICK(7, 2, 1) PICK(7, 2, 2) PICK(7, 2, 4)
  PICK(8, 1, 1) PICK(8, 1, 2) PICK(8, 1, 4) PICK(8, 2, 1) PICK(8, 2, 2) PICK(8, 2, 4)
#undef PICK
  return nullptr;
}

// Decides whether the epoch kernel applies and how the team is shaped.  It needs every
// workgroup of the grid resident at once (checked against the occupancy the runtime reports).
bool fused2_plan(int n_workers, int d0, int d1, int d2, int batch, bool momentum, Fused2Plan* pl) {
  if (d0 < 4 || (d0 & 3) != 0 || d0 > 1024 || (d1 & 15) != 0 || d2 > 64 || batch > 64) return false;
  pl->momentum = momentum ? 1 : 0;
  pl->MT = batch <= 16 ? 1 : batch <= 32 ? 2 : 4;
  const int kb = (d0 + 15) / 16, kbi_need = (kb + kTW - 1) / kTW;
  pl->KBI = kbi_need <= 2 ? 2 : kbi_need <= 4 ? 4 : kbi_need <= 7 ? 7 : 8;
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
    const void* sym = fused2_pick(pl->KBI, pl->NT, pl->MT, momentum);
    if (sym == nullptr) return false;
    if (hipFuncSetAttribute(sym, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return false;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sym, kTT, lds_bytes) != hipSuccess)
      return false;
    if ((long)n_workers * pl->P <= (long)per_cu * cus) return true;
  }
  return false;
}

hipError_t launch_fused2(const Fused2Plan& pl, Fused2Args args, hipStream_t s) {
  const void* sym = fused2_pick(pl.KBI, pl.NT, pl.MT, pl.momentum != 0);
  if (sym == nullptr) return hipErrorInvalidValue;
  if ((pl.momentum != 0) != (args.vel != nullptr)) return hipErrorInvalidValue;
  args.P = pl.P;
  args.d2p = pl.d2p;
  args.ldx = pl.ldx;
  void* kargs[] = {&args};
  // Plain launch: fused2_plan has checked that the whole grid fits on an otherwise idle device at
  // once, and a team member that never shows up (other work holding compute units) ends in the
  // kernel's bounded wait and the abort flag, not in a hang.
  return hipLaunchKernel(sym, dim3((unsigned)(args.n_workers * pl.P)), dim3(kTT), kargs,
                         fused2_lds_bytes(pl), s);
}

}  // namespace prsgd
