// Backward step of the FIRST layer fused with the forward product of the NEXT iteration.
//
// Layer 1 has no delta to pass down, and it is the last kernel of an iteration's backward pass; the
// first kernel of the next iteration's forward pass reads exactly the weights it has just written,
//   H_1^{t+1} = phi(X^{t+1} bf16(W_1^{t}) + b_1^{t}),
// and the minibatch X^{t+1} is already there (zeta_i^{t+1} is drawn during iteration t; it depends
// on nothing iteration t computes).  So the pass over the fp32 master that applies eq. (3),
//   dW_1 = X^{t T} D_1,  db_1 = colsum(D_1),  W_1 <- W_1 - gamma dW_1,  b_1 <- b_1 - gamma db_1,
// also feeds the updated tile, rounded to bf16 in registers (the shadow's value), to the matrix cores
// for the next forward product: W_1 crosses HBM once per iteration instead of twice (the stand-alone
// forward launch and its read of the bf16 shadow are gone).
//
// For the contraction of X^{t+1} W_1 over the rows k of W_1 to stay inside one workgroup, the walk is
// transposed against the other layers' kernel: a workgroup (4 wavefronts) owns 64 COLUMNS n of W_1 of
// one replica and walks down all rows in tiles of 64.  D_1[:, n-band] stays in LDS and the B x 64
// accumulators of the next pre-activation stay in registers; per tile it stages X^t[:, k-tile] and
// X^{t+1}[:, k-tile] (both L2-resident), forms the dW tile, passes it through LDS into the row-major
// layout of the 16-byte weight loads, writes master and shadow, and multiplies X^{t+1}[:, k-tile] with
// the new tile.  Every output block accumulates over k in the order of the stand-alone forward
// product, and the bias is summed as in the other layers' kernel, so H_1^{t+1} and the parameters
// have the bits the two separate launches give.  Whole tiles only (B = 32 MB, d_0 and d_1 multiples
// of 64); straight-line memory operations, first and last two steps peeled, as in the whole-tile
// kernel of the other layers.
#include <atomic>

#include "prsgd_internal.h"

namespace prsgd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

namespace {

constexpr int BT = 64;              // tile edge: weight rows per step, weight columns per workgroup
constexpr int SD = BT + 16;         // LDS row stride of the D_1 band   [b][n]  (bf16 elements)
constexpr int SH = BT + 16;         // LDS row stride of the X^t tile   [b][k]
constexpr int SX = BT + 8;          // LDS row stride of the X^{t+1} tile [b][k] (contraction-contiguous reads)
constexpr int SW = BT + 32;         // LDS row stride of the new W tile [k][n]  (transpose reads)
constexpr int SG = BT + 4;          // LDS row stride of the dW tile    [k][n]  (floats)

__device__ __forceinline__ f32x16_t mfma_bf16(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float act_from_z(float z, int act) {
  return act == PRSGD_TANH ? tanhf(z) : fmaxf(z, 0.0f);
}

constexpr size_t first_lds_bytes(int mb) {
  const size_t br = 32 * (size_t)mb;
  const size_t hk = sizeof(uint16_t) * br * SH, gl = sizeof(float) * BT * SG;
  return sizeof(uint16_t) * (br * SD + br * SX + BT * SW) + (hk > gl ? hk : gl) + sizeof(float) * 5 * BT;
}

// MB: 32-row tiles of the minibatch (B = 32 MB).  NT: non-temporal weight traffic.  SHW: also write
// the bf16 shadow of W_1 (only the stand-alone forward product reads it; the caller may leave it
// stale while this kernel supplies H_1, and refresh it when that chain breaks).  MOM: momentum form
// of the local update, v <- mu v + G, x <- x - gamma v, with the velocity tile streamed beside the
// weights.
template <int MB, bool NT, bool SHW, bool MOM>
__global__ __launch_bounds__(kThreads) void bwd_first_fwd_kernel(BwdArgs p) {
  constexpr int BR = 32 * MB;
  constexpr int S = 2;                                // weight tiles in flight
  constexpr int NZ = (2 * MB + 3) / 4;                // next-activation blocks (32 x 32) per wavefront

  const int bands = p.Nn / BT;
  int g, band;
  if ((p.n_groups & 7) == 0) {                        // all bands of a replica on one XCD
    const int slot = blockIdx.x >> 3;
    g = (blockIdx.x & 7) + 8 * (slot / bands);
    band = slot % bands;
  } else {
    g = blockIdx.x / bands;
    band = blockIdx.x % bands;
  }
  const int n0 = band * BT;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr size_t kHkBytes = sizeof(uint16_t) * BR * SH, kGlBytes = sizeof(float) * BT * SG;
  uint16_t* Dn = reinterpret_cast<uint16_t*>(smem);                      // [BR][SD]  D_1 band, resident
  uint16_t* Hk = Dn + BR * SD;                                           // [BR][SH]  X^t tile ...
  float* Gl = reinterpret_cast<float*>(Hk);                              // ... and, after it, the dW tile [BT][SG]
  uint16_t* Xk = reinterpret_cast<uint16_t*>(reinterpret_cast<unsigned char*>(Hk) +
                                             (kHkBytes > kGlBytes ? kHkBytes : kGlBytes));   // [BR][SX]
  uint16_t* Wl = Xk + BR * SX;                                           // [BT][SW]  new W tile, bf16
  float* Bs = reinterpret_cast<float*>(Wl + BT * SW);                    // [4][BT] partial column sums
  float* Bn = Bs + 4 * BT;                                               // [BT]    new bias of the band

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr32 = lane & 31, kb = lane >> 5;
  const int wk = wave >> 1, wn = wave & 1;

  const uint16_t* h_g = p.h + (size_t)g * p.h_gs;               // X^t      [B][ldh]
  const uint16_t* x_g = p.x_next + (size_t)g * p.x_gs;          // X^{t+1}  [B][ldx]
  const uint16_t* d_g = p.d + (size_t)g * p.d_gs;               // D_1      [B][ldd]
  float* w_g = p.params + (size_t)g * p.p_gs + p.w_off;
  uint16_t* s_g = SHW ? p.shadow + (size_t)g * p.p_gs + p.w_off : nullptr;
  const float* wsrc_g = p.src + (size_t)g * p.src_gs + p.w_off;
  float* v_g = MOM ? p.vel + (size_t)g * p.p_gs + p.w_off : nullptr;
  const bool nt_read = NT && p.src_gs != 0;           // a shared source is re-read by every replica

  const int prow = tid >> 3, pcol = (tid & 7) * 8;              // panels: row q*32 + prow
  const int wrow = tid >> 4, wcol = 4 * (tid & 15);             // weights: row q*16 + wrow
  auto fetch_panel = [&](u32x4_t (&reg)[MB], const uint16_t* src, int ld, int col0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < MB; ++q)
      reg[q] = *reinterpret_cast<const u32x4_t*>(src + (size_t)(q * 32 + prow) * ld + col0 + pcol);
  };
  auto stash_panel = [&](uint16_t* lds, int stride, const u32x4_t (&reg)[MB]) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < MB; ++q)
      *reinterpret_cast<u32x4_t*>(lds + (q * 32 + prow) * stride + pcol) = reg[q];
  };
  auto fetch_w = [&](f32x4_t (&reg)[4], int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4_t* src =
          reinterpret_cast<const f32x4_t*>(wsrc_g + (size_t)(k0 + q * 16 + wrow) * p.ldw + n0 + wcol);
      reg[q] = nt_read ? __builtin_nontemporal_load(src) : *src;
    }
  };
  auto fetch_v = [&](f32x4_t (&reg)[4], int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4_t* src =
          reinterpret_cast<const f32x4_t*>(v_g + (size_t)(k0 + q * 16 + wrow) * p.ldw + n0 + wcol);
      reg[q] = NT ? __builtin_nontemporal_load(src) : *src;
    }
  };

  const int n_t = p.K / BT;                           // steps of the walk down the rows
  u32x4_t hr[MB], xr[MB];
  f32x4_t wr[S][4];
  f32x4_t vr[MOM ? S : 1][4];
  fetch_panel(hr, d_g, p.ldd, n0);                    // the D_1 band first (through hr)
  fetch_w(wr[0], 0);
  if (MOM) fetch_v(vr[0], 0);
  stash_panel(Dn, SD, hr);
  fetch_panel(hr, h_g, p.ldh, 0);
  fetch_panel(xr, x_g, p.ldx, 0);
  fetch_w(wr[1], BT);
  if (MOM) fetch_v(vr[1], BT);
  __syncthreads();

  // b_1 <- b_1 - gamma db_1: four quarter sums over the minibatch rows, added in order
  {
    float cs = 0.0f;
#pragma unroll 8
    for (int b = wave * (BR / 4); b < (wave + 1) * (BR / 4); ++b) cs += bf16_to_f32(Dn[b * SD + lane]);
    Bs[wave * BT + lane] = cs;
  }
  __syncthreads();
  if (tid < BT) {
    float cs = ((Bs[tid] + Bs[BT + tid]) + Bs[2 * BT + tid]) + Bs[3 * BT + tid];
    const size_t bo = p.b_off + (size_t)n0 + tid;
    if (MOM) {
      float* vb = p.vel + (size_t)g * p.p_gs + bo;
      cs = fmaf(p.mu, *vb, cs);
      *vb = cs;
    }
    const float b_new = fmaf(-p.lr, cs, p.src[(size_t)g * p.src_gs + bo]);
    p.params[(size_t)g * p.p_gs + bo] = b_new;
    Bn[tid] = b_new;
  }

  f32x16_t acc_z[NZ];
#pragma unroll
  for (int t = 0; t < NZ; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_z[t][v] = 0.0f;

  // One step of the walk: rows k0 .. k0 + 63 of the band.  PF: fetch the weight tile S steps ahead.
  // NEXT: fetch the next minibatch tiles.  (Both flags are literal at every call site.)
  auto tile_step = [&](int it, f32x4_t (&wr)[4], f32x4_t (&vr)[4], const bool PF, const bool NEXT) __attribute__((always_inline)) {
    const int k0 = it * BT;
    stash_panel(Hk, SH, hr);
    stash_panel(Xk, SX, xr);
    __syncthreads();
    if (NEXT) {
      fetch_panel(hr, h_g, p.ldh, k0 + BT);
      fetch_panel(xr, x_g, p.ldx, k0 + BT);
    }
    // dW tile [k][n] = X^t[:, k-tile]^T D_1[:, n-band]: contraction over the minibatch
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < BR / 16; ++kk)
      acc = mfma_bf16(frag_trans(Hk, SH, wk * 32, kk, lane), frag_trans(Dn, SD, wn * 32, kk, lane), acc);
    __syncthreads();                                  // the dW tile takes the place of the X^t tile
#pragma unroll
    for (int v = 0; v < 16; ++v)
      Gl[(wk * 32 + 8 * (v / 4) + 4 * kb + (v % 4)) * SG + wn * 32 + lr32] = acc[v];
    __syncthreads();
    // eq. (3) on the tile, in the layout of the weight loads; the new tile also goes to LDS as bf16
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = q * 16 + wrow;
      f32x4_t gr = *reinterpret_cast<const f32x4_t*>(Gl + row * SG + wcol);
      const size_t off = (size_t)(k0 + row) * p.ldw + n0 + wcol;
      if (MOM) {
        gr.x = fmaf(p.mu, vr[q].x, gr.x);
        gr.y = fmaf(p.mu, vr[q].y, gr.y);
        gr.z = fmaf(p.mu, vr[q].z, gr.z);
        gr.w = fmaf(p.mu, vr[q].w, gr.w);
        if (NT) __builtin_nontemporal_store(gr, reinterpret_cast<f32x4_t*>(v_g + off));
        else *reinterpret_cast<f32x4_t*>(v_g + off) = gr;
      }
      f32x4_t w = wr[q];
      w.x = fmaf(-p.lr, gr.x, w.x);
      w.y = fmaf(-p.lr, gr.y, w.y);
      w.z = fmaf(-p.lr, gr.z, w.z);
      w.w = fmaf(-p.lr, gr.w, w.w);
      const u32x2_t hv2 = {(uint32_t)f32_to_bf16_rne(w.x) | ((uint32_t)f32_to_bf16_rne(w.y) << 16),
                           (uint32_t)f32_to_bf16_rne(w.z) | ((uint32_t)f32_to_bf16_rne(w.w) << 16)};
      if (NT) {
        __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t*>(w_g + off));
        if (SHW) __builtin_nontemporal_store(hv2, reinterpret_cast<u32x2_t*>(s_g + off));
      } else {
        *reinterpret_cast<f32x4_t*>(w_g + off) = w;
        if (SHW) *reinterpret_cast<u32x2_t*>(s_g + off) = hv2;
      }
      *reinterpret_cast<u32x2_t*>(Wl + row * SW + wcol) = hv2;
    }
    __syncthreads();
    // next pre-activation [b][n] += X^{t+1}[:, k-tile] bf16(W_new tile): contraction over k
#pragma unroll
    for (int t = 0; t < NZ; ++t) {
      const int blk = wave + 4 * t;
      if (blk < 2 * MB) {
        const int mb = blk >> 1, nblk = blk & 1;
#pragma unroll
        for (int kk = 0; kk < BT / 16; ++kk)
          acc_z[t] = mfma_bf16(frag_contig(Xk, SX, mb * 32, kk, lane), frag_trans(Wl, SW, nblk * 32, kk, lane),
                               acc_z[t]);
      }
    }
    if (PF) {
      fetch_w(wr, k0 + S * BT);
      if (MOM) fetch_v(vr, k0 + S * BT);
    }
    __syncthreads();                                  // the tiles in LDS are rewritten by the next step
  };

  int it = 0;
#pragma unroll
  for (int st = 0; st < S; ++st) tile_step(st, wr[st], vr[MOM ? st : 0], true, true);
  for (it = S; it < n_t - S; it += S) {
#pragma unroll
    for (int st = 0; st < S; ++st) tile_step(it + st, wr[st], vr[MOM ? st : 0], true, true);
  }
#pragma unroll
  for (int st = 0; st < S; ++st)                      // the last S tiles: nothing left to prefetch
    tile_step(it + st, wr[st], vr[MOM ? st : 0], false, st + 1 < S);

  // ---- H_1^{t+1} = phi(Z + b_1) for this band ------------------------------------------------------
  uint16_t* hn_g = p.h_next + (size_t)g * p.hn_gs;
#pragma unroll
  for (int t = 0; t < NZ; ++t) {
    const int blk = wave + 4 * t;
    if (blk < 2 * MB) {
      const int mb = blk >> 1, nblk = blk & 1;
      const int n = nblk * 32 + lr32;
      const float bn = Bn[n];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int b = mb * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
        hn_g[(size_t)b * p.ldhn + n0 + n] = f32_to_bf16_rne(act_from_z(acc_z[t][v] + bn, p.act));
      }
    }
  }
}

template <int MB, bool SHW, bool MOM>
hipError_t launch_first_one(const BwdArgs& p, hipStream_t s) {
  constexpr size_t kLds = first_lds_bytes(MB);
  static std::atomic<bool> configured{false};
  if (!configured.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_first_fwd_kernel<MB, true, SHW, MOM>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_first_fwd_kernel<MB, false, SHW, MOM>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e != hipSuccess) return e;
    configured.store(true, std::memory_order_release);
  }
  const int bands = p.Nn / BT;
  if (p.streaming)
    hipLaunchKernelGGL((bwd_first_fwd_kernel<MB, true, SHW, MOM>), dim3((unsigned)(bands * p.n_groups)),
                       dim3(kThreads), kLds, s, p);
  else
    hipLaunchKernelGGL((bwd_first_fwd_kernel<MB, false, SHW, MOM>), dim3((unsigned)(bands * p.n_groups)),
                       dim3(kThreads), kLds, s, p);
  return hipGetLastError();
}

template <int MB>
hipError_t launch_first_mb(const BwdArgs& p, hipStream_t s) {
  const bool shw = p.shadow != nullptr, mom = p.vel != nullptr;
  if (mom) return shw ? launch_first_one<MB, true, true>(p, s) : launch_first_one<MB, false, true>(p, s);
  return shw ? launch_first_one<MB, true, false>(p, s) : launch_first_one<MB, false, false>(p, s);
}

}  // namespace

// Whole tiles, every worker active, and the buffers of the next iteration given.
bool bwd_first_fwd_applies(const BwdArgs& p) {
  if (p.B != 32 && p.B != 64 && p.B != 128) return false;
  if (p.K < 4 * BT || (p.K % (2 * BT)) != 0 || p.Nn < BT || (p.Nn % BT) != 0) return false;
  if (p.worker_steps != nullptr || p.dx != nullptr) return false;
  if (p.x_next == nullptr || p.h_next == nullptr) return false;   // shadow == nullptr: it is left stale
  return (p.ldw % 4) == 0 && (p.ldh % 8) == 0 && (p.ldx % 8) == 0 && (p.ldd % 8) == 0 && (p.w_off % 4) == 0;
}

hipError_t launch_bwd_first_fwd(const BwdArgs& p, hipStream_t s) {
  if (!bwd_first_fwd_applies(p) || p.n_groups <= 0) return hipErrorInvalidValue;
  if (p.B == 32) return launch_first_mb<1>(p, s);
  if (p.B == 64) return launch_first_mb<2>(p, s);
  return launch_first_mb<4>(p, s);
}

}  // namespace prsgd
