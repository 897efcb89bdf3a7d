// One pass over a layer's weights for the whole backward step of the per-worker MLP gradient
//   G_i^t = grad F_i(x_i^{t-1}; zeta_i^t)   and the local update   x_i <- x_i - gamma G_i   (eq. 3)
// with bfloat16 matrix operands:
//   dW_l     = H_{l-1}^T D_l,   db_l = colsum(D_l)
//   W_l     <- W_l - gamma dW_l,   b_l <- b_l - gamma db_l        (fp32 master + bf16 shadow)
//   D_{l-1}  = (D_l bf16(W_l)^T) * phi'(H_{l-1})                  (with the weights before the update)
// Every replica has private weights and only B <= 128 batch rows, so the step is bound by moving
// W_l through HBM.  Computing D_{l-1} from the same fp32 master tile that the update has to read
// anyway (rounded to bf16 in registers: exactly the shadow's value) removes the separate read of
// W_l that a stand-alone backward-data product needs.
//
// A workgroup (4 wavefronts) owns 64 rows k of W_l of one replica and walks over all columns in
// tiles of 64.  H_{l-1}[:, k-rows] stays in LDS for the whole walk and the D_{l-1} accumulators
// (B x 64) stay in registers; per tile it stages D_l[:, n-tile] and bf16(W tile) in LDS, runs both
// products on the matrix cores (v_mfma_f32_32x32x16_bf16), passes the dW tile through LDS into the
// row-major layout of the 16-byte weight loads, and writes master and shadow back.  Weight tiles
// are fetched two tiles ahead, D_l tiles (L2-resident: B x d_l bf16) one tile ahead.  The
// whole-tile variant also comes with 32-row bands, for layers whose 64-row bands would leave
// compute units with a single workgroup and nothing to overlap its waits with.
#include <atomic>

#include "prsgd_internal.h"

namespace prsgd {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

namespace {

constexpr int BMK = 64;            // weight rows (k) per workgroup
constexpr int BN = 64;             // weight columns (n) per tile
constexpr int SH = BMK + 16;       // LDS row stride of H^T panel  [b][k]   (bf16 elements)
constexpr int SD = BN + 16;        // LDS row stride of the D tile [b][n]
constexpr int SW = BN + 8;         // LDS row stride of the W tile [k][n]
constexpr int SG = BN + 4;         // LDS row stride of the dW tile [k][n]  (floats)
#ifndef PRSGD_BWD_STAGES
#define PRSGD_BWD_STAGES 2
#endif

__device__ __forceinline__ f32x16_t mfma_bf16(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float dact_from_h(float h, int act) {
  return act == PRSGD_TANH ? (1.0f - h * h) : (h > 0.0f ? 1.0f : 0.0f);
}

// MB: 32-row tiles of the minibatch held on chip (B <= 32 MB).  DX: also produce D_{l-1}.
// S: weight tiles in flight per workgroup (register sets).  MOM: momentum form of the local
// update, v <- mu v + G, x <- x - gamma v, with the velocity tile streamed beside the weights.
template <int MB, bool DX, int S, bool MOM>
__global__ __launch_bounds__(kThreads) void grouped_bwd_kernel(BwdArgs p) {
  constexpr int BR = 32 * MB;
  constexpr int NTD = DX ? (2 * MB + 3) / 4 : 1;     // D_{l-1} accumulator tiles per wavefront

  // workgroup -> (replica, k-tile); all tiles of a replica on one XCD when N is a multiple of 8
  const int tiles = (p.K + BMK - 1) / BMK;
  int g, tile;
  if ((p.n_groups & 7) == 0) {
    const int slot = blockIdx.x >> 3;
    g = (blockIdx.x & 7) + 8 * (slot / tiles);
    tile = slot % tiles;
  } else {
    g = blockIdx.x / tiles;
    tile = blockIdx.x % tiles;
  }
  if (p.worker_steps != nullptr && p.step >= p.worker_steps[g]) return;
  const int k0 = tile * BMK;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* HT = reinterpret_cast<uint16_t*>(smem);            // [BR][SH]
  uint16_t* Dl = HT + BR * SH;                                 // [BR][SD]
  uint16_t* Wl = Dl + BR * SD;                                 // [BMK][SW]
  float* Gl = reinterpret_cast<float*>(Wl + BMK * SW);         // [BMK][SG]
  float* Bs = Gl + BMK * SG;                                   // [4][BN] partial column sums

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr32 = lane & 31, kb = lane >> 5;

  const uint16_t* h_g = p.h + (size_t)g * p.h_gs;
  const uint16_t* d_g = p.d + (size_t)g * p.d_gs;
  float* w_g = p.params + (size_t)g * p.p_gs + p.w_off;
  uint16_t* s_g = p.shadow + (size_t)g * p.p_gs + p.w_off;
  const float* wsrc_g = p.src + (size_t)g * p.src_gs + p.w_off;     // old weights
  float* v_g = MOM ? p.vel + (size_t)g * p.p_gs + p.w_off : nullptr;   // velocity of W_l
  const bool nt = p.streaming != 0;
  const bool nt_read = nt && p.src_gs != 0;      // a shared source is re-read by every replica

  // ---- staging helpers ---------------------------------------------------------------------
  // B x 64 bf16 panel (H^T columns or a D tile): MB 16-byte vectors per thread, row = q*32 + tid/8
  auto fetch_panel = [&](uint4 (&reg)[MB], const uint16_t* src, int ld, int col0, int n_cols) -> uint32_t {
    uint32_t mask = 0;
#pragma unroll
    for (int q = 0; q < MB; ++q) {
      const int row = q * 32 + (tid >> 3), col = col0 + (tid & 7) * 8;
      const bool ok = row < p.B && col < n_cols;
      reg[q] = *reinterpret_cast<const uint4*>(src + (ok ? (size_t)row * ld + col : (size_t)0));
      mask |= (ok ? 1u : 0u) << q;
    }
    return mask;
  };
  auto stash_panel = [&](uint16_t* lds, int stride, const uint4 (&reg)[MB], uint32_t mask) {
#pragma unroll
    for (int q = 0; q < MB; ++q) {
      const uint32_t keep = 0u - ((mask >> q) & 1u);
      const uint4 v = make_uint4(reg[q].x & keep, reg[q].y & keep, reg[q].z & keep, reg[q].w & keep);
      *reinterpret_cast<uint4*>(lds + (q * 32 + (tid >> 3)) * stride + (tid & 7) * 8) = v;
    }
  };
  // 64 x 64 fp32 weight tile: 4 16-byte vectors per thread, row = q*16 + tid/16, column 4*(tid%16)
  auto fetch_w = [&](f32x4_t (&reg)[4], int n0) -> uint32_t {
    uint32_t mask = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = k0 + q * 16 + (tid >> 4), n = n0 + 4 * (tid & 15);
      const bool ok = k < p.K && n < p.Nn;
      const f32x4_t* src = reinterpret_cast<const f32x4_t*>(wsrc_g + (ok ? (size_t)k * p.ldw + n : (size_t)0));
      reg[q] = nt_read ? __builtin_nontemporal_load(src) : *src;
      mask |= (ok ? 1u : 0u) << q;
    }
    return mask;
  };
  // the velocity tile in the same layout (private to the replica: always a streaming access)
  auto fetch_v = [&](f32x4_t (&reg)[4], int n0, uint32_t mask) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = k0 + q * 16 + (tid >> 4), n = n0 + 4 * (tid & 15);
      const bool ok = (mask >> q) & 1u;
      const f32x4_t* src = reinterpret_cast<const f32x4_t*>(v_g + (ok ? (size_t)k * p.ldw + n : (size_t)0));
      reg[q] = nt ? __builtin_nontemporal_load(src) : *src;
    }
  };
  auto stash_w = [&](const f32x4_t (&reg)[4], uint32_t mask) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool ok = (mask >> q) & 1u;
      uint2 hv;
      hv.x = ok ? ((uint32_t)f32_to_bf16_rne(reg[q].x) | ((uint32_t)f32_to_bf16_rne(reg[q].y) << 16)) : 0u;
      hv.y = ok ? ((uint32_t)f32_to_bf16_rne(reg[q].z) | ((uint32_t)f32_to_bf16_rne(reg[q].w) << 16)) : 0u;
      *reinterpret_cast<uint2*>(Wl + (q * 16 + (tid >> 4)) * SW + 4 * (tid & 15)) = hv;
    }
  };

  // ---- prologue -----------------------------------------------------------------------------
  const int n_t = (p.Nn + BN - 1) / BN;
  // Every workgroup walks all column tiles, each from a different start: workgroups that run in
  // step would otherwise all sit on the same byte offset inside their (power-of-two strided)
  // weight rows, i.e. on the same few memory channels.
  const int rot = (int)(((long)tile * n_t) / tiles + g) % n_t;
  auto col_tile = [&](int i) { const int c = i + rot; return c >= n_t ? c - n_t : c; };
  uint4 pr[MB];
  f32x4_t wr[S][4];
  f32x4_t vr[MOM ? S : 1][4];
  uint32_t wm[S], dm;
  {
    const uint32_t hm = fetch_panel(pr, h_g, p.ldh, k0, p.K);
    wm[0] = fetch_w(wr[0], col_tile(0) * BN);
    if (MOM) fetch_v(vr[0], col_tile(0) * BN, wm[0]);
    stash_panel(HT, SH, pr, hm);
  }
  dm = fetch_panel(pr, d_g, p.ldd, col_tile(0) * BN, p.Nn);
#pragma unroll
  for (int st = 1; st < S; ++st) {
    wm[st] = 0;
    if (st < n_t) {
      wm[st] = fetch_w(wr[st], col_tile(st) * BN);
      if (MOM) fetch_v(vr[st], col_tile(st) * BN, wm[st]);
    }
  }

  f32x16_t acc_dx[NTD];
#pragma unroll
  for (int t = 0; t < NTD; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_dx[t][v] = 0.0f;

  const int wk = wave >> 1, wn = wave & 1;             // this wavefront's 32x32 block of the dW tile
  // db_l: the k-tile workgroups of a replica take the column tiles in turn, so that no
  // workgroup carries all of the bias work (the launch ends with its slowest workgroup)

  // one tile: (wr, wm) holds the weights of tile `it` and is refilled with tile it+S
  auto tile_step = [&](int it, f32x4_t (&wr)[4], f32x4_t (&vr)[4], uint32_t& wm) {
    const int ct = col_tile(it), n0 = ct * BN;
    stash_panel(Dl, SD, pr, dm);
    if (DX) stash_w(wr, wm);
    __syncthreads();
    if (it + 1 < n_t) dm = fetch_panel(pr, d_g, p.ldd, col_tile(it + 1) * BN, p.Nn);

    // dW tile block (wk, wn): contraction over the minibatch
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < BR / 16; ++kk)
      acc = mfma_bf16(frag_trans(HT, SH, wk * 32, kk, lane), frag_trans(Dl, SD, wn * 32, kk, lane), acc);
    // D_{l-1} blocks: contraction over this tile's columns, with the pre-update weights
    if (DX) {
#pragma unroll
      for (int t = 0; t < NTD; ++t) {
        const int blk = wave + 4 * t;
        if (blk < 2 * MB) {
          const int mb = blk >> 1, kblk = blk & 1;
#pragma unroll
          for (int kk = 0; kk < BN / 16; ++kk)
            acc_dx[t] = mfma_bf16(frag_contig(Dl, SD, mb * 32, kk, lane),
                                  frag_contig(Wl, SW, kblk * 32, kk, lane), acc_dx[t]);
        }
      }
    }
    // db: column sums of the (rounded) delta tile; rows beyond B are zero.  Each wavefront sums
    // a quarter of the rows, the four partial sums are added in order after the barrier.
    const bool bias_turn = (ct % tiles) == tile;
    if (bias_turn) {
      float cs = 0.0f;
#pragma unroll 8
      for (int b = wave * (BR / 4); b < (wave + 1) * (BR / 4); ++b) cs += bf16_to_f32(Dl[b * SD + lane]);
      Bs[wave * BN + lane] = cs;
    }
    // accumulator element v of lane (lr32, kb) is C[8 (v/4) + 4 kb + v%4][lr32]
#pragma unroll
    for (int v = 0; v < 16; ++v)
      Gl[(wk * 32 + 8 * (v / 4) + 4 * kb + (v % 4)) * SG + wn * 32 + lr32] = acc[v];
    __syncthreads();

    // eq. (3) on the tile, in the layout of the weight loads
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if ((wm >> q) & 1u) {
        const int row = q * 16 + (tid >> 4), c = 4 * (tid & 15);
        f32x4_t gr = *reinterpret_cast<const f32x4_t*>(Gl + row * SG + c);
        const size_t off = (size_t)(k0 + row) * p.ldw + n0 + c;
        if (MOM) {
          gr.x = fmaf(p.mu, vr[q].x, gr.x);
          gr.y = fmaf(p.mu, vr[q].y, gr.y);
          gr.z = fmaf(p.mu, vr[q].z, gr.z);
          gr.w = fmaf(p.mu, vr[q].w, gr.w);
          if (nt) __builtin_nontemporal_store(gr, reinterpret_cast<f32x4_t*>(v_g + off));
          else *reinterpret_cast<f32x4_t*>(v_g + off) = gr;
        }
        f32x4_t w = wr[q];
        w.x = fmaf(-p.lr, gr.x, w.x);
        w.y = fmaf(-p.lr, gr.y, w.y);
        w.z = fmaf(-p.lr, gr.z, w.z);
        w.w = fmaf(-p.lr, gr.w, w.w);
        uint2 hv;
        hv.x = (uint32_t)f32_to_bf16_rne(w.x) | ((uint32_t)f32_to_bf16_rne(w.y) << 16);
        hv.y = (uint32_t)f32_to_bf16_rne(w.z) | ((uint32_t)f32_to_bf16_rne(w.w) << 16);
        typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t hv2 = {hv.x, hv.y};
        if (nt) {
          __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t*>(w_g + off));
          __builtin_nontemporal_store(hv2, reinterpret_cast<u32x2_t*>(s_g + off));
        } else {
          *reinterpret_cast<f32x4_t*>(w_g + off) = w;
          *reinterpret_cast<u32x2_t*>(s_g + off) = hv2;
        }
      }
    }
    if (bias_turn && tid < BN && n0 + tid < p.Nn) {
      float cs = ((Bs[tid] + Bs[BN + tid]) + Bs[2 * BN + tid]) + Bs[3 * BN + tid];
      if (MOM) {
        float* vb = p.vel + (size_t)g * p.p_gs + p.b_off + n0 + tid;
        cs = fmaf(p.mu, *vb, cs);
        *vb = cs;
      }
      const float b_old = p.src[(size_t)g * p.src_gs + p.b_off + n0 + tid];
      p.params[(size_t)g * p.p_gs + p.b_off + n0 + tid] = fmaf(-p.lr, cs, b_old);
    }
    if (it + S < n_t) {
      wm = fetch_w(wr, col_tile(it + S) * BN);
      if (MOM) fetch_v(vr, col_tile(it + S) * BN, wm);
    }
  };

  for (int base = 0; base < n_t; base += S) {
#pragma unroll
    for (int st = 0; st < S; ++st)
      if (base + st < n_t) tile_step(base + st, wr[st], vr[MOM ? st : 0], wm[st]);
  }

  // ---- D_{l-1} = acc * phi'(H_{l-1}) -------------------------------------------------------
  if (DX) {
    uint16_t* dx_g = p.dx + (size_t)g * p.dx_gs;
#pragma unroll
    for (int t = 0; t < NTD; ++t) {
      const int blk = wave + 4 * t;
      if (blk < 2 * MB) {
        const int mb = blk >> 1, kblk = blk & 1;
        const int k = k0 + kblk * 32 + lr32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int b = mb * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
          if (b < p.B && k < p.K) {
            const float hval = bf16_to_f32(HT[b * SH + kblk * 32 + lr32]);
            dx_g[(size_t)b * p.lddx + k] = f32_to_bf16_rne(acc_dx[t][v] * dact_from_h(hval, p.act));
          }
        }
      }
    }
  }
}

// The same step for layers made of whole tiles only (B = 32 MB, d_{l-1} a multiple of the band
// height KB = 64 or 32, d_l a multiple of 64):
// no masks anywhere, and -- the point of the variant -- every tile step issues the same vector
// memory instructions in the same order on every path: D-tile loads, stores of the updated
// tile, loads of the weight tile S steps ahead.  The hardware counts outstanding memory
// operations in issue order, and the compiler can only leave the younger ones in flight across a
// wait if their number does not depend on the path taken; a conditional load or store anywhere in
// the loop (bounds masks, "is there a next tile", the bias update) makes it wait for everything,
// which serialises the prefetch behind the stores of the previous tile.  So the last S steps are
// peeled off (they prefetch nothing), and the bias work inside the loop touches LDS only: its
// loads and stores run once after the walk.
constexpr int kMaxBiasTiles = 4;   // column tiles whose bias a workgroup may own in this variant

template <int MB, bool DX, int S, bool MOM, bool NT, int KB>
__global__ __launch_bounds__(kThreads) void grouped_bwd_full_kernel(BwdArgs p) {
  constexpr int BR = 32 * MB;
  constexpr int KH = KB / 32;                          // 32-row halves of the band
  constexpr int QW = KB / 16;                          // 16-byte vectors of a weight tile per thread
  constexpr int SHK = KB == 64 ? SH : 32;              // LDS row stride of the H^T panel
  constexpr int NTD = DX ? (KH * MB + 3) / 4 : 1;

  const int tiles = p.K / KB;
  int g, tile;
  if ((p.n_groups & 7) == 0) {
    const int slot = blockIdx.x >> 3;
    g = (blockIdx.x & 7) + 8 * (slot / tiles);
    tile = slot % tiles;
  } else {
    g = blockIdx.x / tiles;
    tile = blockIdx.x % tiles;
  }
  if (p.worker_steps != nullptr && p.step >= p.worker_steps[g]) return;
  const int k0 = tile * KB;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* HT = reinterpret_cast<uint16_t*>(smem);            // [BR][SHK]
  uint16_t* Dl = HT + BR * SHK;                                // [BR][SD]
  uint16_t* Wl = Dl + BR * SD;                                 // [KB][SW]
  float* Gl = reinterpret_cast<float*>(Wl + KB * SW);          // [KB][SG]
  float* Bs = Gl + KB * SG;                                    // [4][BN] partial column sums
  float* Bk = Bs + 4 * BN;                                     // [kMaxBiasTiles][BN] db of owned tiles

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr32 = lane & 31, kb = lane >> 5;

  const uint16_t* h_g = p.h + (size_t)g * p.h_gs;
  const uint16_t* d_g = p.d + (size_t)g * p.d_gs;
  float* w_g = p.params + (size_t)g * p.p_gs + p.w_off;
  uint16_t* s_g = p.shadow + (size_t)g * p.p_gs + p.w_off;
  const float* wsrc_g = p.src + (size_t)g * p.src_gs + p.w_off;
  float* v_g = MOM ? p.vel + (size_t)g * p.p_gs + p.w_off : nullptr;
  const bool nt_read = NT && p.src_gs != 0;      // a shared source is re-read by every replica

  // thread -> (row, 16-byte column) of the panels and of the weight tile
  const int prow = tid >> 3, pcol = (tid & 7) * 8;             // panels: row q*32 + prow
  const int wrow = tid >> 4, wcol = 4 * (tid & 15);            // weights: row q*16 + wrow
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
  auto fetch_w = [&](f32x4_t (&reg)[QW], const float* base, int n0, bool stream) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < QW; ++q) {
      const f32x4_t* src = reinterpret_cast<const f32x4_t*>(base + (size_t)(k0 + q * 16 + wrow) * p.ldw + n0 + wcol);
      reg[q] = stream ? __builtin_nontemporal_load(src) : *src;
    }
  };
  auto stash_w = [&](const f32x4_t (&reg)[QW]) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < QW; ++q) {
      const u32x2_t hv = {(uint32_t)f32_to_bf16_rne(reg[q].x) | ((uint32_t)f32_to_bf16_rne(reg[q].y) << 16),
                          (uint32_t)f32_to_bf16_rne(reg[q].z) | ((uint32_t)f32_to_bf16_rne(reg[q].w) << 16)};
      *reinterpret_cast<u32x2_t*>(Wl + (q * 16 + wrow) * SW + wcol) = hv;
    }
  };

  const int n_t = p.Nn / BN;
  const int rot = (int)(((long)tile * n_t) / tiles + g) % n_t;      // see the general kernel
  auto col_tile = [&](int i) { const int c = i + rot; return c >= n_t ? c - n_t : c; };

  u32x4_t pr[MB];
  f32x4_t wr[S][QW];
  f32x4_t vr[MOM ? S : 1][QW];
  if constexpr (KB == 64) {
    fetch_panel(pr, h_g, p.ldh, k0);
  } else {                                             // a 32-wide panel: four 16-byte vectors per row
#pragma unroll
    for (int q = 0; q < (MB + 1) / 2; ++q)
      if (q * 64 + (tid >> 2) < BR)
        pr[q] = *reinterpret_cast<const u32x4_t*>(h_g + (size_t)(q * 64 + (tid >> 2)) * p.ldh + k0 + (tid & 3) * 8);
  }
  fetch_w(wr[0], wsrc_g, col_tile(0) * BN, nt_read);
  if (MOM) fetch_w(vr[0], v_g, col_tile(0) * BN, NT);
  if constexpr (KB == 64) {
    stash_panel(HT, SHK, pr);
  } else {
#pragma unroll
    for (int q = 0; q < (MB + 1) / 2; ++q)
      if (q * 64 + (tid >> 2) < BR)
        *reinterpret_cast<u32x4_t*>(HT + (q * 64 + (tid >> 2)) * SHK + (tid & 3) * 8) = pr[q];
  }
  fetch_panel(pr, d_g, p.ldd, col_tile(0) * BN);
#pragma unroll
  for (int st = 1; st < S; ++st) {
    fetch_w(wr[st], wsrc_g, col_tile(st) * BN, nt_read);
    if (MOM) fetch_w(vr[st], v_g, col_tile(st) * BN, NT);
  }

  f32x16_t acc_dx[NTD];
#pragma unroll
  for (int t = 0; t < NTD; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_dx[t][v] = 0.0f;

  const int wk = wave >> 1, wn = wave & 1;
  // wavefronts without a block of the weight-gradient tile (32-row bands) take the D_{l-1} blocks first
  const int dxw = KB == 64 ? wave : ((wave + 2) & 3);
  int bias_slot = 0;                                   // owned bias tiles met so far (uniform)

  // PF: fetch the weight tile S steps ahead.  DNEXT: fetch the next D tile.
  // (the two flags are literal at every call site and fold away once the step is inlined)
  auto tile_step = [&](int it, f32x4_t (&wr)[QW], f32x4_t (&vr)[QW], const bool PF, const bool DNEXT) __attribute__((always_inline)) {
    const int ct = col_tile(it), n0 = ct * BN;
    stash_panel(Dl, SD, pr);
    if (DX) stash_w(wr);
    __syncthreads();
    if (DNEXT) fetch_panel(pr, d_g, p.ldd, col_tile(it + 1) * BN);

    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    if (KH == 2 || wk < KH) {
#pragma unroll
      for (int kk = 0; kk < BR / 16; ++kk)
        acc = mfma_bf16(frag_trans(HT, SHK, wk * 32, kk, lane), frag_trans(Dl, SD, wn * 32, kk, lane), acc);
    }
    if (DX) {
#pragma unroll
      for (int t = 0; t < NTD; ++t) {
        const int blk = dxw + 4 * t;
        if (blk < KH * MB) {
          const int mb = blk / KH, kblk = blk % KH;
#pragma unroll
          for (int kk = 0; kk < BN / 16; ++kk)
            acc_dx[t] = mfma_bf16(frag_contig(Dl, SD, mb * 32, kk, lane),
                                  frag_contig(Wl, SW, kblk * 32, kk, lane), acc_dx[t]);
        }
      }
    }
    const bool bias_turn = (ct % tiles) == tile;       // uniform over the workgroup
    if (bias_turn) {
      float cs = 0.0f;
#pragma unroll 8
      for (int b = wave * (BR / 4); b < (wave + 1) * (BR / 4); ++b) cs += bf16_to_f32(Dl[b * SD + lane]);
      Bs[wave * BN + lane] = cs;
    }
    if (KH == 2 || wk < KH) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        Gl[(wk * 32 + 8 * (v / 4) + 4 * kb + (v % 4)) * SG + wn * 32 + lr32] = acc[v];
    }
    __syncthreads();

    // eq. (3) on the tile, in the layout of the weight loads
#pragma unroll
    for (int q = 0; q < QW; ++q) {
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
        __builtin_nontemporal_store(hv2, reinterpret_cast<u32x2_t*>(s_g + off));
      } else {
        *reinterpret_cast<f32x4_t*>(w_g + off) = w;
        *reinterpret_cast<u32x2_t*>(s_g + off) = hv2;
      }
    }
    if (bias_turn) {                                   // db of this tile: kept in LDS until the walk ends
      if (tid < BN) Bk[bias_slot * BN + tid] = ((Bs[tid] + Bs[BN + tid]) + Bs[2 * BN + tid]) + Bs[3 * BN + tid];
      ++bias_slot;
    }
    if (PF) {
      fetch_w(wr, wsrc_g, col_tile(it + S) * BN, nt_read);
      if (MOM) fetch_w(vr, v_g, col_tile(it + S) * BN, NT);
    }
  };

  // The first S steps stand outside the loop as well: they follow the prologue, whose loads are
  // issued in another order than those of a step, and a loop header that joins both could only
  // assume the shorter of the two queues.
  int it = 0;
#pragma unroll
  for (int st = 0; st < S; ++st) tile_step(st, wr[st], vr[MOM ? st : 0], true, true);
  for (it = S; it < n_t - S; it += S) {
#pragma unroll
    for (int st = 0; st < S; ++st) tile_step(it + st, wr[st], vr[MOM ? st : 0], true, true);
  }
#pragma unroll
  for (int st = 0; st < S; ++st)                       // the last S tiles: nothing left to prefetch
    tile_step(it + st, wr[st], vr[MOM ? st : 0], false, st + 1 < S);

  // ---- b_l <- b_l - gamma db_l for the column tiles this workgroup owns ---------------------------
  __syncthreads();
  if (tid < BN) {
    int slot = 0;
    for (int i = 0; i < n_t; ++i) {                    // in walk order, as the slots were filled
      const int ct = col_tile(i);
      if ((ct % tiles) != tile) continue;
      float cs = Bk[slot * BN + tid];
      ++slot;
      const size_t bo = p.b_off + (size_t)ct * BN + tid;
      if (MOM) {
        float* vb = p.vel + (size_t)g * p.p_gs + bo;
        cs = fmaf(p.mu, *vb, cs);
        *vb = cs;
      }
      const float b_old = p.src[(size_t)g * p.src_gs + bo];
      p.params[(size_t)g * p.p_gs + bo] = fmaf(-p.lr, cs, b_old);
    }
  }

  // ---- D_{l-1} = acc * phi'(H_{l-1}) -------------------------------------------------------
  if (DX) {
    uint16_t* dx_g = p.dx + (size_t)g * p.dx_gs;
#pragma unroll
    for (int t = 0; t < NTD; ++t) {
      const int blk = dxw + 4 * t;
      if (blk < KH * MB) {
        const int mb = blk / KH, kblk = blk % KH;
        const int k = k0 + kblk * 32 + lr32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int b = mb * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
          const float hval = bf16_to_f32(HT[b * SHK + kblk * 32 + lr32]);
          dx_g[(size_t)b * p.lddx + k] = f32_to_bf16_rne(acc_dx[t][v] * dact_from_h(hval, p.act));
        }
      }
    }
  }
}

// Whether the whole-tile variant with S tiles in flight applies to the layer described by p.
static bool bwd_full_applies(const BwdArgs& p, int mb, int S, int kb = BMK) {
  if (p.B != 32 * mb || (p.K % kb) != 0 || (p.Nn % BN) != 0) return false;
  const int tiles = p.K / kb, n_t = p.Nn / BN;
  if (n_t < 2 * S || (n_t % S) != 0) return false;
  if ((n_t + tiles - 1) / tiles > kMaxBiasTiles) return false;
  // 16-byte vectors: every row of the operands must start 16-byte aligned
  return (p.ldw % 4) == 0 && (p.ldh % 8) == 0 && (p.ldd % 8) == 0 && (p.w_off % 4) == 0;
}

// Fewer than two workgroups of 64-row bands per compute unit on the current device.
static bool few_bands(const BwdArgs& p) {
  static std::atomic<int> cus{0};
  int n = cus.load(std::memory_order_relaxed);
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      return false;
    cus.store(n, std::memory_order_relaxed);
  }
  return (long)((p.K + BMK - 1) / BMK) * p.n_groups < 2L * n;
}

template <int MB, bool DX, bool MOM, int S, int KB>
hipError_t launch_bwd_full_s(const BwdArgs& p, hipStream_t s) {
  constexpr int BR = 32 * MB;
  constexpr int SHK = KB == 64 ? SH : 32;
  constexpr size_t kLds = sizeof(uint16_t) * (BR * SHK + BR * SD + KB * SW) +
                          sizeof(float) * (KB * SG + 4 * BN + kMaxBiasTiles * BN);
  const int tiles = p.K / KB;
  static std::atomic<bool> configured{false};
  if (!configured.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_bwd_full_kernel<MB, DX, S, MOM, true, KB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_bwd_full_kernel<MB, DX, S, MOM, false, KB>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e != hipSuccess) return e;
    configured.store(true, std::memory_order_release);
  }
  if (p.streaming)
    hipLaunchKernelGGL((grouped_bwd_full_kernel<MB, DX, S, MOM, true, KB>), dim3((unsigned)(tiles * p.n_groups)),
                       dim3(kThreads), kLds, s, p);
  else
    hipLaunchKernelGGL((grouped_bwd_full_kernel<MB, DX, S, MOM, false, KB>), dim3((unsigned)(tiles * p.n_groups)),
                       dim3(kThreads), kLds, s, p);
  return hipGetLastError();
}

template <int MB, bool DX, bool MOM> hipError_t launch_bwd_full2(const BwdArgs& p, hipStream_t s) {
  return launch_bwd_full_s<MB, DX, MOM, 2, 64>(p, s);
}
template <int MB, bool DX, bool MOM> hipError_t launch_bwd_full2_half(const BwdArgs& p, hipStream_t s) {
  return launch_bwd_full_s<MB, DX, MOM, 2, 32>(p, s);
}

template <int MB, bool DX, bool MOM>
hipError_t launch_bwd_one(const BwdArgs& p, hipStream_t s) {
  constexpr int S = PRSGD_BWD_STAGES;
  constexpr int BR = 32 * MB;
  constexpr size_t kLds =
      sizeof(uint16_t) * (BR * SH + BR * SD + BMK * SW) + sizeof(float) * (BMK * SG + 4 * BN);
  auto kernel = grouped_bwd_kernel<MB, DX, S, MOM>;
  static std::atomic<bool> configured{false};   // per kernel instance; setting it twice is harmless
  if (!configured.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e != hipSuccess) return e;
    configured.store(true, std::memory_order_release);
  }
  const int tiles = (p.K + BMK - 1) / BMK;
  hipLaunchKernelGGL(kernel, dim3((unsigned)(tiles * p.n_groups)), dim3(kThreads), kLds, s, p);
  return hipGetLastError();
}

}  // namespace

bool bwd_fused_supported(int batch) { return batch >= 1 && batch <= 128; }

hipError_t launch_bwd_fused(const BwdArgs& p, hipStream_t s) {
  if (p.K <= 0 || p.Nn <= 0 || p.n_groups <= 0) return hipSuccess;
  if (!bwd_fused_supported(p.B)) return hipErrorInvalidValue;
  const bool dx = p.dx != nullptr;
  const bool mom = p.vel != nullptr;
  const int mb = p.B <= 32 ? 1 : p.B <= 64 ? 2 : 4;
#define PRSGD_BWD_PICK(FN)                                                              \
  do {                                                                                  \
    if (mom) {                                                                          \
      if (mb == 1) return dx ? FN<1, true, true>(p, s) : FN<1, false, true>(p, s);      \
      if (mb == 2) return dx ? FN<2, true, true>(p, s) : FN<2, false, true>(p, s);      \
      return dx ? FN<4, true, true>(p, s) : FN<4, false, true>(p, s);                   \
    }                                                                                   \
    if (mb == 1) return dx ? FN<1, true, false>(p, s) : FN<1, false, false>(p, s);      \
    if (mb == 2) return dx ? FN<2, true, false>(p, s) : FN<2, false, false>(p, s);      \
    return dx ? FN<4, true, false>(p, s) : FN<4, false, false>(p, s);                   \
  } while (0)
  // Two weight tiles in flight.  Four (possible without the backward-data product) measured
  // 272 us against 298 us on 4096 x 4096 when the kernel runs alone in a loop, but 297 us against
  // 283 us inside the real step: not kept.
  // A layer whose 64-row bands leave compute units without a second workgroup to overlap with is
  // walked in 32-row bands instead (twice the workgroups, each with half the rows of a tile).
  if (few_bands(p) && bwd_full_applies(p, mb, 2, 32)) PRSGD_BWD_PICK(launch_bwd_full2_half);
  if (bwd_full_applies(p, mb, 2)) PRSGD_BWD_PICK(launch_bwd_full2);
  // A layer whose rows are padded to whole column tiles (ld a multiple of 64, less than one tile of
  // padding) is walked over its padded width: the padding columns of W_l, D_l and b_l are zero,
  // their gradient is zero, and the update leaves them zero.
  if ((p.Nn % BN) != 0 && (p.ldw % BN) == 0 && p.ldw - p.Nn < BN && p.ldd == p.ldw) {
    BwdArgs padded = p;
    padded.Nn = p.ldw;
    if (bwd_full_applies(padded, mb, 2)) {
      const BwdArgs& p = padded;
      PRSGD_BWD_PICK(launch_bwd_full2);
    }
  }
  PRSGD_BWD_PICK(launch_bwd_one);
#undef PRSGD_BWD_PICK
}

}  // namespace prsgd
