// Grouped (replica-batched) matrix products of the per-worker MLP gradient
//   G_i^t = grad F_i(x_i^{t-1}; zeta_i^t)            (Algorithm 1, gradient observation)
// on the CDNA4 matrix cores.  One group = one worker's replica: no weights are shared between
// groups, and every group multiplies a skinny B-row activation block with its own weights.
//
//   forward   H_l    = phi(H_{l-1} W_l + b_l)              M = B,       N = d_l,     Kc = d_{l-1}
//   backward  D_{l-1} = (D_l W_l^T) * phi'(H_{l-1})        M = B,       N = d_{l-1}, Kc = d_l
//   weights   dW_l   = H_{l-1}^T D_l ; db_l = colsum(D_l)  M = d_{l-1}, N = d_l,     Kc = B
//             fused with the local update  W_l <- W_l - gamma dW_l      (Algorithm 1, eq. 3)
// With I = 1 all workers share the node average: the same products then run with one weight stream
// (group stride 0) and the weight-gradient product contracts over the stacked minibatches of all
// workers, M = d_{l-1}, N = d_l, Kc = N B, updating the average in place.
//
// A workgroup is 4 wavefronts (8 on the widest tile); each wavefront owns TM x TN accumulator tiles of 32x32
// (v_mfma_f32_32x32x16_bf16 or v_mfma_f32_32x32x2_f32).  Operand tiles are staged through LDS in
// their natural memory orientation with 16-byte global loads; an operand whose contraction
// index is the strided one is transposed while its MFMA fragments are read out of LDS.
#include <atomic>
#include <type_traits>

#include "prsgd_internal.h"

namespace prsgd {

enum { OP_CONTIG = 0, OP_TRANS = 1 };

struct TF32 {
  using elem = float;
  using frag = float;
  static constexpr int V = 4;        // elements per 16-byte vector
  static constexpr int KSTEP = 2;    // contraction depth of one MFMA
  static constexpr int BK = 32;      // contraction depth of one LDS tile
  static constexpr int PADC = 1;
  static constexpr int PADT = 0;     // row padding of a transposed tile
  static constexpr bool kBf16 = false;
};
struct TBF16 {
  using elem = uint16_t;
  using frag = bf16x8_t;
  static constexpr int V = 8;
  static constexpr int KSTEP = 16;
#ifndef PRSGD_BF16_BK
#define PRSGD_BF16_BK 64
#endif
  static constexpr int BK = PRSGD_BF16_BK;
  static constexpr int PADC = 8;
  // A transpose read (ds_read_b64_tr_b16) is served 32 lanes at a time: 4 consecutive contraction rows
  // times 16 dwords each.  With a row stride of 16 dwords modulo 32 (32 bf16 modulo 64) they fall on
  // 64 distinct banks; the earlier padding of 16 lost 17 % (one transposed operand) to 37 % (two) of the
  // LDS cycles to bank conflicts, this one none (SQ_LDS_BANK_CONFLICT).
  static constexpr int PADT = 32;
  static constexpr bool kBf16 = true;
};

template <typename T> __device__ __forceinline__ typename T::elem to_elem(float v);
template <> __device__ __forceinline__ float to_elem<TF32>(float v) { return v; }
template <> __device__ __forceinline__ uint16_t to_elem<TBF16>(float v) { return f32_to_bf16_rne(v); }
template <typename T> __device__ __forceinline__ float from_elem(typename T::elem v);
template <> __device__ __forceinline__ float from_elem<TF32>(float v) { return v; }
template <> __device__ __forceinline__ float from_elem<TBF16>(uint16_t v) { return bf16_to_f32(v); }

// LDS footprint (elements) of a ROWS x BK operand tile.
template <typename T, int ROWS, int KIND> struct TileShape {
  static constexpr int kStride = (KIND == OP_CONTIG) ? (T::BK + T::PADC) : (ROWS + T::PADT);
  static constexpr int kElems = (KIND == OP_CONTIG) ? ROWS * kStride : T::BK * kStride;
};

// Moves a ROWS x BK operand tile from global memory to LDS in two halves so that the global
// loads of tile k+1 can be in flight while tile k is multiplied: fetch() fills registers with
// 16-byte vectors (zero outside the operand), stash() writes them to LDS.
//   OP_CONTIG: element (r, c) at src[r * ld + c]; LDS [ROWS][BK + PADC]
//   OP_TRANS : element (r, c) at src[c * ld + r]; LDS [BK][ROWS + PADT]
// Vector loads run along the memory-contiguous index; a vector that starts inside the logical
// extent may run into the zero padding every buffer carries up to a multiple of 8 elements.
template <typename T, int ROWS, int KIND, int NTHR = kThreads> struct TileIO {
  using E = typename T::elem;
  static constexpr int V = T::V, BK = T::BK;
  static constexpr int VECS = ROWS * BK / V;
  static constexpr int NPT = VECS / NTHR;                // vectors per thread
  static_assert(VECS % NTHR == 0, "tile must split evenly over the workgroup");
  static constexpr int STRIDE = TileShape<T, ROWS, KIND>::kStride;

  // Returns the validity mask of the NPT vectors (bit q set = inside the operand).
  __device__ static __forceinline__ uint32_t fetch(uint4 (&reg)[NPT], const E* __restrict__ src, int ld,
                                                   int row0, int n_rows, int c0, int n_c, int tid) {
    uint32_t mask = 0;
#pragma unroll
    for (int q = 0; q < NPT; ++q) {
      const int v = q * NTHR + tid;
      // Branch-free: an out-of-range vector loads element (0, 0) instead and is zeroed when it
      // is written to LDS, so nothing waits on the load here and the loads stay countable for
      // the compiler's vmcnt bookkeeping across the pipeline.
      bool ok;
      size_t off;
      if (KIND == OP_CONTIG) {
        constexpr int VPR = BK / V;
        const int row = row0 + v / VPR, c = c0 + (v % VPR) * V;
        ok = row < n_rows && c < n_c;
        off = (size_t)row * ld + c;
      } else {
        constexpr int VPC = ROWS / V;
        const int cc = c0 + v / VPC, row = row0 + (v % VPC) * V;
        ok = cc < n_c && row < n_rows;
        off = (size_t)cc * ld + row;
      }
      reg[q] = *reinterpret_cast<const uint4*>(src + (ok ? off : (size_t)0));
      mask |= (ok ? 1u : 0u) << q;
    }
    return mask;
  }

  __device__ static __forceinline__ void stash(E* __restrict__ lds, const uint4 (&reg_in)[NPT],
                                               uint32_t mask, int tid) {
#pragma unroll
    for (int q = 0; q < NPT; ++q) {
      const int v = q * NTHR + tid;
      const uint32_t keep = 0u - ((mask >> q) & 1u);      // all ones inside the operand, else zero
      uint4 reg[1];
      reg[0] = make_uint4(reg_in[q].x & keep, reg_in[q].y & keep, reg_in[q].z & keep, reg_in[q].w & keep);
      if (KIND == OP_CONTIG) {
        constexpr int VPR = BK / V;
        E* dst = lds + (v / VPR) * STRIDE + (v % VPR) * V;
        if (T::kBf16) {
          *reinterpret_cast<uint4*>(dst) = reg[0];
        } else {                                   // odd row stride: four 4-byte stores
          uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
          d32[0] = reg[0].x; d32[1] = reg[0].y; d32[2] = reg[0].z; d32[3] = reg[0].w;
        }
      } else {
        constexpr int VPC = ROWS / V;
        *reinterpret_cast<uint4*>(lds + (v / VPC) * STRIDE + (v % VPC) * V) = reg[0];
      }
    }
  }
};

// MFMA operand fragment of lane (r = lane % 32, kb = lane / 32) for tile row `row` and the
// kk-th KSTEP slice.  A and B fragments use the same (kb, e) -> contraction index map, which is
// all the instruction needs for the product to be the plain sum over c.
template <int ROWS, int KIND>
__device__ __forceinline__ float load_frag_f32(const float* __restrict__ lds, int row, int kk, int kb) {
  if (KIND == OP_CONTIG) return lds[row * TileShape<TF32, ROWS, KIND>::kStride + kk * 2 + kb];
  return lds[(kk * 2 + kb) * TileShape<TF32, ROWS, KIND>::kStride + row];
}
// bf16 fragment: one 16-byte read of a contraction-contiguous tile, the LDS transpose load for a
// tile stored with the contraction index as its row.
template <int ROWS, int KIND>
__device__ __forceinline__ bf16x8_t load_frag_bf16(const uint16_t* __restrict__ lds, int row_block,
                                                   int kk, int lane) {
  constexpr int STRIDE = TileShape<TBF16, ROWS, KIND>::kStride;
  if (KIND == OP_CONTIG) return frag_contig(lds, STRIDE, row_block, kk, lane);
  return frag_trans(lds, STRIDE, row_block, kk, lane);
}

__device__ __forceinline__ f32x16_t mfma(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// A-operand fragment of all ones: with it one matrix instruction yields the column sums of the
// B fragment (every row of the 32 x 32 result holds them).
template <typename F> __device__ __forceinline__ F ones_frag();
template <> __device__ __forceinline__ float ones_frag<float>() { return 1.0f; }
template <> __device__ __forceinline__ bf16x8_t ones_frag<bf16x8_t>() {
  const u16x8_t u = {0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80};
  return __builtin_bit_cast(bf16x8_t, u);
}

__device__ __forceinline__ float act_fwd(float z, int act) {
  return act == PRSGD_TANH ? tanhf(z) : fmaxf(z, 0.0f);
}
__device__ __forceinline__ float act_bwd_from_h(float h, int act) {
  return act == PRSGD_TANH ? (1.0f - h * h) : (h > 0.0f ? 1.0f : 0.0f);
}

// DEEP: the two-stage, four-register-set pipeline (long contractions); otherwise a single LDS
// stage with a one-tile prefetch (the per-replica weight-gradient product: one or two tiles).
template <typename T, int BM, int BN, int WM, int WN, int AKIND, int BKIND,
          bool DEEP = !(AKIND == OP_TRANS && BKIND == OP_TRANS)>
__global__ __launch_bounds__(64 * WM * WN) void grouped_gemm_kernel(GemmArgs p) {
  using E = typename T::elem;
  constexpr int NTHR = 64 * WM * WN;
  using IOA = TileIO<T, BM, AKIND, NTHR>;
  using IOB = TileIO<T, BN, BKIND, NTHR>;
  constexpr int BK = T::BK;
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  constexpr int A_ELEMS = TileShape<T, BM, AKIND>::kElems, B_ELEMS = TileShape<T, BN, BKIND>::kElems;
  static_assert(WM * WN == 4 || WM * WN == 8, "4 or 8 wavefronts per workgroup");
  static_assert(TM >= 1 && TN >= 1, "tile too small for the wavefront grid");
  static_assert((A_ELEMS * sizeof(E)) % 16 == 0 && (B_ELEMS * sizeof(E)) % 16 == 0, "LDS alignment");

  // Workgroup -> (group, tile).  The hardware deals consecutive workgroups round-robin to the
  // 8 XCDs; when the group count is a multiple of 8 all tiles of a group land on one XCD, so the
  // group's activations and weight panel stay in that XCD's L2.
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int n_splits = p.k_splits > 1 ? p.k_splits : 1;     // contraction ranges per output tile
  const int tiles = tiles_m * tiles_n * n_splits;
  int g, tile;
  if ((p.n_groups & 7) == 0) {
    const int slot = blockIdx.x >> 3;
    g = (blockIdx.x & 7) + 8 * (slot / tiles);
    tile = slot % tiles;
  } else {
    g = blockIdx.x / tiles;
    tile = blockIdx.x % tiles;
  }
  const int ks = tile % n_splits;
  tile /= n_splits;
  if (p.worker_steps != nullptr && p.step >= p.worker_steps[g]) return;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // Two LDS stages of each operand tile; the per-replica weight-gradient product (one or two
  // contraction tiles in all) keeps a single stage so that more workgroups fit on a compute unit.
  constexpr int kStages = DEEP ? 2 : 1;
  E* const a_lds0 = reinterpret_cast<E*>(smem);
  E* const b_lds0 = a_lds0 + kStages * A_ELEMS;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int lr32 = lane & 31, kb = lane >> 5;

  const E* a_src = reinterpret_cast<const E*>(p.a) + (size_t)g * p.a_gs;
  const E* b_src = reinterpret_cast<const E*>(p.b) + (size_t)g * p.b_gs;
  // this workgroup's contraction range [k_lo, k_lo + Kc): whole tiles per split
  int Kc = p.Kc;
  if (n_splits > 1) {
    const int per = ((p.Kc + BK - 1) / BK + n_splits - 1) / n_splits * BK;
    const int k_lo = ks * per;
    Kc = max(0, min(p.Kc - k_lo, per));
    if (Kc > 0) {                                  // an empty range keeps valid base addresses
      a_src += (AKIND == OP_CONTIG) ? (size_t)k_lo : (size_t)k_lo * p.lda;
      b_src += (BKIND == OP_CONTIG) ? (size_t)k_lo : (size_t)k_lo * p.ldb;
    }
  }
  const size_t pg = (size_t)g * p.p_gs;
  constexpr bool kIsDw = (AKIND == OP_TRANS && BKIND == OP_TRANS);   // weight-gradient product
  const bool fused = kIsDw && (p.epi == EPI_DW_FUSED);

  // Weight-update epilogue: the output tile leaves through LDS in row-major order, one 16-byte
  // vector per lane (EV vectors per thread).  Start streaming the old weights in that layout now,
  // they are not needed until the products are done.
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  constexpr int SC = BN + 8;                               // LDS row stride of the output tile (floats)
  constexpr int VPR_C = BN / 4, ROWS_PER_PASS = NTHR / VPR_C, EV = kIsDw ? BM / ROWS_PER_PASS : 1;
  static_assert(!kIsDw || (NTHR % VPR_C == 0 && BM % ROWS_PER_PASS == 0), "output tile must split evenly");
  const int e_row = tid / VPR_C, e_col = 4 * (tid % VPR_C);
  f32x4_t w_old[EV];
  if constexpr (kIsDw) if (fused) {
    const float* wbase = p.params + pg + p.w_off;
#pragma unroll
    for (int q = 0; q < EV; ++q) {
      const int m = m0 + q * ROWS_PER_PASS + e_row, n = n0 + e_col;
      const bool ok = m < p.M && n < p.N;
      const f32x4_t* wp = reinterpret_cast<const f32x4_t*>(wbase + (ok ? (size_t)m * p.ldw + n : (size_t)0));
      w_old[q] = p.streaming ? __builtin_nontemporal_load(wp) : *wp;
    }
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // db_l = colsum(D_l): the workgroups of the first row band feed the delta fragments they hold
  // anyway through one more matrix instruction against an all-ones operand
  const bool bias_wave = kIsDw && m0 == 0 && wm == 0;
  f32x16_t accb[kIsDw ? TN : 1];
#pragma unroll
  for (int j = 0; j < (kIsDw ? TN : 1); ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) accb[j][v] = 0.0f;

  // Software pipeline: two LDS stages and R register sets, so that the global loads of tiles
  // it+2 .. it+1+R are all in flight while tile `it` is multiplied -- one tile of compute is far
  // shorter than the HBM latency it has to hide, and a launch has few workgroups per compute unit.
  // Tile j (j >= 1) travels through register set j % R.  The per-replica weight-gradient product
  // contracts over the minibatch only (one or two tiles): it keeps a single LDS stage and a
  // one-tile prefetch and spends its registers on the streamed weights instead.
  constexpr bool kDeep = DEEP;
  constexpr int R = kDeep ? 4 : 1;
  const int n_k = (Kc + BK - 1) / BK;
  uint4 a_r[R][IOA::NPT], b_r[R][IOB::NPT];
  uint32_t a_m[R], b_m[R];                           // validity masks of the register sets
#pragma unroll
  for (int r = 0; r < R; ++r) { a_m[r] = 0; b_m[r] = 0; }
  a_m[0] = IOA::fetch(a_r[0], a_src, p.lda, m0, p.M, 0, Kc, tid);
  b_m[0] = IOB::fetch(b_r[0], b_src, p.ldb, n0, p.N, 0, Kc, tid);
  IOA::stash(a_lds0, a_r[0], a_m[0], tid);
  IOB::stash(b_lds0, b_r[0], b_m[0], tid);
  if constexpr (kDeep) {
    // Unconditional: a tile past the end of the contraction is fetched masked (all vectors read
    // element (0, 0) and are zeroed on the way to LDS).  Straight-line code keeps the number of
    // loads in flight the same on every path, which the wait-count bookkeeping needs.
#pragma unroll
    for (int j = 1; j <= R; ++j) {
      a_m[j % R] = IOA::fetch(a_r[j % R], a_src, p.lda, m0, p.M, j * BK, Kc, tid);
      b_m[j % R] = IOB::fetch(b_r[j % R], b_src, p.ldb, n0, p.N, j * BK, Kc, tid);
    }
  }
  __syncthreads();

  auto compute = [&](int cur) {
    const E* a_cur = a_lds0 + cur * A_ELEMS;
    const E* b_cur = b_lds0 + cur * B_ELEMS;
    constexpr int KK = BK / T::KSTEP;
    // fragments of contraction step kk + 1 are read from LDS while the matrix instructions of
    // step kk run: two register sets, filled alternately (reading further ahead measured no faster)
    typename T::frag af[2][TM], bf[2][TN];
    auto load_frags = [&](int kk, int set) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rb_ = (wm * TM + i) * 32;
        if constexpr (T::kBf16) af[set][i] = load_frag_bf16<BM, AKIND>(a_cur, rb_, kk, lane);
        else af[set][i] = load_frag_f32<BM, AKIND>(a_cur, rb_ + lr32, kk, kb);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int rb_ = (wn * TN + j) * 32;
        if constexpr (T::kBf16) bf[set][j] = load_frag_bf16<BN, BKIND>(b_cur, rb_, kk, lane);
        else bf[set][j] = load_frag_f32<BN, BKIND>(b_cur, rb_ + lr32, kk, kb);
      }
    };
    load_frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) load_frags(kk + 1, (kk + 1) & 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma(af[kk & 1][i], bf[kk & 1][j], acc[i][j]);
      if constexpr (kIsDw) {
        if (bias_wave) {               // rows beyond Kc were zero-filled in LDS
#pragma unroll
          for (int j = 0; j < TN; ++j) accb[j] = mfma(ones_frag<typename T::frag>(), bf[kk & 1][j], accb[j]);
        }
      }
    }
  };
  if constexpr (kDeep) {
    // One pipeline step on tile `it` (it % R == U): multiply the LDS stage it & 1, move tile
    // it+1 from its register set to the other stage, refill that set with tile it+1+R.
    // Straight-line code without a single conditional load: the hardware counts outstanding
    // memory operations in issue order, and the compiler can only leave the loads of the other
    // register sets in flight across a step if their number is the same on every path (a
    // conditional prologue or drain loop made it wait for ALL of them once per R steps).
    auto step = [&](int it, auto u_tag) {
      constexpr int U = decltype(u_tag)::value;
      constexpr int SET = (U + 1) % R, CUR = U & 1;
      compute(CUR);
      IOA::stash(a_lds0 + (CUR ^ 1) * A_ELEMS, a_r[SET], a_m[SET], tid);
      IOB::stash(b_lds0 + (CUR ^ 1) * B_ELEMS, b_r[SET], b_m[SET], tid);
      a_m[SET] = IOA::fetch(a_r[SET], a_src, p.lda, m0, p.M, (it + 1 + R) * BK, Kc, tid);
      b_m[SET] = IOB::fetch(b_r[SET], b_src, p.ldb, n0, p.N, (it + 1 + R) * BK, Kc, tid);
      __syncthreads();
    };
    static_assert(R == 4, "the unrolled pipeline below is written for four register sets");
    using std::integral_constant;
    // Every group of R steps runs the straight-line form: tiles past the end arrive as zeros
    // (masked fetch) and add nothing, at the cost of at most R - 1 empty steps per workgroup.
    for (int it = 0; it < n_k; it += R) {
      step(it, integral_constant<int, 0>{});
      step(it + 1, integral_constant<int, 1>{});
      step(it + 2, integral_constant<int, 2>{});
      step(it + 3, integral_constant<int, 3>{});
    }
  } else {
    for (int it = 0; it < n_k; ++it) {         // single LDS stage, next tile prefetched in registers
      const bool more = it + 1 < n_k;
      if (more) {
        a_m[0] = IOA::fetch(a_r[0], a_src, p.lda, m0, p.M, (it + 1) * BK, Kc, tid);
        b_m[0] = IOB::fetch(b_r[0], b_src, p.ldb, n0, p.N, (it + 1) * BK, Kc, tid);
      }
      compute(0);
      if (more) {
        __syncthreads();
        IOA::stash(a_lds0, a_r[0], a_m[0], tid);
        IOB::stash(b_lds0, b_r[0], b_m[0], tid);
        __syncthreads();
      }
    }
  }

  // ---- epilogue: accumulator element v of lane (lr32, kb) is C[8*(v/4) + 4*kb + v%4][lr32] ----
  if constexpr (kIsDw) {
    float* wbase = (fused ? p.params : p.grads) + pg + p.w_off;
    // accumulators -> LDS (the operand stages are free now) -> row-major 16-byte accesses
    float* c_lds = reinterpret_cast<float*>(smem);
    __syncthreads();                                       // every wavefront is done with the last tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          c_lds[((wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4)) * SC + (wn * TN + j) * 32 + lr32] =
              acc[i][j][v];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < EV; ++q) {
      const int r = q * ROWS_PER_PASS + e_row;
      const int m = m0 + r, n = n0 + e_col;
      if (m < p.M && n < p.N) {
        const f32x4_t g = *reinterpret_cast<const f32x4_t*>(c_lds + r * SC + e_col);
        const size_t off = (size_t)m * p.ldw + n;
        if (fused) {
          f32x4_t w = w_old[q];
          w.x = fmaf(-p.lr, g.x, w.x);
          w.y = fmaf(-p.lr, g.y, w.y);
          w.z = fmaf(-p.lr, g.z, w.z);
          w.w = fmaf(-p.lr, g.w, w.w);
          typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
          const u32x2_t hv = {(uint32_t)f32_to_bf16_rne(w.x) | ((uint32_t)f32_to_bf16_rne(w.y) << 16),
                              (uint32_t)f32_to_bf16_rne(w.z) | ((uint32_t)f32_to_bf16_rne(w.w) << 16)};
          if (p.streaming) {
            __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t*>(wbase + off));
            if (p.shadow != nullptr)
              __builtin_nontemporal_store(hv, reinterpret_cast<u32x2_t*>(p.shadow + pg + p.w_off + off));
          } else {
            *reinterpret_cast<f32x4_t*>(wbase + off) = w;
            if (p.shadow != nullptr) *reinterpret_cast<u32x2_t*>(p.shadow + pg + p.w_off + off) = hv;
          }
        } else {
          *reinterpret_cast<f32x4_t*>(wbase + off) = g;
        }
      }
    }
    if (bias_wave && kb == 0) {       // row 0 of the ones product: lane lr32 holds column lr32
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + lr32;
        const float colsum = accb[j][0];
        if (n < p.N) {
          if (fused) {
            float* bptr = p.params + pg + p.b_off + n;
            *bptr = fmaf(-p.lr, colsum, *bptr);
          } else {
            p.grads[pg + p.b_off + n] = colsum;
          }
        }
      }
    }
    return;
  }

  const float* bias = (p.epi == EPI_FWD_HIDDEN || p.epi == EPI_FWD_LOGITS)
                          ? p.bias_src + (size_t)g * p.bias_gs + p.b_off : nullptr;
  const E* aux = reinterpret_cast<const E*>(p.aux) + (size_t)g * p.aux_gs;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + (wn * TN + j) * 32 + lr32;
      const bool n_ok = n < p.out_cols;
      // partial sums of a split contraction carry no bias: the loss head adds it once
      const float bn = (bias != nullptr && n_splits == 1) ? bias[n_ok ? n : 0] : 0.0f;
      // all loads of the tile first (they may not be reordered across the stores below)
      float h[16];
      if (p.epi == EPI_DX) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
          const bool ok = n_ok && m < p.M;
          h[v] = from_elem<T>(aux[ok ? (size_t)m * p.ldaux + n : (size_t)0]);
        }
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
        if (!n_ok || m >= p.M) continue;
        const size_t o = (size_t)g * p.out_gs + (size_t)m * p.ldo + n;
        const float c = acc[i][j][v];
        if (p.epi == EPI_FWD_HIDDEN) {
          reinterpret_cast<E*>(p.out)[o] = to_elem<T>(act_fwd(c + bn, p.act));
        } else if (p.epi == EPI_FWD_LOGITS) {
          reinterpret_cast<float*>(p.out)[(size_t)ks * p.split_stride + o] = c + bn;
        } else {  // EPI_DX
          reinterpret_cast<E*>(p.out)[o] = to_elem<T>(c * act_bwd_from_h(h[v], p.act));
        }
      }
    }
}

template <typename T, int BM, int BN, int WM, int WN, int AKIND, int BKIND,
          bool DEEP = !(AKIND == OP_TRANS && BKIND == OP_TRANS)>
static hipError_t launch_one(GemmArgs p, int n_groups, hipStream_t s) {
  if (p.M <= 0 || p.N <= 0 || n_groups <= 0) return hipSuccess;
  using E = typename T::elem;
  constexpr size_t kStages = DEEP ? 2 : 1;
  constexpr bool kIsDw = (AKIND == OP_TRANS && BKIND == OP_TRANS);
  constexpr size_t kStageBytes =
      kStages * sizeof(E) * (TileShape<T, BM, AKIND>::kElems + TileShape<T, BN, BKIND>::kElems);
  // the weight-gradient product parks its fp32 output tile [BM][BN + 8] in the same memory
  constexpr size_t kOutBytes = kIsDw ? sizeof(float) * BM * (BN + 8) : 0;
  constexpr size_t kLds = kStageBytes > kOutBytes ? kStageBytes : kOutBytes;
  auto kernel = grouped_gemm_kernel<T, BM, BN, WM, WN, AKIND, BKIND, DEEP>;
  // double-buffered tiles can exceed the 64 KB default; setting the limit twice is harmless
  static std::atomic<bool> configured{false};
  if (!configured.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e != hipSuccess) return e;
    configured.store(true, std::memory_order_release);
  }
  p.n_groups = n_groups;
  if (p.k_splits > 1 && p.epi != EPI_FWD_LOGITS) return hipErrorInvalidValue;
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN) * (p.k_splits > 1 ? p.k_splits : 1);
  hipLaunchKernelGGL(kernel, dim3((unsigned)(tiles * n_groups)), dim3(64 * WM * WN), kLds, s, p);
  return hipGetLastError();
}

constexpr int kComputeUnits = 256;

// Batch-row products (forward, backward-data): the whole minibatch sits in one M tile when
// B <= 128 so that each weight element is read from HBM exactly once per product.  The wide
// (128-column) tile halves LDS traffic per flop; it is used when it still yields at least one
// workgroup per compute unit.
template <typename T, int AKIND, int BKIND>
static hipError_t launch_rows(const GemmArgs& p, int n_groups, hipStream_t s) {
  if (p.M <= 32) return launch_one<T, 32, 128, 1, 4, AKIND, BKIND>(p, n_groups, s);
  const bool wide = (long)((p.N + 127) / 128) * n_groups * ((p.M + 127) / 128) >= kComputeUnits;
  if (p.M <= 64) {
    if (wide) return launch_one<T, 64, 128, 2, 2, AKIND, BKIND>(p, n_groups, s);
    return launch_one<T, 64, 64, 2, 2, AKIND, BKIND>(p, n_groups, s);
  }
  // eight wavefronts on the widest tile: with one wavefront per SIMD nothing covers the LDS
  // latency between fragment reads and matrix instructions (4096 x 4096, 8 replicas: 74 -> 61 us)
  if (wide) return launch_one<T, 128, 128, 2, 4, AKIND, BKIND>(p, n_groups, s);
  // a narrow layer that would leave compute units idle splits the minibatch rows over two
  // workgroups instead: the second reader of a weight tile finds it in the L2 of the same XCD
  if ((long)((p.N + 63) / 64) * n_groups < kComputeUnits)
    return launch_one<T, 64, 64, 2, 2, AKIND, BKIND>(p, n_groups, s);
  return launch_one<T, 128, 64, 2, 2, AKIND, BKIND>(p, n_groups, s);
}

// Output tiles of the batch-row launch launch_rows() would make for p.
static long rows_launch_tiles(const GemmArgs& p, int n_groups) {
  int bm, bn;
  if (p.M <= 32) { bm = 32; bn = 128; }
  else {
    const bool wide = (long)((p.N + 127) / 128) * n_groups * ((p.M + 127) / 128) >= kComputeUnits;
    const bool narrow = (long)((p.N + 63) / 64) * n_groups < kComputeUnits;
    bm = (p.M <= 64 || (!wide && narrow)) ? 64 : 128;
    bn = wide ? 128 : 64;
  }
  return (long)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn) * n_groups;
}

// A logits product that leaves most compute units idle (few classes) cuts its contraction into
// 2 or 4 ranges of whole tiles, every range non-empty and at least two tiles long.
int gemm_logit_splits(const GemmArgs& p, int n_groups, bool bf16) {
  const int bk = bf16 ? TBF16::BK : TF32::BK;
  const int n_k = (p.Kc + bk - 1) / bk;
  const long wgs = rows_launch_tiles(p, n_groups);
  for (int s = kMaxLogitSplits; s >= 2; s >>= 1) {
    const int per = (n_k + s - 1) / s;
    if (wgs * s <= 2 * kComputeUnits && per >= 2 && (long)per * (s - 1) < n_k) return s;
  }
  return 1;
}

hipError_t launch_gemm_fwd(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s) {
  return bf16 ? launch_rows<TBF16, OP_CONTIG, OP_TRANS>(p, n_groups, s)
              : launch_rows<TF32, OP_CONTIG, OP_TRANS>(p, n_groups, s);
}
hipError_t launch_gemm_dx(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s) {
  return bf16 ? launch_rows<TBF16, OP_CONTIG, OP_CONTIG>(p, n_groups, s)
              : launch_rows<TF32, OP_CONTIG, OP_CONTIG>(p, n_groups, s);
}
hipError_t launch_gemm_dw(const GemmArgs& p, int n_groups, bool bf16, hipStream_t s) {
  return bf16 ? launch_one<TBF16, 128, 64, 2, 2, OP_TRANS, OP_TRANS>(p, n_groups, s)
              : launch_one<TF32, 128, 64, 2, 2, OP_TRANS, OP_TRANS>(p, n_groups, s);
}
// The same product with the minibatches of all workers stacked into one contraction (a single
// group, Kc = N B rows).  Large layers: the deep pipeline on the widest tile.  Layers with few
// tiles: 64 x 64 tiles on the shallow pipeline, several workgroups per compute unit, so that the
// weight read-modify-write of one overlaps the products of another (3072 x 1024 with 1024 stacked
// rows: 22 -> 18 us).
hipError_t launch_gemm_dw_stacked(const GemmArgs& p, hipStream_t s) {
  const long wide_tiles = (long)((p.M + 127) / 128) * ((p.N + 127) / 128);
  if (wide_tiles >= kComputeUnits)
    return launch_one<TBF16, 128, 128, 2, 4, OP_TRANS, OP_TRANS, true>(p, 1, s);
  return launch_one<TBF16, 64, 64, 2, 2, OP_TRANS, OP_TRANS, false>(p, 1, s);
}

}  // namespace prsgd
