// Grouped (replica-batched) matrix products of the per-worker MLP gradient
//   G_i^t = grad F_i(x_i^{t-1}; zeta_i^t)            (Algorithm 1, gradient observation)
// on the CDNA4 matrix cores.  One group = one worker's replica: no weights are shared between
// groups, and every group multiplies a skinny B-row activation block with its own weights.
//
//   forward   H_l    = phi(H_{l-1} W_l + b_l)              M = B,       N = d_l,     Kc = d_{l-1}
//   backward  D_{l-1} = (D_l W_l^T) * phi'(H_{l-1})        M = B,       N = d_{l-1}, Kc = d_l
//   weights   dW_l   = H_{l-1}^T D_l ; db_l = colsum(D_l)  M = d_{l-1}, N = d_l,     Kc = B
//             fused with the local update  W_l <- W_l - gamma dW_l      (Algorithm 1, eq. 3)
//
// A workgroup is 4 wavefronts; each wavefront owns TM x TN accumulator tiles of 32x32
// (v_mfma_f32_32x32x16_bf16 or v_mfma_f32_32x32x2_f32).  Operand tiles are staged through LDS in
// their natural memory orientation with 16-byte global loads; an operand whose contraction
// index is the strided one is transposed while its MFMA fragments are read out of LDS.
#include "prsgd_internal.h"

namespace prsgd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

enum { OP_CONTIG = 0, OP_TRANS = 1 };

struct TF32 {
  using elem = float;
  using frag = float;
  static constexpr int V = 4;        // elements per 16-byte vector
  static constexpr int KSTEP = 2;    // contraction depth of one MFMA
  static constexpr int BK = 32;      // contraction depth of one LDS tile
  static constexpr int PADC = 1;
  static constexpr bool kBf16 = false;
};
struct TBF16 {
  using elem = uint16_t;
  using frag = bf16x8_t;
  static constexpr int V = 8;
  static constexpr int KSTEP = 16;
  static constexpr int BK = 64;
  static constexpr int PADC = 8;
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
  static constexpr int kStride = (KIND == OP_CONTIG) ? (T::BK + T::PADC) : ROWS;
  static constexpr int kElems = (KIND == OP_CONTIG) ? ROWS * kStride : T::BK * ROWS;
};

// Copies a ROWS x BK operand tile from global memory into LDS (zero-filled outside the operand).
//   OP_CONTIG: element (r, c) at src[r * ld + c]; LDS [ROWS][BK + PADC]
//   OP_TRANS : element (r, c) at src[c * ld + r]; LDS [BK][ROWS]
// Vector loads run along the memory-contiguous index; a vector that starts inside the logical
// extent may run into the zero padding every buffer carries up to a multiple of 8 elements.
template <typename T, int ROWS, int KIND>
__device__ __forceinline__ void load_tile(typename T::elem* __restrict__ lds,
                                          const typename T::elem* __restrict__ src, int ld,
                                          int row0, int n_rows, int c0, int n_c, int tid) {
  using E = typename T::elem;
  constexpr int V = T::V, BK = T::BK;
  if (KIND == OP_CONTIG) {
    constexpr int VPR = BK / V;
    constexpr int TOTAL = ROWS * VPR;
    constexpr int STRIDE = TileShape<T, ROWS, KIND>::kStride;
#pragma unroll
    for (int v0 = 0; v0 < TOTAL; v0 += kThreads) {
      const int v = v0 + tid;
      if (TOTAL % kThreads != 0 && v >= TOTAL) break;
      const int r = v / VPR, cv = (v % VPR) * V;
      const int row = row0 + r, c = c0 + cv;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (row < n_rows && c < n_c)
        val = *reinterpret_cast<const uint4*>(src + (size_t)row * ld + c);
      E* dst = lds + r * STRIDE + cv;
      if (T::kBf16) {
        *reinterpret_cast<uint4*>(dst) = val;
      } else {                                   // odd row stride: four 4-byte stores
        uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
        d32[0] = val.x; d32[1] = val.y; d32[2] = val.z; d32[3] = val.w;
      }
    }
  } else {
    constexpr int VPC = ROWS / V;
    constexpr int TOTAL = BK * VPC;
#pragma unroll
    for (int v0 = 0; v0 < TOTAL; v0 += kThreads) {
      const int v = v0 + tid;
      if (TOTAL % kThreads != 0 && v >= TOTAL) break;
      const int c = v / VPC, rv = (v % VPC) * V;
      const int row = row0 + rv, cc = c0 + c;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (cc < n_c && row < n_rows)
        val = *reinterpret_cast<const uint4*>(src + (size_t)cc * ld + row);
      *reinterpret_cast<uint4*>(lds + c * ROWS + rv) = val;
    }
  }
}

// MFMA operand fragment of lane (r = lane % 32, kb = lane / 32) for tile row `row` and the
// kk-th KSTEP slice.  A and B fragments use the same (kb, e) -> contraction index map, which is
// all the instruction needs for the product to be the plain sum over c.
template <typename T, int ROWS, int KIND>
__device__ __forceinline__ typename T::frag load_frag(const typename T::elem* __restrict__ lds,
                                                      int row, int kk, int kb);

template <int ROWS, int KIND>
__device__ __forceinline__ float load_frag_f32(const float* __restrict__ lds, int row, int kk, int kb) {
  if (KIND == OP_CONTIG) return lds[row * TileShape<TF32, ROWS, KIND>::kStride + kk * 2 + kb];
  return lds[(kk * 2 + kb) * ROWS + row];
}
template <int ROWS, int KIND>
__device__ __forceinline__ bf16x8_t load_frag_bf16(const uint16_t* __restrict__ lds, int row, int kk,
                                                   int kb) {
  u16x8_t u;
  if (KIND == OP_CONTIG) {
    u = *reinterpret_cast<const u16x8_t*>(lds + row * TileShape<TBF16, ROWS, KIND>::kStride +
                                          kk * 16 + kb * 8);
  } else {
    const uint16_t* p = lds + (kk * 16 + kb * 8) * ROWS + row;
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = p[e * ROWS];
  }
  return __builtin_bit_cast(bf16x8_t, u);
}

__device__ __forceinline__ f32x16_t mfma(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float act_fwd(float z, int act) {
  return act == PRSGD_TANH ? tanhf(z) : fmaxf(z, 0.0f);
}
__device__ __forceinline__ float act_bwd_from_h(float h, int act) {
  return act == PRSGD_TANH ? (1.0f - h * h) : (h > 0.0f ? 1.0f : 0.0f);
}

template <typename T, int BM, int BN, int WM, int WN, int AKIND, int BKIND>
__global__ __launch_bounds__(kThreads) void grouped_gemm_kernel(GemmArgs p) {
  using E = typename T::elem;
  constexpr int BK = T::BK;
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  static_assert(WM * WN == 4, "4 wavefronts per workgroup");
  static_assert(TM >= 1 && TN >= 1, "tile too small for the wavefront grid");

  const int g = blockIdx.z;
  if (p.worker_steps != nullptr && p.step >= p.worker_steps[g]) return;

  __shared__ __attribute__((aligned(16))) E a_lds[TileShape<T, BM, AKIND>::kElems];
  __shared__ __attribute__((aligned(16))) E b_lds[TileShape<T, BN, BKIND>::kElems];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int lr32 = lane & 31, kb = lane >> 5;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;

  const E* a_src = reinterpret_cast<const E*>(p.a) + (size_t)g * p.a_gs;
  const E* b_src = reinterpret_cast<const E*>(p.b) + (size_t)g * p.b_gs;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const bool bias_wg = (p.epi == EPI_DW_FUSED || p.epi == EPI_DW_GRAD) && blockIdx.x == 0;
  float colsum = 0.0f;                       // db: thread n sums column n of the delta tile

  for (int c0 = 0; c0 < p.Kc; c0 += BK) {
    load_tile<T, BM, AKIND>(a_lds, a_src, p.lda, m0, p.M, c0, p.Kc, tid);
    load_tile<T, BN, BKIND>(b_lds, b_src, p.ldb, n0, p.N, c0, p.Kc, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK / T::KSTEP; ++kk) {
      typename T::frag af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + lr32;
        if constexpr (T::kBf16) af[i] = load_frag_bf16<BM, AKIND>(a_lds, row, kk, kb);
        else af[i] = load_frag_f32<BM, AKIND>(a_lds, row, kk, kb);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = (wn * TN + j) * 32 + lr32;
        if constexpr (T::kBf16) bf[j] = load_frag_bf16<BN, BKIND>(b_lds, row, kk, kb);
        else bf[j] = load_frag_f32<BN, BKIND>(b_lds, row, kk, kb);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma(af[i], bf[j], acc[i][j]);
    }
    if (BKIND == OP_TRANS && bias_wg && tid < BN) {
      // delta tile sits in LDS as [c][n]; rows beyond Kc were zero-filled
#pragma unroll 8
      for (int c = 0; c < BK; ++c) colsum += from_elem<T>(b_lds[c * BN + tid]);
    }
    __syncthreads();
  }

  // ---- epilogue: accumulator element v of lane (lr32, kb) is C[8*(v/4) + 4*kb + v%4][lr32] ----
  const size_t pg = (size_t)g * p.p_gs;
  if (p.epi == EPI_DW_FUSED || p.epi == EPI_DW_GRAD) {
    const bool fused = (p.epi == EPI_DW_FUSED);
    float* wbase = (fused ? p.params : p.grads) + pg + p.w_off;
    float w_old[TM][TN][16];
    if (fused) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int m = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
            const int n = n0 + (wn * TN + j) * 32 + lr32;
            w_old[i][j][v] = (m < p.M && n < p.N) ? wbase[(size_t)m * p.ldw + n] : 0.0f;
          }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
          const int n = n0 + (wn * TN + j) * 32 + lr32;
          if (m < p.M && n < p.N) {
            const size_t off = (size_t)m * p.ldw + n;
            if (fused) {
              const float w_new = fmaf(-p.lr, acc[i][j][v], w_old[i][j][v]);
              wbase[off] = w_new;
              if (p.shadow != nullptr) p.shadow[pg + p.w_off + off] = f32_to_bf16_rne(w_new);
            } else {
              wbase[off] = acc[i][j][v];
            }
          }
        }
    if (bias_wg && tid < BN) {
      const int n = n0 + tid;
      if (n < p.N) {
        if (fused) {
          float* bptr = p.params + pg + p.b_off + n;
          *bptr = fmaf(-p.lr, colsum, *bptr);
        } else {
          p.grads[pg + p.b_off + n] = colsum;
        }
      }
    }
    return;
  }

  const float* bias = (p.epi == EPI_FWD_HIDDEN || p.epi == EPI_FWD_LOGITS)
                          ? p.params + pg + p.b_off : nullptr;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + (wn * TN + j) * 32 + lr32;
      if (n >= p.out_cols) continue;
      const float bn = bias != nullptr ? bias[n] : 0.0f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * kb + (v % 4);
        if (m >= p.M) continue;
        const size_t o = (size_t)g * p.out_gs + (size_t)m * p.ldo + n;
        const float c = acc[i][j][v];
        if (p.epi == EPI_FWD_HIDDEN) {
          reinterpret_cast<E*>(p.out)[o] = to_elem<T>(act_fwd(c + bn, p.act));
        } else if (p.epi == EPI_FWD_LOGITS) {
          reinterpret_cast<float*>(p.out)[o] = c + bn;
        } else {  // EPI_DX
          const float h = from_elem<T>(
              reinterpret_cast<const E*>(p.aux)[(size_t)g * p.aux_gs + (size_t)m * p.ldaux + n]);
          reinterpret_cast<E*>(p.out)[o] = to_elem<T>(c * act_bwd_from_h(h, p.act));
        }
      }
    }
}

template <typename T, int BM, int BN, int WM, int WN, int AKIND, int BKIND>
static hipError_t launch_one(const GemmArgs& p, int n_groups, hipStream_t s) {
  if (p.M <= 0 || p.N <= 0 || n_groups <= 0) return hipSuccess;
  dim3 grid((p.M + BM - 1) / BM, (p.N + BN - 1) / BN, n_groups);
  hipLaunchKernelGGL((grouped_gemm_kernel<T, BM, BN, WM, WN, AKIND, BKIND>), grid, dim3(kThreads), 0,
                     s, p);
  return hipGetLastError();
}

// Batch-row products (forward, backward-data): the whole minibatch sits in one M tile when
// B <= 128 so that each weight element is read from HBM exactly once per product.
template <typename T, int AKIND, int BKIND>
static hipError_t launch_rows(const GemmArgs& p, int n_groups, hipStream_t s) {
  if (p.M <= 32) return launch_one<T, 32, 128, 1, 4, AKIND, BKIND>(p, n_groups, s);
  if (p.M <= 64) return launch_one<T, 64, 64, 2, 2, AKIND, BKIND>(p, n_groups, s);
  return launch_one<T, 128, 64, 4, 1, AKIND, BKIND>(p, n_groups, s);
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
  return bf16 ? launch_one<TBF16, 128, 64, 4, 1, OP_TRANS, OP_TRANS>(p, n_groups, s)
              : launch_one<TF32, 128, 64, 4, 1, OP_TRANS, OP_TRANS>(p, n_groups, s);
}

}  // namespace prsgd
