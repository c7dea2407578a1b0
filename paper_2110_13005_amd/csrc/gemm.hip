// bf16 MFMA GEMM family for gfx950 with fused epilogues.
//
//   C[m][n] = epilogue( sum_k Aop(m,k) * Bop(n,k) ),  fp32 accumulation.
//
// Each operand is either "k-contiguous" (stored [row][k]) or "k-strided" (stored [k][row]);
// the three linear-layer contractions of a transformer layer map onto it as
//   forward  y  = x W        : A k-contiguous, B k-strided   (W is [in,out])
//   dgrad    dx = dy W^T     : A k-contiguous, B k-contiguous
//   wgrad    dW = x^T dy     : A k-strided,    B k-strided
// A block computes a BM x BN tile with WGM x WGN waves; tiles of A and B stream through a
// double-buffered LDS stage (global -> registers -> LDS, one barrier per k-step).  k-contiguous
// tiles are read back with 128-bit LDS loads, k-strided tiles with the transposing LDS load,
// so no operand is ever transposed in HBM.  The MFMA is issued with the B fragment first, so a
// lane of the result owns one row m and runs of 4 consecutive columns n: epilogue loads and
// stores are 8-byte (bf16) or 16-byte (fp32) vectors along the contiguous dimension of C.
#include "common.h"

namespace axonn {

// Chunks of a tile that fall outside the matrix are fetched from here instead, so that every
// load is unconditional and nothing has to be patched after it arrives.
__device__ __align__(16) uint32_t g_zero_chunk[4] = {0u, 0u, 0u, 0u};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // 16-byte chunk kept in registers

template <int ROWS, int BK, bool KC>
struct TileLayout {
  // leading dimension in elements, padded so that fragment reads spread over LDS banks
  static constexpr int LD = KC ? (BK + 8) : (ROWS + 32);
  static constexpr int ELEMS = KC ? ROWS * LD : BK * LD;
};

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_kernel(const GemmArgs g) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  using LA = TileLayout<BM, BK, A_KC>;
  using LB = TileLayout<BN, BK, B_KC>;
  constexpr int A_CH = BM * BK / 8 / NT;  // 16-byte chunks per thread per tile
  constexpr int B_CH = BN * BK / 8 / NT;
  static_assert(A_CH >= 1 && B_CH >= 1, "tile too small for the block");
  static_assert((BM * BK / 8) % NT == 0 && (BN * BK / 8) % NT == 0, "tile/threads mismatch");

  __shared__ __align__(16) bf16_t sA[2][LA::ELEMS];
  __shared__ __align__(16) bf16_t sB[2][LB::ELEMS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroups are dealt round-robin to the 8 XCDs; remap so that each XCD (own L2) works on
  // a contiguous run of tiles, ordered m-fastest so that neighbours share the B panel.
  int pid = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  const int tm = pid % g.tiles_m, tn = pid / g.tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  // Per-thread view of the tile copy: chunk j of this thread is 16 bytes at pa[j] (advanced by
  // one k-step per iteration), valid if its row is inside the matrix (fixed) and its k is (checked
  // per step).  Out-of-range chunks read a zero chunk instead, so the loads are unconditional
  // and stay in registers until the next step stores them to LDS.
  const bf16_t* pa[A_CH];
  const bf16_t* pb[B_CH];
  bool va[A_CH], vb[B_CH];
  int ka[A_CH], kb[B_CH], oa[A_CH], ob[B_CH];
#pragma unroll
  for (int j = 0; j < A_CH; ++j) {
    const int c = tid + j * NT;
    if (A_KC) {
      const int row = c / (BK / 8), kc = c % (BK / 8);
      va[j] = (m0 + row) < g.M; ka[j] = kc * 8;
      pa[j] = g.A + (int64_t)(m0 + row) * g.lda + kc * 8;
      oa[j] = row * LA::LD + kc * 8;
    } else {
      const int kr = c / (BM / 8), rc = c % (BM / 8);
      va[j] = (m0 + rc * 8) < g.M; ka[j] = kr;
      pa[j] = g.A + (int64_t)kr * g.lda + m0 + rc * 8;
      oa[j] = kr * LA::LD + rc * 8;
    }
  }
#pragma unroll
  for (int j = 0; j < B_CH; ++j) {
    const int c = tid + j * NT;
    if (B_KC) {
      const int row = c / (BK / 8), kc = c % (BK / 8);
      vb[j] = (n0 + row) < g.N; kb[j] = kc * 8;
      pb[j] = g.B + (int64_t)(n0 + row) * g.ldb + kc * 8;
      ob[j] = row * LB::LD + kc * 8;
    } else {
      const int kr = c / (BN / 8), rc = c % (BN / 8);
      vb[j] = (n0 + rc * 8) < g.N; kb[j] = kr;
      pb[j] = g.B + (int64_t)kr * g.ldb + n0 + rc * 8;
      ob[j] = kr * LB::LD + rc * 8;
    }
  }
  const int64_t step_a = A_KC ? (int64_t)BK : (int64_t)BK * g.lda;
  const int64_t step_b = B_KC ? (int64_t)BK : (int64_t)BK * g.ldb;
  const int K = g.K;
  const bf16_t* zero_chunk = reinterpret_cast<const bf16_t*>(g_zero_chunk);
  u32x4 ra[A_CH], rb[B_CH];

#define AXONN_GLOAD(k0)                                                        \
  _Pragma("unroll") for (int j = 0; j < A_CH; ++j) {                           \
    const bool ok = va[j] && ((k0) + ka[j] < K);                               \
    ra[j] = *reinterpret_cast<const u32x4*>(ok ? pa[j] : zero_chunk);          \
    pa[j] += step_a;                                                           \
  }                                                                            \
  _Pragma("unroll") for (int j = 0; j < B_CH; ++j) {                           \
    const bool ok = vb[j] && ((k0) + kb[j] < K);                               \
    rb[j] = *reinterpret_cast<const u32x4*>(ok ? pb[j] : zero_chunk);          \
    pb[j] += step_b;                                                           \
  }                                                                            \
  __builtin_amdgcn_sched_barrier(0);
#define AXONN_SSTORE(buf)                                                      \
  _Pragma("unroll") for (int j = 0; j < A_CH; ++j)                             \
    *reinterpret_cast<u32x4*>(&sA[buf][oa[j]]) = ra[j];                        \
  _Pragma("unroll") for (int j = 0; j < B_CH; ++j)                             \
    *reinterpret_cast<u32x4*>(&sB[buf][ob[j]]) = rb[j];

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + BK - 1) / BK;
  AXONN_GLOAD(0)
  AXONN_SSTORE(0)
  AXONN_GLOAD(BK)          // tile 1 (all zeros if there is none)
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    // registers hold tile kt+1: park it in the other buffer, then fetch tile kt+2
    AXONN_SSTORE(cur ^ 1)
    AXONN_GLOAD((kt + 2) * BK)
    const bf16_t* a_s = sA[cur];
    const bf16_t* b_s = sB[cur];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r0 = wm * WTM + i * 32;
        fa[i] = A_KC ? frag_kcontig(a_s + r0 * LA::LD + kk * 16, LA::LD, lane)
                     : frag_kstrided<false>(a_s + (kk * 16) * LA::LD + r0, LA::LD, lane);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r0 = wn * WTN + j * 32;
        fb[j] = B_KC ? frag_kcontig(b_s + r0 * LB::LD + kk * 16, LB::LD, lane)
                     : frag_kstrided<false>(b_s + (kk * 16) * LB::LD + r0, LB::LD, lane);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(fb[j], fa[i], acc[i][j]);
    }
    __syncthreads();
  }
#undef AXONN_GLOAD
#undef AXONN_SSTORE

  // ------------------------------------------------------------------ epilogue
  // lane owns row m = .. + lane%32; register r of tile (i,j) is column 8*(r/4)+4*(lane/32)+r%4
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WTM + i * 32 + (lane & 31);
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * (lane >> 5);
        if (n >= g.N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
        if (EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU) {
          if (g.bias) {
            const bf16x4 bv = *reinterpret_cast<const bf16x4*>(g.bias + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += (float)bv[e];
          }
        }
        if (EPI == EPI_BIAS_RES) {
          const bf16x4 rv = *reinterpret_cast<const bf16x4*>(g.res + (int64_t)m * g.ld_res + n);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
        }
        if (EPI == EPI_BIAS_GELU) {
          bf16x4 pv;
#pragma unroll
          for (int e = 0; e < 4; ++e) { pv[e] = (bf16_t)v[e]; v[e] = gelu_f(v[e]); }
          *reinterpret_cast<bf16x4*>(g.aux + (int64_t)m * g.ld_aux + n) = pv;
        }
        if (EPI == EPI_DGELU) {
          const bf16x4 pv = *reinterpret_cast<const bf16x4*>(g.aux + (int64_t)m * g.ld_aux + n);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f((float)pv[e]);
        }
        if (EPI == EPI_ACC_F32) {
          float* cp = reinterpret_cast<float*>(g.C) + (int64_t)m * g.ldc + n;
          floatx4 o;
          if (g.accumulate) {
            o = *reinterpret_cast<const floatx4*>(cp);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] += v[e];
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = v[e];
          }
          *reinterpret_cast<floatx4*>(cp) = o;
        } else {
          bf16_t* cp = reinterpret_cast<bf16_t*>(g.C) + (int64_t)m * g.ldc + n;
          if (EPI == EPI_ACC_BF16 && g.accumulate) {
            const bf16x4 cv = *reinterpret_cast<const bf16x4*>(cp);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += (float)cv[e];
          }
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)v[e];
          *reinterpret_cast<bf16x4*>(cp) = o;
        }
      }
    }
  }
}

// Only the (layout, epilogue) pairs the layer uses are instantiated: forward maps take the
// bias epilogues, input gradients the plain / GeLU' ones, weight gradients the accumulating ones.
constexpr bool epilogue_allowed(bool a_kc, bool b_kc, int e) {
  if (a_kc && !b_kc) return e == EPI_BIAS || e == EPI_BIAS_RES || e == EPI_BIAS_GELU;
  if (a_kc && b_kc) return e == EPI_BIAS || e == EPI_DGELU;
  if (!a_kc && !b_kc) return e == EPI_ACC_F32 || e == EPI_ACC_BF16;
  return false;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC>
static hipError_t launch_cfg(int epi, GemmArgs g, hipStream_t s) {
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  const dim3 grid(g.tiles_m * g.tiles_n), block(WGM * WGN * 64);
#define AXONN_GEMM_CASE(E)                                                                      \
  case E:                                                                                       \
    if constexpr (epilogue_allowed(A_KC, B_KC, E)) {                                            \
      hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, E>), grid, block, 0, s, g); \
      break;                                                                                    \
    } else {                                                                                    \
      return hipErrorInvalidValue;                                                              \
    }
  switch (epi) {
    AXONN_GEMM_CASE(EPI_BIAS)
    AXONN_GEMM_CASE(EPI_BIAS_RES)
    AXONN_GEMM_CASE(EPI_BIAS_GELU)
    AXONN_GEMM_CASE(EPI_DGELU)
    AXONN_GEMM_CASE(EPI_ACC_F32)
    AXONN_GEMM_CASE(EPI_ACC_BF16)
    default: return hipErrorInvalidValue;
  }
#undef AXONN_GEMM_CASE
  return hipGetLastError();
}

template <bool A_KC, bool B_KC>
static hipError_t launch_layout(int epi, const GemmArgs& g, hipStream_t s) {
  // Large tile when the problem fills the chip with it, smaller tile otherwise.
  const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big_tiles >= 128) return launch_cfg<256, 256, 64, 2, 4, A_KC, B_KC>(epi, g, s);
  return launch_cfg<128, 128, 64, 2, 2, A_KC, B_KC>(epi, g, s);
}

hipError_t launch_gemm(bool a_kc, bool b_kc, int epi, const GemmArgs& g, hipStream_t s) {
  if (a_kc && b_kc) return launch_layout<true, true>(epi, g, s);
  if (a_kc && !b_kc) return launch_layout<true, false>(epi, g, s);
  if (!a_kc && !b_kc) return launch_layout<false, false>(epi, g, s);
  return hipErrorInvalidValue;
}

}  // namespace axonn
