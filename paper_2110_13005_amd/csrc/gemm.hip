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

// Workgroup barrier that orders LDS traffic only: global loads issued before it may still be in
// flight after it (the prefetch of the next k-tile is).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int ROWS, int BK, bool KC>
struct TileLayout {
  // leading dimension in elements, padded so that fragment reads spread over LDS banks
  static constexpr int LD = KC ? (BK + 8) : (ROWS + 32);
  static constexpr int ELEMS = KC ? ROWS * LD : BK * LD;
};

// Writes one wave's TM x TN result tiles.  The MFMA was issued with the B fragment first, so
// lane l owns row m_base + 32*i + l%32 and register r of tile (i,j) is column
// n_base + 32*j + 8*(r/4) + 4*(l/32) + r%4: runs of 4 consecutive columns per lane.
template <int EPI, int TM, int TN>
__device__ __forceinline__ void gemm_epilogue(const floatx16 (&acc)[TM][TN], const GemmArgs& g,
                                              int m_base, int n_base, int lane) {
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m_base + i * 32 + (lane & 31);
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n_base + j * 32 + 8 * q + 4 * (lane >> 5);
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

  // Workgroups are dealt round-robin to the 8 XCDs; remap so that each XCD (own L2) works on a
  // contiguous run of tiles, and order tiles in bands of 8 tile-rows, column by column inside a band:
  // the ~32 tiles an XCD has in flight then form an 8 x 4 patch that shares 8 A panels and 4 B
  // panels instead of streaming 32 + 1.
  int pid = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  constexpr int BAND = 8;
  const int band_tiles = BAND * g.tiles_n;
  const int band = pid / band_tiles, in_band = pid - band * band_tiles;
  const int band_rows = min(BAND, g.tiles_m - band * BAND);
  const int tm = band * BAND + in_band % band_rows, tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;

  // Per-thread view of the tile copy: chunk j of this thread is 16 bytes at offset offa[j] of the
  // current k-segment, advanced by one k-step per iteration; it is valid if its row is inside the
  // matrix (fixed) and its k is inside the segment (checked per step).  Out-of-range chunks read a
  // zero chunk instead, so the loads are unconditional and stay in registers until the next step
  // stores them to LDS.
  const bf16_t* pa[A_CH];
  const bf16_t* pb[B_CH];
  int64_t offa[A_CH], offb[B_CH];
  bool va[A_CH], vb[B_CH];
  int ka[A_CH], kb[B_CH], oa[A_CH], ob[B_CH];
#pragma unroll
  for (int j = 0; j < A_CH; ++j) {
    const int c = tid + j * NT;
    if (A_KC) {
      const int row = c / (BK / 8), kc = c % (BK / 8);
      va[j] = (m0 + row) < g.M; ka[j] = kc * 8;
      offa[j] = (int64_t)(m0 + row) * g.lda + kc * 8;
      oa[j] = row * LA::LD + kc * 8;
    } else {
      const int kr = c / (BM / 8), rc = c % (BM / 8);
      va[j] = (m0 + rc * 8) < g.M; ka[j] = kr;
      offa[j] = (int64_t)kr * g.lda + m0 + rc * 8;
      oa[j] = kr * LA::LD + rc * 8;
    }
    pa[j] = g.A_seg[0] + offa[j];
  }
#pragma unroll
  for (int j = 0; j < B_CH; ++j) {
    const int c = tid + j * NT;
    if (B_KC) {
      const int row = c / (BK / 8), kc = c % (BK / 8);
      vb[j] = (n0 + row) < g.N; kb[j] = kc * 8;
      offb[j] = (int64_t)(n0 + row) * g.ldb + kc * 8;
      ob[j] = row * LB::LD + kc * 8;
    } else {
      const int kr = c / (BN / 8), rc = c % (BN / 8);
      vb[j] = (n0 + rc * 8) < g.N; kb[j] = kr;
      offb[j] = (int64_t)kr * g.ldb + n0 + rc * 8;
      ob[j] = kr * LB::LD + rc * 8;
    }
    pb[j] = g.B_seg[0] + offb[j];
  }
  const int64_t step_a = A_KC ? (int64_t)BK : (int64_t)BK * g.lda;
  const int64_t step_b = B_KC ? (int64_t)BK : (int64_t)BK * g.ldb;
  const int K = g.K;
  const int tps = (K + BK - 1) / BK;      // k-tiles per segment
  const int nk = tps * g.n_seg;
  const bf16_t* zero_chunk = reinterpret_cast<const bf16_t*>(g_zero_chunk);
  u32x4 ra[A_CH], rb[B_CH];
  int ld_seg = 0, ld_kin = 0;            // segment and k-tile within it of the NEXT tile to fetch

  // fetch the next k-tile into registers (zeros once all segments are exhausted)
#define AXONN_GLOAD()                                                          \
  {                                                                            \
    const bool live = ld_seg < g.n_seg;                                        \
    const int k0 = ld_kin * BK;                                                \
    _Pragma("unroll") for (int j = 0; j < A_CH; ++j) {                         \
      const bool ok = live & va[j] & (k0 + ka[j] < K);                         \
      ra[j] = *reinterpret_cast<const u32x4*>(ok ? pa[j] : zero_chunk);        \
      pa[j] += step_a;                                                         \
    }                                                                          \
    _Pragma("unroll") for (int j = 0; j < B_CH; ++j) {                         \
      const bool ok = live & vb[j] & (k0 + kb[j] < K);                         \
      rb[j] = *reinterpret_cast<const u32x4*>(ok ? pb[j] : zero_chunk);        \
      pb[j] += step_b;                                                         \
    }                                                                          \
    if (++ld_kin == tps) {                                                     \
      ld_kin = 0;                                                              \
      ++ld_seg;                                                                \
      const int sidx = ld_seg < g.n_seg ? ld_seg : 0;                          \
      const bf16_t* na = g.A_seg[sidx];                                        \
      const bf16_t* nb = g.B_seg[sidx];                                        \
      _Pragma("unroll") for (int j = 0; j < A_CH; ++j) pa[j] = na + offa[j];   \
      _Pragma("unroll") for (int j = 0; j < B_CH; ++j) pb[j] = nb + offb[j];   \
    }                                                                          \
    /* keep the loads here, at the start of the step: a full step of MFMA work hides them */ \
    __builtin_amdgcn_sched_barrier(0);                                         \
  }
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

  AXONN_GLOAD()
  AXONN_SSTORE(0)
  AXONN_GLOAD()            // tile 1 (all zeros if there is none)
  lds_barrier();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    // registers hold tile kt+1: park it in the other buffer, then fetch tile kt+2
    AXONN_SSTORE(cur ^ 1)
    AXONN_GLOAD()
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
    lds_barrier();
  }
#undef AXONN_GLOAD
#undef AXONN_SSTORE

  gemm_epilogue<EPI, TM, TN>(acc, g, m0 + wm * WTM, n0 + wn * WTN, lane);
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
