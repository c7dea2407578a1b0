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
// double-buffered LDS stage (global -> registers -> LDS, or global -> LDS by the memory pipeline in
// gemm_dma_kernel; one barrier per k-step).  k-contiguous
// tiles are read back with 128-bit LDS loads, k-strided tiles with the transposing LDS load,
// so no operand is ever transposed in HBM.  The MFMA is issued with the B fragment first, so a
// lane of the result owns one row m and runs of 4 consecutive columns n: epilogue loads and
// stores are 8-byte (bf16) or 16-byte (fp32) vectors along the contiguous dimension of C.
#include "common.h"
#include <atomic>
#include <type_traits>

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

// Output tile (tm, tn) of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs, each with an L2 of
// its own; the ids are remapped so that each XCD works on a contiguous run of tiles, and the tiles are ordered
// in bands of 8 tiles across the SHORTER side of the tile grid, walked along the longer side: the ~32 tiles an
// XCD has in flight then form an 8 x 4 patch that shares 8 + 4 operand panels instead of streaming 32 + 1, and
// the eight XCDs together work on few bands at a time (bands across the longer side -- 80 x 20 tiles, the
// weight gradient of the second MLP matrix -- put a different band, with 8 panels of the wide operand, on
// every XCD: 192 MB of panels in flight, beyond what the 256 MB last-level cache holds beside the rest).
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
  int pid = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  constexpr int BAND = 8;
  const bool wide = tiles_m <= tiles_n;                    // bands of tile rows, walked column by column
  const int t_band = wide ? tiles_m : tiles_n, t_walk = wide ? tiles_n : tiles_m;
  const int band_tiles = BAND * t_walk;
  const int band = pid / band_tiles, in_band = pid - band * band_tiles;
  const int band_w = min(BAND, t_band - band * BAND);
  const int a = band * BAND + in_band % band_w, b = in_band / band_w;
  tm = wide ? a : b;
  tn = wide ? b : a;
}

template <int ROWS, int BK, bool KC>
struct TileLayout {
  // leading dimension in elements, padded so that fragment reads spread over LDS banks
  static constexpr int LD = KC ? (BK + 8) : (ROWS + 32);
  static constexpr int ELEMS = KC ? ROWS * LD : BK * LD;
};

// Bias of columns n..n+3 as floats (zeros if there is none or the epilogue takes none).
template <int EPI>
__device__ __forceinline__ void load_bias4(float (&bv)[4], const GemmArgs& g, int n) {
#pragma unroll
  for (int e = 0; e < 4; ++e) bv[e] = 0.f;
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU) {
    if (g.bias) {
      const elemx4 b4 = *reinterpret_cast<const elemx4*>(g.bias + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[e] = (float)b4[e];
    }
  }
}

// What an epilogue reads at the position of its result: the residual, the stored pre-activation, or
// the previous value of an accumulating C.  `raw` holds the 4 values as loaded (bf16 in the low half
// of the words, or fp32); loading is separate from the arithmetic so that a caller can have the loads
// of many positions in flight before it consumes the first.
struct EpiOperand { uint32_t raw[4]; };

template <int EPI>
__device__ __forceinline__ bool epi_reads_operand(const GemmArgs& g) {
  return EPI == EPI_BIAS_RES || EPI == EPI_DGELU ||
         ((EPI == EPI_ACC_F32 || EPI == EPI_ACC_BF16) && g.accumulate);
}

// Leading dimension of what the epilogue reads or writes beside C (residual; stored derivative).
template <int EPI>
__device__ __forceinline__ int64_t epi_ld_side(const GemmArgs& g) {
  return EPI == EPI_BIAS_RES ? g.ld_res : (EPI == EPI_DGELU || EPI == EPI_BIAS_GELU) ? g.ld_aux : g.ldc;
}
// off_c = m * ldc + n, off_side = m * epi_ld_side + n (element offsets of the position).
template <int EPI>
__device__ __forceinline__ EpiOperand epi_load_operand(const GemmArgs& g, int64_t off_c, int64_t off_side) {
  EpiOperand o;
  if (EPI == EPI_ACC_F32) {
    const u32x4 t = *reinterpret_cast<const u32x4*>(reinterpret_cast<const float*>(g.C) + off_c);
    o.raw[0] = t[0]; o.raw[1] = t[1]; o.raw[2] = t[2]; o.raw[3] = t[3];
  } else {
    const elem_t* p = EPI == EPI_BIAS_RES ? g.res + off_side
                    : EPI == EPI_DGELU    ? g.aux + off_side
                                          : reinterpret_cast<const elem_t*>(g.C) + off_c;
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    o.raw[0] = t.x; o.raw[1] = t.y; o.raw[2] = 0u; o.raw[3] = 0u;
  }
  return o;
}

// The 4 operand values as floats.
template <int EPI>
__device__ __forceinline__ void epi_operand_values(const EpiOperand& o, float (&x)[4]) {
  if (EPI == EPI_ACC_F32) {
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = __uint_as_float(o.raw[e]);
  } else {
#ifdef AXONN_ELEM_FP16
    const elemx2 lo = __builtin_bit_cast(elemx2, o.raw[0]), hi = __builtin_bit_cast(elemx2, o.raw[1]);
    x[0] = (float)lo[0]; x[1] = (float)lo[1]; x[2] = (float)hi[0]; x[3] = (float)hi[1];
#else
    x[0] = __uint_as_float(o.raw[0] << 16); x[1] = __uint_as_float(o.raw[0] & 0xffff0000u);
    x[2] = __uint_as_float(o.raw[1] << 16); x[3] = __uint_as_float(o.raw[1] & 0xffff0000u);
#endif
  }
}

// Epilogue of 4 consecutive columns n..n+3 of row m (both inside the matrix): v = the sums, bv = their
// bias, `o` = the operand loaded with epi_load_operand (ignored if the epilogue reads none).
template <int EPI>
__device__ __forceinline__ void epi_finish(float (&v)[4], const float (&bv)[4], const EpiOperand& o,
                                           const GemmArgs& g, int64_t off_c, int64_t off_side) {
  float x[4] = {0.f, 0.f, 0.f, 0.f};
  if (epi_reads_operand<EPI>(g)) epi_operand_values<EPI>(o, x);
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += bv[e];
  }
  if (EPI == EPI_BIAS_RES || EPI == EPI_ACC_F32 || EPI == EPI_ACC_BF16) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += x[e];
  }
  if (EPI == EPI_BIAS_GELU) {
    // the derivative is formed here, from the unrounded pre-activation, and stored in its place: the
    // backward epilogue is then one multiplication
    elemx4 dv;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float y, dy;
      gelu_with_grad_f(v[e], y, dy);
      v[e] = y;
      dv[e] = (elem_t)dy;
    }
    *reinterpret_cast<elemx4*>(g.aux + off_side) = dv;
  }
  if (EPI == EPI_DGELU) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= x[e];
  }
  if (EPI == EPI_ACC_F32) {
    *reinterpret_cast<floatx4*>(reinterpret_cast<float*>(g.C) + off_c) = floatx4{v[0], v[1], v[2], v[3]};
  } else {
    elemx4 ov;
#pragma unroll
    for (int e = 0; e < 4; ++e) ov[e] = (elem_t)v[e];
    *reinterpret_cast<elemx4*>(reinterpret_cast<elem_t*>(g.C) + off_c) = ov;
  }
}

template <int EPI>
__device__ __forceinline__ void epilogue_run(float (&v)[4], const float (&bv)[4], const GemmArgs& g,
                                             int m, int n) {
  EpiOperand o;
  const int64_t off_c = (int64_t)m * g.ldc + n, off_side = (int64_t)m * epi_ld_side<EPI>(g) + n;
  if (epi_reads_operand<EPI>(g)) o = epi_load_operand<EPI>(g, off_c, off_side);
  epi_finish<EPI>(v, bv, o, g, off_c, off_side);
}

// Writes one wave's TM x TN result tiles of the 32x32x16 MFMA.  The MFMA was issued with the B
// fragment first, so lane l owns row m_base + 32*i + l%32 and register r of tile (i,j) is column
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
        float bv[4];
        load_bias4<EPI>(bv, g, n);
        epilogue_run<EPI>(v, bv, g, m, n);
      }
    }
  }
}

// Epilogue of a 128 x 16*TN wave tile held as 8 x TN tiles of the 16x16x32 MFMA (B fragment first: lane
// l owns row 16*i + l%16 and the 4 registers of tile (i,j) are columns 16*j + 4*(l/16) + 0..3).  Stored
// straight from that layout a wave instruction would touch 16 rows with 32 bytes each; instead the wave
// passes its tile, 64 rows at a time, through its own LDS region (row stride 16*TN + 4 floats:
// conflict-free both ways) and comes back with lane l owning columns 4*(l%32)..+3 of rows 2t + l/32: a
// wave instruction then covers two rows with up to 256 (bf16) or 512 (fp32) contiguous bytes each, for C
// as well as for the residual / pre-activation operands.  `stage` is wave-private: no workgroup barrier.
template <int TN>
struct StageLayout {
  static constexpr int LD = 16 * TN + 4;
  static constexpr int FLOATS_PER_WAVE = 64 * LD;
};
template <int EPI, int TN>
__device__ __forceinline__ void gemm_epilogue_staged(const floatx4 (&acc)[8][TN], const GemmArgs& g,
                                                     int m_base, int n_base, int lane, float* stage) {
  constexpr int LD = StageLayout<TN>::LD;
  const int nl = 4 * (lane & 31);                 // column inside the wave tile
  const int n = n_base + nl;
  const bool col_ok = nl < 16 * TN && n < g.N;
  float bv[4];
  if (col_ok) load_bias4<EPI>(bv, g, n);
  // What the epilogue reads at its output positions (residual, stored derivative, accumulating C) is
  // loaded in batches whose loads are all in flight together: the whole wave tile at once (64 row pairs,
  // 2 registers each) for bf16 operands, 16 row pairs at a time for an fp32 C.
  constexpr int OB = (EPI == EPI_ACC_F32) ? 16 : 64;
  EpiOperand opnd[OB];
  const bool reads = epi_reads_operand<EPI>(g);
  // element offsets of this lane's position in row pair 0 and their step from one row pair to the next:
  // additions per position instead of 64-bit multiplications
  const int64_t ld_side = epi_ld_side<EPI>(g);
  const int64_t off_c0 = (int64_t)(m_base + (lane >> 5)) * g.ldc + n, off_s0 = (int64_t)(m_base + (lane >> 5)) * ld_side + n;
  const int64_t step_c = 2 * g.ldc, step_s = 2 * ld_side;
  if (OB == 64 && reads) {
    int64_t oc = off_c0, os = off_s0;
#pragma unroll
    for (int t = 0; t < 64; ++t) {
      const int m = m_base + 2 * t + (lane >> 5);
      if (m < g.M && col_ok) opnd[t] = epi_load_operand<EPI>(g, oc, os);
      oc += step_c; os += step_s;
    }
  }
  int64_t oc_l = off_c0, os_l = off_s0;       // positions of the loads of an fp32 C, 16 row pairs at a time
  int64_t oc = off_c0, os = off_s0;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        *reinterpret_cast<floatx4*>(stage + (16 * ii + (lane & 15)) * LD + 16 * j + 4 * (lane >> 4)) =
            acc[4 * p + ii][j];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      if (OB == 16 && reads) {
#pragma unroll
        for (int tt = 0; tt < 16; ++tt) {
          const int m = m_base + 64 * p + 2 * (16 * hh + tt) + (lane >> 5);
          if (m < g.M && col_ok) opnd[tt] = epi_load_operand<EPI>(g, oc_l, os_l);
          oc_l += step_c; os_l += step_s;
        }
      }
#pragma unroll
      for (int tt = 0; tt < 16; ++tt) {
        const int r = 2 * (16 * hh + tt) + (lane >> 5);
        const int m = m_base + 64 * p + r;
        if (m < g.M && col_ok) {
          const floatx4 x = *reinterpret_cast<const floatx4*>(stage + r * LD + nl);
          float v[4] = {x[0], x[1], x[2], x[3]};
          epi_finish<EPI>(v, bv, opnd[OB == 64 ? 32 * p + 16 * hh + tt : tt], g, oc, os);
        }
        oc += step_c; os += step_s;
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

  __shared__ __align__(16) elem_t sA[2][LA::ELEMS];
  __shared__ __align__(16) elem_t sB[2][LB::ELEMS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroups are dealt round-robin to the 8 XCDs; remap so that each XCD (own L2) works on a
  // contiguous run of tiles, and order tiles in bands of 8 tile-rows, column by column inside a band:
  // the ~32 tiles an XCD has in flight then form an 8 x 4 patch that shares 8 A panels and 4 B
  // panels instead of streaming 32 + 1.
  int tm, tn;
  tile_of_block(g.tiles_m, g.tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  // Per-thread view of the tile copy: chunk j of this thread is 16 bytes at offset offa[j] of the
  // current k-segment, advanced by one k-step per iteration; it is valid if its row is inside the
  // matrix (fixed) and its k is inside the segment (checked per step).  Out-of-range chunks read a
  // zero chunk instead, so the loads are unconditional and stay in registers until the next step
  // stores them to LDS.
  const elem_t* pa[A_CH];
  const elem_t* pb[B_CH];
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
  const elem_t* zero_chunk = reinterpret_cast<const elem_t*>(g_zero_chunk);
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
      const elem_t* na = g.A_seg[sidx];                                        \
      const elem_t* nb = g.B_seg[sidx];                                        \
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
    const elem_t* a_s = sA[cur];
    const elem_t* b_s = sB[cur];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      elemx8 fa[TM], fb[TN];
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

// ---------------------------------------------------------------------------------------------
// Column sums of B beside a weight gradient.  The bias gradient of a linear map is the column sum of the same
// dy whose product with x^T is the weight gradient (Sec. 2: both are sums over the tokens of the microbatches),
// and the tiles of dy pass through the registers of the weight-gradient kernel anyway: the workgroups of tile
// row 0 (one per block of columns) add up their B fragments as they multiply them, so dy is not read from
// memory a second time.  A B fragment of the 16x16x32 MFMA holds, in lane l, 8 consecutive k of column l % 16;
// the sum over its elements, then over the four lanes that share the column, then over all k-steps is the
// column sum over every segment of the launch.  One wave per column half (wm == 0) does it, one pair of
// elements behind each of the first 4*TN MFMAs of a phase (the fragment that MFMA has just used), in a copy of
// the k loop of its own, so that the other waves' loop carries nothing of it.  The summing workgroup of column
// block tn is the one of tile row tn * tiles_m / tiles_n: the extra work is then spread evenly over the launch
// order, and with it over the XCDs (all in tile row 0 it made the XCD of the first band finish last: 20 us per
// launch of the 12B-shape weight gradients).
// Adds elements 2*pair and 2*pair + 1 of a B fragment to the lane's partial sum.
__device__ __forceinline__ void colsum_pair(float& cs, const elemx8& fb, int pair) {
#ifdef AXONN_ELEM_FP16
  cs += (float)fb[2 * pair] + (float)fb[2 * pair + 1];
#else
  const elemx2 ones = {(elem_t)1.0f, (elem_t)1.0f};
  const elemx2 two = {fb[2 * pair], fb[2 * pair + 1]};
  cs = __builtin_amdgcn_fdot2_f32_bf16(two, ones, cs, false);   // fp32 sum of the two and cs
#endif
}
// Stores (or, for an accumulating launch, adds) the sums of the wave's 16*TN columns from n_base on to
// g.colsum, which has the element type of C.
template <int EPI, int TN>
__device__ __forceinline__ void colsum_store(const float (&cs)[TN], const GemmArgs& g, int n_base, int lane) {
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    float v = cs[j];
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    const int n = n_base + 16 * j + lane;
    if (lane < 16 && n < g.N) {
      if (EPI == EPI_ACC_F32) {
        float* o = reinterpret_cast<float*>(g.colsum) + n;
        *o = g.accumulate ? *o + v : v;
      } else {
        elem_t* o = reinterpret_cast<elem_t*>(g.colsum) + n;
        *o = (elem_t)(g.accumulate ? (float)*o + v : v);
      }
    }
  }
}
constexpr bool epilogue_sums_columns(bool a_kc, bool b_kc, int e) {
  return !a_kc && !b_kc && (e == EPI_ACC_F32 || e == EPI_ACC_BF16);
}

// ------------------------------------------------------------------------------------------
// Large-problem kernel: 256 x (32*TN) x 64 block tile, 4 waves (2 x 2), wave tile 128 x 16*TN = 8 x TN
// tiles of the 16x16x32 MFMA held in accumulation registers (all 256 of them for TN = 8), so that each
// byte read from LDS feeds twice the MFMA work of a 128 x 64 wave tile.  TN = 8 is the most efficient
// shape; TN = 5 and 6 (block widths 160 and 192) exist because the tile count of a problem should fill
// the 256 CUs a whole number of times (hidden sizes of 5 * 2^k and 3 * 2^k divide evenly by them).
// One wave per SIMD: latency is hidden inside the wave by software pipelining.  A k-step is two
// phases of 8*TN MFMAs (one 32-wide k slice each); the fragments of a slice are read from LDS one phase
// ahead; the copy of the next tiles (registers -> LDS, then the registers are reloaded from global
// memory) is spread over the MFMAs of both phases, and the single barrier of the step sits just
// after the start of the second phase.
// Tiles are fetched with buffer loads: an offset at or beyond the descriptor's size returns zeros
// without touching memory, which covers rows outside the matrix, the k tail and the tiles past the
// last one without branches or per-chunk pointers.
constexpr uint32_t kOutOfRange = 0x80000000u;


// Item idx of n items spread evenly over the MFMA slots [first, first + span), and its inverse (-1: no
// item at slot q).  span >= n, so that no two items share a slot.
constexpr int spread_slot(int idx, int n, int first, int span) { return first + idx * span / n; }
constexpr int item_at(int q, int n, int first, int span) {
  if (q < first) return -1;
  const int i = ((q - first) * n + span - 1) / span;     // the only candidate: smallest i with slot >= q
  return (i < n && spread_slot(i, n, first, span) == q) ? i : -1;
}

template <bool A_KC, bool B_KC, int EPI, int TN>
__global__ __launch_bounds__(256) void gemm_big_kernel(const GemmArgs g) {
  constexpr int BM = 256, BN = 32 * TN, BK = 64, TM = 8;
  // 16-byte chunks per thread and tile of A and of B.  A k-strided B tile always takes the copy pattern
  // and the LDS layout of the 256-wide tile (8 chunks per thread, 32 per k); the lanes whose columns lie
  // beyond a narrower block read "out of range" (zeros, no memory traffic) into LDS columns nobody uses.
  constexpr int NCA = 8, NCB = B_KC ? TN : 8;
  constexpr int NM = TM * TN;           // MFMAs per phase
  constexpr int NF = TM + TN;           // fragments per k slice
  using LA = TileLayout<BM, BK, A_KC>;
  using LB = TileLayout<B_KC ? BN : 256, BK, B_KC>;
  // one LDS block: A buffers 0,1, then B buffers 0,1; the epilogue reuses it as staging space
  constexpr int LDS_BYTES = 2 * (LA::ELEMS + LB::ELEMS) * (int)sizeof(elem_t);
  static_assert(LDS_BYTES >= 4 * StageLayout<TN>::FLOATS_PER_WAVE * (int)sizeof(float), "staging space of the epilogue");
  __shared__ __align__(16) char smem[LDS_BYTES];
#define sA(buf) (reinterpret_cast<elem_t*>(smem) + (buf) * LA::ELEMS)
#define sB(buf) (reinterpret_cast<elem_t*>(smem) + 2 * LA::ELEMS + (buf) * LB::ELEMS)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // Workgroups are dealt round-robin to the 8 XCDs; remap so that each XCD (own L2) works on a
  // contiguous run of tiles, ordered in bands of 8 tile-rows, column by column inside a band.
  int tm, tn;
  tile_of_block(g.tiles_m, g.tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  // Chunk j of this thread of operand A: byte offset va + j * ja from the segment base, advanced by sa per
  // k-step; it lands at element wa + j * WJA of the LDS tile.  The same for B.
  const uint32_t lda = (uint32_t)g.lda, ldb = (uint32_t)g.ldb;
  uint32_t va, vb, ja, jb, sa, sb, nra, nrb;
  int wa, wb, kca = 0, kcb = 0;
  constexpr int WJA = A_KC ? 32 * LA::LD : 8 * LA::LD;
  constexpr int WJB = B_KC ? 32 * LB::LD : 8 * LB::LD;
  if (A_KC) {
    const int row = tid >> 3, kc = tid & 7;
    va = ((uint32_t)(m0 + row) * lda + kc * 8) * 2u; ja = 32u * lda * 2u; sa = BK * 2u;
    wa = row * LA::LD + kc * 8; kca = kc * 8; nra = (uint32_t)g.M * lda * 2u;
  } else {
    const int kr = tid >> 5, rc = tid & 31;
    va = (m0 + rc * 8 < g.M) ? ((uint32_t)kr * lda + m0 + rc * 8) * 2u : kOutOfRange;
    ja = 8u * lda * 2u; sa = BK * lda * 2u;
    wa = kr * LA::LD + rc * 8; nra = (uint32_t)g.K * lda * 2u;
  }
  if (B_KC) {
    const int row = tid >> 3, kc = tid & 7;
    vb = ((uint32_t)(n0 + row) * ldb + kc * 8) * 2u; jb = 32u * ldb * 2u; sb = BK * 2u;
    wb = row * LB::LD + kc * 8; kcb = kc * 8; nrb = (uint32_t)g.N * ldb * 2u;
  } else {
    const int kr = tid >> 5, rc = tid & 31;
    vb = (rc * 8 < BN && n0 + rc * 8 < g.N) ? ((uint32_t)kr * ldb + n0 + rc * 8) * 2u : kOutOfRange;
    jb = 8u * ldb * 2u; sb = BK * ldb * 2u;
    wb = kr * LB::LD + rc * 8; nrb = (uint32_t)g.K * ldb * 2u;
  }
  const int K = g.K;
  const int tps = (K + BK - 1) / BK;      // k-tiles per segment
  const int nk = tps * g.n_seg;
  __amdgpu_buffer_rsrc_t rsa = make_rsrc(g.A_seg[0], nra), rsb = make_rsrc(g.B_seg[0], nrb);
  u32x4 ra[NCA], rb[NCB];
  int ld_seg = 0, ld_kin = 0;            // segment and k-tile within it of the NEXT tile to fetch

  // Fetch of the next tile, split so that it can be interleaved with MFMAs: BEGIN computes the
  // offsets, LOAD_A/B(c) issue the load of chunk c, END advances to the next tile.
  uint32_t xa, xb;
#define AXONN_GLOAD_BEGIN()                                                                    \
  {                                                                                            \
    const bool live = ld_seg < g.n_seg;                                                        \
    xa = ((live & (!A_KC | (ld_kin * BK + kca < K))) ? va : kOutOfRange) + (uint32_t)ld_kin * sa; \
    xb = ((live & (!B_KC | (ld_kin * BK + kcb < K))) ? vb : kOutOfRange) + (uint32_t)ld_kin * sb; \
  }
#define AXONN_LOAD_A(c) ra[c] = __builtin_amdgcn_raw_buffer_load_b128(rsa, xa + (c) * ja, 0, 0);
#define AXONN_LOAD_B(c) rb[c] = __builtin_amdgcn_raw_buffer_load_b128(rsb, xb + (c) * jb, 0, 0);
#define AXONN_GLOAD_END()                                                                      \
  if (++ld_kin == tps) {                                                                       \
    ld_kin = 0;                                                                                \
    ++ld_seg;                                                                                  \
    const int sidx = ld_seg < g.n_seg ? ld_seg : 0;                                            \
    rsa = make_rsrc(g.A_seg[sidx], nra);                                                       \
    rsb = make_rsrc(g.B_seg[sidx], nrb);                                                       \
  }
#define AXONN_STORE_A(buf, c) *reinterpret_cast<u32x4*>(&sA(buf)[wa + (c) * WJA]) = ra[c];
#define AXONN_STORE_B(buf, c) *reinterpret_cast<u32x4*>(&sB(buf)[wb + (c) * WJB]) = rb[c];
  // Fragment f (0..NF-1) of k slice kk (0 or 1) of the tile in buffer buf -> fragment set F, in the
  // order the MFMAs of the slice consume them: a0 b0..b(TN-1) a1..a7.
#define AXONN_FRAG(F, buf, kk, f)                                                              \
  if ((f) == 0 || (f) > TN) {                                                                  \
    const int i = (f) == 0 ? 0 : (f) - TN;                                                     \
    const int r0 = wm * 128 + i * 16;                                                          \
    fa[F][i] = A_KC ? frag16_kcontig(sA(buf) + r0 * LA::LD + (kk) * 32, LA::LD, lane)          \
                    : frag16_kstrided(sA(buf) + ((kk) * 32) * LA::LD + r0, LA::LD, lane);      \
  } else {                                                                                     \
    const int j = (f) - 1;                                                                     \
    const int r0 = wn * (16 * TN) + j * 16;                                                    \
    fb[F][j] = B_KC ? frag16_kcontig(sB(buf) + r0 * LB::LD + (kk) * 32, LB::LD, lane)          \
                    : frag16_kstrided(sB(buf) + ((kk) * 32) * LB::LD + r0, LB::LD, lane);      \
  }
#define AXONN_CS(F, q) if (CSL && (q) < 4 * TN) colsum_pair(cs[(q) % TN], fb[F][(q) % TN], (q) / TN);
#define AXONN_MFMA(F, q) mfma16_acc(acc[(q) / TN][(q) % TN], fb[F][(q) % TN], fa[F][(q) / TN]); AXONN_CS(F, q)
  // One k-step on the tile kt in buffer CUR: two phases of NM MFMAs (k slices 0 and 1), between which
  // the other memory instructions are spread as evenly as their dependences allow, so that neither the
  // LDS nor the issue port sees bursts:
  //   phase 0: fragment reads of slice 1; the B chunks of tile kt+1 go from registers to buffer CUR^1
  //            (first half), then their registers are reloaded with those chunks of tile kt+2 (second
  //            half);
  //   barrier after MFMA 5 of phase 1: by then all of the above has completed, every wave is done with
  //            buffer CUR and tile kt+1 is complete in buffer CUR^1;
  //   phase 1: fragment reads of slice 0 of tile kt+1; the A chunks of tile kt+2 go to buffer CUR and
  //            are reloaded with those of tile kt+3.
  // Every chunk is so in flight for one whole k-step.
#define AXONN_KSTEP(CUR)                                                                       \
  _Pragma("unroll") for (int q = 0; q < NM; ++q) {                                             \
    AXONN_MFMA(0, q)                                                                           \
    { const int f = item_at(q, NF, 0, NM - 3); if (f >= 0) { AXONN_FRAG(1, CUR, 1, f) } }      \
    { const int c = item_at(q, NCB, 1, NM / 2 - 1); if (c >= 0) { AXONN_STORE_B((CUR) ^ 1, c) } } \
    { const int c = item_at(q, NCB, NM / 2 + 1, NM / 2 - 1); if (c >= 0) { AXONN_LOAD_B(c) } } \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }                                                                                            \
  AXONN_GLOAD_END()                                                                            \
  AXONN_GLOAD_BEGIN()                                                                          \
  _Pragma("unroll") for (int q = 0; q < 6; ++q) {                                              \
    AXONN_MFMA(1, q)                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }                                                                                            \
  lds_barrier();                                                                               \
  _Pragma("unroll") for (int q = 6; q < NM; ++q) {                                             \
    AXONN_MFMA(1, q)                                                                           \
    { const int f = item_at(q, NF, 8, NM - 8); if (f >= 0) { AXONN_FRAG(0, (CUR) ^ 1, 0, f) } } \
    { const int c = item_at(q, NCA, 9, NM - 12); if (c >= 0) { AXONN_STORE_A(CUR, c) } }       \
    { const int c = item_at(q, NCA, 11, NM - 12); if (c >= 0) { AXONN_LOAD_A(c) } }            \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }

  floatx4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
  elemx8 fa[2][TM], fb[2][TN];
  constexpr bool CS = epilogue_sums_columns(A_KC, B_KC, EPI);
  const bool cs_on = CS && g.colsum != nullptr && wm == 0 &&              // the same for all lanes of a wave
                     tm == (int)((int64_t)tn * g.tiles_m / g.tiles_n);
  float cs[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) cs[j] = 0.f;

  // prologue: tile 0 in buffer 0; the A chunks of tile 1 in buffer 1 and its B chunks in registers;
  // the A chunks of tile 2 on their way (tiles that do not exist read as zeros)
  AXONN_GLOAD_BEGIN()
#pragma unroll
  for (int c = 0; c < NCA; ++c) { AXONN_LOAD_A(c) }
#pragma unroll
  for (int c = 0; c < NCB; ++c) { AXONN_LOAD_B(c) }
  AXONN_GLOAD_END()
#pragma unroll
  for (int c = 0; c < NCA; ++c) { AXONN_STORE_A(0, c) }
#pragma unroll
  for (int c = 0; c < NCB; ++c) { AXONN_STORE_B(0, c) }
  AXONN_GLOAD_BEGIN()
#pragma unroll
  for (int c = 0; c < NCA; ++c) { AXONN_LOAD_A(c) }
#pragma unroll
  for (int c = 0; c < NCB; ++c) { AXONN_LOAD_B(c) }
  AXONN_GLOAD_END()
#pragma unroll
  for (int c = 0; c < NCA; ++c) { AXONN_STORE_A(1, c) }
  AXONN_GLOAD_BEGIN()
#pragma unroll
  for (int c = 0; c < NCA; ++c) { AXONN_LOAD_A(c) }
  lds_barrier();
#pragma unroll
  for (int f = 0; f < NF; ++f) { AXONN_FRAG(0, 0, 0, f) }
  asm volatile("s_nop 7" ::: "memory");      // accumulators were just zeroed: settle before the first MFMA
  // two k-steps per iteration so that the buffer index is a constant; an odd tile count is padded
  // with a tile of zeros
  auto k_loop = [&](auto with_colsum) {
    constexpr bool CSL = decltype(with_colsum)::value;
    for (int kt = 0; kt < nk; kt += 2) {
      AXONN_KSTEP(0)
      AXONN_KSTEP(1)
    }
  };
  if (CS && cs_on) k_loop(std::true_type{}); else k_loop(std::false_type{});
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // last MFMAs drain before the results are read
#undef AXONN_GLOAD_BEGIN
#undef AXONN_LOAD_A
#undef AXONN_LOAD_B
#undef AXONN_GLOAD_END
#undef AXONN_STORE_A
#undef AXONN_STORE_B
#undef AXONN_FRAG
#undef AXONN_MFMA
#undef AXONN_CS
#undef AXONN_KSTEP

  lds_barrier();                                          // every wave is done with the tiles in LDS
  gemm_epilogue_staged<EPI, TN>(acc, g, m0 + wm * 128, n0 + wn * (16 * TN), lane,
                                reinterpret_cast<float*>(smem) + wave * StageLayout<TN>::FLOATS_PER_WAVE);
  if (CS) { if (cs_on) colsum_store<EPI, TN>(cs, g, n0 + wn * (16 * TN), lane); }
#undef sA
#undef sB
}

// ---------------------------------------------------------------------------------------------
// gemm_dma_kernel: the tiling of gemm_big_kernel (256 x 32*TN x 64 block, 2 x 2 waves, one wave per
// SIMD, 128 x 16*TN wave tile of 16x16x32 MFMAs) with the tiles copied global -> LDS by the memory
// pipeline itself (`buffer_load_dwordx4 ... lds`): no staging registers, no LDS store instructions, no
// vector ALU work for addresses inside the loop.  For problems whose K is a multiple of 64.
//
// One such instruction writes the 64 chunks of 16 bytes its lanes fetch to 1 KB of consecutive LDS
// bytes in lane order (M0 holds the start), so the LDS tiles cannot be padded; instead the lanes
// fetch a permutation of the chunks, chosen so that the fragment reads stay free of bank conflicts:
//   k-contiguous tile  [row][64 k]: 128 bytes per row; slot p of row r holds chunk p ^ ((r >> 1) & 7).
//                      An instruction covers 8 rows.
//   k-strided tile     [k][256 rows]: 512 bytes per k, in natural order.  An instruction covers the k
//                      rows 8c + w and 8c + w + 4 (one per half wave); its 1 KB block is followed by
//                      32 bytes of padding, so that the 8 k rows a transposing read touches in one
//                      pass (k0 .. k0+3 and k0+8 .. k0+11, 32 bytes each) fall into different banks.
// Two stages of one 64-wide k tile each.  A k-step (tile kt in stage CUR) is two phases of 8*TN MFMAs:
// phase 0 multiplies k slice 0 while the fragments of slice 1 are read, phase 1 multiplies slice 1 while the
// slice-0 fragments of tile kt+1 are read from stage CUR^1.  Stage CUR is refilled with tile kt+2 as its
// parts fall free:
//   a k-strided tile by halves (copy instructions c < 4 hold k slice 0, the others slice 1): a few MFMAs
//     into phase 0 a barrier tells that nobody reads slice 0 of stage CUR any more, and that half is copied
//     during the rest of phase 0; the other half likewise behind the barrier of phase 1;
//   a k-contiguous tile (each instruction spans both slices) behind the barrier of phase 1 only.
// The wave waits for its own copies in front of each barrier: `s_waitcnt vmcnt(n)` with n = the number of
// younger copies that may still be in flight; every copy has (nearly) a whole k-step to arrive.  With all 16
// copies of a (k-strided, k-strided) problem behind the one barrier of phase 1 (the previous form, one copy
// per 3.5 MFMAs) the memory pipeline did not keep up, and an MFMA behind a copy that cannot issue yet waits
// with it; spread over both phases (one per 7 MFMAs) the weight-gradient shapes of the 12B stage gained
// 4 % (1212 -> 1262 TFLOP/s).  Splitting k-contiguous tiles the same way needs copies of 64 bytes per row,
// half a cache line: measured 3-6 % slower than whole lines behind one barrier.
// The copies are inline assembly: the compiler neither sees them nor counts them in vmcnt, so the
// waits on them are written out here, and the loop contains no other vector memory instruction.
__device__ __forceinline__ void dma_chunk16(u32x4 rsrc, uint32_t voffset, uint32_t soffset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory");
}
// One MFMA with a copy around it: M0 is written in front of the MFMA and consumed behind it (the MFMA is
// the independent instruction the hardware wants between the two).  One statement, so that nothing the
// compiler emits can come between the write of M0 and its use.
__device__ __forceinline__ void mfma16_acc_dma(floatx4& c, elemx8 a, elemx8 b, u32x4 rsrc, uint32_t voffset,
                                               uint32_t soffset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %3\n\t" AXONN_MFMA_16X16X32_ASM " %0, %1, %2, %0\n\t"
               "buffer_load_dwordx4 %4, %5, %6 offen lds"
               : "+a"(c)
               : "v"(a), "v"(b), "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory");
}
__device__ __forceinline__ void dma_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Buffer descriptor words of `bytes` bytes at p (raw buffer, offsets at or beyond `bytes` read zeros).
__device__ __forceinline__ u32x4 rsrc_words(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  u32x4 r;
  r[0] = (uint32_t)a; r[1] = (uint32_t)(a >> 32) & 0xffffu; r[2] = bytes; r[3] = 0x00020000u;
  return r;
}

// The copy instructions of a k-step in the order they are issued.  Phase 0: the first halves of the
// k-strided operands and the "early" rows of a k-contiguous A.  Phase 1: the rest of the k-contiguous
// operands, then the second halves of the k-strided ones.
// The early rows of a k-contiguous A are those of the fragments i < 4 of either wave row (tile rows 0..63 and
// 128..191, copy instructions 0, 1, 4, 5): an MFMA phase uses A fragment i in MFMAs i*TN .. i*TN + TN-1 only, so
// the registers of the fragments i < 4 of k slice 1 are free half way through phase 1, and that half of the phase
// reads into them the same fragments of the NEXT tile (which a k-contiguous copy has delivered together with its
// slice 0).  Those rows of the stage are then free one phase earlier than the others.
// Returns c for copy instruction c of A, nca + c for copy instruction c of B.
constexpr bool kDmaEarlyRows = true;
constexpr int dma_count(bool a_kc, bool b_kc, int nca, int ncb, int phase) {
  const bool a_split = !a_kc || kDmaEarlyRows;
  return phase == 0 ? (a_split ? nca / 2 : 0) + (b_kc ? 0 : ncb / 2) : (a_split ? nca / 2 : nca) + (b_kc ? ncb : ncb / 2);
}
constexpr int dma_early_row_item(int d, bool early) {      // 0, 1, 4, 5 / 2, 3, 6, 7
  return (d & 1) + 4 * (d >> 1) + (early ? 0 : 2);
}
constexpr int dma_item(bool a_kc, bool b_kc, int nca, int ncb, int phase, int d) {
  if (phase == 0) {
    if (!a_kc || kDmaEarlyRows) { if (d < nca / 2) return a_kc ? dma_early_row_item(d, true) : d; d -= nca / 2; }
    return nca + d;
  }
  if (a_kc && kDmaEarlyRows) { if (d < nca / 2) return dma_early_row_item(d, false); d -= nca / 2; }
  if (a_kc && !kDmaEarlyRows) { if (d < nca) return d; d -= nca; }
  if (b_kc) { if (d < ncb) return nca + d; d -= ncb; }
  if (!a_kc) { if (d < nca / 2) return nca / 2 + d; d -= nca / 2; }
  return nca + ncb / 2 + d;
}
// Fragment f (0: a0, 1..tn: b0.., tn+1..: a1..) that is the k-th one read in a phase; with early rows the
// fragments a0..a3 of slice 1 are not read in phase 0.
constexpr int frag_count(bool a_early, int tn, int phase) { return 8 + tn - (a_early && phase == 0 ? 4 : 0); }
constexpr int frag_item(bool a_early, int tn, int phase, int k) {
  if (!(a_early && phase == 0)) return k;
  return k < tn ? k + 1 : k + 4;      // b0 .. b(tn-1), then a4 .. a7
}

template <bool A_KC, bool B_KC, int EPI, int TN>
__global__ __launch_bounds__(256) void gemm_dma_kernel(const GemmArgs g) {
  constexpr int BM = 256, BN = 32 * TN, BK = 64, TM = 8;
  constexpr int NCA = 8, NCB = B_KC ? TN : 8;     // copy instructions per wave and tile
  constexpr int NM = TM * TN, NF = TM + TN, ND = NCA + NCB;
  // copies per phase; of those of phase 1, the ones that belong to k-strided operands (issued last)
  constexpr int N0 = dma_count(A_KC, B_KC, NCA, NCB, 0), N1 = dma_count(A_KC, B_KC, NCA, NCB, 1);
  constexpr int N1S = (A_KC ? 0 : NCA / 2) + (B_KC ? 0 : NCB / 2);
  static_assert(N0 + N1 == ND && 2 * (N0 + N1) < 64, "copy bookkeeping");
  constexpr bool A_EARLY = A_KC && kDmaEarlyRows;
  constexpr int KS_BLOCK = 1024 + 32;             // two k rows of a k-strided tile and their padding
  constexpr int SA = A_KC ? BM * BK * 2 : 32 * KS_BLOCK;              // bytes of one stage of A
  constexpr int SB = B_KC ? BN * BK * 2 : 32 * KS_BLOCK;              // and of B
  constexpr int TILE_BYTES = 2 * (SA + SB);
  constexpr int EPI_BYTES = 4 * StageLayout<TN>::FLOATS_PER_WAVE * (int)sizeof(float);
  constexpr int LDS_BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
  __shared__ __align__(1024) char smem[LDS_BYTES];   // A stage 0, A stage 1, B stage 0, B stage 1

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  int tm, tn;
  tile_of_block(g.tiles_m, g.tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  // Copy instruction c of this wave: the byte offset of each lane's chunk from the segment base in
  // k-tile 0 (kOutOfRange for rows outside the matrix), and the bytes to add per k-tile (uniform).
  const uint32_t lda = (uint32_t)g.lda, ldb = (uint32_t)g.ldb;
  uint32_t va[NCA], vb[NCB];
  uint32_t sa, sb, nra, nrb;
  if (A_KC) {
    const int q = (lane & 7) ^ (((wave & 1) << 2) + (lane >> 4));
#pragma unroll
    for (int c = 0; c < NCA; ++c) {
      const int row = m0 + (c * 4 + wave) * 8 + (lane >> 3);
      va[c] = row < g.M ? ((uint32_t)row * lda + q * 8) * 2u : kOutOfRange;
    }
    sa = BK * 2u; nra = (uint32_t)g.M * lda * 2u;
  } else {
#pragma unroll
    for (int c = 0; c < NCA; ++c) {
      const int k = 8 * c + wave + 4 * (lane >> 5);
      const int col = m0 + ((lane & 31) << 3);
      va[c] = col < g.M ? ((uint32_t)k * lda + col) * 2u : kOutOfRange;
    }
    sa = BK * lda * 2u; nra = (uint32_t)g.K * lda * 2u;
  }
  if (B_KC) {
    const int q = (lane & 7) ^ (((wave & 1) << 2) + (lane >> 4));
#pragma unroll
    for (int c = 0; c < NCB; ++c) {
      const int row = n0 + (c * 4 + wave) * 8 + (lane >> 3);
      vb[c] = row < g.N ? ((uint32_t)row * ldb + q * 8) * 2u : kOutOfRange;
    }
    sb = BK * 2u; nrb = (uint32_t)g.N * ldb * 2u;
  } else {
#pragma unroll
    for (int c = 0; c < NCB; ++c) {
      const int k = 8 * c + wave + 4 * (lane >> 5);
      const int cl = (lane & 31) << 3;
      vb[c] = (cl < BN && n0 + cl < g.N) ? ((uint32_t)k * ldb + n0 + cl) * 2u : kOutOfRange;
    }
    sb = BK * ldb * 2u; nrb = (uint32_t)g.K * ldb * 2u;
  }

  // Fragment reads: per-lane byte offsets into `smem` that do not depend on stage and k slice.
  //   k-contiguous: rows r0 + lane%16 (r0 a multiple of 16), chunk 4*kk + lane/16 of the row; one offset
  //                 per k slice, fragment i adds i * 16 rows.
  //   k-strided:    k rows 32*kk + 8*(lane/16) + (lane%16)/4 (+4 for the second half: the other half of
  //                 the same block), elements r0 + 4*(lane%4) .. +3; one offset.
  const int ft = lane & 15, fg = lane >> 4;
  uint32_t fa_off[A_KC ? 2 : 1], fb_off[B_KC ? 2 : 1];
  if (A_KC) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
      fa_off[kk] = (uint32_t)((wm * 128 + ft) * 128 + ((((kk << 2) + fg) ^ ((lane >> 1) & 7)) << 4));
  } else {
    fa_off[0] = (uint32_t)((4 * fg + (ft >> 2)) * KS_BLOCK + (wm * 128 + 4 * (ft & 3)) * 2);
  }
  if (B_KC) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
      fb_off[kk] = (uint32_t)(2 * SA + (wn * 16 * TN + ft) * 128 + ((((kk << 2) + fg) ^ ((lane >> 1) & 7)) << 4));
  } else {
    fb_off[0] = (uint32_t)(2 * SA + (4 * fg + (ft >> 2)) * KS_BLOCK + (wn * 16 * TN + 4 * (ft & 3)) * 2);
  }

  const int tps = g.K / BK;               // k-tiles per segment (K is a multiple of BK)
  const int nk = tps * g.n_seg;
  int ld_seg = 0, ld_kin = 0;             // segment and k-tile within it of the NEXT tile to fetch
  u32x4 rsa = rsrc_words(g.A_seg[0], nra), rsb = rsrc_words(g.B_seg[0], nrb);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(AXONN_LDS char*)smem;

  // Copy instruction d (A chunks first, then B chunks) of the next tile into stage `buf`.
#define AXONN_DMA(buf, d)                                                                      \
  if ((d) < NCA) {                                                                             \
    dma_chunk16(rsa, va[(d) < NCA ? (d) : 0], (uint32_t)ld_kin * sa,                           \
                lds0 + (buf) * SA + ((d) * 4 + wave) * (A_KC ? 1024 : KS_BLOCK));              \
  } else {                                                                                     \
    dma_chunk16(rsb, vb[(d) >= NCA ? (d) - NCA : 0], (uint32_t)ld_kin * sb,                    \
                lds0 + 2 * SA + (buf) * SB + (((d) - NCA) * 4 + wave) * (B_KC ? 1024 : KS_BLOCK)); \
  }
  // The tile after the last one of the last segment does not exist: a descriptor of size 0 makes its
  // copies write zeros (the tile that pads an odd tile count is multiplied, the others are not read).
#define AXONN_MFMA_DMA(F, q, buf, d)                                                           \
  if ((d) < NCA) {                                                                             \
    mfma16_acc_dma(acc[(q) / TN][(q) % TN], fb[F][(q) % TN], fa[F][(q) / TN], rsa,             \
                   va[(d) < NCA ? (d) : 0], (uint32_t)ld_kin * sa,                             \
                   lds0 + (buf) * SA + ((d) * 4 + wave) * (A_KC ? 1024 : KS_BLOCK));           \
  } else {                                                                                     \
    mfma16_acc_dma(acc[(q) / TN][(q) % TN], fb[F][(q) % TN], fa[F][(q) / TN], rsb,             \
                   vb[(d) >= NCA ? (d) - NCA : 0], (uint32_t)ld_kin * sb,                      \
                   lds0 + 2 * SA + (buf) * SB + (((d) - NCA) * 4 + wave) * (B_KC ? 1024 : KS_BLOCK)); \
  }
#define AXONN_DMA_NEXT()                                                                       \
  if (++ld_kin == tps) {                                                                       \
    ld_kin = 0;                                                                                \
    ++ld_seg;                                                                                  \
    const bool live = ld_seg < g.n_seg;                                                        \
    const int sidx = live ? ld_seg : 0;                                                        \
    rsa = rsrc_words(g.A_seg[sidx], live ? nra : 0u);                                          \
    rsb = rsrc_words(g.B_seg[sidx], live ? nrb : 0u);                                          \
  }
#define AXONN_FRAG(F, buf, kk, f)                                                              \
  if ((f) == 0 || (f) > TN) {                                                                  \
    const int i = (f) == 0 ? 0 : (f) - TN;                                                     \
    if (A_KC) {                                                                                \
      fa[F][i] = *reinterpret_cast<const elemx8*>(smem + fa_off[A_KC ? (kk) : 0] + (buf) * SA + i * 2048); \
    } else {                                                                                   \
      const char* pf = smem + fa_off[0] + (buf) * SA + (kk) * 16 * KS_BLOCK + i * 32;          \
      union { elemx8 v; short4v h[2]; } u;                                                     \
      u.h[0] = lds_read_tr16(reinterpret_cast<const elem_t*>(pf));                             \
      u.h[1] = lds_read_tr16(reinterpret_cast<const elem_t*>(pf + 512));                       \
      fa[F][i] = u.v;                                                                          \
    }                                                                                          \
  } else {                                                                                     \
    const int j = (f) - 1;                                                                     \
    if (B_KC) {                                                                                \
      fb[F][j] = *reinterpret_cast<const elemx8*>(smem + fb_off[B_KC ? (kk) : 0] + (buf) * SB + j * 2048); \
    } else {                                                                                   \
      const char* pf = smem + fb_off[0] + (buf) * SB + (kk) * 16 * KS_BLOCK + j * 32;          \
      union { elemx8 v; short4v h[2]; } u;                                                     \
      u.h[0] = lds_read_tr16(reinterpret_cast<const elem_t*>(pf));                             \
      u.h[1] = lds_read_tr16(reinterpret_cast<const elem_t*>(pf + 512));                       \
      fb[F][j] = u.v;                                                                          \
    }                                                                                          \
  }
#define AXONN_CS(F, q) if (CSL && (q) < 4 * TN) colsum_pair(cs[(q) % TN], fb[F][(q) % TN], (q) / TN);
#define AXONN_MFMA(F, q) mfma16_acc(acc[(q) / TN][(q) % TN], fb[F][(q) % TN], fa[F][(q) / TN]); AXONN_CS(F, q)
  // One phase: multiplies the fragments of set FMUL; reads k slice RDKK of stage RDBUF into set FRD and
  // issues the copies of phase PH of the next tile to fetch into stage DMABUF.  Phase 0 of a problem without a
  // k-strided operand has no copies, no wait and no barrier.
#define AXONN_PHASE(FMUL, FRD, RDBUF, RDKK, DMABUF, PH)                                          \
  if ((PH) == 1 || N0 > 0) {                                                                     \
    _Pragma("unroll") for (int q = 0; q < 6; ++q) {                                              \
      AXONN_MFMA(FMUL, q)                                                                        \
      __builtin_amdgcn_sched_barrier(0);                                                         \
    }                                                                                            \
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"((PH) == 0 ? N0 + N1 : N1S + N0) : "memory");      \
    lds_barrier();                                                                               \
    _Pragma("unroll") for (int q = 6; q < NM; ++q) {                                             \
      const int dd = item_at(q, (PH) == 0 ? N0 : N1, 7, NM - 8);                                 \
      if (dd >= 0) {                                                                             \
        AXONN_MFMA_DMA(FMUL, q, DMABUF, dma_item(A_KC, B_KC, NCA, NCB, PH, dd))                  \
        AXONN_CS(FMUL, q)                                                                        \
      } else {                                                                                   \
        AXONN_MFMA(FMUL, q)                                                                      \
      }                                                                                          \
      { const int k = item_at(q, frag_count(A_EARLY, TN, PH), 8, NM - 8);                        \
        if (k >= 0) { AXONN_FRAG(FRD, RDBUF, RDKK, frag_item(A_EARLY, TN, PH, k)) } }            \
      if (A_EARLY && (PH) == 1) {      /* a0..a3 of slice 1 of the same tile, into registers that are free by now */ \
        const int e = item_at(q, 4, 4 * TN + 2, NM - 4 * TN - 3);                                \
        if (e >= 0) { AXONN_FRAG(FMUL, RDBUF, 1, e == 0 ? 0 : TN + e) }                          \
      }                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                         \
    }                                                                                            \
  } else {                                                                                       \
    _Pragma("unroll") for (int q = 0; q < NM; ++q) {                                             \
      AXONN_MFMA(FMUL, q)                                                                        \
      { const int f = item_at(q, NF, 0, NM - 3); if (f >= 0) { AXONN_FRAG(FRD, RDBUF, RDKK, f) } } \
      __builtin_amdgcn_sched_barrier(0);                                                         \
    }                                                                                            \
  }
#define AXONN_KSTEP(CUR)                                                                         \
  AXONN_PHASE(0, 1, CUR, 1, CUR, 0)                                                              \
  AXONN_PHASE(1, 0, (CUR) ^ 1, 0, CUR, 1)                                                        \
  AXONN_DMA_NEXT()

  floatx4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
  elemx8 fa[2][TM], fb[2][TN];
  constexpr bool CS = epilogue_sums_columns(A_KC, B_KC, EPI);
  const bool cs_on = CS && g.colsum != nullptr && wm == 0 &&              // the same for all lanes of a wave
                     tm == (int)((int64_t)tn * g.tiles_m / g.tiles_n);
  float cs[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) cs[j] = 0.f;

  // prologue: tiles 0 and 1 into stages 0 and 1, in the order of the loop
#pragma unroll
  for (int t = 0; t < 2; ++t) {
#pragma unroll
    for (int d = 0; d < N0; ++d) { AXONN_DMA(t, dma_item(A_KC, B_KC, NCA, NCB, 0, d)) }
#pragma unroll
    for (int d = 0; d < N1; ++d) { AXONN_DMA(t, dma_item(A_KC, B_KC, NCA, NCB, 1, d)) }
    AXONN_DMA_NEXT()
  }
  // k slice 0 of tile 0 has arrived once the only copies in flight are its second halves and tile 1
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N1S + N0 + N1) : "memory");
  lds_barrier();
#pragma unroll
  for (int f = 0; f < NF; ++f) { AXONN_FRAG(0, 0, 0, f) }
  if (A_EARLY) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { AXONN_FRAG(1, 0, 1, e == 0 ? 0 : TN + e) }
  }
  asm volatile("s_nop 7" ::: "memory");      // accumulators were just zeroed: settle before the first MFMA
  auto k_loop = [&](auto with_colsum) {
    constexpr bool CSL = decltype(with_colsum)::value;
    for (int kt = 0; kt < nk; kt += 2) {
      AXONN_KSTEP(0)
      AXONN_KSTEP(1)
    }
  };
  if (CS && cs_on) k_loop(std::true_type{}); else k_loop(std::false_type{});
  dma_wait_all();                            // copies of tiles past the end still write (zeros) to LDS
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // last MFMAs drain before the results are read
#undef AXONN_DMA
#undef AXONN_MFMA_DMA
#undef AXONN_PHASE
#undef AXONN_DMA_NEXT
#undef AXONN_FRAG
#undef AXONN_MFMA
#undef AXONN_CS
#undef AXONN_KSTEP

  lds_barrier();                                          // every wave is done with the tiles in LDS
  gemm_epilogue_staged<EPI, TN>(acc, g, m0 + wm * 128, n0 + wn * (16 * TN), lane,
                                reinterpret_cast<float*>(smem) + wave * StageLayout<TN>::FLOATS_PER_WAVE);
  if (CS) { if (cs_on) colsum_store<EPI, TN>(cs, g, n0 + wn * (16 * TN), lane); }
}

// Only the (layout, epilogue) pairs the layer uses are instantiated: forward maps take the
// bias epilogues, input gradients the plain / GeLU' ones, weight gradients the accumulating ones.
constexpr bool epilogue_allowed(bool a_kc, bool b_kc, int e) {
  if (a_kc && !b_kc) return e == EPI_BIAS || e == EPI_BIAS_RES || e == EPI_BIAS_GELU;
  if (a_kc && b_kc) return e == EPI_BIAS || e == EPI_DGELU;
  if (!a_kc && !b_kc) return e == EPI_ACC_F32 || e == EPI_ACC_BF16;
  return false;
}

// The column sums a launch asks for (g.colsum) by the stand-alone kernels, segment by segment: for the kernels
// that do not form them on the way.  g.colsum_ws: what launch_colsum needs for K rows of N columns.
static hipError_t colsum_separately(int epi, const GemmArgs& g, hipStream_t s) {
  if (!g.colsum) return hipSuccess;
  if (!g.colsum_ws || !(epi == EPI_ACC_F32 || epi == EPI_ACC_BF16)) return hipErrorInvalidValue;
  for (int i = 0; i < g.n_seg; ++i) {
    const hipError_t e = launch_colsum(g.K, g.N, g.B_seg[i], g.ldb, g.colsum, (g.accumulate || i > 0) ? 2 : 1,
                                       epi == EPI_ACC_F32, g.colsum_ws, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
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
  const hipError_t e = hipGetLastError();
  return e != hipSuccess ? e : colsum_separately(epi, g, s);   // these kernels leave the column sums to others
}

// Launcher settings that axonn_tuning() can change (process-wide; -1 = the built-in rule).
static std::atomic<int64_t> g_tune_copy_mask{-1}, g_tune_big_min_tiles{-1}, g_tune_tile_n{-1};

bool set_gemm_tuning(int knob, int64_t value) {
  if (value < -1) return false;
  switch (knob) {
    case 0: if (value > 15) return false; g_tune_copy_mask = value; return true;
    case 1: g_tune_big_min_tiles = value; return true;
    case 2: if (value != -1 && value != 0 && value != 160 && value != 192 && value != 256) return false;
            g_tune_tile_n = value; return true;
    default: return false;
  }
}

template <bool A_KC, bool B_KC, int TN>
static hipError_t launch_big(int epi, GemmArgs g, hipStream_t s) {
  g.tiles_m = (g.M + 255) / 256;
  g.tiles_n = (g.N + 32 * TN - 1) / (32 * TN);
  const dim3 grid(g.tiles_m * g.tiles_n), block(256);
  // The kernel with copies by the memory pipeline needs whole k tiles.  It is the faster one for every layout
  // with a 16-bit result (single launches of the 12B-shape problems: forward +11 %, input gradients +4 %, weight
  // gradients +8 % over the register-staged kernel; whole batches of the 12B / 24B / 100B stage shapes 3.4 / 3.3 /
  // 4.3 % faster than with the previous choice); with an fp32 read-modify-write result the register-staged
  // kernel stays ahead (110.3 vs 111.0 ms per 12B batch).
  // axonn_tuning(AXONN_TUNE_GEMM_COPY_MASK, m) fixes the choice per class instead (bit 0 (kc,kc), bit 1 (kc,ks),
  // bit 2 (ks,ks) with a 16-bit result, bit 3 (ks,ks) with an fp32 result): the tests run every case through
  // both kernels with it.
  const int64_t mask_set = g_tune_copy_mask.load();
  const int64_t dma_mask = mask_set >= 0 ? mask_set : 7;
  const int dma_bit = A_KC ? (B_KC ? 0 : 1) : (epi == EPI_ACC_F32 ? 3 : 2);
  const bool use_dma = ((dma_mask >> dma_bit) & 1) && g.K % 64 == 0;
#define AXONN_GEMM_CASE(E)                                                                      \
  case E:                                                                                       \
    if constexpr (epilogue_allowed(A_KC, B_KC, E)) {                                            \
      if (use_dma)                                                                              \
        hipLaunchKernelGGL((gemm_dma_kernel<A_KC, B_KC, E, TN>), grid, block, 0, s, g);         \
      else                                                                                      \
        hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, E, TN>), grid, block, 0, s, g);         \
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
  return hipGetLastError();          // both kernels form the column sums of a weight gradient themselves
}

// The large-problem kernel addresses an operand with 32-bit byte offsets from the segment base.
static bool fits_32bit_offsets(int64_t rows, int64_t ld) {
  return ld > 0 && (rows + 1024) * ld * 2 < (int64_t(1) << 31);
}

// Number of 256 x 256 tiles from which the large-problem kernel is used: half the CUs, unless
// axonn_tuning(AXONN_TUNE_GEMM_BIG_MIN_TILES, n) says otherwise (the tests send small ragged problems through
// the large-problem kernels with it).
static int64_t big_tile_threshold() {
  const int64_t v = g_tune_big_min_tiles.load();
  return v >= 0 ? v : 128;
}

// Block width of the large-problem kernel for an M x N x (nk k-steps) problem: when other kernels share the chip
// (they fill the CUs a partly filled round leaves idle), the widest and most efficient one; when the launch has
// the chip to itself, the one with the lowest modelled time: a round (up to 256 tiles, one per CU) costs a fixed
// part (fill, epilogue) plus nk k-steps whose duration grows with the number of MFMAs (8 * TN per phase) on top of
// a part that does not (the A tile is fetched whatever the width).  Constants in microseconds, fitted to full
// rounds of the 12B-class shapes; on the forward and input-gradient shapes of the 24B and 100B stages the choice
// is the fastest of the three widths, or within 3 % of it, in all 16 cases (single launches, each width forced in
// turn with AXONN_TUNE_GEMM_TILE_N).
static int choose_tn(int64_t M, int64_t N, int64_t nk, bool concurrent) {
  const int64_t forced = g_tune_tile_n.load();
  if (forced == 160) return 5;
  if (forced == 192) return 6;
  if (forced == 256 || concurrent) return 8;
  const int cand[3] = {8, 6, 5};
  int best = 8;
  double best_cost = 0;
  for (int tn : cand) {
    const int64_t tiles = ((M + 255) / 256) * ((N + 32 * tn - 1) / (32 * tn));
    const int64_t rounds = (tiles + 255) / 256;
    const double cost = rounds * (20.0 + nk * (0.55 + 0.15 * tn));
    if (best_cost == 0 || cost < best_cost * 0.98) { best = tn; best_cost = cost; }
  }
  return best;
}

template <bool A_KC, bool B_KC>
static hipError_t launch_layout(int epi, const GemmArgs& g, hipStream_t s) {
  // Large tile when the problem fills the chip with it, smaller tile otherwise.
  const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big_tiles >= big_tile_threshold()) {
    if (fits_32bit_offsets(A_KC ? g.M : g.K, g.lda) && fits_32bit_offsets(B_KC ? g.N : g.K, g.ldb)) {
      const int64_t nk = (int64_t)((g.K + 63) / 64) * g.n_seg;
      switch (choose_tn(g.M, g.N, nk, g.concurrent != 0)) {
        case 5: return launch_big<A_KC, B_KC, 5>(epi, g, s);
        case 6: return launch_big<A_KC, B_KC, 6>(epi, g, s);
        default: return launch_big<A_KC, B_KC, 8>(epi, g, s);
      }
    }
    return launch_cfg<256, 256, 64, 2, 4, A_KC, B_KC>(epi, g, s);
  }
  return launch_cfg<128, 128, 64, 2, 2, A_KC, B_KC>(epi, g, s);
}

hipError_t launch_gemm(bool a_kc, bool b_kc, int epi, const GemmArgs& g, hipStream_t s) {
  if (a_kc && b_kc) return launch_layout<true, true>(epi, g, s);
  if (a_kc && !b_kc) return launch_layout<true, false>(epi, g, s);
  if (!a_kc && !b_kc) return launch_layout<false, false>(epi, g, s);
  return hipErrorInvalidValue;
}

}  // namespace axonn
