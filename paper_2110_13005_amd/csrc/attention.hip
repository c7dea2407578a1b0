// Fused causal self-attention for gfx950: forward (online softmax, never materialises the
// s x s matrix in HBM) and backward (probabilities recomputed from the stored log-sum-exp).
//
// All contractions run on v_mfma_f32_32x32x16_bf16.  The kernels are arranged so that the
// score tile comes out of the MFMA with the index that is contracted NEXT held in registers
// and the other index on lanes; the rounded tile is then fed straight back as an MFMA operand
// from registers (no LDS round trip):
//   forward, dQ kernel : S^T[key][query] -> lane = query, so max / sum / lse / delta are
//                        per-lane scalars; next contraction is over keys (P V, dS K).
//   dK/dV kernel       : S[query][key]   -> lane = key; next contraction is over queries
//                        (P^T dO, dS^T Q).
// Operands whose contracted index is not contiguous in the [row][d] tiles (V, and Q / dO / K
// in the backward kernels) are fetched with the transposing LDS read.
#include "common.h"

namespace axonn {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The kernels are compiled for head dimensions D = 64, 128 and 192.  EXACT: the head dimension is D.
// Otherwise the real head dimension d (a multiple of 4, d <= D) is a run-time argument and the columns
// d .. D-1 of every head read as zero and are never written: zero columns add nothing to q.k, and the
// padded columns of V give output columns nobody stores.  Heads then start at multiples of 8 bytes only, so
// the 8 elements at columns [col, col + 8) of a head row are fetched as two 8-byte halves.
template <bool EXACT>
__device__ __forceinline__ uint4 load_cols8(const elem_t* p, int col, int d) {
  if (EXACT) return *reinterpret_cast<const uint4*>(p);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (col + 4 <= d) {
    const uint2 lo = *reinterpret_cast<const uint2*>(p);
    v.x = lo.x; v.y = lo.y;
  }
  if (col + 8 <= d) {
    const uint2 hi = *reinterpret_cast<const uint2*>(p + 4);
    v.z = hi.x; v.w = hi.y;
  }
  return v;
}

// Cooperative copy of a ROWS x D bf16 tile (rows row0.., zero beyond n_rows) by 256 threads:
// global -> registers, then registers -> LDS with leading dimension LD.
template <int ROWS, int D>
struct TileRegs {
  static constexpr int NCH = ROWS * D / 8 / 256;
  uint4 r[NCH];
  template <bool EXACT>
  __device__ __forceinline__ void load(const elem_t* base, int64_t ld, int row0, int n_rows, int d, int tid) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c = tid + j * 256;
      const int row = c / (D / 8), ch = c % (D / 8);
      r[j] = (row0 + row < n_rows)
                 ? load_cols8<EXACT>(base + (int64_t)(row0 + row) * ld + ch * 8, ch * 8, d)
                 : make_uint4(0, 0, 0, 0);
    }
  }
  // The same tile of an exact-size head through buffer loads, with next to no address arithmetic per tile:
  // `off0` = byte offset, from the descriptor's base, of this thread's first chunk in the tile that starts at
  // row 0 (see offset0); the tile starts at row0; rows outside the descriptor's range read as zeros.
  static __device__ __forceinline__ uint32_t offset0(uint32_t row_bytes, int tid) {
    return (uint32_t)(tid / (D / 8)) * row_bytes + (uint32_t)(tid % (D / 8)) * 16u;
  }
  __device__ __forceinline__ void load_buffer(__amdgpu_buffer_rsrc_t rsrc, uint32_t off0, uint32_t row_bytes, int row0) {
    constexpr int RSTEP = 256 / (D / 8);        // rows between consecutive chunks of a thread
    const uint32_t base = off0 + (uint32_t)row0 * row_bytes;
#pragma unroll
    for (int j = 0; j < NCH; ++j)
      r[j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, base + (uint32_t)(j * RSTEP) * row_bytes, 0, 0));
  }
  template <int LD>
  __device__ __forceinline__ void store(elem_t* lds, int tid) const {
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c = tid + j * 256;
      *reinterpret_cast<uint4*>(lds + (c / (D / 8)) * LD + (c % (D / 8)) * 8) = r[j];
    }
  }
};

__device__ __forceinline__ elemx8 pack8(const floatx16& t, int first) {
  elemx8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (elem_t)t[first + e];
  return o;
}

// Row fragment straight from global memory: lane holds row (row0 + lane%32), elements
// [k0 + 8*(lane/32), +8) -- the MFMA operand layout.  Rows >= n_rows read as zero.
template <bool EXACT>
__device__ __forceinline__ elemx8 global_frag(const elem_t* base, int64_t ld, int row, int n_rows,
                                              int k0, int lane, int d) {
  uint4 v = make_uint4(0, 0, 0, 0);
  const int col = k0 + 8 * (lane >> 5);
  if (row < n_rows) v = load_cols8<EXACT>(base + (int64_t)row * ld + col, col, d);
  return __builtin_bit_cast(elemx8, v);
}

// Work assignment of the attention kernels: block id of a 1-D grid of n_tiles * n_bh blocks -> (rank of
// the tile, batch*head index).  Workgroups are dealt round-robin to the 8 XCDs, each with an L2 of its
// own, so XCD x gets ids x, x+8, ...: those are mapped to a contiguous range of (batch, head) pairs, so
// that the K/V (or Q/dO) rows of a head are fetched into one L2 instead of all eight; inside the range
// the tiles of rank 0 (the longest-running ones under causal masking) of every head come first.
__device__ __forceinline__ void attn_block(int n_bh, int& rank, int& bh) {
  const int id = blockIdx.x;
  if ((gridDim.x & 7) == 0 && (n_bh & 7) == 0) {
    const int per_xcd = n_bh >> 3, j = id >> 3;        // j-th block of XCD id % 8
    rank = j / per_xcd;
    bh = (id & 7) * per_xcd + j % per_xcd;
  } else {
    rank = id / n_bh;
    bh = id % n_bh;
  }
}

// Row stride (elements) of an LDS tile of D-element rows that is read both ways: with 128-bit reads of 16 rows
// at one column (conflict-free when the stride is an odd multiple of 4 words) and with the transposing 64-bit
// reads that take 32 bytes from each of 4 consecutive rows (conflict-free when 4 consecutive rows start at
// least 8 words apart modulo the 64 banks).  12 or 52 words modulo 64 satisfy both.
template <int D>
struct BothWaysStride {
  static constexpr int WORDS_MOD = (D / 2) % 64;
  static constexpr int PAD_WORDS = (12 - WORDS_MOD + 64) % 64 <= (52 - WORDS_MOD + 64) % 64 ? (12 - WORDS_MOD + 64) % 64
                                                                                            : (52 - WORDS_MOD + 64) % 64;
  static constexpr int LD = D + 2 * PAD_WORDS;
  static_assert((LD / 2) % 64 == 12 || (LD / 2) % 64 == 52, "stride class");
};

// =============================================================================== forward
// grid: (ceil(s/128), b*a); 4 waves; wave w owns queries q0 + 32w .. +31.
template <int D, bool EXACT>
__global__ __launch_bounds__(256, D > 128 ? 1 : 2) void attn_fwd_kernel(int s, int a, int n_bh, int d_arg,
                                                       const elem_t* __restrict__ qkv,
                                                       elem_t* __restrict__ o,
                                                       float* __restrict__ lse) {
  constexpr int BKV = 64, LDK = D + 8, LDV = D + 32, DT = D / 32, KK = D / 16;
  __shared__ __align__(16) elem_t sK[BKV * LDK];
  __shared__ __align__(16) elem_t sV[BKV * LDV];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int rank, bh;
  attn_block(n_bh, rank, bh);
  const int qt = (s + 127) / 128 - 1 - rank;  // longest rows first
  const int bi = bh / a, hd = bh % a;
  const int d = EXACT ? D : d_arg;
  const int h = a * d;
  const int64_t ld = 3 * (int64_t)h;
  const elem_t* qb = qkv + (int64_t)bi * s * ld + hd * d;
  const elem_t* kb = qb + h;
  const elem_t* vb = qb + 2 * h;
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, qi = qw0 + (lane & 31);
  const float scale_log2 = kLog2e * rsqrtf((float)d);

  elemx8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk] = global_frag<EXACT>(qb, ld, qi, s, kk * 16, lane, d);

  floatx16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int kv_end = min(s, q0 + 128);
  const int n_kt = (kv_end + BKV - 1) / BKV;
  TileRegs<BKV, D> rk, rv;
  // exact-size heads: tiles through buffer loads over the rows of this (batch, head)
  const uint32_t row_bytes = (uint32_t)ld * 2u, tile_bytes = EXACT ? (uint32_t)(((int64_t)(s - 1) * ld + D) * 2) : 0u;
  const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kb, tile_bytes), v_rsrc = make_rsrc(vb, tile_bytes);
  const uint32_t off0 = TileRegs<BKV, D>::offset0(row_bytes, tid);
  auto fetch = [&](int row0) {
    if (EXACT) {
      rk.load_buffer(k_rsrc, off0, row_bytes, row0);
      rv.load_buffer(v_rsrc, off0, row_bytes, row0);
    } else {
      rk.template load<EXACT>(kb, ld, row0, s, d, tid);
      rv.template load<EXACT>(vb, ld, row0, s, d, tid);
    }
  };
  fetch(0);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int k0 = kt * BKV;
    __syncthreads();
    rk.template store<LDK>(sK, tid);
    rv.template store<LDV>(sV, tid);
    __syncthreads();
    if (kt + 1 < n_kt) fetch(k0 + BKV);
    if (k0 > qw0 + 31) continue;  // every key of the tile is in this wave's future

    floatx16 sacc[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[ks][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        sacc[ks] = mfma32(frag_kcontig(sK + (32 * ks) * LDK + kk * 16, LDK, lane), qf[kk], sacc[ks]);
    }
    // Keys beyond the query are masked in the tiles that straddle the diagonal only: a real (wave-uniform)
    // branch, so that the other tiles do not pay for the comparisons.
    if (k0 + BKV - 1 > qw0) {
      asm volatile("" ::: "memory");            // keeps the compiler from turning the branch into selects
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * ks + 8 * (r >> 2) + 4 * g + (r & 3);
          if (key > qi) sacc[ks][r] = -INFINITY;
        }
    }
    // Row maximum of the raw scores; in units of the exponent (log2) it is mx * scale_log2 (the scale is positive).
    float mx = sacc[0][0];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[ks][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
    // m_run is the reference point of the exponentials, not necessarily the running maximum: it moves (and the
    // sums so far are rescaled) only when some row's maximum has grown by more than 2^8 since it was set, so
    // most tiles skip the rescaling; p stays <= 256 and the result is the same up to rounding.
    if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
    const float neg_m = -m_run;
    float psum = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(fmaf(sacc[ks][r], scale_log2, neg_m));
        sacc[ks][r] = p;
        psum += p;
      }
    l_run += psum;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const elemx8 pf = pack8(sacc[ks], 8 * c);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          oacc[dt] = mfma32(frag_kstrided<true>(sV + (32 * ks + 16 * c) * LDV + dt * 32, LDV, lane),
                            pf, oacc[dt]);
      }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < s) {
    const float inv = 1.f / l_tot;
    elem_t* orow = o + ((int64_t)bi * s + qi) * h + hd * d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        elemx4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (elem_t)(oacc[dt][4 * q + e] * inv);
        if (EXACT || dt * 32 + 8 * q + 4 * g < d) *reinterpret_cast<elemx4*>(orow + dt * 32 + 8 * q + 4 * g) = v;
      }
    if (g == 0) lse[((int64_t)bi * a + hd) * s + qi] = (m_run + __log2f(l_tot)) * kLn2;
  }
}

// ============================================================================ backward
// delta[b][a][i] = sum_d dO[i][d] * O[i][d]
template <int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(int64_t n_chunks, int s, int a,
                                                         const elem_t* __restrict__ o,
                                                         const elem_t* __restrict__ dout,
                                                         float* __restrict__ delta) {
  constexpr int LPR = D / 8;  // lanes per (row, head)
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  float p = 0.f;
  if (c < n_chunks) {
    const elemx8 ov = *reinterpret_cast<const elemx8*>(o + c * 8);
    const elemx8 dv = *reinterpret_cast<const elemx8*>(dout + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) p += (float)ov[e] * (float)dv[e];
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) p += __shfl_xor(p, off, 64);
  if (c < n_chunks && (c % LPR) == 0) {
    const int64_t hc = a * (int64_t)LPR;  // chunks per row
    const int64_t row = c / hc;
    const int hd = (int)((c % hc) / LPR);
    const int64_t bi = row / s, i = row % s;
    delta[(bi * a + hd) * s + i] = p;
  }
}

// The same for any head dimension d that is a multiple of 4: 16 lanes per (row, head), 4 elements per lane
// and step.
__global__ __launch_bounds__(256) void attn_delta_general_kernel(int64_t n_pairs, int s, int a, int d,
                                                                 const elem_t* __restrict__ o,
                                                                 const elem_t* __restrict__ dout,
                                                                 float* __restrict__ delta) {
  const int64_t pair = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);   // (row, head)
  const int j = threadIdx.x & 15;
  float p = 0.f;
  if (pair < n_pairs) {
    const elem_t* op = o + pair * d;          // rows are a * d long: pair * d = row * a * d + head * d
    const elem_t* dp = dout + pair * d;
    for (int c = 4 * j; c < d; c += 64) {
      const elemx4 ov = *reinterpret_cast<const elemx4*>(op + c);
      const elemx4 dv = *reinterpret_cast<const elemx4*>(dp + c);
#pragma unroll
      for (int e = 0; e < 4; ++e) p += (float)ov[e] * (float)dv[e];
    }
  }
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) p += __shfl_xor(p, off, 64);
  if (pair < n_pairs && j == 0) {
    const int64_t row = pair / a;
    const int hd = (int)(pair % a);
    const int64_t bi = row / s, i = row % s;
    delta[(bi * a + hd) * s + i] = p;
  }
}

// dK / dV: grid (ceil(s/128), b*a); wave w owns keys k0 + 32w .. +31 and walks the query tiles
// at or below the diagonal.
template <int D, bool EXACT>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_kernel(
    int s, int a, int n_bh, int d_arg, const elem_t* __restrict__ qkv, const elem_t* __restrict__ dout,
    const float* __restrict__ lse, const float* __restrict__ delta, elem_t* __restrict__ dqkv) {
  constexpr int BQ = 64, LDQ = BothWaysStride<D>::LD, DT = D / 32, KK = D / 16;
  __shared__ __align__(16) elem_t sQ[BQ * LDQ];
  __shared__ __align__(16) elem_t sdO[BQ * LDQ];
  __shared__ __align__(16) float s_lse[BQ];
  __shared__ __align__(16) float s_delta[BQ];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int rank, bh;
  attn_block(n_bh, rank, bh);                  // key tile `rank` walks n_tiles - rank query tiles: longest first
  const int bi = bh / a, hd = bh % a;
  const int d = EXACT ? D : d_arg;
  const int h = a * d;
  const int64_t ld = 3 * (int64_t)h;
  const elem_t* qb = qkv + (int64_t)bi * s * ld + hd * d;
  const elem_t* kb = qb + h;
  const elem_t* vb = qb + 2 * h;
  const elem_t* dob = dout + (int64_t)bi * s * h + hd * d;
  const float* lse_b = lse + ((int64_t)bi * a + hd) * s;
  const float* delta_b = delta + ((int64_t)bi * a + hd) * s;
  const int k0 = rank * 128, kw0 = k0 + 32 * wave, kj = kw0 + (lane & 31);
  const float scale = rsqrtf((float)d), scale_log2 = kLog2e * scale;

  elemx8 kf[KK], vf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    kf[kk] = global_frag<EXACT>(kb, ld, kj, s, kk * 16, lane, d);
    vf[kk] = global_frag<EXACT>(vb, ld, kj, s, kk * 16, lane, d);
  }
  floatx16 dvacc[DT], dkacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dvacc[dt][r] = dkacc[dt][r] = 0.f;

  const int qt_begin = k0 / BQ, n_qt = (s + BQ - 1) / BQ;
  TileRegs<BQ, D> rq, rdo;
  float r_lse = 0.f, r_delta = 0.f;
  const uint32_t q_row_bytes = (uint32_t)ld * 2u, do_row_bytes = (uint32_t)h * 2u;
  const __amdgpu_buffer_rsrc_t q_rsrc = make_rsrc(qb, EXACT ? (uint32_t)(((int64_t)(s - 1) * ld + D) * 2) : 0u);
  const __amdgpu_buffer_rsrc_t do_rsrc = make_rsrc(dob, EXACT ? (uint32_t)(((int64_t)(s - 1) * h + D) * 2) : 0u);
  const uint32_t q_off0 = TileRegs<BQ, D>::offset0(q_row_bytes, tid), do_off0 = TileRegs<BQ, D>::offset0(do_row_bytes, tid);
  auto prefetch = [&](int qt) {
    if (EXACT) {
      rq.load_buffer(q_rsrc, q_off0, q_row_bytes, qt * BQ);
      rdo.load_buffer(do_rsrc, do_off0, do_row_bytes, qt * BQ);
    } else {
      rq.template load<EXACT>(qb, ld, qt * BQ, s, d, tid);
      rdo.template load<EXACT>(dob, h, qt * BQ, s, d, tid);
    }
    if (tid < BQ) {
      const int qrow = qt * BQ + tid;
      r_lse = qrow < s ? lse_b[qrow] : 0.f;
      r_delta = qrow < s ? delta_b[qrow] : 0.f;
    }
  };
  prefetch(qt_begin);
  for (int qt = qt_begin; qt < n_qt; ++qt) {
    const int q0 = qt * BQ;
    __syncthreads();
    rq.template store<LDQ>(sQ, tid);
    rdo.template store<LDQ>(sdO, tid);
    if (tid < BQ) {
      s_lse[tid] = r_lse * kLog2e;
      s_delta[tid] = r_delta;
    }
    __syncthreads();
    if (qt + 1 < n_qt) prefetch(qt + 1);
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      const int qq0 = q0 + 32 * qs;
      if (qq0 + 31 < kw0) continue;  // all these queries precede every key of this wave
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = pacc[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        sacc = mfma32(frag_kcontig(sQ + (32 * qs) * LDQ + kk * 16, LDQ, lane), kf[kk], sacc);
        pacc = mfma32(frag_kcontig(sdO + (32 * qs) * LDQ + kk * 16, LDQ, lane), vf[kk], pacc);
      }
      // lane = key kj; register r = query qq0 + 8*(r/4) + 4g + r%4
      // masking in the blocks that straddle the diagonal only (a wave-uniform branch, kept as one)
      if (kw0 + 31 > qq0) {
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qrow = qq0 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kj > qrow) sacc[r] = -INFINITY;
        }
      }
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const floatx4 l4 = *reinterpret_cast<const floatx4*>(&s_lse[32 * qs + 8 * q4 + 4 * g]);
        const floatx4 d4 = *reinterpret_cast<const floatx4*>(&s_delta[32 * qs + 8 * q4 + 4 * g]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * q4 + e;
          const float p = fast_exp2(fmaf(sacc[r], scale_log2, -l4[e]));
          sacc[r] = p;
          pacc[r] = p * (pacc[r] - d4[e]);
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const elemx8 pf = pack8(sacc, 8 * c);
        const elemx8 dsf = pack8(pacc, 8 * c);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dvacc[dt] = mfma32(frag_kstrided<true>(sdO + (32 * qs + 16 * c) * LDQ + dt * 32, LDQ, lane),
                             pf, dvacc[dt]);
          dkacc[dt] = mfma32(frag_kstrided<true>(sQ + (32 * qs + 16 * c) * LDQ + dt * 32, LDQ, lane),
                             dsf, dkacc[dt]);
        }
      }
    }
  }
  if (kj < s) {
    elem_t* dk_row = dqkv + ((int64_t)bi * s + kj) * ld + h + hd * d;
    elem_t* dv_row = dk_row + h;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        elemx4 kv4, vv4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kv4[e] = (elem_t)(dkacc[dt][4 * q + e] * scale);
          vv4[e] = (elem_t)dvacc[dt][4 * q + e];
        }
        if (EXACT || dt * 32 + 8 * q + 4 * g < d) {
          *reinterpret_cast<elemx4*>(dk_row + dt * 32 + 8 * q + 4 * g) = kv4;
          *reinterpret_cast<elemx4*>(dv_row + dt * 32 + 8 * q + 4 * g) = vv4;
        }
      }
  }
}

// dQ: grid (ceil(s/128), b*a); wave w owns queries q0 + 32w .. +31 and walks the key tiles up
// to the diagonal (same traversal as the forward kernel).
template <int D, bool EXACT>
__global__ __launch_bounds__(256, D > 128 ? 1 : 2) void attn_bwd_dq_kernel(
    int s, int a, int n_bh, int d_arg, const elem_t* __restrict__ qkv, const elem_t* __restrict__ dout,
    const float* __restrict__ lse, const float* __restrict__ delta, elem_t* __restrict__ dqkv) {
  constexpr int BKV = 64, LDK = BothWaysStride<D>::LD, DT = D / 32, KK = D / 16;
  __shared__ __align__(16) elem_t sK[BKV * LDK];
  __shared__ __align__(16) elem_t sV[BKV * LDK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
  int rank, bh;
  attn_block(n_bh, rank, bh);
  const int qt = (s + 127) / 128 - 1 - rank;
  const int bi = bh / a, hd = bh % a;
  const int d = EXACT ? D : d_arg;
  const int h = a * d;
  const int64_t ld = 3 * (int64_t)h;
  const elem_t* qb = qkv + (int64_t)bi * s * ld + hd * d;
  const elem_t* kb = qb + h;
  const elem_t* vb = qb + 2 * h;
  const elem_t* dob = dout + (int64_t)bi * s * h + hd * d;
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, qi = qw0 + (lane & 31);
  const float scale = rsqrtf((float)d), scale_log2 = kLog2e * scale;
  const float lse_q = (qi < s) ? lse[((int64_t)bi * a + hd) * s + qi] * kLog2e : 0.f;
  const float delta_q = (qi < s) ? delta[((int64_t)bi * a + hd) * s + qi] : 0.f;

  elemx8 qf[KK], dof[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    qf[kk] = global_frag<EXACT>(qb, ld, qi, s, kk * 16, lane, d);
    dof[kk] = global_frag<EXACT>(dob, h, qi, s, kk * 16, lane, d);
  }
  floatx16 dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[dt][r] = 0.f;

  const int kv_end = min(s, q0 + 128);
  const int n_kt = (kv_end + BKV - 1) / BKV;
  TileRegs<BKV, D> rk, rv;
  const uint32_t row_bytes = (uint32_t)ld * 2u, tile_bytes = EXACT ? (uint32_t)(((int64_t)(s - 1) * ld + D) * 2) : 0u;
  const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kb, tile_bytes), v_rsrc = make_rsrc(vb, tile_bytes);
  const uint32_t off0 = TileRegs<BKV, D>::offset0(row_bytes, tid);
  auto fetch = [&](int row0) {
    if (EXACT) {
      rk.load_buffer(k_rsrc, off0, row_bytes, row0);
      rv.load_buffer(v_rsrc, off0, row_bytes, row0);
    } else {
      rk.template load<EXACT>(kb, ld, row0, s, d, tid);
      rv.template load<EXACT>(vb, ld, row0, s, d, tid);
    }
  };
  fetch(0);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int k0 = kt * BKV;
    __syncthreads();
    rk.template store<LDK>(sK, tid);
    rv.template store<LDK>(sV, tid);
    __syncthreads();
    if (kt + 1 < n_kt) fetch(k0 + BKV);
    if (k0 > qw0 + 31) continue;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = pacc[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        sacc = mfma32(frag_kcontig(sK + (32 * ks) * LDK + kk * 16, LDK, lane), qf[kk], sacc);
        pacc = mfma32(frag_kcontig(sV + (32 * ks) * LDK + kk * 16, LDK, lane), dof[kk], pacc);
      }
      // lane = query qi; register r = key k0 + 32ks + 8*(r/4) + 4g + r%4
      // masking in the blocks that straddle the diagonal only (a wave-uniform branch, kept as one)
      if (k0 + 32 * ks + 31 > qw0) {
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * ks + 8 * (r >> 2) + 4 * g + (r & 3);
          if (key > qi) sacc[r] = -INFINITY;
        }
      }
      const float neg_lse = -lse_q;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(fmaf(sacc[r], scale_log2, neg_lse));
        pacc[r] = p * (pacc[r] - delta_q);
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const elemx8 dsf = pack8(pacc, 8 * c);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          dqacc[dt] = mfma32(frag_kstrided<true>(sK + (32 * ks + 16 * c) * LDK + dt * 32, LDK, lane),
                             dsf, dqacc[dt]);
      }
    }
  }
  if (qi < s) {
    elem_t* dq_row = dqkv + ((int64_t)bi * s + qi) * ld + hd * d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        elemx4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (elem_t)(dqacc[dt][4 * q + e] * scale);
        if (EXACT || dt * 32 + 8 * q + 4 * g < d) *reinterpret_cast<elemx4*>(dq_row + dt * 32 + 8 * q + 4 * g) = v;
      }
  }
}

// ------------------------------------------------------------------------- launchers
// d = 64 or 128: the kernels compiled for exactly that head dimension.  Any other multiple of 4 up to 192:
// the next compiled size with the columns beyond d masked.
// The exact-size kernels address the rows of a (batch, head) with 32-bit byte offsets (buffer loads): for sequences
// too long for that (s * 3 * a * d * 2 bytes beyond 2^31) the general kernels take over.
#define AXONN_ATTN_DISPATCH(KERNEL, ...)                                                              \
  do {                                                                                                \
    const bool off32 = ((int64_t)s + 256) * 3 * a * d * 2 < (int64_t(1) << 31);                       \
    if (d == 64 && off32) hipLaunchKernelGGL((KERNEL<64, true>), grid, dim3(256), 0, st, __VA_ARGS__);         \
    else if (d == 128 && off32) hipLaunchKernelGGL((KERNEL<128, true>), grid, dim3(256), 0, st, __VA_ARGS__);  \
    else if (d <= 64) hipLaunchKernelGGL((KERNEL<64, false>), grid, dim3(256), 0, st, __VA_ARGS__);    \
    else if (d <= 128) hipLaunchKernelGGL((KERNEL<128, false>), grid, dim3(256), 0, st, __VA_ARGS__); \
    else hipLaunchKernelGGL((KERNEL<192, false>), grid, dim3(256), 0, st, __VA_ARGS__);               \
  } while (0)

static bool head_dim_supported(int d) { return d >= 4 && d <= 192 && d % 4 == 0; }

hipError_t launch_attention_fwd(int b, int s, int a, int d, const void* qkv, void* o, float* lse,
                                hipStream_t st) {
  if (!head_dim_supported(d)) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(((s + 127) / 128) * b * a));
  AXONN_ATTN_DISPATCH(attn_fwd_kernel, s, a, b * a, d, (const elem_t*)qkv, (elem_t*)o, lse);
  return hipGetLastError();
}

hipError_t launch_attention_bwd(int b, int s, int a, int d, const void* qkv, const void* o,
                                const float* lse, const void* dout, void* dqkv, float* delta,
                                hipStream_t st) {
  if (!head_dim_supported(d)) return hipErrorInvalidValue;
  if (d == 64 || d == 128) {
    const int64_t n_chunks = (int64_t)b * s * a * d / 8;
    const dim3 gd((unsigned)((n_chunks + 255) / 256));
    if (d == 128)
      hipLaunchKernelGGL(attn_delta_kernel<128>, gd, dim3(256), 0, st, n_chunks, s, a, (const elem_t*)o, (const elem_t*)dout, delta);
    else
      hipLaunchKernelGGL(attn_delta_kernel<64>, gd, dim3(256), 0, st, n_chunks, s, a, (const elem_t*)o, (const elem_t*)dout, delta);
  } else {
    const int64_t n_pairs = (int64_t)b * s * a;
    hipLaunchKernelGGL(attn_delta_general_kernel, dim3((unsigned)((n_pairs + 15) / 16)), dim3(256), 0, st, n_pairs, s, a, d,
                       (const elem_t*)o, (const elem_t*)dout, delta);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)(((s + 127) / 128) * b * a));
  AXONN_ATTN_DISPATCH(attn_bwd_dkdv_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)dout, lse, (const float*)delta, (elem_t*)dqkv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  AXONN_ATTN_DISPATCH(attn_bwd_dq_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)dout, lse, (const float*)delta, (elem_t*)dqkv);
  return hipGetLastError();
}
#undef AXONN_ATTN_DISPATCH

}  // namespace axonn
