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

#include <type_traits>

namespace axonn {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max(v of this lane, v of lane ^ 32) with v_permlane32_swap: given the same register twice it leaves the lower half-wave's
// values in both halves of one result and the upper half-wave's in both halves of the other.  Unlike a shuffle it does
// not go through the LDS queue, whose results return in order: a shuffle behind a batch of fragment reads waits for all
// of them.
__device__ __forceinline__ float max_with_other_half(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

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
  // chunk j alone: for kernels that spread a tile's loads and stores over their instruction stream
  __device__ __forceinline__ void load_buffer_one(int j, __amdgpu_buffer_rsrc_t rsrc, uint32_t off0, uint32_t row_bytes, int row0) {
    constexpr int RSTEP = 256 / (D / 8);
    r[j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off0 + (uint32_t)(row0 + j * RSTEP) * row_bytes, 0, 0));
  }
  template <int LD>
  __device__ __forceinline__ void store_one(int j, elem_t* lds, int tid) const {
    const int c = tid + j * 256;
    *reinterpret_cast<uint4*>(lds + (c / (D / 8)) * LD + (c % (D / 8)) * 8) = r[j];
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

// The rows a wave owns (32 of the workgroup's 128) enter and leave the kernels of the exact head dimensions through
// LDS.  Fetched or stored straight from the MFMA layout, every lane touches a row of its own, 16 or 8 bytes at a time:
// a memory instruction then covers 32 different lines, and the workgroups' first loads and last stores alone took a
// fifth of the dK / dV kernel's time.  Staged, a load or store instruction covers whole rows (16 bytes per lane).
//
// stage_rows_in: the 128 x D tile at rows row0.. of a descriptor into LDS with row stride LD (all 256 threads; rows
// beyond the descriptor's range read as zeros); the caller puts barriers around its use.
template <int D, int LD>
__device__ __forceinline__ void stage_rows_in(elem_t* lds, __amdgpu_buffer_rsrc_t rsrc, uint32_t row_bytes, int row0, int tid) {
  TileRegs<128, D> t;
  t.load_buffer(rsrc, TileRegs<128, D>::offset0(row_bytes, tid), row_bytes, row0);
  t.template store<LD>(lds, tid);
}
// store_rows_out: one wave's 32 x D result (the MFMA result layout: lane = row lane % 32, registers 4q .. 4q+3 of
// tile dt = columns 32 dt + 8 q + 4 (lane / 32) ..) times `mul`, rounded, to rows of `ld` elements at `dst`; `stage`
// is 32 x (D + 8) elements of LDS that only this wave touches (no barrier: a wave's LDS operations keep their order).
template <int D>
__device__ __forceinline__ void store_rows_out(elem_t* stage, const floatx16* acc, float mul, elem_t* dst, int64_t ld,
                                               int n_rows, int lane) {
  constexpr int LDO = D + 8, DT = D / 32, CPR = D / 8;      // 16-byte chunks per row
  const int g = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      elemx4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (elem_t)(acc[dt][4 * q + e] * mul);
      *reinterpret_cast<elemx4*>(stage + (lane & 31) * LDO + dt * 32 + 8 * q + 4 * g) = v;
    }
#pragma unroll
  for (int j = 0; j < 32 * CPR / 64; ++j) {
    const int idx = lane + 64 * j, row = idx / CPR, ch = idx % CPR;
    const uint4 v = *reinterpret_cast<const uint4*>(stage + row * LDO + ch * 8);
    if (row < n_rows) *reinterpret_cast<uint4*>(dst + (int64_t)row * ld + ch * 8) = v;
  }
}

// =============================================================================== forward
// grid: (ceil(s/128), b*a); 4 waves; wave w owns queries q0 + 32w .. +31.
template <int D, bool EXACT>
__global__ __launch_bounds__(256, D > 128 ? 1 : 2) void attn_fwd_kernel(int s, int a, int n_bh, int d_arg,
                                                       const elem_t* __restrict__ qkv,
                                                       elem_t* __restrict__ o,
                                                       float* __restrict__ lse) {
  constexpr int BKV = 64, LDK = D + 8, LDV = D + 32, DT = D / 32, KK = D / 16;
  __shared__ __align__(16) elem_t smem[BKV * (LDK + LDV)];      // K and V tile; at the ends the staged Q and O rows
  static_assert(BKV * (LDK + LDV) >= 128 * (D + 8), "the workgroup's 128 rows fit the tile buffers");
  elem_t* sK = smem;
  elem_t* sV = smem + BKV * LDK;
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
  if (EXACT) {
    stage_rows_in<D, D + 8>(smem, make_rsrc(qb, (uint32_t)(((int64_t)(s - 1) * ld + D) * 2)), (uint32_t)ld * 2u, q0, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = frag_kcontig(smem + (32 * wave) * (D + 8) + kk * 16, D + 8, lane);
  } else {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = global_frag<EXACT>(qb, ld, qi, s, kk * 16, lane, d);
  }

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

    // All the K fragments of the tile are requested before the first MFMA, and the V fragments behind the last one,
    // ahead of the exponentials: left to the compiler, every MFMA follows the LDS round trip of a read of its own.
    // (Not where the fragments of a whole tile do not fit the registers: D = 192, and D = 128 with masked columns.)
    constexpr bool BATCH = D <= 64 || (D <= 128 && EXACT);
    elemx8 kfr[2][KK];
    if (BATCH) {
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) kfr[ks][kk] = frag_kcontig(sK + (32 * ks) * LDK + kk * 16, LDK, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    floatx16 sacc[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[ks][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        sacc[ks] = mfma32(BATCH ? kfr[ks][kk] : frag_kcontig(sK + (32 * ks) * LDK + kk * 16, LDK, lane), qf[kk], sacc[ks]);
    elemx8 vfr[4][DT];
    if (BATCH) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vfr[kc][dt] = frag_kstrided<true>(sV + (16 * kc) * LDV + dt * 32, LDV, lane);
      __builtin_amdgcn_sched_barrier(0);
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
    mx = max_with_other_half(mx) * scale_log2;
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
          oacc[dt] = mfma32(BATCH ? vfr[2 * ks + c][dt] : frag_kstrided<true>(sV + (32 * ks + 16 * c) * LDV + dt * 32, LDV, lane),
                            pf, oacc[dt]);
      }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (EXACT) {
    __syncthreads();              // the tiles in LDS are done with
    store_rows_out<D>(smem + wave * (32 * (D + 8)), oacc, 1.f / l_tot, o + ((int64_t)bi * s + qw0) * h + hd * d, h, s - qw0, lane);
    if (g == 0 && qi < s) lse[((int64_t)bi * a + hd) * s + qi] = (m_run + __log2f(l_tot)) * kLn2;
    return;
  }
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
        if (dt * 32 + 8 * q + 4 * g < d) *reinterpret_cast<elemx4*>(orow + dt * 32 + 8 * q + 4 * g) = v;
      }
    if (g == 0) lse[((int64_t)bi * a + hd) * s + qi] = (m_run + __log2f(l_tot)) * kLn2;
  }
}

// ============================================================================ backward
// delta[b][a][i] = sum_d dO[i][d] * O[i][d]
// For any head dimension d that is a multiple of 4: 16 lanes per (row, head), 4 elements per lane and step.
// (Launched in front of the general kernels only: the exact-size dQ kernel forms delta itself.)
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

// dK / dV: grid (ceil(s/128), b*a); wave w owns keys k0 + 32w .. +31 and walks the query tiles at or below the
// diagonal.  The Q / dO tiles alternate between two LDS buffers: the next tile is fetched into registers at the top
// of a step and stored to the other buffer at the end, so one barrier per tile is enough.
//
// A wave is alone on its SIMD (accumulators and K / V fragments take most of the register file), so nothing hides the
// MFMA phases of a 32-query block behind its exponentials, or an LDS round trip behind an MFMA, unless the instruction
// stream does.  Up to D = 128 a tile has 128 queries, four blocks, processed as two pairs in four phases each: S and
// dP of the first block; S and dP of the second next to the exponentials of the first; the dV / dK MFMAs of the first
// next to the exponentials of the second; the dV / dK MFMAs of the second.  A phase is a run of slots: one MFMA, the
// LDS read of the fragment that the MFMA W - 1 slots later needs (a ring of W fragments, so the reads run ahead
// across the phase boundaries and only the first few of a tile are waited for), and a share of the other block's
// exponentials.  The MFMAs are volatile assembly: they keep this order, and the reads stay between them where they
// are written.  The tile on the diagonal takes the same path with the mask applied to every element (a block above
// the diagonal comes out as zeros; the wave with the lowest keys needs all four blocks anyway).
// At D = 192 the registers do not hold two blocks: tiles of 64 queries, block by block.
template <int D, bool EXACT>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_kernel(
    int s, int a, int n_bh, int d_arg, const elem_t* __restrict__ qkv, const elem_t* __restrict__ dout,
    const float* __restrict__ lse, const float* __restrict__ delta, elem_t* __restrict__ dqkv) {
  constexpr bool PAIR = D <= 128;
  constexpr int BQ = PAIR ? 128 : 64, LDQ = BothWaysStride<D>::LD, DT = D / 32, KK = D / 16;
  constexpr int NBUF = 2;
  __shared__ __align__(16) elem_t sQ_[NBUF][BQ * LDQ];
  __shared__ __align__(16) elem_t sdO_[NBUF][BQ * LDQ];
  __shared__ __align__(16) float s_lse_[NBUF][BQ];
  __shared__ __align__(16) float s_delta_[NBUF][BQ];
  static_assert(NBUF * BQ * LDQ >= 128 * LDQ, "the workgroup's 128 keys fit the tile buffers");
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
  if (EXACT) {
    const uint32_t kv_bytes = (uint32_t)(((int64_t)(s - 1) * ld + D) * 2);
    stage_rows_in<D, LDQ>(&sQ_[0][0], make_rsrc(kb, kv_bytes), (uint32_t)ld * 2u, k0, tid);
    stage_rows_in<D, LDQ>(&sdO_[0][0], make_rsrc(vb, kv_bytes), (uint32_t)ld * 2u, k0, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf[kk] = frag_kcontig(&sQ_[0][0] + (32 * wave) * LDQ + kk * 16, LDQ, lane);
      vf[kk] = frag_kcontig(&sdO_[0][0] + (32 * wave) * LDQ + kk * 16, LDQ, lane);
    }
    __syncthreads();
  } else {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf[kk] = global_frag<EXACT>(kb, ld, kj, s, kk * 16, lane, d);
      vf[kk] = global_frag<EXACT>(vb, ld, kj, s, kk * 16, lane, d);
    }
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
  auto prefetch_stats = [&](int qt) {
    if (tid < BQ) {
      const int qrow = qt * BQ + tid;
      r_lse = qrow < s ? lse_b[qrow] : 0.f;
      r_delta = qrow < s ? delta_b[qrow] : 0.f;
    }
  };
  auto store_stats = [&](int buf) {
    if (tid < BQ) {
      s_lse_[buf][tid] = r_lse * kLog2e;
      s_delta_[buf][tid] = r_delta;
    }
  };
  auto prefetch = [&](int qt) {
    if (EXACT) {
      rq.load_buffer(q_rsrc, q_off0, q_row_bytes, qt * BQ);
      rdo.load_buffer(do_rsrc, do_off0, do_row_bytes, qt * BQ);
    } else {
      rq.template load<EXACT>(qb, ld, qt * BQ, s, d, tid);
      rdo.template load<EXACT>(dob, h, qt * BQ, s, d, tid);
    }
    prefetch_stats(qt);
  };
  auto store_tile = [&](int buf) {
    rq.template store<LDQ>(sQ_[buf], tid);
    rdo.template store<LDQ>(sdO_[buf], tid);
    store_stats(buf);
  };
  // P and dS of one 32-query block from its scores and dP, in place, then rounded into MFMA operands:
  // lane = key kj; register r = query 8*(r/4) + 4g + r%4 of the block
  auto softmax_block = [&](const float* lse32, const float* delta32, floatx16& sacc, floatx16& pacc, elemx8* pf, elemx8* dsf) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const floatx4 l4 = *reinterpret_cast<const floatx4*>(&lse32[8 * q4 + 4 * g]);
      const floatx4 d4 = *reinterpret_cast<const floatx4*>(&delta32[8 * q4 + 4 * g]);
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
      pf[c] = pack8(sacc, 8 * c);
      dsf[c] = pack8(pacc, 8 * c);
    }
  };

  prefetch(qt_begin);
  store_tile(0);
  if constexpr (!PAIR) {
    for (int qt = qt_begin; qt < n_qt; ++qt) {
      const int q0 = qt * BQ, buf = (qt - qt_begin) & 1;
      const elem_t* sQ = sQ_[buf];
      const elem_t* sdO = sdO_[buf];
      const float* s_lse = s_lse_[buf];
      const float* s_delta = s_delta_[buf];
      const bool more = qt + 1 < n_qt;
      __syncthreads();            // tile qt is in LDS; every wave has left tile qt - 1, whose buffer the next store takes
      if (more) prefetch(qt + 1);
#pragma unroll
      for (int qs = 0; qs < BQ / 32; ++qs) {
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
        // masking in the blocks that straddle the diagonal only (a wave-uniform branch, kept as one)
        if (kw0 + 31 > qq0) {
          asm volatile("" ::: "memory");
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qrow = qq0 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (kj > qrow) sacc[r] = -INFINITY;
          }
        }
        elemx8 pf[2], dsf[2];
        softmax_block(s_lse + 32 * qs, s_delta + 32 * qs, sacc, pacc, pf, dsf);
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            dvacc[dt] = mfma32(frag_kstrided<true>(sdO + (32 * qs + 16 * c) * LDQ + dt * 32, LDQ, lane),
                               pf[c], dvacc[dt]);
            dkacc[dt] = mfma32(frag_kstrided<true>(sQ + (32 * qs + 16 * c) * LDQ + dt * 32, LDQ, lane),
                               dsf[c], dkacc[dt]);
          }
      }
    if (more) store_tile(buf ^ 1);
    }
  } else {
    // K and V fragments move to the accumulation registers, which the MFMAs below read them from
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" : "+a"(kf[kk]), "+a"(vf[kk]));
    constexpr int NS = 2 * KK, NG = 4 * DT, PS = 2 * NS + 2 * NG, NSLOT = 2 * PS, W = 8;
    constexpr int EPS = 16 / NS, EPG = 16 / NG;      // elements of a block per slot of the phase beside it
    static_assert(16 % NS == 0 && 16 % NG == 0, "whole elements per slot");
    // One tile: `masked` is a std::integral_constant (the tile on the diagonal: keys beyond the query get no weight)
    // `fetch_row0` >= 0: the tile at that row is fetched on the way and stored to the other buffer (exact head
    // dimensions): one 16-byte piece per thread and slot, the loads in the first score phase and the stores in the
    // last gradient phase, whose slots have no exponentials beside their MFMAs.  Issued in one go, the loads of the
    // four waves wait for the memory pipeline, and the stores for the LDS, with nothing to do meanwhile.
    constexpr int NCH = TileRegs<BQ, D>::NCH, STORE_SLOT0 = NSLOT - 2 * NCH;
    static_assert(2 * NCH <= NS && 2 * NCH <= NG, "a piece per slot of one phase");
    auto tile_stream = [&](int q0, int buf, int fetch_row0, auto masked) {
      constexpr bool MASKED = decltype(masked)::value;
      const elem_t* sQ = sQ_[buf];
      const elem_t* sdO = sdO_[buf];
      const float* s_lse = s_lse_[buf];
      const float* s_delta = s_delta_[buf];
      floatx16 sacc[2], pacc[2];          // of the pair in flight
      uint32_t pfw[2][8], dsw[2][8];      // P and dS of a block rounded to 16 bits, two per word: MFMA operands
      floatx4 l4[2], d4[2];               // log-sum-exp and delta of the four queries of a group; two groups in flight
      elemx8 ring[W];
      auto load_stats = [&](int blk, int q4) {
        l4[q4 & 1] = *reinterpret_cast<const floatx4*>(&s_lse[32 * blk + 8 * q4 + 4 * g]);
        d4[q4 & 1] = *reinterpret_cast<const floatx4*>(&s_delta[32 * blk + 8 * q4 + 4 * g]);
      };
      // element r of block blk (half hf of its pair): P = exp(S - lse), dS = P (dP - delta), rounded once a pair of
      // elements is complete
      auto softmax_elem = [&](int blk, int r) {
        const int hf = blk & 1, q4 = r >> 2;
        float x = fmaf(sacc[hf][r], scale_log2, -l4[q4 & 1][r & 3]);
        if (MASKED && kj > q0 + 32 * blk + 8 * q4 + 4 * g + (r & 3)) x = -INFINITY;
        const float p = fast_exp2(x);
        sacc[hf][r] = p;
        pacc[hf][r] = p * (pacc[hf][r] - d4[q4 & 1][r & 3]);
        if (r & 1) {
          elemx2 pp, dd;
          pp[0] = (elem_t)sacc[hf][r - 1]; pp[1] = (elem_t)sacc[hf][r];
          dd[0] = (elem_t)pacc[hf][r - 1]; dd[1] = (elem_t)pacc[hf][r];
          pfw[hf][r >> 1] = __builtin_bit_cast(uint32_t, pp);
          dsw[hf][r >> 1] = __builtin_bit_cast(uint32_t, dd);
        }
        if ((r & 3) == 3 && q4 + 2 < 4) load_stats(blk, q4 + 2);     // the group after next, into the pair just used up
      };
      auto operand = [&](const uint32_t* w, int c) {
        return __builtin_bit_cast(elemx8, make_uint4(w[4 * c], w[4 * c + 1], w[4 * c + 2], w[4 * c + 3]));
      };
      // slot j: pair j / PS; within the pair, score slots of its two blocks, then gradient slots of its two blocks
      auto load_frag = [&](int j) -> elemx8 {
        const int pair = j / PS, jj = j % PS;
        if (jj < 2 * NS) {
          const int blk = 2 * pair + jj / NS, i = jj % NS, kk = i >> 1;
          return frag_kcontig(((i & 1) ? sdO : sQ) + (32 * blk) * LDQ + kk * 16, LDQ, lane);
        }
        const int blk = 2 * pair + (jj - 2 * NS) / NG, i = (jj - 2 * NS) % NG, c = i / (2 * DT), dt = (i % (2 * DT)) >> 1;
        return frag_kstrided<true>(((i & 1) ? sQ : sdO) + (32 * blk + 16 * c) * LDQ + dt * 32, LDQ, lane);
      };
      auto slot_mfma = [&](int j, elemx8 f) {
        const int jj = j % PS;
        if (jj < 2 * NS) {
          const int hf = jj / NS, i = jj % NS, kk = i >> 1;
          if (i & 1) {
            if (kk == 0) mfma32_vgpr_zero_ba(pacc[hf], f, vf[kk]);
            else if (kk == KK - 1) mfma32_vgpr_settled_ba(pacc[hf], f, vf[kk]);     // the phase's last: its block's scores settle
            else mfma32_vgpr_ba(pacc[hf], f, vf[kk]);
          } else {
            if (kk == 0) mfma32_vgpr_zero_ba(sacc[hf], f, kf[kk]); else mfma32_vgpr_ba(sacc[hf], f, kf[kk]);
          }
        } else {
          const int hf = (jj - 2 * NS) / NG, i = (jj - 2 * NS) % NG, c = i / (2 * DT), dt = (i % (2 * DT)) >> 1;
          if (i & 1) mfma32_agpr(dkacc[dt], f, operand(dsw[hf], c));
          else mfma32_agpr(dvacc[dt], f, operand(pfw[hf], c));
        }
      };
#pragma unroll
      for (int j = 0; j < W - 1; ++j) ring[j] = load_frag(j);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NSLOT; ++j) {
        const int pair = j / PS, jj = j % PS;
        slot_mfma(j, ring[j % W]);
        if (j + W - 1 < NSLOT) ring[(j + W - 1) % W] = load_frag(j + W - 1);   // into the fragment of the slot before
        if (jj == NS - 1) { load_stats(2 * pair, 0); load_stats(2 * pair, 1); }
        if (EXACT && fetch_row0 >= 0) {
          if (j < 2 * NCH) {
            const int k = j;
            if (k < NCH) rq.load_buffer_one(k, q_rsrc, q_off0, q_row_bytes, fetch_row0);
            else rdo.load_buffer_one(k - NCH, do_rsrc, do_off0, do_row_bytes, fetch_row0);
          }
          if (j >= STORE_SLOT0) {
            const int k = j - STORE_SLOT0;
            if (k < NCH) rq.template store_one<LDQ>(k, sQ_[buf ^ 1], tid);
            else rdo.template store_one<LDQ>(k - NCH, sdO_[buf ^ 1], tid);
          }
        }
        if (jj >= NS && jj < 2 * NS) {
#pragma unroll
          for (int e = 0; e < EPS; ++e) softmax_elem(2 * pair, (jj - NS) * EPS + e);
          if (jj == 2 * NS - 1) { load_stats(2 * pair + 1, 0); load_stats(2 * pair + 1, 1); }
        } else if (jj >= 2 * NS && jj < 2 * NS + NG) {
#pragma unroll
          for (int e = 0; e < EPG; ++e) softmax_elem(2 * pair + 1, (jj - 2 * NS) * EPG + e);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // the tile on the diagonal, then the others in a loop of their own (so that the accumulators keep one place in
    // the register files throughout it)
    {
      const bool more = qt_begin + 1 < n_qt;
      __syncthreads();
      if (more) { if (EXACT) prefetch_stats(qt_begin + 1); else prefetch(qt_begin + 1); }
      tile_stream(qt_begin * BQ, 0, more ? (qt_begin + 1) * BQ : -1, std::true_type{});
      if (more) { if (EXACT) store_stats(1); else store_tile(1); }
    }
    for (int qt = qt_begin + 1; qt < n_qt; ++qt) {
      const int buf = (qt - qt_begin) & 1;
      const bool more = qt + 1 < n_qt;
      __syncthreads();            // tile qt is in LDS; every wave has left tile qt - 1, whose buffer the next store takes
      if (more) { if (EXACT) prefetch_stats(qt + 1); else prefetch(qt + 1); }
      tile_stream(qt * BQ, buf, more ? (qt + 1) * BQ : -1, std::false_type{});
      if (more) { if (EXACT) store_stats(buf ^ 1); else store_tile(buf ^ 1); }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) mfma32_settle_agpr(dvacc[dt], dkacc[dt]);
  }
  if (EXACT) {
    __syncthreads();              // the tiles in LDS are done with
    elem_t* dk_rows = dqkv + ((int64_t)bi * s + kw0) * ld + h + hd * d;
    store_rows_out<D>(&sQ_[0][0] + wave * (32 * (D + 8)), dkacc, scale, dk_rows, ld, s - kw0, lane);
    store_rows_out<D>(&sdO_[0][0] + wave * (32 * (D + 8)), dvacc, 1.f, dk_rows + h, ld, s - kw0, lane);
    return;
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
        if (dt * 32 + 8 * q + 4 * g < d) {
          *reinterpret_cast<elemx4*>(dk_row + dt * 32 + 8 * q + 4 * g) = kv4;
          *reinterpret_cast<elemx4*>(dv_row + dt * 32 + 8 * q + 4 * g) = vv4;
        }
      }
  }
}

// dQ: grid (ceil(s/128), b*a); wave w owns queries q0 + 32w .. +31 and walks the key tiles up
// to the diagonal (same traversal as the forward kernel).
// The exact-size kernels also form delta (above) for their 128 queries, from the rows of dO they stage anyway and
// the same rows of O, and leave it in `delta` for the dK / dV kernel, which then has to run behind this one: no
// launch of its own for it, and dO is read once less.  The general kernels read `delta` and ignore `o`.
template <int D, bool EXACT>
__global__ __launch_bounds__(256, D > 128 ? 1 : 2) void attn_bwd_dq_kernel(
    int s, int a, int n_bh, int d_arg, const elem_t* __restrict__ qkv, const elem_t* __restrict__ o,
    const elem_t* __restrict__ dout, const float* __restrict__ lse, float* __restrict__ delta,
    elem_t* __restrict__ dqkv) {
  constexpr int BKV = 64, LDK = BothWaysStride<D>::LD, DT = D / 32, KK = D / 16;
  __shared__ __align__(16) elem_t smem[2 * BKV * LDK];          // K and V tile; at the ends the staged Q, dO and dQ rows
  static_assert(2 * BKV * LDK >= 128 * (D + 8), "the workgroup's 128 rows fit the tile buffers");
  elem_t* sK = smem;
  elem_t* sV = smem + BKV * LDK;
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
  float delta_q;
  __shared__ float s_delta[128];

  elemx8 qf[KK], dof[KK];
  if (EXACT) {
    // dO and O rows of the workgroup's queries, chunk for chunk in the same registers of the same threads: the
    // D / 8 lanes that hold a row's chunks add up its products
    using Rows = TileRegs<128, D>;
    constexpr int LPR = D / 8, RSTEP = 256 / LPR;
    const uint32_t o_bytes = (uint32_t)(((int64_t)(s - 1) * h + D) * 2), o_off0 = Rows::offset0((uint32_t)h * 2u, tid);
    Rows r_q, r_do, r_o;         // all three requested at once; Q, needed first, in front
    r_q.load_buffer(make_rsrc(qb, (uint32_t)(((int64_t)(s - 1) * ld + D) * 2)), Rows::offset0((uint32_t)ld * 2u, tid),
                    (uint32_t)ld * 2u, q0);
    r_do.load_buffer(make_rsrc(dob, o_bytes), o_off0, (uint32_t)h * 2u, q0);
    r_o.load_buffer(make_rsrc(o + (int64_t)bi * s * h + hd * d, o_bytes), o_off0, (uint32_t)h * 2u, q0);
    r_q.template store<D + 8>(smem, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = frag_kcontig(smem + (32 * wave) * (D + 8) + kk * 16, D + 8, lane);
    __syncthreads();
    r_do.template store<D + 8>(smem, tid);
#pragma unroll
    for (int j = 0; j < Rows::NCH; ++j) {
      const elemx8 ov = __builtin_bit_cast(elemx8, r_o.r[j]), dv = __builtin_bit_cast(elemx8, r_do.r[j]);
      float p = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) p += (float)ov[e] * (float)dv[e];
#pragma unroll
      for (int off = LPR / 2; off > 0; off >>= 1) p += __shfl_xor(p, off, 64);
      const int row = tid / LPR + j * RSTEP;
      if (tid % LPR == 0) {
        s_delta[row] = p;
        if (q0 + row < s) delta[((int64_t)bi * a + hd) * s + q0 + row] = p;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) dof[kk] = frag_kcontig(smem + (32 * wave) * (D + 8) + kk * 16, D + 8, lane);
    delta_q = s_delta[32 * wave + (lane & 31)];
  } else {
    delta_q = (qi < s) ? delta[((int64_t)bi * a + hd) * s + qi] : 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qf[kk] = global_frag<EXACT>(qb, ld, qi, s, kk * 16, lane, d);
      dof[kk] = global_frag<EXACT>(dob, h, qi, s, kk * 16, lane, d);
    }
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
  if (EXACT) {
    __syncthreads();              // the tiles in LDS are done with
    store_rows_out<D>(smem + wave * (32 * (D + 8)), dqacc, scale, dqkv + ((int64_t)bi * s + qw0) * ld + hd * d, ld, s - qw0, lane);
    return;
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
  const dim3 grid((unsigned)(((s + 127) / 128) * b * a));
  // the exact-size dQ kernel (the dispatch's condition for it) forms delta itself and runs first
  const bool dq_forms_delta = (d == 64 || d == 128) && ((int64_t)s + 256) * 3 * a * d * 2 < (int64_t(1) << 31);
  hipError_t e;
  if (dq_forms_delta) {
    AXONN_ATTN_DISPATCH(attn_bwd_dq_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)o, (const elem_t*)dout, lse, delta, (elem_t*)dqkv);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    AXONN_ATTN_DISPATCH(attn_bwd_dkdv_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)dout, lse, (const float*)delta, (elem_t*)dqkv);
    return hipGetLastError();
  }
  const int64_t n_pairs = (int64_t)b * s * a;
  hipLaunchKernelGGL(attn_delta_general_kernel, dim3((unsigned)((n_pairs + 15) / 16)), dim3(256), 0, st, n_pairs, s, a, d,
                     (const elem_t*)o, (const elem_t*)dout, delta);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  AXONN_ATTN_DISPATCH(attn_bwd_dkdv_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)dout, lse, (const float*)delta, (elem_t*)dqkv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  AXONN_ATTN_DISPATCH(attn_bwd_dq_kernel, s, a, b * a, d, (const elem_t*)qkv, (const elem_t*)o, (const elem_t*)dout, lse, delta, (elem_t*)dqkv);
  return hipGetLastError();
}
#undef AXONN_ATTN_DISPATCH

}  // namespace axonn
