// HBM-bound kernels of the stage: LayerNorm forward / backward, column sums (bias and
// LayerNorm parameter gradients), small accumulate / convert helpers and the Adam bucket
// kernel.  All of them move 16-byte vectors per lane along the contiguous dimension and
// reduce with wavefront shuffles; none of them uses atomics, so results are reproducible.
#include "common.h"

namespace axonn {

// One workgroup of 4 wavefronts per row: the row lives in registers (MAXC chunks of 8 bf16 per
// lane, chunk c of thread t is chunk c*256 + t of the row), so the mean and the variance are the
// plain two-pass definitions computed from one HBM read; the four wavefront sums are combined
// through LDS in a fixed order.  MAXC is the smallest power of two that covers the row, so that a
// thread holds few registers and many rows are in flight per CU.
constexpr int LN_THREADS = 256;
constexpr int LN_MAX_COLS = 16 * LN_THREADS * 8;   // 32768

__device__ __forceinline__ float block_sum4(float v, float (&red)[4], int lane, int wave) {
  v = wave_sum(v);
  __syncthreads();                 // previous use of red[] is over
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return ((red[0] + red[1]) + red[2]) + red[3];
}

template <int MAXC>
__global__ __launch_bounds__(LN_THREADS) void layernorm_fwd_kernel(
    int T, int h, const elem_t* __restrict__ x, const elem_t* __restrict__ gamma,
    const elem_t* __restrict__ beta, float eps, elem_t* __restrict__ out,
    elem_t* __restrict__ out_lo, float* __restrict__ stats) {
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int nch = h >> 3;
  const elem_t* xr = x + (int64_t)row * h;
  elemx8 v[MAXC];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * LN_THREADS + tid;
    if (ch < nch) {
      v[c] = *reinterpret_cast<const elemx8*>(xr + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += (float)v[c][e];
    }
  }
  const float mean = block_sum4(sum, red, lane, wave) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * LN_THREADS + tid;
    if (ch < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = (float)v[c][e] - mean;
        sq += d * d;
      }
    }
  }
  const float rstd = rsqrtf(block_sum4(sq, red, lane, wave) / (float)h + eps);
  if (tid == 0) {
    stats[2 * (int64_t)row] = mean;
    stats[2 * (int64_t)row + 1] = rstd;
  }
  elem_t* orow = out + (int64_t)row * h;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * LN_THREADS + tid;
    if (ch < nch) {
      const elemx8 gv = *reinterpret_cast<const elemx8*>(gamma + ch * 8);
      const elemx8 bv = *reinterpret_cast<const elemx8*>(beta + ch * 8);
      elemx8 o, lo;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float val = (float)gv[e] * (((float)v[c][e] - mean) * rstd) + (float)bv[e];
        o[e] = (elem_t)val;
        lo[e] = (elem_t)(val - (float)o[e]);   // what the rounding to bf16 dropped
      }
      *reinterpret_cast<elemx8*>(orow + ch * 8) = o;
      if (out_lo) *reinterpret_cast<elemx8*>(out_lo + (int64_t)row * h + ch * 8) = lo;
    }
  }
}

// dx = res + rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)),  dxhat = dout * gamma
template <int MAXC>
__global__ __launch_bounds__(LN_THREADS) void layernorm_bwd_dx_kernel(
    int T, int h, const elem_t* __restrict__ dout, const elem_t* __restrict__ x,
    const float* __restrict__ stats, const elem_t* __restrict__ gamma,
    const elem_t* __restrict__ res, elem_t* __restrict__ dx) {
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int nch = h >> 3;
  const float mean = stats[2 * (int64_t)row], rstd = stats[2 * (int64_t)row + 1];
  const elem_t* xr = x + (int64_t)row * h;
  const elem_t* dr = dout + (int64_t)row * h;
  elemx8 xv[MAXC], dv[MAXC];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * LN_THREADS + tid;
    if (ch < nch) {
      xv[c] = *reinterpret_cast<const elemx8*>(xr + ch * 8);
      dv[c] = *reinterpret_cast<const elemx8*>(dr + ch * 8);
      const elemx8 gv = *reinterpret_cast<const elemx8*>(gamma + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float dxh = (float)dv[c][e] * (float)gv[e];
        const float xh = ((float)xv[c][e] - mean) * rstd;
        s1 += dxh;
        s2 += dxh * xh;
      }
    }
  }
  const float m1 = block_sum4(s1, red, lane, wave) / (float)h;
  const float m2 = block_sum4(s2, red, lane, wave) / (float)h;
  elem_t* orow = dx + (int64_t)row * h;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int ch = c * LN_THREADS + tid;
    if (ch < nch) {
      const elemx8 gv = *reinterpret_cast<const elemx8*>(gamma + ch * 8);
      elemx8 rv;
      if (res) rv = *reinterpret_cast<const elemx8*>(res + (int64_t)row * h + ch * 8);
      elemx8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float dxh = (float)dv[c][e] * (float)gv[e];
        const float xh = ((float)xv[c][e] - mean) * rstd;
        float r = rstd * (dxh - m1 - xh * m2);
        if (res) r += (float)rv[e];
        o[e] = (elem_t)r;
      }
      *reinterpret_cast<elemx8*>(orow + ch * 8) = o;
    }
  }
}

// Column partial sums over a block of 64 rows.  Each wave owns 512 columns (8 per lane) of
// a 16-row quarter of the block; quarters are combined through LDS.  MODE 0: sum y.
// MODE 1: sum y and sum y * xhat with xhat = (x - mean) * rstd (LayerNorm gain gradient).
// partial layout: [row_block][MODE+1][ncols].
constexpr int CS_ROWS = 64;
template <int MODE>
__global__ __launch_bounds__(256) void colsum_partial_kernel(
    int T, int N, const elem_t* __restrict__ y, int64_t ldy, const elem_t* __restrict__ x,
    const float* __restrict__ stats, float* __restrict__ partial) {
  __shared__ float red[3][2][64][8];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + lane) * 8;
  const int r_begin = blockIdx.y * CS_ROWS + q * (CS_ROWS / 4);
  float a0[8], a1[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a0[e] = a1[e] = 0.f;
  if (col < N) {
    // the rows of a batch are all requested before the first is added: with one load in flight per lane every
    // row costs a round trip to HBM
    constexpr int QR = CS_ROWS / 4;
    constexpr int HB = MODE == 1 ? 4 : 8;  // rows per batch of loads (two operands and the row statistics in mode 1)
#pragma unroll
    for (int i0 = 0; i0 < QR; i0 += HB) {
      elemx8 yv[HB], xv[HB];
      float mean[HB], rstd[HB];
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        // rows past the end re-read the last row and are left out of the sums below
        const int r = min(r_begin + i0 + i, T - 1);
        yv[i] = *reinterpret_cast<const elemx8*>(y + (int64_t)r * ldy + col);
        if (MODE == 1) {
          xv[i] = *reinterpret_cast<const elemx8*>(x + (int64_t)r * N + col);
          mean[i] = stats[2 * (int64_t)r];
          rstd[i] = stats[2 * (int64_t)r + 1];
        }
      }
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        const bool in_range = r_begin + i0 + i < T;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float v = in_range ? (float)yv[i][e] : 0.f;
          a0[e] += v;
          if (MODE == 1) a1[e] += v * (((float)xv[i][e] - mean[i]) * rstd[i]);
        }
      }
    }
  }
  if (q > 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[q - 1][0][lane][e] = a0[e];
      if (MODE == 1) red[q - 1][1][lane][e] = a1[e];
    }
  }
  __syncthreads();
  if (q == 0 && col < N) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // fixed order q = 0,1,2,3 keeps the sum reproducible
      a0[e] = ((a0[e] + red[0][0][lane][e]) + red[1][0][lane][e]) + red[2][0][lane][e];
      if (MODE == 1) a1[e] = ((a1[e] + red[0][1][lane][e]) + red[1][1][lane][e]) + red[2][1][lane][e];
    }
    float* p0 = partial + ((int64_t)blockIdx.y * (MODE + 1)) * N + col;
    *reinterpret_cast<floatx4*>(p0) = floatx4{a0[0], a0[1], a0[2], a0[3]};
    *reinterpret_cast<floatx4*>(p0 + 4) = floatx4{a0[4], a0[5], a0[6], a0[7]};
    if (MODE == 1) {
      float* p1 = p0 + N;
      *reinterpret_cast<floatx4*>(p1) = floatx4{a1[0], a1[1], a1[2], a1[3]};
      *reinterpret_cast<floatx4*>(p1 + 4) = floatx4{a1[4], a1[5], a1[6], a1[7]};
    }
  }
}

// out[k][n] = sum over row blocks of partial[rb][k][n], k < KSUM.  The sums are either stored as
// fp32 (acc_mode 0), or stored into / added to gradient vectors of the accumulation type
// (acc_mode 1 / 2; dst_fp32 says whether that type is fp32 or bf16).
template <typename T>
__device__ __forceinline__ void put_sum(T* dst, int n, float v, int acc_mode) {
  dst[n] = (T)((acc_mode == 2 ? (float)dst[n] : 0.f) + v);
}
// A block owns 64 columns; its four wavefronts each sum every fourth row block (loads independent of one
// another, so they are all in flight at once), and the four sums are combined through LDS in a fixed order.
template <int KSUM>
__global__ __launch_bounds__(256) void colsum_final_kernel(int nrb, int N,
                                                           const float* __restrict__ partial,
                                                           void* __restrict__ out0,
                                                           void* __restrict__ out1,
                                                           int acc_mode, int dst_fp32) {
  __shared__ float red[3][KSUM][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  float s0 = 0.f, s1 = 0.f;
  if (n < N) {
#pragma unroll 8
    for (int rb = q; rb < nrb; rb += 4) {
      s0 += partial[((int64_t)rb * KSUM) * N + n];
      if (KSUM == 2) s1 += partial[((int64_t)rb * KSUM + 1) * N + n];
    }
  }
  if (q > 0) {
    red[q - 1][0][lane] = s0;
    if (KSUM == 2) red[q - 1][KSUM - 1][lane] = s1;
  }
  __syncthreads();
  if (q != 0 || n >= N) return;
  s0 = ((s0 + red[0][0][lane]) + red[1][0][lane]) + red[2][0][lane];
  if (KSUM == 2) s1 = ((s1 + red[0][KSUM - 1][lane]) + red[1][KSUM - 1][lane]) + red[2][KSUM - 1][lane];
  if (acc_mode == 0 || dst_fp32) {
    put_sum(reinterpret_cast<float*>(out0), n, s0, acc_mode);
    if (KSUM == 2) put_sum(reinterpret_cast<float*>(out1), n, s1, acc_mode);
  } else {
    put_sum(reinterpret_cast<elem_t*>(out0), n, s0, acc_mode);
    if (KSUM == 2) put_sum(reinterpret_cast<elem_t*>(out1), n, s1, acc_mode);
  }
}

__global__ __launch_bounds__(256) void f32_to_elem_kernel(uint64_t n8, uint64_t n,
                                                          const float* __restrict__ src,
                                                          elem_t* __restrict__ dst) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    const floatx4 a = *reinterpret_cast<const floatx4*>(src + i * 8);
    const floatx4 b = *reinterpret_cast<const floatx4*>(src + i * 8 + 4);
    elemx8 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) { o[e] = (elem_t)a[e]; o[4 + e] = (elem_t)b[e]; }
    *reinterpret_cast<elemx8*>(dst + i * 8) = o;
  }
  if (blockIdx.x == 0) {
    for (uint64_t i = n8 * 8 + threadIdx.x; i < n; i += 256) dst[i] = (elem_t)src[i];
  }
}

__global__ __launch_bounds__(256) void fill_elem_kernel(uint64_t n, elem_t* dst, float value) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  const elem_t v = (elem_t)value;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = v;
}

// Adam with decoupled weight decay on one resident bucket: per element 12 B of fp32 state and
// 2 B of bf16 gradient in, 12 B of state and 2 B of bf16 parameter out.
struct AdamConsts {
  float lr, b1, b2, omb1, omb2, eps, wd, grad_scale, inv_bc1, inv_bc2;
};
__device__ __forceinline__ void adam_elem(float& th, float& m, float& v, float g16,
                                          const AdamConsts& c) {
  const float g = c.grad_scale * g16;
  m = c.b1 * m + c.omb1 * g;
  v = c.b2 * v + c.omb2 * g * g;
  const float mhat = m * c.inv_bc1;
  const float vhat = v * c.inv_bc2;
  th = th - c.lr * (mhat / (sqrtf(vhat) + c.eps) + c.wd * th);
}
// theta16 = the 16-bit rounding of the fp32 theta that is stored, not of the unrounded update: for half
// precision the compiler would otherwise fuse the last multiply-add with the conversion (one rounding from
// the exact result), which differs from rounding the stored value where that is an exact tie.
__device__ __forceinline__ elem_t round_stored(float a) {
  asm volatile("" : "+v"(a));
  return (elem_t)a;
}
__global__ __launch_bounds__(256) void adam_kernel(uint64_t n8, uint64_t n, float* __restrict__ theta,
                                                   float* __restrict__ m, float* __restrict__ v,
                                                   const elem_t* __restrict__ g16,
                                                   elem_t* __restrict__ p16, AdamConsts c) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    const uint64_t o = i * 8;
    floatx4 t0 = *reinterpret_cast<const floatx4*>(theta + o), t1 = *reinterpret_cast<const floatx4*>(theta + o + 4);
    floatx4 m0 = *reinterpret_cast<const floatx4*>(m + o), m1 = *reinterpret_cast<const floatx4*>(m + o + 4);
    floatx4 v0 = *reinterpret_cast<const floatx4*>(v + o), v1 = *reinterpret_cast<const floatx4*>(v + o + 4);
    const elemx8 gv = *reinterpret_cast<const elemx8*>(g16 + o);
    elemx8 pv;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float a = t0[e], b = m0[e], d = v0[e];
      adam_elem(a, b, d, (float)gv[e], c);
      t0[e] = a; m0[e] = b; v0[e] = d; pv[e] = round_stored(a);
      a = t1[e]; b = m1[e]; d = v1[e];
      adam_elem(a, b, d, (float)gv[4 + e], c);
      t1[e] = a; m1[e] = b; v1[e] = d; pv[4 + e] = round_stored(a);
    }
    *reinterpret_cast<floatx4*>(theta + o) = t0; *reinterpret_cast<floatx4*>(theta + o + 4) = t1;
    *reinterpret_cast<floatx4*>(m + o) = m0; *reinterpret_cast<floatx4*>(m + o + 4) = m1;
    *reinterpret_cast<floatx4*>(v + o) = v0; *reinterpret_cast<floatx4*>(v + o + 4) = v1;
    *reinterpret_cast<elemx8*>(p16 + o) = pv;
  }
  if (blockIdx.x == 0) {
    for (uint64_t i = n8 * 8 + threadIdx.x; i < n; i += 256) {
      float a = theta[i], b = m[i], d = v[i];
      adam_elem(a, b, d, (float)g16[i], c);
      theta[i] = a; m[i] = b; v[i] = d; p16[i] = round_stored(a);
    }
  }
}

// ------------------------------------------------------------------------- launchers
#define AXONN_LN_DISPATCH(KERNEL, ...)                                                        \
  {                                                                                           \
    const dim3 grid((unsigned)T), block(LN_THREADS);                                          \
    const int64_t per_thread = (h + LN_THREADS * 8 - 1) / (LN_THREADS * 8);                   \
    if (per_thread <= 1) hipLaunchKernelGGL(KERNEL<1>, grid, block, 0, s, __VA_ARGS__);       \
    else if (per_thread <= 2) hipLaunchKernelGGL(KERNEL<2>, grid, block, 0, s, __VA_ARGS__);  \
    else if (per_thread <= 4) hipLaunchKernelGGL(KERNEL<4>, grid, block, 0, s, __VA_ARGS__);  \
    else if (per_thread <= 8) hipLaunchKernelGGL(KERNEL<8>, grid, block, 0, s, __VA_ARGS__);  \
    else hipLaunchKernelGGL(KERNEL<16>, grid, block, 0, s, __VA_ARGS__);                      \
  }

hipError_t launch_layernorm_fwd(int64_t T, int64_t h, const void* x, const void* gamma,
                                const void* beta, float eps, void* out, void* out_lo, float* stats,
                                hipStream_t s) {
  if (h > LN_MAX_COLS || T <= 0) return hipErrorInvalidValue;
  AXONN_LN_DISPATCH(layernorm_fwd_kernel, (int)T, (int)h, (const elem_t*)x, (const elem_t*)gamma,
                    (const elem_t*)beta, eps, (elem_t*)out, (elem_t*)out_lo, stats)
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd(int64_t T, int64_t h, const void* dout, const void* x,
                                const float* stats, const void* gamma, const void* res_grad,
                                void* dx, void* dgamma, void* dbeta, int acc_mode, bool dst_fp32,
                                float* ws, hipStream_t s) {
  if (h > LN_MAX_COLS || T <= 0) return hipErrorInvalidValue;
  AXONN_LN_DISPATCH(layernorm_bwd_dx_kernel, (int)T, (int)h, (const elem_t*)dout, (const elem_t*)x,
                    stats, (const elem_t*)gamma, (const elem_t*)res_grad, (elem_t*)dx)
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int nrb = (int)((T + CS_ROWS - 1) / CS_ROWS);
  const dim3 g2((unsigned)((h + 511) / 512), (unsigned)nrb);
  hipLaunchKernelGGL(colsum_partial_kernel<1>, g2, dim3(256), 0, s, (int)T, (int)h,
                     (const elem_t*)dout, (int64_t)h, (const elem_t*)x, stats, ws);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_final_kernel<2>, dim3((unsigned)((h + 63) / 64)), dim3(256), 0, s, nrb,
                     (int)h, (const float*)ws, dbeta, dgamma, acc_mode, dst_fp32 ? 1 : 0);
  return hipGetLastError();
}
#undef AXONN_LN_DISPATCH

hipError_t launch_colsum(int64_t T, int64_t N, const void* y, int64_t ldy, void* out, int acc_mode,
                         bool dst_fp32, float* ws, hipStream_t s) {
  const int nrb = (int)((T + CS_ROWS - 1) / CS_ROWS);
  const dim3 g2((unsigned)((N + 511) / 512), (unsigned)nrb);
  hipLaunchKernelGGL(colsum_partial_kernel<0>, g2, dim3(256), 0, s, (int)T, (int)N,
                     (const elem_t*)y, ldy, (const elem_t*)nullptr, (const float*)nullptr, ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_final_kernel<1>, dim3((unsigned)((N + 63) / 64)), dim3(256), 0, s, nrb,
                     (int)N, (const float*)ws, out, (void*)nullptr, acc_mode, dst_fp32 ? 1 : 0);
  return hipGetLastError();
}

static unsigned grid_for(uint64_t work_items) {
  uint64_t b = (work_items + 255) / 256;
  if (b < 1) b = 1;
  if (b > 256 * 16) b = 256 * 16;  // 16 blocks per CU, grid-stride beyond
  return (unsigned)b;
}

// Number of elements of x[0..n) that are not finite (infinity or NaN): what a dynamic loss scaler looks for
// in the 16-bit gradients.  kNonfiniteBlocks workgroups write one partial count each, a second launch adds
// them in a fixed order: no atomics, no buffer to clear.  ws holds kNonfiniteBlocks + 1 counters; the total
// lands in ws[kNonfiniteBlocks].
constexpr int kNonfiniteBlocks = 1024;
__global__ __launch_bounds__(256) void nonfinite_partial_kernel(uint64_t n, const elem_t* __restrict__ x,
                                                                unsigned long long* __restrict__ ws) {
  __shared__ unsigned int red[4];
  const uint64_t n8 = n / 8;
  unsigned int c = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (uint64_t)kNonfiniteBlocks * 256) {
    const elemx8 v = *reinterpret_cast<const elemx8*>(x + i * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float f = (float)v[e];
      c += (f - f == 0.f) ? 0u : 1u;          // inf - inf and NaN - NaN are NaN
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(n - n8 * 8)) {
    const float f = (float)x[n8 * 8 + threadIdx.x];
    c += (f - f == 0.f) ? 0u : 1u;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) ws[blockIdx.x] = (unsigned long long)red[0] + red[1] + red[2] + red[3];
}
__global__ __launch_bounds__(256) void nonfinite_final_kernel(unsigned long long* __restrict__ ws) {
  __shared__ unsigned long long red[4];
  unsigned long long c = 0;
  for (int i = threadIdx.x; i < kNonfiniteBlocks; i += 256) c += ws[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) ws[kNonfiniteBlocks] = red[0] + red[1] + red[2] + red[3];
}
hipError_t launch_count_nonfinite(uint64_t n, const void* x, uint64_t* ws, hipStream_t s) {
  hipLaunchKernelGGL(nonfinite_partial_kernel, dim3(kNonfiniteBlocks), dim3(256), 0, s, n, (const elem_t*)x,
                     (unsigned long long*)ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(nonfinite_final_kernel, dim3(1), dim3(256), 0, s, (unsigned long long*)ws);
  return hipGetLastError();
}

hipError_t launch_f32_to_elem(uint64_t n, const float* src, void* dst, hipStream_t s) {
  hipLaunchKernelGGL(f32_to_elem_kernel, dim3(grid_for(n / 8)), dim3(256), 0, s, n / 8, n, src,
                     (elem_t*)dst);
  return hipGetLastError();
}

hipError_t launch_fill_elem(uint64_t n, void* dst, float value, hipStream_t s) {
  hipLaunchKernelGGL(fill_elem_kernel, dim3(grid_for(n)), dim3(256), 0, s, n, (elem_t*)dst, value);
  return hipGetLastError();
}

hipError_t launch_adam(uint64_t n, float* theta, float* m, float* v, const void* g16, void* p16,
                       double lr, double b1, double b2, double eps, double wd, int64_t step,
                       double grad_scale, hipStream_t s) {
  AdamConsts c;
  c.lr = (float)lr; c.b1 = (float)b1; c.b2 = (float)b2; c.eps = (float)eps; c.wd = (float)wd;
  c.grad_scale = (float)grad_scale;
  // 1 - beta and the bias corrections in double on the host: they lose digits in float for
  // beta near 1
  c.omb1 = (float)(1.0 - b1); c.omb2 = (float)(1.0 - b2);
  c.inv_bc1 = (float)(1.0 / (1.0 - pow(b1, (double)step)));
  c.inv_bc2 = (float)(1.0 / (1.0 - pow(b2, (double)step)));
  hipLaunchKernelGGL(adam_kernel, dim3(grid_for(n / 8)), dim3(256), 0, s, n / 8, n, theta, m, v,
                     (const elem_t*)g16, (elem_t*)p16, c);
  return hipGetLastError();
}

}  // namespace axonn
