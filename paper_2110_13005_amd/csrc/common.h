// Shared declarations of libaxonn_stage: vector types, MFMA fragment helpers for gfx950,
// wavefront reductions and the internal launch functions the stage runtime calls.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace axonn {

// The 16-bit element type of activations, parameters and gradients: bfloat16, or IEEE half precision (the
// paper's arithmetic, Sec. 2 "Mixed precision") when the sources are compiled with AXONN_ELEM_FP16: the
// same kernels, the other conversion and MFMA instructions.  Both formats round to nearest even on
// conversion from fp32; fp16 overflows to infinity beyond 65504, which is what the loss scaler looks for.
#ifdef AXONN_ELEM_FP16
typedef _Float16 elem_t;
#define AXONN_ELEM_TYPE_ID 1
#define AXONN_MFMA_32X32X16 __builtin_amdgcn_mfma_f32_32x32x16_f16
#define AXONN_MFMA_16X16X32 __builtin_amdgcn_mfma_f32_16x16x32_f16
#define AXONN_MFMA_16X16X32_ASM "v_mfma_f32_16x16x32_f16"
#define AXONN_MFMA_32X32X16_ASM "v_mfma_f32_32x32x16_f16"
#else
typedef __bf16 elem_t;
#define AXONN_ELEM_TYPE_ID 0
#define AXONN_MFMA_32X32X16 __builtin_amdgcn_mfma_f32_32x32x16_bf16
#define AXONN_MFMA_16X16X32 __builtin_amdgcn_mfma_f32_16x16x32_bf16
#define AXONN_MFMA_16X16X32_ASM "v_mfma_f32_16x16x32_bf16"
#define AXONN_MFMA_32X32X16_ASM "v_mfma_f32_32x32x16_bf16"
#endif
typedef __attribute__((__vector_size__(2 * sizeof(elem_t)))) elem_t elemx2;
typedef __attribute__((__vector_size__(4 * sizeof(elem_t)))) elem_t elemx4;
typedef __attribute__((__vector_size__(8 * sizeof(elem_t)))) elem_t elemx8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

#define AXONN_LDS __attribute__((address_space(3)))

#ifdef __HIPCC__
// ---------------------------------------------------------------------------------
// v_mfma_f32_32x32x16_{bf16,f16} register layout (checked on hardware):
//   operand X (either input): lane l holds X[row = l%32][k = 8*(l/32) + i], i = 0..7
//   result D[m][n]:           lane l, register r holds n = l%32, m = 8*(r/4) + 4*(l/32) + r%4
// D = first_operand(rows -> m) x second_operand(rows -> n).
// ---------------------------------------------------------------------------------
__device__ __forceinline__ floatx16 mfma32(elemx8 a, elemx8 b, floatx16 c) {
  return AXONN_MFMA_32X32X16(a, b, c, 0, 0, 0);
}

// v_mfma_f32_16x16x32_{bf16,f16} register layout:
//   operand X (either input): lane l holds X[row = l%16][k = 8*(l/16) + i], i = 0..7
//   result D[m][n]:           lane l, register r holds n = l%16, m = 4*(l/16) + r
// Same work per cycle as the 32x32x16 form, but it draws less power per FLOP (less accumulator
// traffic), which matters once the whole chip runs MFMAs and the clock is power-limited.
__device__ __forceinline__ floatx4 mfma16(elemx8 a, elemx8 b, floatx4 c) {
  return AXONN_MFMA_16X16X32(a, b, c, 0, 0, 0);
}
// Raw buffer descriptor over `bytes` bytes at p: a load at an offset at or beyond `bytes` returns zeros
// without touching memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// The same instruction with the accumulator pinned to the accumulation registers (a[...]): a kernel
// whose 256 accumulators fill that file exactly needs every one of them there, and the register
// allocator does not get this right by itself.  The compiler does not see an MFMA here, so the
// caller keeps MFMA hazards itself: a few idle cycles between writing an accumulator with another
// instruction and the first MFMA on it, and >= 18 between the last MFMA and reading the result.
__device__ __forceinline__ void mfma16_acc(floatx4& c, elemx8 a, elemx8 b) {
  asm volatile(AXONN_MFMA_16X16X32_ASM " %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// The 32x32x16 form as inline assembly, for kernels that fix the order of their MFMAs and the register file of every
// accumulator themselves (volatile statements keep their order, and memory operations do not move across them): a
// kernel with more than 256 registers per lane gets the accumulation-register form of the builtin for every MFMA, and
// results that vector instructions consume next would be copied out one register at a time.
//   mfma32_agpr:      c += a x b, c in the accumulation registers (long-lived accumulators)
//   mfma32_vgpr_*_ba: c in ordinary registers, b in the accumulation registers; plain: c += a x b, _zero: c = a x b
// The compiler does not know these are MFMAs and keeps none of their hazards, so the statements carry them:
//   * two wait states ahead of every MFMA: the distance a register written by a vector instruction needs before an
//     MFMA reads it, and the compiler may place such a write (a copy, an initialisation, the conversion that produces
//     an operand) directly in front of the statement;
//   * _settled: 20 wait states behind the MFMA, inside the statement, so that nothing can come between: more than
//     the eight passes plus the distance the rules ask for before another kind of instruction reads (or the
//     compiler copies) the result.  They pass while the MFMA executes.  A chain's last MFMA is issued this way, or
//     one MFMA before such a one; mfma32_settle_agpr does the same for accumulators at the end of a kernel.
#define AXONN_MFMA32_GAP "s_nop 1\n\t"
#define AXONN_MFMA32_SETTLE "\n\ts_nop 7\n\ts_nop 7\n\ts_nop 3"
__device__ __forceinline__ void mfma32_agpr(floatx16& c, elemx8 a, elemx8 b) {
  asm volatile(AXONN_MFMA32_GAP AXONN_MFMA_32X32X16_ASM " %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma32_vgpr_ba(floatx16& c, elemx8 a, elemx8 b) {
  asm volatile(AXONN_MFMA32_GAP AXONN_MFMA_32X32X16_ASM " %0, %1, %2, %0" : "+v"(c) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma32_vgpr_zero_ba(floatx16& c, elemx8 a, elemx8 b) {
  asm volatile(AXONN_MFMA32_GAP AXONN_MFMA_32X32X16_ASM " %0, %1, %2, 0" : "=&v"(c) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma32_vgpr_settled_ba(floatx16& c, elemx8 a, elemx8 b) {
  asm volatile(AXONN_MFMA32_GAP AXONN_MFMA_32X32X16_ASM " %0, %1, %2, %0" AXONN_MFMA32_SETTLE : "+v"(c) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma32_settle_agpr(floatx16& c0, floatx16& c1) {
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+a"(c0), "+a"(c1));
}

// Fragment of a 32(row) x 16(k) operand block from an LDS tile stored [row][k] (k
// contiguous, `ld` elements per row).  `base` points at (row0, k0).
__device__ __forceinline__ elemx8 frag_kcontig(const elem_t* base, int ld, int lane) {
  return *reinterpret_cast<const elemx8*>(base + (lane & 31) * ld + 8 * (lane >> 5));
}

// ds_read_b64_tr_b16 (checked on hardware): within each group of 16 lanes, lane t supplies
// the address of 4 consecutive 16-bit values; lane t receives element t%4 of the values
// addressed by lanes t/4, 4 + t/4, 8 + t/4, 12 + t/4.  So if lane t addresses
// [k = kb + t/4][r = rb + 4*(t%4) .. +3] of a [k][r] tile, lane t ends up holding
// r = rb + t for k = kb .. kb+3.
__device__ __forceinline__ short4v lds_read_tr16(const elem_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (AXONN_LDS short4v*)p);
}

// Fragment of a 32(row) x 16(k) operand block from an LDS tile stored [k][row] (row
// contiguous, `ld` elements per k).  `base` points at (k0, row0).
// PERM = false: register i of lane l holds k = k0 + 8*(l/32) + i (same convention as
//               frag_kcontig, to pair with any other operand).
// PERM = true:  register j of lane l holds k = k0 + 8*(j/4) + 4*(l/32) + j%4, which is the
//               order in which an MFMA result tile keeps its m index in registers 0..7 --
//               to pair with an operand built in registers from a result tile.
template <bool PERM>
__device__ __forceinline__ elemx8 frag_kstrided(const elem_t* base, int ld, int lane) {
  const int t = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const int kq = t >> 2, r = 16 * half + 4 * (t & 3);
  const int k_a = PERM ? 4 * g : 8 * g;
  const int k_b = PERM ? 8 + 4 * g : 8 * g + 4;
  union { elemx8 v; short4v h[2]; } u;
  u.h[0] = lds_read_tr16(base + (k_a + kq) * ld + r);
  u.h[1] = lds_read_tr16(base + (k_b + kq) * ld + r);
  return u.v;
}

// The same two fragment readers for a 16(row) x 32(k) operand block of the 16x16x32 MFMA.
__device__ __forceinline__ elemx8 frag16_kcontig(const elem_t* base, int ld, int lane) {
  return *reinterpret_cast<const elemx8*>(base + (lane & 15) * ld + 8 * (lane >> 4));
}
__device__ __forceinline__ elemx8 frag16_kstrided(const elem_t* base, int ld, int lane) {
  const int t = lane & 15, g = lane >> 4;
  const int kq = t >> 2, r = 4 * (t & 3);
  union { elemx8 v; short4v h[2]; } u;
  u.h[0] = lds_read_tr16(base + (8 * g + kq) * ld + r);
  u.h[1] = lds_read_tr16(base + (8 * g + 4 + kq) * ld + r);
  return u.v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ float bf2f(elem_t v) { return (float)v; }
__device__ __forceinline__ elem_t f2bf(float v) { return (elem_t)v; }

// GeLU pieces in the exact (erf) form: Phi(x) = 0.5*(1+erf(x/sqrt2)), phi(x) = exp(-x^2/2)/sqrt(2pi).
// erfc(z), z >= 0, is evaluated as a degree-5 polynomial in 1/(1 + p z) times exp(-z^2) (Abramowitz &
// Stegun 7.1.26, absolute error <= 1.5e-7, i.e. one fp32 ulp of values near 1); Phi takes erfc(|x|/sqrt2)
// on the side of the tail, so there is no cancellation for negative x.  `e` returns exp(-x^2/2), which
// the derivative needs as well.
__device__ __forceinline__ float normal_cdf_f(float x, float& e) {
  const float z = fabsf(x) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * z);   // v_rcp_f32 (1 ulp), not the 10-instruction IEEE division
  e = __expf(-z * z);
  float p = 1.061405429f;
  p = p * t - 1.453152027f;
  p = p * t + 1.421413741f;
  p = p * t - 0.284496736f;
  p = p * t + 0.254829592f;
  const float half_erfc = 0.5f * p * t * e;
  return x >= 0.f ? 1.0f - half_erfc : half_erfc;
}
__device__ __forceinline__ float gelu_f(float x) {
  float e;
  return x * normal_cdf_f(x, e);
}
__device__ __forceinline__ float gelu_grad_f(float x) {
  float e;
  const float cdf = normal_cdf_f(x, e);
  return cdf + x * e * 0.39894228040143267794f;
}
// GeLU(x) and GeLU'(x) together (they share Phi and the exponential).
__device__ __forceinline__ void gelu_with_grad_f(float x, float& y, float& dy) {
  float e;
  const float cdf = normal_cdf_f(x, e);
  y = x * cdf;
  dy = cdf + x * e * 0.39894228040143267794f;
}
#endif  // __HIPCC__

// --------------------------------------------------------------------- host launchers
enum GemmEpilogue {
  EPI_BIAS = 0, EPI_BIAS_RES = 1, EPI_BIAS_GELU = 2, EPI_DGELU = 3,
  EPI_ACC_F32 = 4, EPI_ACC_BF16 = 5
};

// The contraction index may be split into up to kMaxKSegments segments of K elements each that
// live in different buffers (same shape and leading dimension): segment s of operand A starts at
// A_seg[s].  This is how a weight gradient is summed over several microbatches in one launch.
constexpr int kMaxKSegments = 16;
struct GemmArgs {
  const elem_t* A_seg[kMaxKSegments];
  const elem_t* B_seg[kMaxKSegments];
  void* C;
  const elem_t* bias; const elem_t* res; elem_t* aux;
  int64_t lda, ldb, ldc, ld_res, ld_aux;
  int M, N, K;       // K = length of ONE segment
  int n_seg;
  int accumulate;
  int concurrent;    // other kernels share the chip with this launch: prefer the most efficient tile shape
                     // over one whose tile count fills the CUs a whole number of times
  int tiles_m, tiles_n;
  // Weight gradients (both operands k-strided, accumulating epilogues) only: if colsum is not null, the sums
  // over k (all segments) of B's N columns are stored in colsum[0..N), or added to it if `accumulate`; colsum
  // has C's element type.  The large-problem kernels form them on the way; for the others colsum_ws must hold
  // ceil(K/64) * N floats of workspace.
  void* colsum;
  float* colsum_ws;
};

// All return hipError_t of the launch (hipGetLastError) and validate nothing: callers check.
hipError_t launch_gemm(bool a_kc, bool b_kc, int epilogue, const GemmArgs& g, hipStream_t s);
// Launcher settings behind axonn_tuning(): knob 0 copy-kernel mask, 1 large-kernel threshold in tiles, 2 forced
// block width (0 or -1: the launcher's rule).  false: unknown knob or value out of range.
bool set_gemm_tuning(int knob, int64_t value);
hipError_t launch_layernorm_fwd(int64_t T, int64_t h, const void* x, const void* gamma,
                                const void* beta, float eps, void* out, void* out_lo, float* stats,
                                hipStream_t s);
// dgamma / dbeta and the column sums of launch_colsum go to `out` vectors: acc_mode 0 stores fp32
// sums; acc_mode 1 stores and acc_mode 2 adds to vectors of the gradient accumulation type (fp32 if
// dst_fp32, else bf16).
hipError_t launch_layernorm_bwd(int64_t T, int64_t h, const void* dout, const void* x,
                                const float* stats, const void* gamma, const void* res_grad,
                                void* dx, void* dgamma, void* dbeta, int acc_mode, bool dst_fp32,
                                float* ws, hipStream_t s);
hipError_t launch_colsum(int64_t T, int64_t N, const void* y, int64_t ldy, void* out, int acc_mode,
                         bool dst_fp32, float* ws, hipStream_t s);
hipError_t launch_f32_to_elem(uint64_t n, const float* src, void* dst, hipStream_t s);
hipError_t launch_fill_elem(uint64_t n, void* dst, float value, hipStream_t s);
// Counts the non-finite elements of x[0..n) into ws[kNonfiniteWsCounters - 1]; ws: kNonfiniteWsCounters
// 64-bit counters of device memory, all overwritten.
constexpr int kNonfiniteWsCounters = 1025;
hipError_t launch_count_nonfinite(uint64_t n, const void* x, uint64_t* ws, hipStream_t s);
hipError_t launch_attention_fwd(int b, int s, int a, int d, const void* qkv, void* o,
                                float* lse, hipStream_t st);
hipError_t launch_attention_bwd(int b, int s, int a, int d, const void* qkv, const void* o,
                                const float* lse, const void* dout, void* dqkv, float* delta,
                                hipStream_t st);
hipError_t launch_embed_fwd(int T, int h, int s, int vocab, const int* tokens, const void* wte, const void* wpe,
                            void* x, hipStream_t st);
hipError_t launch_embed_bwd(int b, int s, int h, int vocab, const int* tokens, const void* dx, void* dwte,
                            void* dwpe, int accumulate, hipStream_t st);
// Cross-entropy over bf16 logits [T, V]: token_loss[t] and loss[0] = sum_t token_loss[t] / (T * n_microbatches);
// the logits are overwritten by dloss/dlogits.
hipError_t launch_xent(int T, int V, void* logits, const int* targets, int n_microbatches, float loss_scale,
                       float* token_loss, float* loss, hipStream_t st);
hipError_t launch_adam(uint64_t n, float* theta, float* m, float* v, const void* g16,
                       void* p16, double lr, double b1, double b2, double eps, double wd,
                       int64_t step, double grad_scale, hipStream_t s);

}  // namespace axonn
