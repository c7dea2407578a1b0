// HBM-bound kernels of the first and the last pipeline stage (Alg. 2's special cases): token +
// position embedding and its gradient, and the cross-entropy over the LM head's logits with the
// loss pre-divided by the number of microbatches (Sec. 4.2).  16-byte vectors along the contiguous
// dimension, wavefront shuffles for reductions, no atomics: results are reproducible.
//
// Token and target ids outside [0, vocab) never reach an address: they are clamped into range.
#include "common.h"

namespace axonn {

constexpr int ENDS_THREADS = 256;

__device__ __forceinline__ int clamp_id(int id, int vocab) { return id < 0 ? 0 : (id >= vocab ? vocab - 1 : id); }

// x[t, :] = wte[tokens[t], :] + wpe[t % s, :]; one workgroup per token, 8 columns per lane and step.
__global__ __launch_bounds__(ENDS_THREADS) void embed_fwd_kernel(
    int T, int h, int s, int vocab, const int* __restrict__ tokens, const elem_t* __restrict__ wte,
    const elem_t* __restrict__ wpe, elem_t* __restrict__ x) {
  const int t = blockIdx.x;
  const int id = clamp_id(tokens[t], vocab);
  const elem_t* e = wte + (int64_t)id * h;
  const elem_t* p = wpe + (int64_t)(t % s) * h;
  elem_t* o = x + (int64_t)t * h;
  for (int c = threadIdx.x * 8; c < h; c += ENDS_THREADS * 8) {
    const elemx8 a = *reinterpret_cast<const elemx8*>(e + c);
    const elemx8 b = *reinterpret_cast<const elemx8*>(p + c);
    elemx8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (elem_t)((float)a[i] + (float)b[i]);
    *reinterpret_cast<elemx8*>(o + c) = r;
  }
}

// dwte[id, :] (+)= sum of dx[t', :] over the tokens t' of this microbatch with tokens[t'] == id.
// One workgroup per token t; it works only if t is the first occurrence of its id, and then adds the
// rows of all occurrences in token order (fp32), so every table row has exactly one writer.  Rows
// whose id does not occur are not touched (the caller clears the table before a batch's first pass).
__global__ __launch_bounds__(ENDS_THREADS) void embed_bwd_wte_kernel(
    int T, int h, int vocab, const int* __restrict__ tokens, const elem_t* __restrict__ dx,
    elem_t* __restrict__ dwte, int accumulate) {
  __shared__ int first_flag;
  const int t = blockIdx.x, tid = threadIdx.x;
  const int id = clamp_id(tokens[t], vocab);
  if (tid == 0) first_flag = 1;
  __syncthreads();
  for (int u = tid; u < t; u += ENDS_THREADS)
    if (clamp_id(tokens[u], vocab) == id) first_flag = 0;   // benign race: every writer stores 0
  __syncthreads();
  if (!first_flag) return;
  elem_t* g = dwte + (int64_t)id * h;
  for (int c = tid * 8; c < h; c += ENDS_THREADS * 8) {
    float acc[8];
    if (accumulate) {
      const elemx8 old = *reinterpret_cast<const elemx8*>(g + c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = (float)old[i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    }
    for (int u = t; u < T; ++u) {
      if (clamp_id(tokens[u], vocab) != id) continue;   // uniform over the workgroup
      const elemx8 v = *reinterpret_cast<const elemx8*>(dx + (int64_t)u * h + c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += (float)v[i];
    }
    elemx8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (elem_t)acc[i];
    *reinterpret_cast<elemx8*>(g + c) = r;
  }
}

// dwpe[p, :] (+)= sum over the b sequences of dx[b*s + p, :]; one workgroup per position.
__global__ __launch_bounds__(ENDS_THREADS) void embed_bwd_wpe_kernel(
    int b, int s, int h, const elem_t* __restrict__ dx, elem_t* __restrict__ dwpe, int accumulate) {
  const int p = blockIdx.x;
  elem_t* g = dwpe + (int64_t)p * h;
  for (int c = threadIdx.x * 8; c < h; c += ENDS_THREADS * 8) {
    float acc[8];
    if (accumulate) {
      const elemx8 old = *reinterpret_cast<const elemx8*>(g + c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = (float)old[i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    }
    for (int q = 0; q < b; ++q) {
      const elemx8 v = *reinterpret_cast<const elemx8*>(dx + ((int64_t)q * s + p) * h + c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += (float)v[i];
    }
    elemx8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (elem_t)acc[i];
    *reinterpret_cast<elemx8*>(g + c) = r;
  }
}

__device__ __forceinline__ float block_reduce4(float v, float (&red)[4], int lane, int wave, bool is_max) {
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : ((red[0] + red[1]) + red[2]) + red[3];
}

// One workgroup per token row of the logits [T, V] (bf16).  First sweep: row maximum and
// sum of exp(l - max) per lane with the running-maximum recurrence, combined over the workgroup;
// token_loss[t] = max + log(sum) - l[target].  Second sweep: the row is overwritten by the gradient
// of the microbatch's loss, (softmax - onehot) * scale with scale = 1 / (T * n_microbatches).
__global__ __launch_bounds__(ENDS_THREADS) void xent_kernel(
    int T, int V, elem_t* __restrict__ logits, const int* __restrict__ targets, float scale,
    float* __restrict__ token_loss) {
  __shared__ float red[4];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  elem_t* row = logits + (int64_t)t * V;
  const int tgt = clamp_id(targets[t], V);
  float m = -INFINITY, sum = 0.f;
  for (int c = tid * 8; c < V; c += ENDS_THREADS * 8) {
    const elemx8 v = *reinterpret_cast<const elemx8*>(row + c);
    float cm = (float)v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) cm = fmaxf(cm, (float)v[i]);
    const float nm = fmaxf(m, cm);
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) part += __expf((float)v[i] - nm);
    sum = sum * __expf(m - nm) + part;     // m = -inf at first: exp(-inf) = 0
    m = nm;
  }
  const float M = block_reduce4(m, red, lane, wave, true);
  const float total = block_reduce4(m == -INFINITY ? 0.f : sum * __expf(m - M), red, lane, wave, false);
  const float lse = M + __logf(total);
  if (tid == 0) token_loss[t] = lse - (float)row[tgt];
  __syncthreads();   // the target logit is read before any lane overwrites the row
  for (int c = tid * 8; c < V; c += ENDS_THREADS * 8) {
    const elemx8 v = *reinterpret_cast<const elemx8*>(row + c);
    elemx8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p = __expf((float)v[i] - lse);
      r[i] = (elem_t)((p - ((c + i) == tgt ? 1.f : 0.f)) * scale);
    }
    *reinterpret_cast<elemx8*>(row + c) = r;
  }
}

// loss[0] = scale * sum_t token_loss[t], one workgroup, fixed order.
__global__ __launch_bounds__(ENDS_THREADS) void loss_sum_kernel(int T, const float* __restrict__ token_loss,
                                                               float scale, float* __restrict__ loss) {
  __shared__ float red[4];
  const int tid = threadIdx.x;
  float s = 0.f;
  for (int t = tid; t < T; t += ENDS_THREADS) s += token_loss[t];
  const float total = block_reduce4(s, red, tid & 63, tid >> 6, false);
  if (tid == 0) loss[0] = total * scale;
}

hipError_t launch_embed_fwd(int T, int h, int s, int vocab, const int* tokens, const void* wte, const void* wpe,
                            void* x, hipStream_t st) {
  hipLaunchKernelGGL(embed_fwd_kernel, dim3((unsigned)T), dim3(ENDS_THREADS), 0, st, T, h, s, vocab, tokens,
                     (const elem_t*)wte, (const elem_t*)wpe, (elem_t*)x);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(int b, int s, int h, int vocab, const int* tokens, const void* dx, void* dwte,
                            void* dwpe, int accumulate, hipStream_t st) {
  hipLaunchKernelGGL(embed_bwd_wte_kernel, dim3((unsigned)(b * s)), dim3(ENDS_THREADS), 0, st, b * s, h, vocab,
                     tokens, (const elem_t*)dx, (elem_t*)dwte, accumulate);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(embed_bwd_wpe_kernel, dim3((unsigned)s), dim3(ENDS_THREADS), 0, st, b, s, h,
                     (const elem_t*)dx, (elem_t*)dwpe, accumulate);
  return hipGetLastError();
}

hipError_t launch_xent(int T, int V, void* logits, const int* targets, int n_microbatches, float loss_scale,
                       float* token_loss, float* loss, hipStream_t st) {
  const float scale = 1.0f / ((float)T * (float)n_microbatches);
  // the gradient carries the loss scale (Sec. 2, mixed precision), the reported loss does not
  hipLaunchKernelGGL(xent_kernel, dim3((unsigned)T), dim3(ENDS_THREADS), 0, st, T, V, (elem_t*)logits, targets,
                     scale * loss_scale, token_loss);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(ENDS_THREADS), 0, st, T, (const float*)token_loss, scale, loss);
  return hipGetLastError();
}

}  // namespace axonn
