// Rank-r side products of the QAT-LoRA layer (Sec. 3.1; Eq. lora_forward / lora_backward): the LoRA path kept
// next to the quantized weight instead of being merged into it.
//
//   down   U[T,r]   = Xs[T,n] . M            M = A^T (U = X A^T)  or  M = B (U = dY B)
//   up     Out[T,n] = Out + gamma U[T,r] . M  M = B^T (Y += gamma (X A^T) B^T)  or  M = A (dX += gamma (dY B) A)
//   tn     G[r,n]   = sum_t U[t,:]^T Xs[t,:]  per block of 128 tokens, summed in fixed order by reduce_partials_kernel
//                                             (dA = gamma (dY B)^T X,  dB^T = gamma (X A^T)^T dY)
// All three stream their large operand once per chunk of 16 ranks and are bound by HBM; U is binary32 and
// accumulation is binary32.  The small matrix is read either as [r, n] (rank-major, A) or as [n, r] (B).
#include "l4q_device.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

constexpr int LR_KC = 16;  // ranks per pass

// element (k, j) of the small matrix: rank-major [r, n] or [n, r]
template <class S, bool NR>
__device__ __forceinline__ float small_at(const S* __restrict__ M, int64_t n, int r, int k, int64_t j) {
  return load1(NR ? M + j * r + k : M + (int64_t)k * n + j);
}

// one wave per token row: U[t, k0 .. k0 + 15] = sum_j Xs[t, j] M(k, j)
template <class S, bool NR>
__global__ __launch_bounds__(256) void lora_down_kernel(const S* __restrict__ Xs, int64_t T, int64_t n,
                                                         const S* __restrict__ M, int r, float* __restrict__ U) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const S* xrow = Xs + t * n;
  for (int k0 = 0; k0 < r; k0 += LR_KC) {
    float acc[LR_KC];
#pragma unroll
    for (int k = 0; k < LR_KC; ++k) acc[k] = 0.f;
    for (int64_t j = lane; j < n; j += 64) {
      const float x = load1(xrow + j);
#pragma unroll
      for (int k = 0; k < LR_KC; ++k)
        if (k0 + k < r) acc[k] = fmaf(x, small_at<S, NR>(M, n, r, k0 + k, j), acc[k]);
    }
#pragma unroll
    for (int k = 0; k < LR_KC; ++k) {
      const float v = wave_sum_width(acc[k], 64);
      if (lane == 0 && k0 + k < r) U[t * r + k0 + k] = v;
    }
  }
}

template <class S> __device__ __forceinline__ float to_f32(S v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// Out[t, j] += gamma * sum_k U[t, k] M(k, j); one thread per element, rows of 256 columns per block
template <class S, bool NR>
__global__ __launch_bounds__(256) void lora_up_kernel(S* __restrict__ Out, int64_t T, int64_t n,
                                                       const float* __restrict__ U, const S* __restrict__ M, int r,
                                                       float gamma) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t t = blockIdx.y;
  if (j >= n) return;
  const float* u = U + t * r;  // uniform per block
  float acc = 0.f;
  for (int k = 0; k < r; ++k) acc = fmaf(u[k], small_at<S, NR>(M, n, r, k, j), acc);
  S* dst = Out + t * n + j;
  store1(dst, to_f32<S>(*dst) + gamma * acc);
}

// part[tb][k][j] (or [tb][j][k] when NR) = sum over the 128 tokens of block tb of U[t, k] Xs[t, j]
constexpr int LR_TB = 128;
template <class S, bool NR>
__global__ __launch_bounds__(256) void lora_tn_partial_kernel(const float* __restrict__ U, const S* __restrict__ Xs,
                                                               int64_t T, int64_t n, int r,
                                                               float* __restrict__ part) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tb = blockIdx.y;
  const int k0 = blockIdx.z * LR_KC;
  const int64_t t_begin = tb * LR_TB, t_end = t_begin + LR_TB < T ? t_begin + LR_TB : T;
  float acc[LR_KC];
#pragma unroll
  for (int k = 0; k < LR_KC; ++k) acc[k] = 0.f;
  if (j < n) {
    for (int64_t t = t_begin; t < t_end; ++t) {
      const float x = load1(Xs + t * n + j);
      const float* u = U + t * r + k0;  // uniform
#pragma unroll
      for (int k = 0; k < LR_KC; ++k)
        if (k0 + k < r) acc[k] = fmaf(u[k], x, acc[k]);
    }
    float* dst = part + tb * (int64_t)r * n;
#pragma unroll
    for (int k = 0; k < LR_KC; ++k)
      if (k0 + k < r) dst[NR ? j * r + k0 + k : (int64_t)(k0 + k) * n + j] = acc[k];
  }
}

}  // namespace

template <class S>
void launch_lora_down(const S* Xs, int64_t T, int64_t n, const S* M, int r, bool m_is_n_by_r, float* U,
                      hipStream_t stream) {
  dim3 grid((unsigned)((T + 3) / 4));
  if (m_is_n_by_r) hipLaunchKernelGGL((lora_down_kernel<S, true>), grid, dim3(256), 0, stream, Xs, T, n, M, r, U);
  else hipLaunchKernelGGL((lora_down_kernel<S, false>), grid, dim3(256), 0, stream, Xs, T, n, M, r, U);
}

template <class S>
void launch_lora_up(S* Out, int64_t T, int64_t n, const float* U, const S* M, int r, bool m_is_n_by_r, float gamma,
                    hipStream_t stream) {
  dim3 grid((unsigned)((n + 255) / 256), (unsigned)T);
  if (m_is_n_by_r) hipLaunchKernelGGL((lora_up_kernel<S, true>), grid, dim3(256), 0, stream, Out, T, n, U, M, r, gamma);
  else hipLaunchKernelGGL((lora_up_kernel<S, false>), grid, dim3(256), 0, stream, Out, T, n, U, M, r, gamma);
}

int64_t lora_tn_blocks(int64_t T) { return (T + LR_TB - 1) / LR_TB; }

template <class S>
void launch_lora_tn(const float* U, const S* Xs, int64_t T, int64_t n, int r, bool out_n_by_r, float* partial,
                    float gamma, float* out, bool accumulate, hipStream_t stream) {
  const int64_t nb = lora_tn_blocks(T);
  dim3 grid((unsigned)((n + 255) / 256), (unsigned)nb, (unsigned)((r + LR_KC - 1) / LR_KC));
  if (out_n_by_r) hipLaunchKernelGGL((lora_tn_partial_kernel<S, true>), grid, dim3(256), 0, stream, U, Xs, T, n, r, partial);
  else hipLaunchKernelGGL((lora_tn_partial_kernel<S, false>), grid, dim3(256), 0, stream, U, Xs, T, n, r, partial);
  launch_reduce_partials(partial, nb, (int64_t)r * n, gamma, out, accumulate, stream);
}

template void launch_lora_down<float>(const float*, int64_t, int64_t, const float*, int, bool, float*, hipStream_t);
template void launch_lora_down<bf16_t>(const bf16_t*, int64_t, int64_t, const bf16_t*, int, bool, float*, hipStream_t);
template void launch_lora_up<float>(float*, int64_t, int64_t, const float*, const float*, int, bool, float, hipStream_t);
template void launch_lora_up<bf16_t>(bf16_t*, int64_t, int64_t, const float*, const bf16_t*, int, bool, float, hipStream_t);
template void launch_lora_tn<float>(const float*, const float*, int64_t, int64_t, int, bool, float*, float, float*, bool,
                                    hipStream_t);
template void launch_lora_tn<bf16_t>(const float*, const bf16_t*, int64_t, int64_t, int, bool, float*, float, float*, bool,
                                     hipStream_t);

}  // namespace l4q
