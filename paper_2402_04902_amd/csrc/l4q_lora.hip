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

// A wave (one per workgroup) takes LR_RB token rows, so that what it reads of the small matrix is used LR_RB times:
// U[t, k0 .. k0 + 15] = sum_j Xs[t, j] M(k, j).  Rank-major M (A, n % 4 == 0): a lane walks 4 consecutive columns
// with vector loads.  M as [n, r] (B): a lane walks single columns and reads that column's ranks contiguously.
constexpr int LR_RB = 4;

template <class S, bool NR>
__global__ __launch_bounds__(64) void lora_down_kernel(const S* __restrict__ Xs, int64_t T, int64_t n,
                                                         const S* __restrict__ M, int r, float* __restrict__ U) {
  const int lane = threadIdx.x & 63;
  const int64_t t0 = (int64_t)blockIdx.x * LR_RB;  // one wave per block
  if (t0 >= T) return;
  const S* xrow[LR_RB];
#pragma unroll
  for (int q = 0; q < LR_RB; ++q) xrow[q] = Xs + (t0 + q < T ? t0 + q : T - 1) * n;
  for (int k0 = 0; k0 < r; k0 += LR_KC) {
    float acc[LR_RB][LR_KC];
#pragma unroll
    for (int q = 0; q < LR_RB; ++q)
#pragma unroll
      for (int k = 0; k < LR_KC; ++k) acc[q][k] = 0.f;
    if (!NR) {
      for (int64_t j = (int64_t)lane * 4; j < n; j += 256) {
        float x[LR_RB][4];
#pragma unroll
        for (int q = 0; q < LR_RB; ++q) load4(xrow[q] + j, x[q]);
#pragma unroll
        for (int k = 0; k < LR_KC; ++k) {
          float a[4];
          load4(M + (int64_t)(k0 + k < r ? k0 + k : r - 1) * n + j, a);
          if (k0 + k >= r) a[0] = a[1] = a[2] = a[3] = 0.f;
#pragma unroll
          for (int q = 0; q < LR_RB; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[q][k] = fmaf(x[q][c], a[c], acc[q][k]);
        }
      }
    } else {
      for (int64_t j = lane; j < n; j += 64) {
        float m[LR_KC];
#pragma unroll
        for (int k = 0; k < LR_KC; ++k) m[k] = k0 + k < r ? load1(M + j * r + k0 + k) : 0.f;
#pragma unroll
        for (int q = 0; q < LR_RB; ++q) {
          const float x = load1(xrow[q] + j);
#pragma unroll
          for (int k = 0; k < LR_KC; ++k) acc[q][k] = fmaf(x, m[k], acc[q][k]);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < LR_RB; ++q)
#pragma unroll
      for (int k = 0; k < LR_KC; ++k) {
        const float v = wave_sum_width(acc[q][k], 64);
        if (lane == 0 && k0 + k < r && t0 + q < T) U[(t0 + q) * r + k0 + k] = v;
      }
  }
}

template <class S> __device__ __forceinline__ float to_f32(S v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// Out[t, j] += gamma * sum_k U[t, k] M(k, j).  A thread owns one column and LR_UT consecutive tokens: its column
// of the small matrix is read once per rank chunk and stays in registers; U[t, :] is uniform over the block.
constexpr int LR_UT = 16;

template <class S, bool NR>
__global__ __launch_bounds__(256) void lora_up_kernel(S* __restrict__ Out, int64_t T, int64_t n,
                                                       const float* __restrict__ U, const S* __restrict__ M, int r,
                                                       float gamma) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t t0 = (int64_t)blockIdx.y * LR_UT;
  if (j >= n) return;
  float acc[LR_UT];
#pragma unroll
  for (int q = 0; q < LR_UT; ++q) acc[q] = 0.f;
  for (int k0 = 0; k0 < r; k0 += LR_KC) {
    float m[LR_KC];
#pragma unroll
    for (int k = 0; k < LR_KC; ++k) m[k] = k0 + k < r ? small_at<S, NR>(M, n, r, k0 + k, j) : 0.f;
#pragma unroll
    for (int q = 0; q < LR_UT; ++q) {
      const float* u = U + (t0 + q < T ? t0 + q : T - 1) * r + k0;  // uniform over the block
#pragma unroll
      for (int k = 0; k < LR_KC; ++k)
        if (k0 + k < r) acc[q] = fmaf(u[k], m[k], acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < LR_UT; ++q)
    if (t0 + q < T) {
      S* dst = Out + (t0 + q) * n + j;
      store1(dst, to_f32<S>(*dst) + gamma * acc[q]);
    }
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
  dim3 grid((unsigned)((T + LR_RB - 1) / LR_RB));
  if (m_is_n_by_r) hipLaunchKernelGGL((lora_down_kernel<S, true>), grid, dim3(64), 0, stream, Xs, T, n, M, r, U);
  else hipLaunchKernelGGL((lora_down_kernel<S, false>), grid, dim3(64), 0, stream, Xs, T, n, M, r, U);
}

template <class S>
void launch_lora_up(S* Out, int64_t T, int64_t n, const float* U, const S* M, int r, bool m_is_n_by_r, float gamma,
                    hipStream_t stream) {
  dim3 grid((unsigned)((n + 255) / 256), (unsigned)((T + LR_UT - 1) / LR_UT));
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
