// Straightforward kernels: a strided binary32 GEMM, the unfused quantizer-gradient pass and the
// two-pass dA reduction.  They serve the binary32 mode end to end and the unfused backward of
// the bfloat16 mode; they make no assumption on shapes beyond the library's divisibility rules.
#include "l4q_device.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

// ------------------------------------------------------------------ strided SGEMM
// 64 x 64 output tile, 16-deep k step, 256 threads, 4 x 4 outputs per thread.
constexpr int SG_BM = 64, SG_BN = 64, SG_BK = 16;

__global__ __launch_bounds__(256) void sgemm_kernel(const float* __restrict__ A, int64_t a_rs, int64_t a_cs,
                                                     const float* __restrict__ B, int64_t b_rs, int64_t b_cs,
                                                     float* __restrict__ C, int64_t ldc, int64_t M, int64_t N,
                                                     int64_t K, float scale) {
  __shared__ float As[SG_BK][SG_BM + 4];
  __shared__ float Bs[SG_BK][SG_BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * SG_BM, n0 = (int64_t)blockIdx.x * SG_BN;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += SG_BK) {
    // 64 x 16 elements per operand, 4 per thread.  The faster-varying thread index follows the
    // operand's unit-stride axis where there is one.
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = tid + e * 256;
      int mm, kk;
      if (a_cs == 1) { kk = idx & 15; mm = idx >> 4; } else { mm = idx & 63; kk = idx >> 6; }
      const int64_t m = m0 + mm, k = k0 + kk;
      As[kk][mm] = (m < M && k < K) ? A[m * a_rs + k * a_cs] : 0.f;
      int nn, kb;
      if (b_rs == 1) { kb = idx & 15; nn = idx >> 4; } else { nn = idx & 63; kb = idx >> 6; }
      const int64_t n = n0 + nn, k2 = k0 + kb;
      Bs[kb][nn] = (n < N && k2 < K) ? B[k2 * b_rs + n * b_cs] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SG_BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t m = m0 + ty * 4 + u;
    if (m >= M) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int64_t n = n0 + tx * 4 + v;
      if (n < N) C[m * ldc + n] = scale * acc[u][v];
    }
  }
}

// ------------------------------------------------------------------ quantizer gradients, unfused
// One wave per weight row p; a lane owns 4 consecutive columns per 256-column step.
//   dscale[p,q] = sum_j dWq * (m ? code - w : code)   (Eq. quant_lsq_s and App. A.1 case list)
//   dzero [p,q] = sum_j dWq * (m ? 0 : 1)             (Eq. appen_lsq_b)
//   dWq <- m * dWq                                    (Eq. appen_ste)
//   dB[p,k]     = gamma * sum_j (m * dWq)[p,j] A[k,j] (Eq. appen_l4q_b)
constexpr int QG_KCHUNK = 16;

template <class T>
__global__ __launch_bounds__(256) void quant_grads_kernel(LayerDims d, const T* __restrict__ W0,
                                                           const T* __restrict__ A, const T* __restrict__ B,
                                                           const float* __restrict__ scale,
                                                           const float* __restrict__ zero, float* __restrict__ dW,
                                                           float* __restrict__ dscale, float* __restrict__ dzero,
                                                           float* __restrict__ dB) {
  const int lane = threadIdx.x & 63;
  const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (p >= d.o) return;
  const int64_t G = d.i / d.g;
  const int lanes_per_group = d.g / 4;
  const int width = lanes_per_group < 64 ? lanes_per_group : 64;
  const int steps_per_group = lanes_per_group <= 64 ? 1 : lanes_per_group / 64;

  // pass 0 does everything for LoRA ranks 0..15; further passes only add dB for ranks 16.., re-reading
  // the already masked dW.
  for (int k0 = 0; k0 < d.r; k0 += QG_KCHUNK) {
    const int kn = d.r - k0 < QG_KCHUNK ? d.r - k0 : QG_KCHUNK;
    float dBacc[QG_KCHUNK];
#pragma unroll
    for (int k = 0; k < QG_KCHUNK; ++k) dBacc[k] = 0.f;
    float ds = 0.f, db = 0.f;
    int step_in_group = 0;
    for (int64_t base = 0; base < d.i; base += 256) {
      const int64_t j0 = base + lane * 4;
      const bool active = j0 < d.i;
      float g4[4] = {0.f, 0.f, 0.f, 0.f};
      if (active) {
        load4(dW + p * d.i + j0, g4);
        if (k0 == 0) {
          const int64_t q = j0 / d.g;
          const float s = scale[p * G + q], b = zero[p * G + q];
          float wc[4];
          merged_weight4<T>(W0 + p * d.i, A, B + p * d.r, d.i, d.r, j0, d.gamma, wc);
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const QuantOut qo = quantize_elem(wc[c], s, b, d.qn, d.qp);
            const float dwq_ds = qo.in_range ? qo.code - qo.w : qo.code;
            ds = fmaf(g4[c], dwq_ds, ds);
            db += qo.in_range ? 0.f : g4[c];
            g4[c] = qo.in_range ? g4[c] : 0.f;
          }
          store4(dW + p * d.i + j0, g4);
        }
#pragma unroll
        for (int k = 0; k < QG_KCHUNK; ++k) {
          if (k < kn) {
            float a[4];
            load4(A + (int64_t)(k0 + k) * d.i + j0, a);
#pragma unroll
            for (int c = 0; c < 4; ++c) dBacc[k] = fmaf(g4[c], a[c], dBacc[k]);
          }
        }
      }
      if (k0 == 0 && ++step_in_group == steps_per_group) {
        step_in_group = 0;
        const float ds_sum = wave_sum_width(ds, width);
        const float db_sum = wave_sum_width(db, width);
        if (active && (lane & (width - 1)) == 0) {
          const int64_t q = j0 / d.g;
          dscale[p * G + q] = d.accumulate ? dscale[p * G + q] + ds_sum : ds_sum;
          dzero[p * G + q] = d.accumulate ? dzero[p * G + q] + db_sum : db_sum;
        }
        ds = 0.f;
        db = 0.f;
      }
    }
#pragma unroll
    for (int k = 0; k < QG_KCHUNK; ++k) {
      const float tot = wave_sum_width(dBacc[k], 64);
      if (lane == 0 && k < kn) {
        const float v = d.gamma * tot;
        dB[p * d.r + k0 + k] = d.accumulate ? dB[p * d.r + k0 + k] + v : v;
      }
    }
  }
}

// ------------------------------------------------------------------ dA = gamma * B^T dWp
// pass 1: a thread owns one column j and sums B[p,k] * dWp[p,j] over a block of rows
template <class T>
__global__ __launch_bounds__(256) void dA_partial_kernel(LayerDims d, const T* __restrict__ B,
                                                          const float* __restrict__ dWp,
                                                          float* __restrict__ partial) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t p0 = (int64_t)blockIdx.y * kDaRowBlock;
  const int64_t p1 = p0 + kDaRowBlock < d.o ? p0 + kDaRowBlock : d.o;
  if (j >= d.i) return;
  for (int k0 = 0; k0 < d.r; k0 += QG_KCHUNK) {
    const int kn = d.r - k0 < QG_KCHUNK ? d.r - k0 : QG_KCHUNK;
    float acc[QG_KCHUNK];
#pragma unroll
    for (int k = 0; k < QG_KCHUNK; ++k) acc[k] = 0.f;
    for (int64_t p = p0; p < p1; ++p) {
      const float gv = dWp[p * d.i + j];
#pragma unroll
      for (int k = 0; k < QG_KCHUNK; ++k)
        if (k < kn) acc[k] = fmaf(load1(B + p * d.r + k0 + k), gv, acc[k]);
    }
#pragma unroll
    for (int k = 0; k < QG_KCHUNK; ++k)
      if (k < kn) partial[((int64_t)blockIdx.y * d.r + k0 + k) * d.i + j] = acc[k];
  }
}

}  // namespace

// pass 2 (also used by the fused backward): out[e] = scale * sum_b partial[b * n + e], b ascending
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int64_t nblocks,
                                                               int64_t n, float scale, float* __restrict__ out,
                                                               bool accumulate) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float acc = 0.f;
  for (int64_t b = 0; b < nblocks; ++b) acc += partial[b * n + e];
  out[e] = accumulate ? out[e] + scale * acc : scale * acc;
}

void launch_reduce_partials(const float* partial, int64_t nblocks, int64_t n, float scale, float* out,
                            bool accumulate, hipStream_t stream) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partial,
                     nblocks, n, scale, out, accumulate);
}

// Both reductions of the fused backward in one launch; 4 consecutive elements per thread (n % 4 == 0).
// A block is 64 element quads x 4 slices of the partial index: slice q sums partials [q*per, (q+1)*per) in
// ascending order and the four slice sums are added in ascending q, so the summation order is fixed.
__global__ __launch_bounds__(256) void reduce_two_partials_kernel(const float* __restrict__ pa, int nba, int64_t na,
                                                                   float* __restrict__ outa,
                                                                   const float* __restrict__ pb, int nbb, int64_t nb,
                                                                   float* __restrict__ outb, float scale,
                                                                   int blocks_a, bool accumulate) {
  __shared__ float4 slice_sum[3][64];
  const bool second = (int)blockIdx.x >= blocks_a;
  const float* __restrict__ part = second ? pb : pa;
  float* __restrict__ out = second ? outb : outa;
  const int nblocks = second ? nbb : nba;
  const int64_t n = second ? nb : na;
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int64_t e = ((int64_t)(second ? blockIdx.x - blocks_a : blockIdx.x) * 64 + lane) * 4;
  const int per = (nblocks + 3) / 4;
  const int b0 = q * per, b1 = min(nblocks, b0 + per);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (e < n) {
#pragma unroll 4
    for (int b = b0; b < b1; ++b) {
      const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)b * n + e);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  if (q > 0) slice_sum[q - 1][lane] = acc;
  __syncthreads();
  if (q > 0 || e >= n) return;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const float4 v = slice_sum[k][lane];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  float4 r = make_float4(scale * acc.x, scale * acc.y, scale * acc.z, scale * acc.w);
  if (accumulate) {
    const float4 old = *reinterpret_cast<const float4*>(out + e);
    r = make_float4(old.x + r.x, old.y + r.y, old.z + r.z, old.w + r.w);
  }
  *reinterpret_cast<float4*>(out + e) = r;
}

void launch_reduce_two_partials(const float* pa, int nba, int64_t na, float* outa, const float* pb, int nbb,
                                int64_t nb, float* outb, float scale, bool accumulate, hipStream_t stream) {
  const int blocks_a = (int)((na / 4 + 63) / 64), blocks_b = (int)((nb / 4 + 63) / 64);
  hipLaunchKernelGGL(reduce_two_partials_kernel, dim3((unsigned)(blocks_a + blocks_b)), dim3(256), 0, stream, pa, nba,
                     na, outa, pb, nbb, nb, outb, scale, blocks_a, accumulate);
}

// ------------------------------------------------------------------ AdamW step on {A, B, scale, zero}
// One launch over the concatenation [A | B | scale | zero]; the moments m, v are stored in that order.
__global__ __launch_bounds__(256) void adamw_kernel(AdamwArgs a) {
  const int64_t n = a.n[0] + a.n[1] + a.n[2] + a.n[3];
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) {
    int t = 0;
    int64_t k = e;
    while (k >= a.n[t]) { k -= a.n[t]; ++t; }
    const float g = a.grad[t][k];
    float p = a.param[t][k];
    const float m = a.beta1 * a.m[e] + (1.f - a.beta1) * g;
    const float v = a.beta2 * a.v[e] + (1.f - a.beta2) * g * g;
    a.m[e] = m;
    a.v[e] = v;
    const float mhat = m / a.bias1, vhat = v / a.bias2;
    p = p - a.lr * a.weight_decay * p - a.lr * mhat / (sqrtf(vhat) + a.eps);
    a.param[t][k] = p;
    if (t < 2 && a.copy_bf16[t]) a.copy_bf16[t][k] = f32_to_bf16(p);
  }
}

void launch_adamw(const AdamwArgs& a, hipStream_t stream) {
  const int64_t n = a.n[0] + a.n[1] + a.n[2] + a.n[3];
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
}

void launch_sgemm(const float* A, int64_t a_rs, int64_t a_cs, const float* B, int64_t b_rs, int64_t b_cs,
                  float* C, int64_t ldc, int64_t M, int64_t N, int64_t K, float scale, hipStream_t stream) {
  dim3 grid((unsigned)((N + SG_BN - 1) / SG_BN), (unsigned)((M + SG_BM - 1) / SG_BM));
  hipLaunchKernelGGL(sgemm_kernel, grid, dim3(256), 0, stream, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, M, N, K, scale);
}

template <class T>
void launch_quant_grads(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, float* dWq_inout, float* dscale, float* dzero, float* dB,
                        hipStream_t stream) {
  dim3 grid((unsigned)((d.o + 3) / 4));
  hipLaunchKernelGGL(quant_grads_kernel<T>, grid, dim3(256), 0, stream, d, W0, A, B, scale, zero, dWq_inout, dscale,
                     dzero, dB);
}

template <class T>
void launch_dA(const LayerDims& d, const T* B, const float* dWp, float* partial, float* dA, hipStream_t stream) {
  const int64_t nrb = (d.o + kDaRowBlock - 1) / kDaRowBlock;
  dim3 grid((unsigned)((d.i + 255) / 256), (unsigned)nrb);
  hipLaunchKernelGGL(dA_partial_kernel<T>, grid, dim3(256), 0, stream, d, B, dWp, partial);
  const int64_t n = (int64_t)d.r * d.i;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partial, nrb, n,
                     d.gamma, dA, d.accumulate);
}

template void launch_quant_grads<float>(const LayerDims&, const float*, const float*, const float*, const float*,
                                        const float*, float*, float*, float*, float*, hipStream_t);
template void launch_quant_grads<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*,
                                         const float*, const float*, float*, float*, float*, float*, hipStream_t);
template void launch_dA<float>(const LayerDims&, const float*, const float*, float*, float*, hipStream_t);
template void launch_dA<bf16_t>(const LayerDims&, const bf16_t*, const float*, float*, float*, hipStream_t);

}  // namespace l4q
