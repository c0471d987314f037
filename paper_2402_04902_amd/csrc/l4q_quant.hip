// Merge + quantize pass, integer-code export, min/max initialisation, 16-bit transpose.
//
// merge_quant_kernel is the HBM-streaming prologue of both passes: it reads W0 once with
// coalesced 8/16-byte loads, adds the rank-r update from registers/L2, applies the group-wise
// quantizer and writes whichever outputs were asked for (dequantized Wq, int8 codes, the
// binary32 merged weight, the straight-through mask).
#include "l4q_device.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

constexpr int kThreads = 256;
constexpr int kColsPerThread = 4;
constexpr int kColsPerBlock = kThreads * kColsPerThread;  // 1024
constexpr int kRowsPerBlock = 16;

template <class T>
__global__ __launch_bounds__(kThreads) void merge_quant_kernel(LayerDims d, const T* __restrict__ W0,
                                                                const T* __restrict__ A, const T* __restrict__ B,
                                                                const float* __restrict__ scale,
                                                                const float* __restrict__ zero, T* __restrict__ wq,
                                                                int8_t* __restrict__ codes, float* __restrict__ wcomb,
                                                                uint8_t* __restrict__ mask) {
  const int64_t j0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * kColsPerThread;
  if (j0 >= d.i) return;
  const int64_t p0 = (int64_t)blockIdx.y * kRowsPerBlock;
  const int64_t p1 = p0 + kRowsPerBlock < d.o ? p0 + kRowsPerBlock : d.o;
  const int64_t G = d.i / d.g;
  const int64_t q = j0 / d.g;  // 4 consecutive columns lie in one group because g % 4 == 0
  for (int64_t p = p0; p < p1; ++p) {
    float wc[4];
    merged_weight4<T>(W0 + p * d.i, A, B + p * d.r, d.i, d.r, j0, d.gamma, wc);
    const float s = scale[p * G + q];
    const float b = zero[p * G + q];
    float wqv[4];
    uint32_t cpack = 0, mpack = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const QuantOut qo = quantize_elem(wc[c], s, b, d.qn, d.qp);
      wqv[c] = dequant_elem(qo.code, s, b);
      cpack |= ((uint32_t)(uint8_t)(int8_t)(int)qo.code) << (8 * c);
      mpack |= (qo.in_range ? 1u : 0u) << (8 * c);
    }
    const int64_t off = p * d.i + j0;
    if (wq) store4(wq + off, wqv);
    if (codes) *reinterpret_cast<uint32_t*>(codes + off) = cpack;
    if (mask) *reinterpret_cast<uint32_t*>(mask + off) = mpack;
    if (wcomb) store4(wcomb + off, wc);
  }
}

// One wave per weight row; each lane owns 4 consecutive columns per 256-column step.
template <class T>
__global__ __launch_bounds__(kThreads) void init_qparams_kernel(LayerDims d, const T* __restrict__ W0,
                                                                 const T* __restrict__ A, const T* __restrict__ B,
                                                                 int method, float* __restrict__ scale,
                                                                 float* __restrict__ zero) {
  const int lane = threadIdx.x & 63;
  const int64_t p = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (p >= d.o) return;
  const int64_t G = d.i / d.g;
  const int lanes_per_group = d.g / 4;               // power of two
  const int width = lanes_per_group < 64 ? lanes_per_group : 64;
  const int steps_per_group = lanes_per_group <= 64 ? 1 : lanes_per_group / 64;
  const float inf = __builtin_huge_valf();
  float lo = inf, hi = -inf;
  int step_in_group = 0;
  for (int64_t base = 0; base < d.i; base += 256) {
    const int64_t j0 = base + lane * 4;
    if (j0 < d.i) {
      float wc[4];
      merged_weight4<T>(W0 + p * d.i, A, B + p * d.r, d.i, d.r, j0, d.gamma, wc);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        lo = fminf(lo, wc[c]);
        hi = fmaxf(hi, wc[c]);
      }
    }
    if (++step_in_group < steps_per_group) continue;
    step_in_group = 0;
    for (int off = width >> 1; off > 0; off >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, off, 64));
      hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    }
    if (j0 < d.i && (lane & (width - 1)) == 0) {
      float s, b = 0.f;
      if (method == 0) {  // asymmetric min/max
        s = __fdiv_rn(hi - lo, d.qp - d.qn);
        b = lo - s * d.qn;
      } else if (method == 1) {  // symmetric
        s = __fdiv_rn(fmaxf(fabsf(lo), fabsf(hi)), -d.qn);
      } else {  // L4Q_init (Eq. l4q_quant_init)
        s = fmaxf(fabsf(__fdiv_rn(lo, d.qn)), fabsf(__fdiv_rn(hi, d.qp)));
      }
      const int64_t q = j0 / d.g;
      scale[p * G + q] = s;
      zero[p * G + q] = b;
    }
    lo = inf;
    hi = -inf;
  }
}

// 64 x 64 tile through LDS; 16-byte global accesses on both sides.
__global__ __launch_bounds__(256) void transpose_u16_kernel(const uint16_t* __restrict__ in, int64_t rows,
                                                             int64_t cols, uint16_t* __restrict__ out,
                                                             int64_t ld_out) {
  __shared__ uint32_t tile[64][33];  // 64 rows of 64 halves; 33-dword stride keeps column reads conflict-free
  const int64_t r0 = (int64_t)blockIdx.y * 64;
  const int64_t c0 = (int64_t)blockIdx.x * 64;
  const int tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = tid + it * 256;
    const int rr = idx >> 3, ch = idx & 7;
    const int64_t r = r0 + rr, c = c0 + ch * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < rows && c < cols) v = *reinterpret_cast<const uint4*>(in + r * cols + c);
    tile[rr][ch * 4 + 0] = v.x;
    tile[rr][ch * 4 + 1] = v.y;
    tile[rr][ch * 4 + 2] = v.z;
    tile[rr][ch * 4 + 3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = tid + it * 256;
    const int cc = idx >> 3, ch = idx & 7;  // output row cc, 8 consecutive input rows ch*8..
    const int64_t c = c0 + cc, r = r0 + ch * 8;
    if (c < cols && r < ld_out) {
      uint32_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = (tile[ch * 8 + e][cc >> 1] >> (16 * (cc & 1))) & 0xFFFFu;
      uint4 v;
      v.x = h[0] | (h[1] << 16);
      v.y = h[2] | (h[3] << 16);
      v.z = h[4] | (h[5] << 16);
      v.w = h[6] | (h[7] << 16);
      *reinterpret_cast<uint4*>(out + c * ld_out + r) = v;
    }
  }
}

}  // namespace

template <class T>
void launch_merge_quant(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, T* wq, int8_t* codes, float* wcomb, uint8_t* mask,
                        hipStream_t stream) {
  dim3 grid((unsigned)((d.i + kColsPerBlock - 1) / kColsPerBlock), (unsigned)((d.o + kRowsPerBlock - 1) / kRowsPerBlock));
  hipLaunchKernelGGL(merge_quant_kernel<T>, grid, dim3(kThreads), 0, stream, d, W0, A, B, scale, zero, wq, codes,
                     wcomb, mask);
}

template <class T>
void launch_init_qparams(const LayerDims& d, const T* W0, const T* A, const T* B, int method, float* scale,
                         float* zero, hipStream_t stream) {
  const int rows_per_block = kThreads / 64;
  dim3 grid((unsigned)((d.o + rows_per_block - 1) / rows_per_block));
  hipLaunchKernelGGL(init_qparams_kernel<T>, grid, dim3(kThreads), 0, stream, d, W0, A, B, method, scale, zero);
}

void launch_transpose_u16(const uint16_t* in, int64_t rows, int64_t cols, uint16_t* out, int64_t ld_out,
                          hipStream_t stream) {
  dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((ld_out + 63) / 64));
  hipLaunchKernelGGL(transpose_u16_kernel, grid, dim3(256), 0, stream, in, rows, cols, out, ld_out);
}

template void launch_merge_quant<float>(const LayerDims&, const float*, const float*, const float*, const float*,
                                        const float*, float*, int8_t*, float*, uint8_t*, hipStream_t);
template void launch_merge_quant<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*,
                                         const float*, const float*, bf16_t*, int8_t*, float*, uint8_t*,
                                         hipStream_t);
template void launch_init_qparams<float>(const LayerDims&, const float*, const float*, const float*, int, float*,
                                         float*, hipStream_t);
template void launch_init_qparams<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*, int,
                                          float*, float*, hipStream_t);

}  // namespace l4q
