// Device-side helpers shared by the L4Q kernels: storage-type loads, the binary32 quantizer
// chain (Sec. 2.2 Eq. quant; Sec. 3.2 Eqs. l4q_Wcombine / l4q_Wquant / l4q_Wdequant;
// App. A.1 Eq. appen_ste), and small wave-level reductions.
//
// The whole library is compiled with -ffp-contract=off: a written `a * b + c` is two rounded
// operations; a fused multiply-add happens only where fmaf() is spelled out.  Codes and masks
// therefore come out the same in every kernel that recomputes them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace l4q {

typedef uint16_t bf16_t;  // raw bfloat16 storage: the upper half of a binary32

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  // round to nearest even; gfx950 has a native convert for this
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- loads of 4 consecutive elements as floats (pointer must be 4-element aligned) ----
__device__ __forceinline__ void load4(const float* __restrict__ p, float (&v)[4]) {
  float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const bf16_t* __restrict__ p, float (&v)[4]) {
  uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
}
__device__ __forceinline__ float load1(const float* __restrict__ p) { return *p; }
__device__ __forceinline__ float load1(const bf16_t* __restrict__ p) { return bf16_to_f32(*p); }

__device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
  uint2 t;
  t.x = pack_bf16x2(v[0], v[1]);
  t.y = pack_bf16x2(v[2], v[3]);
  *reinterpret_cast<uint2*>(p) = t;
}

// ---- the low-rank accumulation step: acc + B[p,k] * A[k,j] ----
// binary32 inputs: product and sum are rounded separately (the stated operation order).
// bfloat16 inputs: the product of two 8-bit significands is exact in binary32, so the fused
// form rounds once to the same value and costs one instruction.
template <class T> __device__ __forceinline__ float lora_mac(float acc, float b, float a);
template <> __device__ __forceinline__ float lora_mac<float>(float acc, float b, float a) { return acc + b * a; }
template <> __device__ __forceinline__ float lora_mac<bf16_t>(float acc, float b, float a) { return fmaf(b, a, acc); }

// Merged weight of 4 consecutive columns j0..j0+3 of row p:  Wc = W0 + gamma * sum_k B[p,k] A[k,j]
// (Eq. l4q_Wcombine), k ascending.
template <class T>
__device__ __forceinline__ void merged_weight4(const T* __restrict__ W0row, const T* __restrict__ A,
                                               const T* __restrict__ Brow, int64_t i, int r, int64_t j0,
                                               float gamma, float (&wc)[4]) {
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < r; ++k) {
    const float bk = load1(Brow + k);
    float a[4];
    load4(A + (int64_t)k * i + j0, a);
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = lora_mac<T>(acc[c], bk, a[c]);
  }
  float w0[4];
  load4(W0row + j0, w0);
#pragma unroll
  for (int c = 0; c < 4; ++c) wc[c] = w0[c] + gamma * acc[c];
}

struct QuantOut {
  float w;     // pre-round value (Wc - b) / s
  float code;  // round(clamp(w)), integer valued
  bool in_range;
};

// Eq. quant / l4q_Wquant and the straight-through condition of Eq. appen_ste.
__device__ __forceinline__ QuantOut quantize_elem(float wc, float s, float b, float qn, float qp) {
  QuantOut q;
  q.w = __fdiv_rn(wc - b, s);
  q.code = rintf(fminf(fmaxf(q.w, qn), qp));
  q.in_range = (q.w >= qn) && (q.w <= qp);
  return q;
}

// Eq. l4q_Wdequant
__device__ __forceinline__ float dequant_elem(float code, float s, float b) { return fmaf(code, s, b); }

// ---- wave-level sums (64-wide wavefront) ----
__device__ __forceinline__ float wave_sum_width(float v, int width) {
  // sum over aligned segments of `width` lanes (power of two, <= 64); every lane gets its segment's sum
  for (int off = width >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

}  // namespace l4q
