// Host-side launch functions of the L4Q kernels (internal; the public surface is include/l4q.h).
// Every launcher enqueues on `stream` and returns; none synchronises.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace l4q {

typedef uint16_t bf16_t;

struct LayerDims {
  int64_t T, i, o;
  int r, bits, g;
  float gamma;   // (float)alpha / (float)r
  float qn, qp;  // Q_N, Q_P as floats
  int64_t G() const { return i / g; }
};

// ---- merge + quantize pass (Eqs. l4q_Wcombine, l4q_Wquant, l4q_Wdequant) ----
// Any of the outputs may be null.  wq has the storage type T and leading dimension i.
template <class T>
void launch_merge_quant(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, T* wq, int8_t* codes, float* wcomb, uint8_t* mask,
                        hipStream_t stream);

// ---- per-group min/max initialisation (App. B, Eq. quant_inits) ----
template <class T>
void launch_init_qparams(const LayerDims& d, const T* W0, const T* A, const T* B, int method, float* scale,
                         float* zero, hipStream_t stream);

// ---- out[c, r] = in[r, c] for 16-bit elements; out has leading dimension ld_out >= rows and
// the columns rows..ld_out-1 of every output row are zero-filled ----
void launch_transpose_u16(const uint16_t* in, int64_t rows, int64_t cols, uint16_t* out, int64_t ld_out,
                          hipStream_t stream);

// ---- bf16 MFMA GEMM  C[M,N] = A[M,K] . B[N,K]^T, fp32 accumulate ----
// A, B row-major with leading dimensions lda, ldb (elements, multiples of 8); K multiple of 8.
void launch_gemm_bf16_nt(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                         int64_t K, bf16_t* C_bf16, float* C_f32, int64_t ldc, hipStream_t stream);

// ---- binary32 GEMM with arbitrary strides: C[m,n] = scale * sum_k A[m*a_rs + k*a_cs] B[k*b_rs + n*b_cs] ----
void launch_sgemm(const float* A, int64_t a_rs, int64_t a_cs, const float* B, int64_t b_rs, int64_t b_cs,
                  float* C, int64_t ldc, int64_t M, int64_t N, int64_t K, float scale, hipStream_t stream);

// ---- unfused quantizer gradients: reads dWq [o,i] (binary32), recomputes w, code, mask; writes
// dscale, dzero [o,G], dB partial-free result dB [o,r], and overwrites dWq with mask * dWq ----
template <class T>
void launch_quant_grads(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, float* dWq_inout, float* dscale, float* dzero, float* dB,
                        hipStream_t stream);

// ---- dA = gamma * B^T . dWp  (reduction over the o rows), two deterministic passes ----
// partial: [ceil(o / kDaRowBlock), r, i] floats
constexpr int kDaRowBlock = 128;
template <class T>
void launch_dA(const LayerDims& d, const T* B, const float* dWp, float* partial, float* dA, hipStream_t stream);

}  // namespace l4q
