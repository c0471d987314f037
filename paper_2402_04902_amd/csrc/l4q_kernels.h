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
  bool accumulate = false;  // backward: add dA, dB, dscale, dzero to what the outputs hold instead of overwriting
  int64_t G() const { return i / g; }
};

// ---- merge + quantize pass (Eqs. l4q_Wcombine, l4q_Wquant, l4q_Wdequant) ----
// Every output is optional (null = not written).
template <class T>
struct MergeQuantOut {
  // bfloat16 storage: Wq and Wq^T are written for the matrix-core GEMM's B operand, in blocks of 32 k-values:
  //   wq  [ld_wq / 32][o][32]:  Wq[p, j]  at ((j / 32) o + p) 32 + j % 32;  columns i..ld_wq-1 zeros
  //   wqT [ld_wqT / 32][i][32]: Wq[p, j]  at ((p / 32) i + j) 32 + p % 32;  rows o..ld_wqT-1 zeros
  // binary32 storage: wq [o, ld_wq] row-major.
  T* wq = nullptr;
  int64_t ld_wq = 0;         // multiple of 32 (bfloat16)
  bf16_t* wqT = nullptr;
  int64_t ld_wqT = 0;        // multiple of 32
  bf16_t* bT = nullptr;      // B^T [r, ld_wqT] bf16 for the fused backward; columns o..ld_wqT-1 zeros (bf16 mode only)
  uint16_t* fgrad = nullptr; // [o,i] binary16: d(Wq)/d(scale) = code - w in range, code (= Q_N or Q_P) when clipped;
                             // |value| <= 1/2 exactly when the element is in range
  int8_t* codes = nullptr;   // [o,i]
  float* wcomb = nullptr;    // [o,i] binary32 merged weight
  uint8_t* mask = nullptr;   // [o,i] 1 where Q_N <= w <= Q_P
};
template <class T>
void launch_merge_quant(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, const MergeQuantOut<T>& out, hipStream_t stream);


// Streaming form of the pass for bfloat16 storage (l4q_merge_stream.hip): the forward output set (wq alone) or the
// fused-backward set (wqT + fgrad [+ bT]), rank a multiple of 8, group size >= 32.  launch_merge_quant uses it where
// it applies.
bool merge_quant_stream_supported(const LayerDims& d, const MergeQuantOut<bf16_t>& out);
void launch_merge_quant_stream(const LayerDims& d, const bf16_t* W0, const bf16_t* A, const bf16_t* B,
                               const float* scale, const float* zero, const MergeQuantOut<bf16_t>& out,
                               hipStream_t stream);
// Check of the streaming form's reciprocal-based quotient against the IEEE divide for `count` significands of the
// scale starting at `first`; counts (device, zeroed by the caller): wrong reciprocals, wrong quotients, quotients compared.
void launch_check_fast_divide(uint32_t first, uint32_t count, unsigned long long* counts, hipStream_t stream);

// ---- per-group min/max initialisation (App. B, Eq. quant_inits) ----
template <class T>
void launch_init_qparams(const LayerDims& d, const T* W0, const T* A, const T* B, int method, float* scale,
                         float* zero, hipStream_t stream);

// ---- quantization / clipping error sums (App. B, Table 5): out2[0] = sum |Wc - Wq|, out2[1] = sum |Wc - (clamp(w) s + b)| ----
// partial: [o * ceil(i / 256) * 2] floats of scratch
template <class T>
void launch_quant_errors(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                         const float* zero, float* partial, float* out2, hipStream_t stream);

// compute units of the current device (asked once per device, then cached)
int device_compute_units();

// ---- bf16 MFMA GEMM  C[M,N] = A[M,K] . B[N,K]^T, fp32 accumulate, bf16 output ----
// A row-major and K-contiguous with leading dimension lda (elements, a multiple of 8); rows of A end at K_a (a
// multiple of 8, K - 32 < K_a <= K) and are not read past it.  B K-contiguous in blocks of 32 k-values,
// B[k / 32][n][k % 32] with the N rows of a block contiguous (what the merge + quantize pass writes; ldb unused), K
// rounded up to 32 with zeros for k in [K_a, K).  Every operand below 1 GiB, N % 4 == 0, ldc % 4 == 0.
// Few tiles (small M: few tokens): the k range is split into `slices` = gemm_nt_splitk_slices(M, N, K) > 1 runs of
// whole stage pairs, one workgroup per (tile, slice); the slices' binary32 tiles go to `partial`
// [slices][M][N] and a second launch adds them in slice order (the result does not depend on the run) and rounds to
// bf16.  With `partial` == nullptr, or one slice, the product is a single pass.
int gemm_nt_splitk_slices(int64_t M, int64_t N, int64_t K);
void launch_gemm_bf16_nt(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                         int64_t K, int64_t K_a, bf16_t* C, int64_t ldc, hipStream_t stream,
                         float* partial = nullptr);

// ---- matrix-core-only probe: `workgroups` x 4 waves x `iterations` x 16 MFMA 32x32x16 on fragments taken from the
// first 64 KiB of `data`; sink [workgroups * 256] floats.  Returns the FLOPs the launch performs. ----
double launch_mfma_probe(const bf16_t* data, int iterations, int workgroups, float* sink, hipStream_t stream);

// ---- C[M,N] (float) = A[K,M]^T . B[K,N]: both operands K-major (rows = k), any K ----
void launch_gemm_bf16_kmajor_f32(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                                 int64_t K, float* C, int64_t ldc, hipStream_t stream);

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

// out[e] = scale * sum_b partial[b * n + e], b ascending (fixed summation order); accumulate: added to out[e]
void launch_reduce_partials(const float* partial, int64_t nblocks, int64_t n, float scale, float* out,
                            bool accumulate, hipStream_t stream);

// ---- AdamW step (App. C) on the four trainable tensors, in the order A, B, scale, zero ----
struct AdamwArgs {
  float* param[4];        // binary32 master parameters, updated in place
  const float* grad[4];
  int64_t n[4];
  float* m;               // first / second moments, concatenated in the same order
  float* v;
  bf16_t* copy_bf16[2];   // optional bfloat16 copies of the new A and B (null: none)
  float lr, beta1, beta2, eps, weight_decay;
  float bias1, bias2;     // 1 - beta1^t, 1 - beta2^t
};
void launch_adamw(const AdamwArgs& a, hipStream_t stream);

// ---- fully quantized layer: bit-packing of int8 codes [o,i] (i % 32 == 0) and Y = X . dequant(packed)^T ----
void launch_pack_codes(const int8_t* codes, int64_t o, int64_t i, int bits, uint32_t* packed, hipStream_t stream);
bool qgemm_supported(const LayerDims& d);
// partial: optional room for fp32 partial sums (qgemm_workspace_bytes(d); ignored when null or smaller)
size_t qgemm_workspace_bytes(const LayerDims& d);
void launch_qgemm(const LayerDims& d, const bf16_t* X, const uint32_t* packed, const float* scale, const float* zero,
                  bf16_t* Y, float* partial, size_t partial_bytes, hipStream_t stream);

// outa = scale * sum of nba partials of na elements, outb likewise, in one launch (na, nb multiples of 4)
void launch_reduce_two_partials(const float* pa, int nba, int64_t na, float* outa, const float* pb, int nbb,
                                int64_t nb, float* outb, float scale, bool accumulate, hipStream_t stream);

// ---- weight-gradient GEMM with fused quantizer backward (bf16 mode) ----
// dY [T, o], X [T, i] as the caller holds them; fgrad [o, i] binary16 from launch_merge_quant;
// BT [r, ld_bt]: B^T as the backward merge pass leaves it (MergeQuantOut::bT).  Writes dscale, dzero [o, G] and the partial sums
// dA_part [tiles_m, r, i], dB_part [2 * tiles_n, o, r] (no gamma applied yet).
bool dw_fused_supported(const LayerDims& d);
void dw_fused_tiles(const LayerDims& d, int* tiles_m, int* tiles_n);
void launch_dw_fused(const LayerDims& d, const bf16_t* dY, const bf16_t* X, const uint16_t* fgrad, const bf16_t* A,
                     const bf16_t* BT, int64_t ld_bt, float* dscale, float* dzero, float* dA_part, float* dB_part,
                     hipStream_t stream);


// Second form for ranks 33 .. 256 (see l4q_bwd_fused.hip): dscale, dzero as above, and the masked gradient m * dWq
// written as bfloat16 dWm [o, i]; then launch_dw_masked_products forms
//   rawA [slices_a][r, i] = B^T . dWm  and  rawB [slices_b][o, r] = dWm . A^T   (binary32, no gamma yet)
// with the library's GEMM kernels, each product split along k into dw_masked_product_slices() partial results that
// the caller adds in slice order.
bool dw_masked_supported(const LayerDims& d);
void launch_dw_masked(const LayerDims& d, const bf16_t* dY, const bf16_t* X, const uint16_t* fgrad, float* dscale,
                      float* dzero, bf16_t* dWm, hipStream_t stream);
void dw_masked_product_slices(const LayerDims& d, int* slices_a, int* slices_b);
void launch_dw_masked_products(const LayerDims& d, const bf16_t* dWm, const bf16_t* A, const bf16_t* B, float* rawA,
                               float* rawB, hipStream_t stream);

// ---- rank-r side products of the QAT-LoRA layer (Sec. 3.1): U binary32 [T, r]; the small matrix M is read as
// [r, n] (A) or, with m_is_n_by_r, as [n, r] (B) ----
template <class S>
void launch_lora_down(const S* Xs, int64_t T, int64_t n, const S* M, int r, bool m_is_n_by_r, float* U,
                      hipStream_t stream);                    // U = Xs . M^T  (sum over n)
template <class S>
void launch_lora_up(S* Out, int64_t T, int64_t n, const float* U, const S* M, int r, bool m_is_n_by_r, float gamma,
                    hipStream_t stream);                      // Out += gamma U . M
int64_t lora_tn_blocks(int64_t T);                            // token blocks of the partial sums below
// out = gamma * sum_t U[t,:]^T Xs[t,:] as [r, n], or as [n, r] with out_n_by_r; partial: lora_tn_blocks(T) * r * n floats
template <class S>
void launch_lora_tn(const float* U, const S* Xs, int64_t T, int64_t n, int r, bool out_n_by_r, float* partial,
                    float gamma, float* out, bool accumulate, hipStream_t stream);

}  // namespace l4q
