/*
 * l4q.h - C ABI of the MI355X (gfx950) implementation of the L4Q quantization-aware
 * LoRA linear layer (arXiv 2402.04902, Sec. 3.2 and App. A).
 *
 * Orientation.  The paper writes Y = Wq X with X in R^{i x s x b}.  This library uses the
 * row-major "tokens first" statement of the same product:
 *
 *     Y[T,o] = X[T,i] . Wq[o,i]^T ,   T = batch * sequence.
 *
 * Symbols (paper's notation): i / o in- and out-features, r LoRA rank, n bit width,
 * g quantization group size (g consecutive elements along i within one weight row),
 * G = i / g groups per row, gamma = alpha / r the merge constant (the paper's "alpha"),
 * Q_N = -2^(n-1), Q_P = 2^(n-1) - 1.
 *
 * Tensors.  All pointers are DEVICE pointers, row-major, contiguous, 16-byte aligned.
 *   X [T,i], dY [T,o], Y [T,o], dX [T,i], W0 [o,i], A [r,i], B [o,r] :
 *       float (dtype = L4Q_DTYPE_F32) or bfloat16 (dtype = L4Q_DTYPE_BF16; upper half of
 *       an IEEE binary32).
 *   scale, zero, dscale, dzero [o,G] : float always.  "zero" is the real-valued additive
 *       bias b of Eq. (quant): w = (W - b) / s, Wq = w~ s + b.  It is not an integer zero point.
 *   dA [r,i], dB [o,r] : float always.
 * Outputs are overwritten; the one exception is L4Q_FLAG_ACCUMULATE_GRADS (below), under which l4q_backward and
 * l4q_qatlora_backward add the four parameter gradients to what their arrays hold.
 *
 * Ownership.  The caller owns every buffer, workspace included.  The library allocates
 * nothing, keeps no pointer after a call returns and has no global state (the opt-in
 * benchmark switch l4q_profile_gemm and the fixed scratch array of l4q_quant_errors_static aside), so calls on
 * different streams may run concurrently as long as their output and workspace buffers are
 * distinct.
 *
 * Streams.  `hip_stream` is a hipStream_t (NULL = the default stream).  All work is
 * enqueued on it; no entry point synchronises with the host.
 *
 * Errors.  Every entry point validates its arguments before it launches anything and
 * returns L4Q_OK (0) or a negative l4q_status.  Nothing is printed and nothing aborts.
 * scale <= 0, NaN or Inf inputs are not detected: results are then undefined (a non-finite value in X or dY
 * stays within the rows of Y / dX that the product's definition gives it).
 *
 * Arithmetic contract for the discrete part (codes and straight-through mask).  All kernels
 * evaluate, in IEEE binary32 with one rounding per written operation and no fused
 * multiply-add,
 *     acc = 0;  for k = 0..r-1: acc = acc + B[p,k] * A[k,j]
 *     Wc  = W0[p,j] + gamma * acc           gamma = (float)alpha / (float)r
 *     w   = (Wc - zero[p,q]) / scale[p,q]   correctly rounded divide (or any sequence proved to give its result)
 *     w~  = rint(min(max(w, Q_N), Q_P))     ties to even
 *     m   = (Q_N <= w) && (w <= Q_P)
 * so codes and masks are reproducible bit for bit on any IEEE machine.
 */
#ifndef L4Q_H
#define L4Q_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define L4Q_VERSION 100

typedef enum l4q_status {
  L4Q_OK = 0,
  L4Q_ERR_NULL = -1,      /* a required pointer is NULL */
  L4Q_ERR_SHAPE = -2,     /* non-positive dimension, i % g != 0, or a divisibility rule below */
  L4Q_ERR_BITS = -3,      /* bits outside 2..8 */
  L4Q_ERR_DTYPE = -4,     /* dtype not F32 / BF16, or flags has unknown bits */
  L4Q_ERR_ALIGN = -5,     /* a pointer is not 16-byte aligned */
  L4Q_ERR_WORKSPACE = -6, /* workspace NULL or smaller than l4q_workspace_bytes reports */
  L4Q_ERR_LAUNCH = -7,    /* a kernel launch failed (hipGetLastError was not hipSuccess) */
  L4Q_ERR_METHOD = -8,    /* unknown initialisation method */
  L4Q_ERR_TOO_LARGE = -9  /* l4q_quant_errors_static: the problem needs more than L4Q_STATIC_SCRATCH_BYTES */
} l4q_status;

enum { L4Q_DTYPE_F32 = 0, L4Q_DTYPE_BF16 = 1 };

/* flags */
enum {
  L4Q_FLAG_NONE = 0,
  /* bf16 only: run the backward pass through the unfused kernels (dWq written to the
   * workspace in binary32, quantizer gradients in a separate pass).  Slower; exists so the
   * fused epilogue can be cross-checked and as the path for group sizes the fused kernel
   * does not cover. */
  L4Q_FLAG_UNFUSED_BACKWARD = 1,
  /* l4q_backward adds dA, dB, dscale and dzero to what the output arrays hold instead of overwriting
   * them (gradient accumulation over micro-batches; App. C trains with an effective batch of 128).
   * dX is always overwritten.  Each call's own contribution is computed as without the flag and
   * added with one binary32 addition per element.  Ignored by the other entry points. */
  L4Q_FLAG_ACCUMULATE_GRADS = 2
};

/* Shape rules: tokens, in_features, out_features, rank >= 1; group_size a power of two >= 4,
 * in_features % group_size == 0; 2 <= bits <= 8; rank <= 256.
 * BF16 additionally: group_size % 8 == 0 and out_features % 8 == 0 (16-byte rows), and each of
 * tokens*in_features, tokens*out_features, out_features*ceil32(in_features), in_features*ceil32(out_features)
 * below 2^29 - 2^20 elements (ceil32: rounded up to a multiple of 32). */
typedef struct l4q_desc {
  int64_t tokens;       /* T */
  int64_t in_features;  /* i */
  int64_t out_features; /* o */
  int32_t rank;         /* r */
  int32_t bits;         /* n */
  int32_t group_size;   /* g */
  float alpha;          /* LoRA alpha; the merge uses gamma = alpha / rank */
  int32_t dtype;        /* L4Q_DTYPE_* */
  int32_t flags;        /* L4Q_FLAG_* */
} l4q_desc;

/* Bytes of device workspace l4q_forward and l4q_backward need for this descriptor (all of its fields count: at
 * few tokens a bfloat16 layer's forward and dX products are split along k over the compute units, and the
 * slices' binary32 tiles live in the workspace).  Either output pointer may be NULL.  The workspace must be
 * 256-byte aligned. */
int l4q_workspace_bytes(const l4q_desc* desc, size_t* forward_bytes, size_t* backward_bytes);

/* Forward pass (Sec. 3.2, Eqs. l4q_Wcombine, l4q_Wquant, l4q_Wdequant, l4q_forward):
 *   Wc = W0 + gamma B A;  w~ = round(clamp((Wc - zero)/scale, Q_N, Q_P));  Wq = w~ scale + zero;
 *   Y = X Wq^T.
 * Nothing is kept for the backward pass: the workspace content is dead when the call's work
 * has finished. */
int l4q_forward(const l4q_desc* desc, const void* X, const void* W0, const void* A, const void* B,
                const float* scale, const float* zero, void* Y,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward pass (Sec. 3.2 "Memory Efficient QAT" / "Efficient LoRA Training"; App. A.1, A.2).
 * Takes only the forward INPUTS plus dY; Wq, w and the mask are recomputed (App. D.2).
 *   dX     = dY Wq
 *   dWq    = dY^T X                                       (Eq. appen_wq; never returned)
 *   dscale = sum over the group of dWq * (m ? w~ - w : w~) (Eq. quant_lsq_s, App. A.1 cases)
 *   dzero  = sum over the group of dWq * (m ? 0 : 1)       (Eq. appen_lsq_b)
 *   dA     = gamma B^T (m * dWq),  dB = gamma (m * dWq) A^T (Eqs. appen_l4q_a, appen_l4q_b)
 * with m the straight-through mask on the pre-round w (Eq. appen_ste). */
int l4q_backward(const l4q_desc* desc, const void* X, const void* dY, const void* W0,
                 const void* A, const void* B, const float* scale, const float* zero,
                 void* dX, float* dA, float* dB, float* dscale, float* dzero,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* QAT-LoRA layer, the straightforward integration the paper starts from (Sec. 3.1): only the frozen weight
 * goes through the quantizer and the LoRA path stays next to it in high precision,
 *   Y  = X . Q(W0)^T + gamma (X A^T) B^T
 *   dX = dY . Q(W0) + gamma (dY B) A;   dWq = dY^T X is written to the workspace in binary32 (the memory overhead
 *   the section names) and d(scale), d(zero) are taken from it with Eq. quant_lsq_s / quant_lsq_b;
 *   dA = gamma (dY B)^T X,  dB = gamma dY^T (X A^T)              (Eq. lora_backward).
 * Arguments, layouts, dtypes, flags (L4Q_FLAG_ACCUMULATE_GRADS) and error behaviour as l4q_forward / l4q_backward;
 * L4Q_FLAG_UNFUSED_BACKWARD has no effect.  The side products X A^T and dY B are binary32; in BF16 mode Y and dX
 * are rounded once by the main product and once more when the LoRA term is added.  Provided to measure the
 * memory / time gap to the L4Q layer on the same device; it shares the L4Q kernels. */
int l4q_qatlora_workspace_bytes(const l4q_desc* desc, size_t* forward_bytes, size_t* backward_bytes);
int l4q_qatlora_forward(const l4q_desc* desc, const void* X, const void* W0, const void* A, const void* B,
                        const float* scale, const float* zero, void* Y,
                        void* workspace, size_t workspace_bytes, void* hip_stream);
int l4q_qatlora_backward(const l4q_desc* desc, const void* X, const void* dY, const void* W0,
                         const void* A, const void* B, const float* scale, const float* zero,
                         void* dX, float* dA, float* dB, float* dscale, float* dzero,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Integer codes of the fully quantized layer (what inference consumes; Sec. 3.2, Eq. l4q_Wquant).
 *   codes [o,i] int8 in [Q_N, Q_P] (may be NULL);
 *   wcomb [o,i] float: the binary32 merged weight Wc the codes were taken from (may be NULL);
 *   mask  [o,i] uint8: 1 where Q_N <= w <= Q_P (may be NULL).
 * `tokens` of the descriptor is ignored.  Needs no workspace. */
int l4q_export_codes(const l4q_desc* desc, const void* W0, const void* A, const void* B,
                     const float* scale, const float* zero,
                     int8_t* codes, float* wcomb, uint8_t* mask, void* hip_stream);

/* Packed export of the fully quantized layer (Sec. 3.2).  packed: out_features * bits * in_features / 32
 * 32-bit words; the unsigned field u = w~ - Q_N of column j occupies bits [bits*j, bits*j + bits) of the row's
 * little-endian bit string.  in_features % 32 == 0.  workspace: out_features * in_features bytes,
 * 256-byte aligned.  `tokens` is ignored. */
int l4q_export_packed(const l4q_desc* desc, const void* W0, const void* A, const void* B,
                      const float* scale, const float* zero, uint32_t* packed,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Forward pass of the fully quantized layer from the packed codes alone (no W0, A, B):
 *   Y[T,o] = X[T,i] . (w~ scale + zero)^T        (Eq. l4q_forward with Eq. l4q_Wdequant)
 * BF16 only (X, Y bfloat16); bits in {2,3,4,8}; in_features % 64 == 0.  Meant for decode-sized T:
 * the packed weights are streamed once per pass of at most 64 tokens (32 or 48 for some shapes), so the
 * cost grows with T beyond that.
 * workspace (device memory, 256-byte aligned) is optional: NULL / 0 is always accepted.  Layers with few output
 * rows and long rows run faster from about 8 tokens on when given
 * l4q_quantized_forward_workspace_bytes() of it
 * (the row is then cut into k-slices over the compute units, whose partial sums are added in a fixed order);
 * a workspace smaller than that is ignored.  The result does not depend on the stream's other work, but with and
 * without the workspace it may differ in the last bit of the fp32 sum before the rounding to bfloat16. */
int l4q_quantized_forward(const l4q_desc* desc, const void* X, const uint32_t* packed,
                          const float* scale, const float* zero, void* Y,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace l4q_quantized_forward can make use of for this layer (0 for most shapes; does not depend on
 * `tokens`). */
int l4q_quantized_forward_workspace_bytes(const l4q_desc* desc, size_t* bytes);

/* Quantization-parameter initialisation from the merged weight (Sec. 3.3, Eq. l4q_quant_init;
 * App. B, Eq. quant_inits).  Writes scale, zero [o,G].
 *   L4Q_INIT_ASYMM : s = (max - min) / (Q_P - Q_N),  b = min - s Q_N
 *   L4Q_INIT_SYMM  : s = max|W| / 2^(n-1),           b = 0
 *   L4Q_INIT_L4Q   : s = max(|min / Q_N|, |max / Q_P|), b = 0
 *   L4Q_INIT_LSQPLUS : s = max(|mu - 3 sigma|, |mu + 3 sigma|) / 2^(n-1), b = 0, mu / sigma the mean and
 *                      (population) standard deviation of the group; group_size <= 256 only
 * The first three are evaluated in binary32, one rounding per written operation (bit-reproducible);
 * LSQ+ sums in binary32 in an unspecified order.  `tokens` is ignored. */
enum { L4Q_INIT_ASYMM = 0, L4Q_INIT_SYMM = 1, L4Q_INIT_L4Q = 2, L4Q_INIT_LSQPLUS = 3 };
int l4q_init_qparams(const l4q_desc* desc, const void* W0, const void* A, const void* B,
                     int method, float* scale, float* zero, void* hip_stream);

/* Quantization and clipping error of the current parameters (App. B, the E_quant / E_clip columns of the
 * initialisation table; the paper names them without formulas, read here as)
 *   errors[0] = sum over the weight of |Wc - Wq|,   errors[1] = sum of |Wc - (clamp(w, Q_N, Q_P) scale + zero)|.
 * errors: 2 floats on the device.  workspace: out_features * ceil(in_features / 256) * 8 bytes, 256-byte
 * aligned.  `tokens` is ignored. */
int l4q_quant_errors(const l4q_desc* desc, const void* W0, const void* A, const void* B,
                     const float* scale, const float* zero, float* errors,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* l4q_quant_errors for callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels, with the partial sums in a device array that is
 * part of the library image (L4Q_STATIC_SCRATCH_BYTES per GPU, resident until the process ends).  Calls no
 * allocator.  Arguments, result and errors as l4q_quant_errors, without the workspace; additionally
 * L4Q_ERR_TOO_LARGE when out_features * ceil(in_features / 256) * 8 exceeds L4Q_STATIC_SCRATCH_BYTES (nothing is
 * launched then).  All calls on one GPU share the one array: calls that may overlap there (different streams,
 * concurrent graph launches) race and must be ordered by the caller.  Nothing of an earlier call's content is read. */
#define L4Q_STATIC_SCRATCH_BYTES (8u << 20)
int l4q_quant_errors_static(const l4q_desc* desc, const void* W0, const void* A, const void* B,
                            const float* scale, const float* zero, float* errors, void* hip_stream);

/* One AdamW step (decoupled weight decay; App. C: weight decay 0.01) on the layer's four trainable tensors.
 *   m <- beta1 m + (1 - beta1) g;   v <- beta2 v + (1 - beta2) g^2
 *   p <- p - lr wd p - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * A32 [r,i], B32 [o,r], scale, zero [o,G]: binary32 master parameters, updated in place; dA .. dzero: their
 * gradients (what l4q_backward writes); m, v: moments, r*i + o*r + 2*o*G floats each, laid out
 * [A | B | scale | zero].  A_copy / B_copy (BF16 descriptors only, may be NULL): bfloat16 copies of the new A and
 * B for the next forward.  The paper fixes neither betas nor eps; common values are 0.9, 0.999, 1e-8.
 * `step` counts from 1.  `tokens` is ignored.  Arithmetic is binary32. */
typedef struct l4q_adamw {
  float lr, beta1, beta2, eps, weight_decay;
  int32_t step;
} l4q_adamw;
int l4q_adamw_step(const l4q_desc* desc, const l4q_adamw* hp,
                   float* A32, float* B32, float* scale, float* zero,
                   const float* dA, const float* dB, const float* dscale, const float* dzero,
                   float* m, float* v, void* A_copy, void* B_copy, void* hip_stream);

/* Learning rate of 0-based `step` (host function): linear warm-up lr_max (step + 1) / W over the first
 * W = ceil(warmup_fraction * total_steps) steps, then half a cosine from lr_max to 0 at total_steps
 * (App. C: cosine decay with linear warm-up through 10 % of the steps; the end value is this file's reading). */
float l4q_cosine_lr(int64_t step, int64_t total_steps, double lr_max, double warmup_fraction);

/* Opt-in timing of the library's bf16 GEMM and merge + quantize launches, for benchmarks (not for use under graph
 * capture: it creates HIP events).  While enabled, every such launch of l4q_forward / l4q_backward (and the GEMMs of
 * the QAT-LoRA entry points) is bracketed by two events recorded on the caller's stream.  This switch and its event
 * list are process-wide state.  l4q_profile_gemm(1) clears earlier records and starts recording, l4q_profile_gemm(0)
 * stops and clears.  l4q_profile_read waits for the recorded events of one kind (host-blocking) and returns their
 * summed kernel time in milliseconds, the number of launches and their algorithmic work; any pointer may be NULL.
 *   L4Q_PROFILE_GEMM            work = FLOPs, 2 M N K per launch with the unpadded K
 *   L4Q_PROFILE_MERGE_FORWARD   the merge + quantize pass of l4q_forward (Eqs. l4q_Wcombine .. l4q_Wdequant);
 *                               work = bytes: W0 read (2 o i) + scale and zero (8 o G) + Wq written (2 o i)
 *   L4Q_PROFILE_MERGE_BACKWARD  the recompute pass of l4q_backward; work = bytes: the same reads + Wq^T (2 o i) and,
 *                               for the fused weight-gradient kernel, the binary16 d(Wq)/d(scale) factor (2 o i)
 * l4q_profile_gemm_read is l4q_profile_read(L4Q_PROFILE_GEMM, ...). */
enum { L4Q_PROFILE_GEMM = 0, L4Q_PROFILE_MERGE_FORWARD = 1, L4Q_PROFILE_MERGE_BACKWARD = 2 };
int l4q_profile_gemm(int enable);
int l4q_profile_read(int kind, double* total_ms, int64_t* launches, double* total_work);
int l4q_profile_gemm_read(double* total_ms, int64_t* launches, double* total_flops);

/* Diagnostic for the merge + quantize pass, whose bf16 kernels replace the division w = (Wc - zero) / scale of the
 * arithmetic contract above by a multiplication with the correctly rounded reciprocal of the scale and one
 * exact-remainder correction.  For `count` (<= 2^23) significands of the scale starting at `first_significand`, at
 * three exponents each, the device compares (a) that reciprocal with the IEEE 1 / s and (b) the kernels' quotient
 * with the IEEE x / s for every x = s t moved by -5 .. +5 units in the last place, t running over every rounding tie
 * k + 1/2 (-128 <= k < 128) and every grid end Q_N, Q_P of 2 .. 8 bits.  counts: 3 x uint64 on the device, zeroed by
 * the caller; the call adds the number of wrong reciprocals, of wrong quotients, and of quotients compared. */
int l4q_check_fast_divide(uint32_t first_significand, uint32_t count, uint64_t* counts, void* hip_stream);

/* Matrix-core-only microbenchmark (for benchmarks): `workgroups` workgroups of 4 waves each run
 * `iterations` x 16 v_mfma_f32_32x32x16_bf16 on operand fragments taken from the first 64 KiB of
 * `data` (device, bf16), with the register shape of the library's GEMM and no memory traffic in
 * the loop.  sink: device, workgroups * 256 floats (written once at the end).  *flops receives the
 * FLOPs of the launch.  What it sustains depends on the operand values (power). */
int l4q_mfma_probe(const void* data, int iterations, int workgroups, float* sink, double* flops, void* hip_stream);

/* Static, NUL-terminated description of a status code. */
const char* l4q_status_string(int status);

/* L4Q_VERSION the library was built from. */
int l4q_version(void);

#ifdef __cplusplus
}
#endif
#endif /* L4Q_H */
