// The fully quantized layer (Sec. 3.2: inference runs on w~, scale and zero alone; Eq. l4q_forward):
// bit-packing of the integer codes and Y = X . dequant(codes)^T for small token counts (decode).
//
// Packed layout: the unsigned field u = w~ - Q_N of column j occupies bits [n j, n j + n) of the
// row's little-endian bit string; rows are n * i / 32 words.
//
// qgemm_kernel: one workgroup = 32 weight rows, 4 waves splitting k in interleaved 64-wide chunks.
// A lane owns one weight row: per chunk it loads the n words holding its 32 consecutive codes
// (lane group 0: k 0..31 of the chunk, group 1: k 32..63), expands them to bf16 (w~ s + b, the same
// values the training forward multiplies with) and feeds them to the matrix core as the row operand;
// the token operand comes straight from X (L1/L2 resident at decode sizes).  The k-slot order inside
// a chunk differs from memory order, identically for both operands, which a contraction allows.
// Partial sums of the 4 waves meet in LDS.  The weight stream is read once: HBM-bound.
#include "l4q_device.h"
#include "l4q_gemm_core.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

typedef gemm::bf16x8_t bf16x8_t;
typedef gemm::f32x16_t f32x16_t;

__global__ __launch_bounds__(256) void pack_codes_kernel(const int8_t* __restrict__ codes, int64_t o, int64_t i,
                                                          int bits, int qn, uint32_t* __restrict__ packed) {
  const int64_t words_per_row = bits * i / 32;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= o * words_per_row) return;
  const int64_t p = idx / words_per_row, w = idx % words_per_row;
  const int64_t bit0 = 32 * w;
  uint32_t word = 0;
  for (int64_t j = bit0 / bits; j < i && bits * j < bit0 + 32; ++j) {
    const uint32_t u = (uint32_t)((int)codes[p * i + j] - qn);
    const int pos = (int)(bits * j - bit0);
    word |= pos >= 0 ? u << pos : u >> -pos;
  }
  packed[idx] = word;
}

constexpr int QG_TOK = 64;  // tokens per pass

template <int BITS>
__global__ __launch_bounds__(256) void qgemm_kernel(const bf16_t* __restrict__ X, const uint32_t* __restrict__ packed,
                                                     const float* __restrict__ scale,
                                                     const float* __restrict__ zero, bf16_t* __restrict__ Y, int T,
                                                     int o, int i, int g, float qn) {
  __shared__ float red[4][2][16][64];
#if defined(__HIP_DEVICE_COMPILE__)
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int p = blockIdx.x * 32 + l32;
  const bool p_ok = p < o;
  const int pc = p_ok ? p : o - 1;
  const int words_per_row = BITS * (i / 32);
  const int G = i / g;
  const uint32_t* wrow = packed + (int64_t)pc * words_per_row;
  const int nchunks = i / 64;
  constexpr uint32_t MASK = (1u << BITS) - 1u;

  for (int t0 = 0; t0 < T; t0 += QG_TOK) {
    f32x16_t acc[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[tb][e] = 0.f;
    const int t_a = t0 + l32, t_b = t0 + 32 + l32;
    const bf16_t* xa = X + (int64_t)(t_a < T ? t_a : T - 1) * i;
    const bf16_t* xb = X + (int64_t)(t_b < T ? t_b : T - 1) * i;

    for (int c = wave; c < nchunks; c += 4) {
      const int krun = c * 64 + lh * 32;  // first k of this lane group's 32-code run
      uint32_t w[BITS + 1];
#pragma unroll
      for (int q = 0; q < BITS; ++q) w[q] = wrow[(krun / 32) * BITS + q];
      w[BITS] = 0;
      float s = scale[(int64_t)pc * G + krun / g], b = zero[(int64_t)pc * G + krun / g];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        if (g < 32 && m > 0) {  // a group can end inside the run: refresh per fragment
          s = scale[(int64_t)pc * G + (krun + 8 * m) / g];
          b = zero[(int64_t)pc * G + (krun + 8 * m) / g];
        }
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int bit = (8 * m + e) * BITS;
          const int idx = bit >> 5, sh = bit & 31;
          uint32_t v = w[idx] >> sh;
          if (sh + BITS > 32) v |= w[idx + 1] << (32 - sh);
          f[e] = p_ok ? fmaf((float)(v & MASK) + qn, s, b) : 0.f;
        }
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 wp = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                          pack_bf16x2(f[6], f[7])};
        const bf16x8_t wfrag = __builtin_bit_cast(bf16x8_t, wp);
        uint4 ra = *reinterpret_cast<const uint4*>(xa + krun + 8 * m);
        uint4 rb = *reinterpret_cast<const uint4*>(xb + krun + 8 * m);
        if (t_a >= T) ra = make_uint4(0, 0, 0, 0);
        if (t_b >= T) rb = make_uint4(0, 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, __builtin_bit_cast(bf16x8_t, ra), acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, __builtin_bit_cast(bf16x8_t, rb), acc[1], 0, 0, 0);
      }
    }

    // accumulator: lane = token (second operand's index), register e = weight row 8 (e/4) + 4 (lane/32) + e%4
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) red[wave][tb][e][lane] = acc[tb][e];
    __syncthreads();
    if (wave < 2) {  // wave 0 finishes token block 0, wave 1 token block 1
      const int t = t0 + wave * 32 + l32;
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          v[e] = (red[0][wave][4 * eg + e][lane] + red[1][wave][4 * eg + e][lane]) +
                 (red[2][wave][4 * eg + e][lane] + red[3][wave][4 * eg + e][lane]);
        const int prow = blockIdx.x * 32 + 8 * eg + 4 * lh;
        if (t < T && prow < o) store4(Y + (int64_t)t * o + prow, v);
      }
    }
    __syncthreads();
  }
#endif
}

}  // namespace

void launch_pack_codes(const int8_t* codes, int64_t o, int64_t i, int bits, uint32_t* packed, hipStream_t stream) {
  const int64_t n = o * (bits * i / 32);
  hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, codes, o, i, bits,
                     -(1 << (bits - 1)), packed);
}

bool qgemm_supported(const LayerDims& d) { return (d.bits == 2 || d.bits == 3 || d.bits == 4 || d.bits == 8) && d.i % 64 == 0 && d.g >= 8; }

void launch_qgemm(const LayerDims& d, const bf16_t* X, const uint32_t* packed, const float* scale, const float* zero,
                  bf16_t* Y, hipStream_t stream) {
  dim3 grid((unsigned)((d.o + 31) / 32));
#define L4Q_QGEMM(B)                                                                                              \
  hipLaunchKernelGGL(qgemm_kernel<B>, grid, dim3(256), 0, stream, X, packed, scale, zero, Y, (int)d.T, (int)d.o, \
                     (int)d.i, d.g, d.qn)
  if (d.bits == 2) L4Q_QGEMM(2);
  else if (d.bits == 3) L4Q_QGEMM(3);
  else if (d.bits == 4) L4Q_QGEMM(4);
  else L4Q_QGEMM(8);
#undef L4Q_QGEMM
}

}  // namespace l4q
