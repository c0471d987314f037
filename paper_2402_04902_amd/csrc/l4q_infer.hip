// The fully quantized layer (Sec. 3.2: inference runs on w~, scale and zero alone; Eq. l4q_forward):
// bit-packing of the integer codes and Y = X . dequant(codes)^T for small token counts (decode).
//
// Packed layout: the unsigned field u = w~ - Q_N of column j occupies bits [n j, n j + n) of the
// row's little-endian bit string; rows are n * i / 32 words.
//
// Five kernels compute the product, chosen by launch_qgemm from the code width, the token count and the layer's
// shape (each is described where it is defined): qgemm_wreg_kernel (2 / 3 / 4 / 8 bits, groups of 128 and more, one
// token to a few token blocks: the packed codes resident in registers, the activations streamed),
// qgemm_decode_kernel (2 / 4 / 8 bits, activations resident in LDS, the weights streamed through rings),
// qgemm_stream_kernel (4 / 8 bits, up to 32 tokens per pass), qgemm_tile_kernel (3 / 4 / 8 bits, 64-row tiles, up to
// 64 tokens per pass, optionally in k-slices whose partial sums qgemm_slices_sum_kernel adds), and qgemm_kernel,
// which covers every other layout:
// qgemm_kernel: one workgroup = 32 weight rows, 8 waves splitting k in interleaved 64-wide chunks.
// A lane owns one weight row: per chunk it loads the n words holding its 32 consecutive codes
// (lane group 0: k 0..31 of the chunk, group 1: k 32..63), turns them into bf16 operands (integer codes with the
// affine part applied to the accumulator when g >= 64, else w~ s + b itself) and feeds them to the matrix core
// as the row operand; the token operand comes straight from X (L1/L2 resident at decode sizes).  The k-slot
// order inside a chunk differs from memory order, identically for both operands, which a contraction allows.
// Partial sums of the 8 waves meet in LDS.  The weight stream is read once per pass: HBM-bound.
#include <type_traits>

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

constexpr int QG_WAVES = 8;   // k-split inside a workgroup

// Integer code fields -> bf16 matrix operand without a per-element convert:
//  * n <= 7: the bf16 bit pattern 0x4300 | u is the exact value 128 + u, so the matrix core multiplies
//    X with (w~ + K0), K0 = 128 - Q_N, and the shift is undone together with the zero term below;
//  * n == 8: v_cvt_f32_ubyte + (-128) gives w~ itself (|w~| <= 128 is exact in bf16), K0 = 0.
// The affine part of Eq. l4q_Wdequant is applied to the accumulator, once per 64-wide k chunk (one group
// or a whole number of groups when g < 64 -- then per 8-wide fragment):
//   sum_k X (w~ s + b) = s * sum_k X (w~ + K0) + (b - K0 s) * sum_k X.
// The matrix op is issued as D = Xfrag . Wfrag^T, so a lane of D is a weight row (scale / zero are per
// lane) and its 16 registers are tokens; sum_k X comes from a second matrix op against a fragment of ones.
template <int BITS, int NTB, bool PER_FRAG>
__global__ __launch_bounds__(QG_WAVES * 64) void qgemm_kernel(const bf16_t* __restrict__ X,
                                                               const uint32_t* __restrict__ packed,
                                                               const float* __restrict__ scale,
                                                               const float* __restrict__ zero,
                                                               bf16_t* __restrict__ Y, int T, int o, int i, int g,
                                                               float qn) {
  __shared__ float red[QG_WAVES][2][16][64];
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
  const float* srow = scale + (int64_t)pc * G;
  const float* brow = zero + (int64_t)pc * G;
  const int nchunks = i / 64;
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  constexpr float K0 = BITS == 8 ? 0.f : 128.f + (float)(1 << (BITS - 1));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, ones_bits);
  constexpr bool per_frag = PER_FRAG;  // g < 64: a chunk holds several groups

  for (int t0 = 0; t0 < T; t0 += 32 * NTB) {
    constexpr bool two_blocks = NTB == 2;  // a pass covers 32 * NTB tokens
    f32x16_t acc[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[tb][e] = 0.f;
    const int t_a = t0 + l32, t_b = t0 + 32 + l32;
    const bf16_t* xa = X + (int64_t)(t_a < T ? t_a : T - 1) * i;
    const bf16_t* xb = X + (int64_t)(t_b < T ? t_b : T - 1) * i;

    // Operands of one 64-wide k chunk.  Lane group h = lane / 32 owns k = 64 c + 32 h .. + 31 in both operands.
    struct Chunk {
      uint32_t w[BITS + 1];
      float s[4], b[4];
      uint4 xa[4], xb[4];
    };
    auto fetch = [&](int c, Chunk& ck) {
      const int cc = c < nchunks ? c : nchunks - 1;  // clamped: a fetch past the end is never consumed
      const int krun = cc * 64 + lh * 32;
#pragma unroll
      for (int q = 0; q < BITS; ++q) ck.w[q] = wrow[(krun / 32) * BITS + q];
      ck.w[BITS] = 0;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        if (g < 32 || m == 0) {
          const int kq = g >= 32 ? krun : krun + 8 * m;
          ck.s[m] = srow[kq / g];
          ck.b[m] = brow[kq / g];
        } else {
          ck.s[m] = ck.s[0];
          ck.b[m] = ck.b[0];
        }
        ck.xa[m] = *reinterpret_cast<const uint4*>(xa + krun + 8 * m);
        if (two_blocks) ck.xb[m] = *reinterpret_cast<const uint4*>(xb + krun + 8 * m);
      }
    };
    auto wfrag_of = [&](const Chunk& ck, int m) -> bf16x8_t {
      uint32_t d[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        uint32_t u[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int bit = (8 * m + 2 * e2 + h) * BITS;
          const int idx = bit >> 5, sh = bit & 31;
          uint32_t v = ck.w[idx] >> sh;
          if (sh + BITS > 32) v |= ck.w[idx + 1] << (32 - sh);
          u[h] = v & MASK;
        }
        if (BITS == 8) d[e2] = pack_bf16x2((float)u[0] - 128.f, (float)u[1] - 128.f);
        else d[e2] = (u[0] | (u[1] << 16)) | 0x43004300u;
      }
      const u32x4 wp = {d[0], d[1], d[2], d[3]};
      return __builtin_bit_cast(bf16x8_t, wp);
    };
    // The two lane groups of a wave hold different k ranges of the chunk and, for g < 64, different groups:
    // the matrix op sums both groups' k-slots into one accumulator, so the affine part can only be applied
    // per chunk when scale and zero are the same for both halves, i.e. g >= 64.  Smaller groups take the
    // slower route of scaling the operand itself.
    auto consume = [&](const Chunk& ck) {
      if constexpr (!per_frag) {
        f32x16_t tw[2], tx[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 16; ++e) { tw[tb][e] = 0.f; tx[tb][e] = 0.f; }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const bf16x8_t wf = wfrag_of(ck, m);
          const bf16x8_t xfa = __builtin_bit_cast(bf16x8_t, ck.xa[m]);  // tokens past T: clamped row, never stored
          tw[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xfa, wf, tw[0], 0, 0, 0);
          tx[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xfa, ones, tx[0], 0, 0, 0);
          if (two_blocks) {
            const bf16x8_t xfb = __builtin_bit_cast(bf16x8_t, ck.xb[m]);
            tw[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xfb, wf, tw[1], 0, 0, 0);
            tx[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xfb, ones, tx[1], 0, 0, 0);
          }
        }
        // g >= 64: both lane groups share the chunk's scale / zero; take them from the row's own lane
        const float sc = ck.s[0], bz = ck.b[0] - K0 * ck.s[0];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          if (tb == 1 && !two_blocks) break;
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[tb][e] = fmaf(bz, tx[tb][e], fmaf(sc, tw[tb][e], acc[tb][e]));
        }
      } else {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          // dequantize the operand itself: w~ s + b rounded to bf16, as the training forward does
          float f[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int bit = (8 * m + e) * BITS;
            const int idx = bit >> 5, sh = bit & 31;
            uint32_t v = ck.w[idx] >> sh;
            if (sh + BITS > 32) v |= ck.w[idx + 1] << (32 - sh);
            f[e] = fmaf((float)(v & MASK) + qn, ck.s[m], ck.b[m]);
          }
          const u32x4 wp = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                            pack_bf16x2(f[6], f[7])};
          const bf16x8_t wf = __builtin_bit_cast(bf16x8_t, wp);
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ck.xa[m]), wf, acc[0], 0, 0, 0);
          if (two_blocks) {
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ck.xb[m]), wf, acc[1], 0, 0, 0);
          }
        }
      }
    };
    if constexpr (per_frag) {
      Chunk c0, c1;
      fetch(wave, c0);
      for (int c = wave; c < nchunks; c += 2 * QG_WAVES) {
        fetch(c + QG_WAVES, c1);
        consume(c0);
        fetch(c + 2 * QG_WAVES, c0);
        if (c + QG_WAVES < nchunks) consume(c1);
      }
    } else {
      // g >= 64.  The weight stream is what has to come from HBM, and a wave sees only a few dozen chunks:
      // to keep enough bytes in flight it requests the packed words (and scale / zero) of QG_NB chunks at a
      // time, one batch ahead of the batch being consumed; X (cache resident) is fetched one chunk ahead.
      constexpr int QG_NB = 4;
      struct Batch {
        uint32_t w[QG_NB][BITS + 1];
        float s[QG_NB], b[QG_NB];
      };
      auto chunk_of = [&](int bt, int q) { return wave + QG_WAVES * (bt * QG_NB + q); };
      auto fetch_batch = [&](int bt, Batch& B) {
#pragma unroll
        for (int q = 0; q < QG_NB; ++q) {
          const int c = chunk_of(bt, q);
          const int krun = (c < nchunks ? c : nchunks - 1) * 64 + lh * 32;
#pragma unroll
          for (int v = 0; v < BITS; ++v) B.w[q][v] = wrow[(krun / 32) * BITS + v];
          B.w[q][BITS] = 0;
          B.s[q] = srow[krun / g];
          B.b[q] = brow[krun / g];
        }
      };
      auto fetch_x = [&](int c, Chunk& ck) {
        const int krun = (c < nchunks ? c : nchunks - 1) * 64 + lh * 32;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          ck.xa[m] = *reinterpret_cast<const uint4*>(xa + krun + 8 * m);
          if (two_blocks) ck.xb[m] = *reinterpret_cast<const uint4*>(xb + krun + 8 * m);
        }
      };
      auto consume_batch = [&](int bt, const Batch& B) {
        Chunk cx[2];
        fetch_x(chunk_of(bt, 0), cx[0]);
#pragma unroll
        for (int q = 0; q < QG_NB; ++q) {
          if (q + 1 < QG_NB) fetch_x(chunk_of(bt, q + 1), cx[(q + 1) & 1]);
          if (chunk_of(bt, q) < nchunks) {  // wave-uniform
            Chunk& ck = cx[q & 1];
#pragma unroll
            for (int v = 0; v <= BITS; ++v) ck.w[v] = B.w[q][v];
            ck.s[0] = B.s[q];
            ck.b[0] = B.b[q];
            consume(ck);
          }
        }
      };
      const int nbatches = (nchunks + QG_WAVES * QG_NB - 1) / (QG_WAVES * QG_NB);
      Batch b0, b1;
      fetch_batch(0, b0);
      for (int bt = 0; bt < nbatches; bt += 2) {
        fetch_batch(bt + 1, b1);
        consume_batch(bt, b0);
        fetch_batch(bt + 2, b0);
        if (bt + 1 < nbatches) consume_batch(bt + 1, b1);
      }
    }

    // accumulator: lane = weight row (second operand's index), register e = token 8 (e/4) + 4 (lane/32) + e%4
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) red[wave][tb][e][lane] = acc[tb][e];
    __syncthreads();
    if (wave < 2 && (wave == 0 || two_blocks)) {  // wave 0 finishes token block 0, wave 1 token block 1
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < QG_WAVES; ++q) v += red[q][wave][e][lane];
        const int t = t0 + wave * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (t < T && p_ok) Y[(int64_t)t * o + p] = f32_to_bf16(v);
      }
    }
    __syncthreads();
  }
#endif
}


// ---------------------------------------------------------------------------------------------
// Streaming form of the same product for the common layouts: bits in {4, 8}, rows of packed words a
// whole number of 128-byte cache lines, group size a multiple of the codes of a sub-step.
//
// One workgroup = ROWS weight rows (32, or 16 for up to 16 tokens: the 16x16x32 matrix op then does the
// same work in a quarter of the matrix-core time), 4 waves; the row's 128-byte stages go round-robin to
// the waves and each wave runs a private pipeline, so there is no barrier until the final sum.  A stage
// (ROWS rows x 128 bytes) travels HBM -> LDS with buffer_load ... lds instructions whose lanes read whole
// cache lines (8 lanes per row) -- the per-lane row ownership of qgemm_kernel touches 32 lines for 32
// bytes each instead.  LDS keeps the rows 128 bytes apart; the 16-byte chunk c of row r sits at position
// c ^ ((r / 2) % 8), which makes the fragment reads (lane = row) conflict-free.  In sub-step h a lane of
// lane group kg reads chunk KG h + kg of its row: 128 / bits codes = 16 / bits operand fragments, the
// f-th of which is its 8 k-slots in the f-th matrix op of the sub-step.
// Ring of 4 stages per wave: three stages are in flight while one is consumed.  X fragments and scale /
// zero are fetched one stage ahead into registers; every load is issued in a fixed order so that one
// partial s_waitcnt covers the stage.
// Operand fragment f (8 consecutive codes) of a 16-byte chunk of packed codes, as bf16 values without a convert.
// 4 bits: byte r holds codes 2r (low nibble) and 2r + 1; times 0x1001 puts a copy of the byte 12 bits up, so one mask
// leaves code 2r in bits 0..3 and code 2r + 1 in bits 16..19, and OR-ing 0x4300 into both halves makes the bf16 pair
// 128 + u (the caller's K0 takes the 128 and the code offset out again).  8 bits: code - 128, converted.
typedef uint32_t code_chunk_t __attribute__((ext_vector_type(4)));
template <int BITS>
__device__ __forceinline__ bf16x8_t code_fragment(const code_chunk_t& w, int f) {
  code_chunk_t d;
  if (BITS == 4) {
    const uint32_t v = w[f];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t spread = __builtin_amdgcn_ubfe(v, 8 * r, 8) * 0x1001u;
      // ((x & mask) | bias as one v_and_or_b32: the constants are made opaque so that they stay in registers - the op
      // takes no literals; the op itself is left to the compiler: as inline assembly it would hide that a vector op wrote
      // the register, and the wait states a matrix op needs before it reads such a register would be missing)
      uint32_t mask = 0x000F000Fu, bias = 0x43004300u;
      asm("" : "+s"(mask));
      asm("" : "+v"(bias));
      d[r] = (spread & mask) | bias;
    }
  } else if (BITS == 2) {
    // the chunk's first two dwords hold 32 codes; fragment f is the 16-bit half f % 2 of dword f / 2, its code pairs are
    // 4-bit fields: times 0x4001 puts a copy 14 bits up, the mask leaves code 2r in bits 0..1 and code 2r + 1 in bits
    // 16..17 (the caller's K0 is 128 + 2)
    const uint32_t v = w[f >> 1];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t spread = __builtin_amdgcn_ubfe(v, 16 * (f & 1) + 4 * r, 4) * 0x4001u;
      d[r] = (spread & 0x00030003u) | 0x43004300u;
    }
  } else if (BITS == 3) {
    // the chunk's first three dwords hold 32 codes; fragment f is the 24-bit window from bit 24 f, its code pairs are
    // 6-bit fields: times 0x2001 puts a copy 13 bits up, the mask leaves code 2r in bits 0..2 and code 2r + 1 in bits
    // 16..18 (the caller's K0 is 128 + 4)
    const uint32_t win = f == 0 ? w[0] : f == 1 ? (w[0] >> 24) | (w[1] << 8) : f == 2 ? (w[1] >> 16) | (w[2] << 16) : w[2] >> 8;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t spread = __builtin_amdgcn_ubfe(win, 6 * r, 6) * 0x2001u;
      d[r] = (spread & 0x00070007u) | 0x43004300u;
    }
  } else {
    const uint32_t v0 = w[(2 * f) & 3], v1 = w[(2 * f + 1) & 3];  // 4 + 4 codes
    d[0] = pack_bf16x2((float)(v0 & 0xFFu) - 128.f, (float)((v0 >> 8) & 0xFFu) - 128.f);
    d[1] = pack_bf16x2((float)((v0 >> 16) & 0xFFu) - 128.f, (float)(v0 >> 24) - 128.f);
    d[2] = pack_bf16x2((float)(v1 & 0xFFu) - 128.f, (float)((v1 >> 8) & 0xFFu) - 128.f);
    d[3] = pack_bf16x2((float)((v1 >> 16) & 0xFFu) - 128.f, (float)(v1 >> 24) - 128.f);
  }
  return __builtin_bit_cast(bf16x8_t, d);
}

constexpr int QS_NSW = 4;             // ring stages per wave

template <int ROWS> struct QsMfma;
template <> struct QsMfma<32> {
  typedef f32x16_t acc_t;
  static constexpr int NACC = 16;
  static __device__ __forceinline__ acc_t mma(bf16x8_t a, bf16x8_t b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  // token (row of D) held in register e by a lane of lane group kg
  static __device__ __forceinline__ int token(int e, int kg) { return 8 * (e >> 2) + 4 * kg + (e & 3); }
};
template <> struct QsMfma<16> {
  typedef float acc_t __attribute__((ext_vector_type(4)));
  static constexpr int NACC = 4;
  static __device__ __forceinline__ acc_t mma(bf16x8_t a, bf16x8_t b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int token(int e, int kg) { return 4 * kg + e; }
};

template <int BITS, int ROWS>
__global__ __launch_bounds__(256, 2) void qgemm_stream_kernel(const bf16_t* __restrict__ X,
                                                               const uint32_t* __restrict__ packed,
                                                               const float* __restrict__ scale,
                                                               const float* __restrict__ zero,
                                                               bf16_t* __restrict__ Y, int T, int t0, int o, int i,
                                                               int g) {
  constexpr int STAGE = ROWS * 128;  // bytes of a stage
  __shared__ __attribute__((aligned(1024))) unsigned char lds[4 * QS_NSW * STAGE];
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(BITS == 4 || BITS == 8, "bits");
  typedef QsMfma<ROWS> M;
  typedef typename M::acc_t acc_t;
  constexpr int NACC = M::NACC;
  constexpr int KG = 64 / ROWS;    // lane groups of the matrix op (k-slot groups)
  constexpr int NH = 8 / KG;       // sub-steps per stage
  constexpr int NDMA = ROWS / 8;   // wave-wide loads per stage
  constexpr int CH = 128 / BITS;   // codes per 16-byte chunk
  constexpr int KS = 8 * CH;       // codes per stage
  constexpr int FR = CH / 8;       // operand fragments per chunk
  constexpr int SUB = KG * CH;     // codes per sub-step
  constexpr int NXL = NH * FR + 2 * NH;  // register loads per stage: X fragments, scale and zero per sub-step
  constexpr float K0 = BITS == 8 ? 0.f : 128.f + (float)(1 << (BITS - 1));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef gemm::lds_ptr_t lds_ptr_t;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane % ROWS, kg = lane / ROWS;
  const int p0 = blockIdx.x * ROWS;
  const int p = p0 + ln;
  const int pc = p < o ? p : o - 1;
  const int rb = i / 8 * BITS;     // bytes of a packed row
  const int nst = rb / 128;        // stages of a row
  const int G = i / g;
  const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, ones_bits);

  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(packed), 0, (int)((int64_t)o * rb), 0x00020000);
  unsigned voff[NDMA];
#pragma unroll
  for (int q = 0; q < NDMA; ++q) {
    const int r = 8 * q + (lane >> 3);
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    voff[q] = p0 + r < o ? (unsigned)((p0 + r) * rb + chunk * 16) : gemm::OOB_OFFSET;
  }
  unsigned char* ring = lds + wave * (QS_NSW * STAGE);
  const unsigned frag_row = ln * 128;
  const int swz = (ln >> 1) & 7;
  const int tok = t0 + ln < T ? t0 + ln : T - 1;
  const bf16_t* xrow = X + (int64_t)tok * i;
  const float* srow = scale + (int64_t)pc * G;
  const float* brow = zero + (int64_t)pc * G;
  const int nj = wave < nst ? (nst - wave + 3) / 4 : 0;  // stages of this wave: wave, wave + 4, ...

  auto issue_dma = [&](int j) {  // stage j of this wave into ring slot j % QS_NSW; past the end: no traffic
    const unsigned kb = j < nj ? (unsigned)(wave + 4 * j) * 128u : gemm::PAST_END_OFFSET;
    unsigned char* dst = ring + (j % QS_NSW) * STAGE;
#pragma unroll
    for (int q = 0; q < NDMA; ++q)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(dst + q * 1024), 16, voff[q] + kb, 0, 0, 0);
  };
  struct StageRegs {
    uint4 x[NH][FR];
    float s[NH], b[NH];
  };
  auto fetch_regs = [&](int j, StageRegs& R) {  // clamped: a fetch past the end is never consumed
    const int st = wave + 4 * (j < nj ? j : (nj > 0 ? nj - 1 : 0));
    const int k0 = (st < nst ? st : nst - 1) * KS;
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
      for (int f = 0; f < FR; ++f)
        R.x[h][f] = *reinterpret_cast<const uint4*>(xrow + k0 + (KG * h + kg) * CH + 8 * f);
#pragma unroll
    for (int h = 0; h < NH; ++h) {  // scale / zero of the group each sub-step lies in
      const int grp = (k0 + h * SUB) / g;
      R.s[h] = srow[grp];
      R.b[h] = brow[grp];
    }
  };

  acc_t acc;
#pragma unroll
  for (int e = 0; e < NACC; ++e) acc[e] = 0.f;

  auto consume = [&](int j, const StageRegs& R) {
    const bool live = j < nj;
    const unsigned char* src = ring + (j % QS_NSW) * STAGE + frag_row;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(src + (((KG * h + kg) ^ swz) << 4));
      acc_t tw, tx;
#pragma unroll
      for (int e = 0; e < NACC; ++e) { tw[e] = 0.f; tx[e] = 0.f; }
#pragma unroll
      for (int f = 0; f < FR; ++f) {
        const bf16x8_t wf = code_fragment<BITS>(w, f);
        const bf16x8_t xf = __builtin_bit_cast(bf16x8_t, R.x[h][f]);  // tokens past T: clamped row, never stored
        tw = M::mma(xf, wf, tw);
        tx = M::mma(xf, ones, tx);
      }
      // the sub-step lies inside one group: sum_k X (w~ s + b) = s sum_k X (w~ + K0) + (b - K0 s) sum_k X.
      // A stage past the end (the pipeline always runs an even number) gets scale = zero = 0: it adds nothing.
      const float sc = live ? R.s[h] : 0.f, bz = live ? R.b[h] - K0 * sc : 0.f;
#pragma unroll
      for (int e = 0; e < NACC; ++e) acc[e] = fmaf(bz, tx[e], fmaf(sc, tw[e], acc[e]));
    }
  };

  // Issue order (every wave, every iteration): registers of stage j + 1, then the DMA of stage j + 3.  When
  // stage j is consumed, what was issued after its own loads is DMA j + 2, registers j + 1 and DMA j + 3.
  StageRegs r0, r1;
  issue_dma(0);
  issue_dma(1);
  fetch_regs(0, r0);
  issue_dma(2);
  __builtin_amdgcn_sched_barrier(0);  // the scheduler keeps each phase where it is written
  for (int j = 0; j < nj; j += 2) {
    fetch_regs(j + 1, r1);
    __builtin_amdgcn_sched_barrier(0);
    issue_dma(j + 3);
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(NDMA + NXL + NDMA));
    __builtin_amdgcn_sched_barrier(0);
    consume(j, r0);
    __builtin_amdgcn_sched_barrier(0);
    fetch_regs(j + 2, r0);
    __builtin_amdgcn_sched_barrier(0);
    issue_dma(j + 4);
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(NDMA + NXL + NDMA));
    __builtin_amdgcn_sched_barrier(0);
    consume(j + 1, r1);
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(0));
  __syncthreads();  // every wave is done with its ring: the LDS is reused for the sum over the waves

  // accumulator: lane = weight row, register e = token M::token(e, kg)
  float* red = reinterpret_cast<float*>(lds);
#pragma unroll
  for (int e = 0; e < NACC; ++e) red[(wave * NACC + e) * 64 + lane] = acc[e];
  __syncthreads();
  {  // wave w finishes registers NACC / 4 * w .. + NACC / 4 - 1
#pragma unroll
    for (int e4 = 0; e4 < NACC / 4; ++e4) {
      const int e = wave * (NACC / 4) + e4;
      const float v = (red[(0 * NACC + e) * 64 + lane] + red[(1 * NACC + e) * 64 + lane]) +
                      (red[(2 * NACC + e) * 64 + lane] + red[(3 * NACC + e) * 64 + lane]);
      const int t = t0 + M::token(e, kg);
      if (t < T && p < o) Y[(int64_t)t * o + p] = f32_to_bf16(v);
    }
  }
#endif
}

// The same pipeline for the smallest batches (single-token decode first of all), 16-row tiles.  In the kernel above
// every stage costs a wave 8 wave-wide register loads of X fragments and 4 of scale / zero, which together occupy the
// vector-memory path four times as long as the two loads that bring the weights themselves.  Here the activations
// of the whole pass (T rows of X, at most QD_X_MAX bytes) and the tile's scale / zero rows are put into LDS once per
// workgroup, and the stage loop issues nothing but the weight stream: fragments, scale and zero are LDS reads
// (lanes of one token and k-group read the same address, which the LDS serves as a broadcast).  NSW = ring stages
// per wave: 4 when several workgroups share a compute unit, 8 when there is at most one per unit and a wave has to
// keep more of the stream in flight by itself, 2 where the activations leave room for no more.
constexpr int QD_X_MAX = 132 * 1024;  // bytes of X held in LDS
constexpr int QD_SB_MAX = 17 * 1024;  // bytes of scale + zero held in LDS (up to 128 groups per row)
constexpr int QD_LDS_MAX = 160 * 1024; // LDS of a compute unit

template <int BITS, int NSW>
__global__ __launch_bounds__(256, 2) void qgemm_decode_kernel(const bf16_t* __restrict__ X,
                                                               const uint32_t* __restrict__ packed,
                                                               const float* __restrict__ scale,
                                                               const float* __restrict__ zero,
                                                               bf16_t* __restrict__ Y, int T, int o, int i, int g,
                                                               int xpitch, int sb_pitch) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char dlds[];
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(BITS == 2 || BITS == 4 || BITS == 8, "bits");
  constexpr int ROWS = 16;
  constexpr int STAGE = ROWS * 128;
  typedef QsMfma<ROWS> M;
  typedef typename M::acc_t acc_t;
  constexpr int NACC = M::NACC;
  // A lane group's share of a sub-step: 16 bytes of its row's stage, or 8 for 2 bits (32 codes either way at 2 and 4
  // bits), so that a sub-step's 4 x 32 codes never span more than one group of 128.
  constexpr int LB = BITS == 2 ? 8 : 16;
  constexpr int KG = 64 / ROWS, NDMA = ROWS / 8;
  constexpr int CH = LB * 8 / BITS, KS = 128 * 8 / BITS, FR = CH / 8, SUB = KG * CH, NH = KS / SUB;
  constexpr float K0 = BITS == 8 ? 0.f : 128.f + (float)(1 << (BITS - 1));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef gemm::lds_ptr_t lds_ptr_t;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane % ROWS, kg = lane / ROWS;
  const int p0 = blockIdx.x * ROWS;
  const int p = p0 + ln;
  const int rb = i / 8 * BITS;
  // A row need not be a whole number of 128-byte stages: its last stage then runs into the next row's codes (or past
  // the matrix: zeros), which meet activations that are zero (every token's row in LDS is zero beyond k = i) and
  // scale / zero values that are the zeros of the table's padding.
  const int nst = (rb + 127) / 128;
  const int G = i / g;
  const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, ones_bits);

  unsigned char* ring = dlds + wave * (NSW * STAGE);
  // [T][xpitch bytes] bf16: a token's row, zero from k = i to the end of its last stage; rows 16 bytes apart in the
  // banks, so that the tokens of a fragment read spread over the bank groups
  unsigned char* xl = dlds + 4 * NSW * STAGE;
  float* sl = reinterpret_cast<float*>(xl + T * xpitch);        // [16][sb_pitch], odd pitch: conflict-free columns
  float* bl = sl + ROWS * sb_pitch;

  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(packed), 0, (int)((int64_t)o * rb), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcX = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(X), 0, (int)((int64_t)T * i * 2), 0x00020000);
  unsigned voff[NDMA];
#pragma unroll
  for (int q = 0; q < NDMA; ++q) {
    const int r = 8 * q + (lane >> 3);
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    voff[q] = p0 + r < o ? (unsigned)((p0 + r) * rb + chunk * 16) : gemm::OOB_OFFSET;
  }
  const int nj = wave < nst ? (nst - wave + 3) / 4 : 0;
  auto issue_dma = [&](int j) {
    const unsigned kb = j < nj ? (unsigned)(wave + 4 * j) * 128u : gemm::PAST_END_OFFSET;
    unsigned char* dst = ring + (j % NSW) * STAGE;
#pragma unroll
    for (int q = 0; q < NDMA; ++q)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(dst + q * 1024), 16, voff[q] + kb, 0, 0, 0);
  };

  // the first NSW - 1 weight stages, then X (1 KiB pieces round-robin over the waves; bytes past the end of X read
  // as zero), then scale / zero of the tile's rows, all by DMA into LDS
#pragma unroll
  for (int j = 0; j < NSW - 1; ++j) issue_dma(j);
  {
    const int npc = xpitch / 1024;  // 1 KiB pieces of a token's row
    for (int q = wave; q < T * npc; q += 4) {
      const int t = q / npc, c = q - t * npc;
      const int byte = c * 1024 + lane * 16;
      const unsigned off = byte < i * 2 ? (unsigned)((int64_t)t * i * 2 + byte) : gemm::OOB_OFFSET;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcX, (lds_ptr_t)(xl + t * xpitch + c * 1024), 16, off, 0, 0, 0);
    }
  }
  {
    // Per table row ceil(G / 64) wave-wide loads of 4 bytes per lane, straight into the padded LDS row: nothing passes
    // through registers and nothing waits before the common wait below (a loop of load - wait - store rounds cost a
    // memory latency per round: same box, [4096 x 11008] at one token 8.9 against 10.0 us).  Lanes past the row's G
    // values and rows past o get out-of-range offsets and write zeros, which the pitch (a multiple of 64, plus 1)
    // keeps inside the row's own padding.
    const __amdgpu_buffer_rsrc_t rsrcS = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(scale), 0, (int)((int64_t)o * G * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcZ = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(zero), 0, (int)((int64_t)o * G * 4), 0x00020000);
    const int per_row = (sb_pitch - 1) / 64;  // (the pitch covers the groups of the padded row)
    for (int u = wave; u < ROWS * per_row; u += 4) {
      const int row = u / per_row, c = u - row * per_row;
      const int idx = c * 64 + lane;
      const unsigned off = idx < G && p0 + row < o ? (unsigned)(((p0 + row) * G + idx) * 4) : gemm::OOB_OFFSET;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcS, (lds_ptr_t)(sl + row * sb_pitch + c * 64), 4, off, 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcZ, (lds_ptr_t)(bl + row * sb_pitch + c * 64), 4, off, 0, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(0));
  __syncthreads();

  const unsigned frag_row = ln * 128;
  const int swz = (ln >> 1) & 7;
  const int tok = ln < T ? ln : T - 1;
  const unsigned char* xrow = xl + (size_t)tok * xpitch;
  const float* srow = sl + ln * sb_pitch;
  const float* brow = bl + ln * sb_pitch;

  acc_t acc;
#pragma unroll
  for (int e = 0; e < NACC; ++e) acc[e] = 0.f;

  for (int j = 0; j < nj; ++j) {
    issue_dma(j + NSW - 1);
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm((NSW - 1) * NDMA));  // stage j has landed; the NSW - 1 after it may be in flight
    __builtin_amdgcn_sched_barrier(0);                       // the LDS reads below stay behind the wait
    const unsigned char* src = ring + (j % NSW) * STAGE + frag_row;
    const int k0 = (wave + 4 * j) * KS;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      u32x4 w;
      if constexpr (BITS == 2) {  // half a 16-byte chunk: piece KG h + kg of the row's sixteen
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const int piece = KG * h + kg;
        const u32x2 w2 = *reinterpret_cast<const u32x2*>(src + ((((piece >> 1) ^ swz) << 4) | ((piece & 1) << 3)));
        w = u32x4{w2[0], w2[1], 0u, 0u};
      } else {
        w = *reinterpret_cast<const u32x4*>(src + (((KG * h + kg) ^ swz) << 4));
      }
      const int grp = (k0 + h * SUB) / g;
      const float sc = srow[grp], bz = brow[grp] - K0 * sc;
      acc_t tw, tx;
#pragma unroll
      for (int e = 0; e < NACC; ++e) { tw[e] = 0.f; tx[e] = 0.f; }
#pragma unroll
      for (int f = 0; f < FR; ++f) {
        const bf16x8_t wf = code_fragment<BITS>(w, f);
        const bf16x8_t xf = *reinterpret_cast<const bf16x8_t*>(xrow + (size_t)(k0 + (KG * h + kg) * CH + 8 * f) * 2);
        tw = M::mma(xf, wf, tw);
        tx = M::mma(xf, ones, tx);
      }
#pragma unroll
      for (int e = 0; e < NACC; ++e) acc[e] = fmaf(bz, tx[e], fmaf(sc, tw[e], acc[e]));
    }
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(0));
  __syncthreads();  // every wave is done with its ring: the LDS is reused for the sum over the waves

  float* red = reinterpret_cast<float*>(dlds);
#pragma unroll
  for (int e = 0; e < NACC; ++e) red[(wave * NACC + e) * 64 + lane] = acc[e];
  __syncthreads();
  {
    const int e = wave;  // wave w finishes register w: token 4 kg + w
    const float v = (red[(0 * NACC + e) * 64 + lane] + red[(1 * NACC + e) * 64 + lane]) +
                    (red[(2 * NACC + e) * 64 + lane] + red[(3 * NACC + e) * 64 + lane]);
    const int t = M::token(e, kg);
    if (t < T && p < o) Y[(int64_t)t * o + p] = f32_to_bf16(v);
  }
#endif
}

// Batches of up to 64 tokens per pass on wide layers (the smallest ones only when their activations do not fit the
// kernel above).  One workgroup = 64 weight rows in four 16-row tiles, every wave walking its tile's whole row (or the
// workgroup's k-slice of it), so all waves consume the same k-stage at the same time and can share its activations: a
// stage of X (TB x 16 tokens x 128 / BITS x 8 k-values) is put into LDS once per workgroup by DMA, swizzled (chunk c
// of token t at position c ^ (t % 16)) so that the fragment reads of 16 tokens hit 16 different bank groups.  NWV = 4:
// one wave per row tile with all TB token blocks.  NWV = 8 (even TB): two waves per row tile, each with half of the
// token blocks; they share the tile's weight ring (each issues half of its loads) and both turn the codes into
// operands, but a SIMD now holds two waves, and one's LDS round trips and integer work run under the other's matrix
// ops (measured at [11008 x 4096]: 21 vs 23 us at 32 tokens, 28 vs 35 at 64).  The weights are streamed as in the
// kernels above (a ring of 2 KB stages per row tile).  The ring is as deep as 160 KB of LDS allow for the stage size
// (8 stages for one token block, 3 for four): memory returns in order, so the weight stream from HBM and the
// activations from the L2 share one prefetch distance.  One barrier per stage makes the stage visible to every wave
// and frees the slot that is refilled next.
// The zero-point term needs sum_k X per (token, group), which does not depend on the weight row: wave w < TB forms it
// for token block w with one extra matrix op per fragment (against ones), chained over the sub-steps of a group, and
// stores the running sum into a table in LDS (no read-modify-write, whose LDS round trips a wave pays in full);
// after the loop every lane adds sum_g (zero - K0 scale)[row, g] * table[token, g] to its outputs, the first factor
// fetched before the loop, held in registers and staged through the LDS the rings have left.  The scales of the 64
// rows sit in LDS too (odd row pitch), so the stage loop issues DMA loads only and its partial waits are exact.
// BITS = 3: the activation side is that of 4 bits (256 k-values per stage, 32 codes per lane group and sub-step); the
// weights of a row tile are streamed in units of three 128-byte stages = 1024 codes = four activation stages, held in
// a ring of two units, and read as 12-byte pieces: lane group kg of sub-step h of a unit owns codes 32 (4 h + kg) .. +
// 31 = the 12 bytes from (4 h + kg) 12 of the row's 384, three dwords that may straddle two 16-byte chunks or two
// stages of the swizzled layout; fragment f of a piece is a 24-bit window whose code pairs are 6-bit fields.  The
// activation ring has three stages for every token-block count.
constexpr int qt_ring_stages(int token_blocks) { return token_blocks == 1 ? 8 : token_blocks == 2 ? 5 : token_blocks == 3 ? 4 : 3; }
constexpr int QT_SLICES_MAX = 8;  // k-slices of a row tile at most
constexpr int QT_ROWQ = 6;  // 16-byte pieces of a 64-row scale / zero block per thread: groups per row <= 96

template <int BITS, int TB, int NWV>
__global__ __launch_bounds__(NWV * 64) void qgemm_tile_kernel(const bf16_t* __restrict__ X,
                                                         const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ scale,
                                                         const float* __restrict__ zero, bf16_t* __restrict__ Y,
                                                         float* __restrict__ part, int T, int t0, int o, int i, int g,
                                                         int sx_pitch) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char tlds[];
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(BITS == 3 || BITS == 4 || BITS == 8, "bits");
  static_assert(TB >= 1 && TB <= 4, "token blocks of 16");
  static_assert(NWV == 4 || (NWV == 8 && TB % 2 == 0), "4 waves, or 8 with the token blocks split in two halves");
  constexpr bool W3 = BITS == 3;  // 3-bit codes: weights in units of three stages (see below), same activation stages as 4 bits
  typedef QsMfma<16> M;
  typedef typename M::acc_t acc_t;
  constexpr int TH = NWV / 4;        // waves per 16-row tile, each with TBW of the token blocks
  constexpr int TBW = TB / TH;
  constexpr int NT = NWV * 64;
  constexpr int KG = 4, NH = 2, NDMA = 2 / TH;  // NDMA: this wave's loads of its row tile's weight stage
  constexpr int QT_NS = W3 ? 3 : qt_ring_stages(TB);
  constexpr int CH = W3 ? 32 : 128 / BITS, KS = 8 * CH, FR = CH / 8, SUB = KG * CH;
  constexpr int WSTAGE = 16 * 128;            // bytes of a weight stage of one row tile
  // ring of a row tile's weights: QT_NS stages, or (3 bits) two units of three stages
  constexpr int WSLOT = W3 ? 3 * WSTAGE : WSTAGE;
  constexpr int WRING = W3 ? 2 * WSLOT : QT_NS * WSTAGE;
  constexpr int XROW = KS * 2;                // bytes of a token's activations in a stage
  constexpr int XSTAGE = TB * 16 * XROW;      // bytes of the shared activation stage
  constexpr int NXW = XSTAGE / 1024 / NWV;    // wave-wide activation loads per wave and stage
  static_assert(NXW >= 1 && NXW * 1024 * NWV == XSTAGE, "the activation stage divides over the waves");
  constexpr int LOADS = NDMA + NXW;           // DMA loads per wave and stage
  constexpr float K0 = BITS == 8 ? 0.f : 128.f + (float)(1 << (BITS - 1));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef gemm::lds_ptr_t lds_ptr_t;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane % 16, kg = lane / 16;
  const int rt = wave & 3, th = wave >> 2;    // row tile and token half of this wave
  const int p0 = blockIdx.x * 64 + rt * 16;   // first row of this wave's tile
  const int p = p0 + ln;
  const int rb = i / 8 * BITS;
  const int G = i / g;
  // k-slice of this workgroup: stages j0 .. j0 + nst - 1 of the row (the whole row when the grid has one slice)
  // (3 bits: a stage here is an activation stage of KS k-values, and slices are whole units of four of them)
  const int nst_row = W3 ? i / KS : rb / 128, slices = gridDim.y, slice = blockIdx.y;
  const int nun = W3 ? (nst_row + 3) / 4 : nst_row, unit = W3 ? 4 : 1;
  const int u0 = slice * (nun / slices) + (slice < nun % slices ? slice : nun % slices);
  const int ucnt = nun / slices + (slice < nun % slices ? 1 : 0);
  const int j0 = u0 * unit;
  const int nst = ((u0 + ucnt) * unit < nst_row ? (u0 + ucnt) * unit : nst_row) - j0;
  const int n_pass = T - t0 < 16 * TB ? T - t0 : 16 * TB;  // tokens of this pass
  // the groups this slice meets: the tables in LDS hold these only, indexed from grp_first
  const int grp_first = j0 * KS / g, groups = ((j0 + nst) * KS - 1) / g - grp_first + 1;
  const int ppr = (groups + 3) / 4;  // 16-byte pieces of a table row
  const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, ones_bits);

  unsigned char* wring = tlds + rt * WRING;  // shared by the waves of the row tile
  unsigned char* xring = tlds + 4 * WRING;
  float* sx = reinterpret_cast<float*>(xring + QT_NS * XSTAGE);  // [TB * 16][sx_pitch] sums of X per token and group
  float* sl = sx + TB * 16 * sx_pitch;                           // [64][sx_pitch] scale of the workgroup's rows

  const __amdgpu_buffer_rsrc_t rsrcW = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(packed), 0, (int)((int64_t)o * rb), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcX = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(X), 0, (int)((int64_t)T * i * 2), 0x00020000);
  unsigned voffW[NDMA], voffX[NXW];
#pragma unroll
  for (int q = 0; q < NDMA; ++q) {  // wave-wide load th NDMA + q of the row tile's stage: rows 8 (th NDMA + q) .. + 7
    const int r = 8 * (th * NDMA + q) + (lane >> 3);
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    voffW[q] = p0 + r < o ? (unsigned)((p0 + r) * rb + chunk * 16) : gemm::OOB_OFFSET;
  }
#pragma unroll
  for (int q = 0; q < NXW; ++q) {  // this wave's pieces of the shared stage: LDS bytes [(wave NXW + q) 1024 + 16 lane, +16)
    const int pos = (wave * NXW + q) * 1024 + lane * 16;
    const int tok = pos / XROW, cpos = (pos % XROW) / 16;
    const int chunk = cpos ^ (tok & 15);
    voffX[q] = t0 + tok < T ? (unsigned)(((int64_t)(t0 + tok) * i) * 2 + chunk * 16) : gemm::OOB_OFFSET;
  }
  auto issue_dma = [&](int j) {  // stage j into ring slot j % QT_NS; past the end of k: zeros, no traffic
    const bool live = j < nst;
    const unsigned kx = live ? (unsigned)(j0 + j) * (unsigned)XROW : gemm::PAST_END_OFFSET;
    unsigned char* xdst = xring + (j % QT_NS) * XSTAGE + wave * NXW * 1024;
    if constexpr (!W3) {
      const unsigned kw = live ? (unsigned)(j0 + j) * 128u : gemm::PAST_END_OFFSET;
      unsigned char* wdst = wring + (j % QT_NS) * WSTAGE;
#pragma unroll
      for (int q = 0; q < NDMA; ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcW, (lds_ptr_t)(wdst + (th * NDMA + q) * 1024), 16, voffW[q] + kw,
                                                 0, 0, 0);
    } else if (j >= 1) {
      // Three stages of weights (1024 codes) serve four activation stages.  Every group of loads carries one stage's
      // worth, so that the count per group - and with it the partial waits - stays what it is for 4 bits: group j
      // brings part (j - 1) % 4 of unit (j - 1) / 4 + 1 (parts 0 .. 2 = its three stages, part 3 = loads that fetch
      // nothing and write zeros over stage 0 of the unit before, which its last two activation stages no longer read
      // and which the next group refills).  The unit is complete with group 4 c, one group before activation stage
      // 4 c, its first user, is waited for; part 0 overwrites stage 0 of the unit two back while that unit's last
      // activation stage reads its stage 2 only.
      const int part = (j - 1) & 3, un = (j - 1) / 4 + 1;
      const bool real = part < 3 && 4 * un < nst;
      const unsigned kb = real ? (unsigned)(3 * (u0 + un) + part) * 128u : gemm::PAST_END_OFFSET;
      unsigned char* wdst = wring + (part < 3 ? (un & 1) * WSLOT + part * WSTAGE : ((un - 1) & 1) * WSLOT);
#pragma unroll
      for (int q = 0; q < NDMA; ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcW, (lds_ptr_t)(wdst + (th * NDMA + q) * 1024), 16, voffW[q] + kb,
                                                 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < NXW; ++q)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcX, (lds_ptr_t)(xdst + q * 1024), 16, voffX[q] + kx, 0, 0, 0);
  };
  const float* srow = sl + (rt * 16 + ln) * sx_pitch;

  // The scale / zero values of the workgroup's 64 weight rows and the slice's groups: each thread fetches up to QT_ROWQ
  // pieces of 4 floats (piece q4 of a row = groups grp_first + 4 q4 .. + 3; rows past the matrix read as zero through
  // the buffer range, values past the slice's groups are fetched but not kept), all requested before the first is used,
  // and puts them into rows of odd pitch.
  const __amdgpu_buffer_rsrc_t rsrcS = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(scale), 0, (int)((int64_t)o * G * 4), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcZ = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(zero), 0, (int)((int64_t)o * G * 4), 0x00020000);
  int piece_row[QT_ROWQ], piece_q4[QT_ROWQ];
#pragma unroll
  for (int q = 0; q < QT_ROWQ; ++q) {
    const int piece = q * NT + (int)threadIdx.x;
    piece_row[q] = piece / ppr;
    piece_q4[q] = piece - piece_row[q] * ppr;
  }
  auto load_rows = [&](const __amdgpu_buffer_rsrc_t& rsrc, float4 (&rows)[QT_ROWQ]) {
#pragma unroll
    for (int q = 0; q < QT_ROWQ; ++q) {
      const int64_t at = ((int64_t)blockIdx.x * 64 + piece_row[q]) * G + grp_first + 4 * piece_q4[q];
      const unsigned off = q * NT + (int)threadIdx.x < 64 * ppr ? (unsigned)(at * 4) : gemm::OOB_OFFSET;
      rows[q] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
    }
  };
  auto store_rows = [&](const float4 (&rows)[QT_ROWQ], float* table) {
#pragma unroll
    for (int q = 0; q < QT_ROWQ; ++q) {
      const float v[4] = {rows[q].x, rows[q].y, rows[q].z, rows[q].w};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (q * NT + (int)threadIdx.x < 64 * ppr && 4 * piece_q4[q] + c < groups)
          table[piece_row[q] * sx_pitch + 4 * piece_q4[q] + c] = v[c];
    }
  };

  acc_t acc[TBW];  // token blocks th TBW .. th TBW + TBW - 1 of this wave's 16 rows
#pragma unroll
  for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[tb][e] = 0.f;

  const unsigned frag_row = ln * 128;
  const int swz = (ln >> 1) & 7;

  const int own = wave < TB ? wave : TB - 1;
  acc_t tx;          // running sums of X over the group in progress, token block `own`
  int tx_grp = -1;   // that group
#pragma unroll
  for (int e = 0; e < 4; ++e) tx[e] = 0.f;
  auto consume = [&](int j) {
    const unsigned char* wsrc = wring + (W3 ? ((j >> 2) & 1) * WSLOT : (j % QT_NS) * WSTAGE) + frag_row;
    const unsigned char* xsrc = xring + (j % QT_NS) * XSTAGE;
    const int st = j0 + (j < nst ? j : nst - 1);
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      // every LDS read of the sub-step is issued before the first use: one exposed latency per sub-step
      u32x4 w;
      if constexpr (!W3) {
        w = *reinterpret_cast<const u32x4*>(wsrc + (((KG * h + kg) ^ swz) << 4));
      } else {
        // sub-step 2 (j % 4) + h of the unit: this lane group's 32 codes are the 12 bytes from (4 sub-step + kg) 12 of
        // the row's 384, three dwords of the swizzled stages (a piece may straddle two chunks or two stages)
        const int piece = (4 * (2 * (j & 3) + h) + kg) * 12;
#pragma unroll
        for (int dw = 0; dw < 3; ++dw) {
          const int byte = piece + 4 * dw;
          const int b = byte & 127;
          w[dw] = *reinterpret_cast<const uint32_t*>(wsrc + (byte >> 7) * WSTAGE + (((b >> 4) ^ swz) << 4) + (b & 15));
        }
        w[3] = 0u;
      }
      bf16x8_t xf[FR][TBW], xo[FR];
#pragma unroll
      for (int f = 0; f < FR; ++f) {
        const int cpos = ((KG * h + kg) * FR + f) ^ ln;  // swizzled chunk position of this lane's token
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
          xf[f][tb] = *reinterpret_cast<const bf16x8_t*>(xsrc + ((th * TBW + tb) * 16 + ln) * XROW + cpos * 16);
        // wave w < TB also sums token block w (read by every wave, so that the reads stay one straight block)
        xo[f] = *reinterpret_cast<const bf16x8_t*>(xsrc + (own * 16 + ln) * XROW + cpos * 16);
      }
      const int grp = (st * KS + h * SUB) / g - grp_first;  // position in the tables
      const float sc = srow[grp];
      __builtin_amdgcn_sched_barrier(0);
      acc_t tw[TBW];
#pragma unroll
      for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
        for (int e = 0; e < 4; ++e) tw[tb][e] = 0.f;
#pragma unroll
      for (int f = 0; f < FR; ++f) {
        const bf16x8_t wf = code_fragment<BITS>(w, f);
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb) tw[tb] = M::mma(xf[f][tb], wf, tw[tb]);
      }
#pragma unroll
      for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[tb][e] = fmaf(sc, tw[tb][e], acc[tb][e]);
      if (wave < TB) {  // (uniform over the wave)
        if (grp != tx_grp) {  // a group starts (the groups are whole numbers of sub-steps)
          tx_grp = grp;
#pragma unroll
          for (int e = 0; e < 4; ++e) tx[e] = 0.f;
        }
#pragma unroll
        for (int f = 0; f < FR; ++f) tx = M::mma(xo[f], ones, tx);
        // Every column of tx holds the same sums: one lane per token stores the running sum of the group (plain
        // stores, the last one of a group leaves the whole sum; this wave is the only writer of the cell).
        if (ln == 0 && j < nst) {
#pragma unroll
          for (int e = 0; e < 4; ++e) sx[(wave * 16 + M::token(e, kg)) * sx_pitch + grp] = tx[e];
        }
      }
    }
  };

  // The first QT_NS - 1 stages are requested, then the scale / zero rows of the 64 weight rows are fetched: the scales
  // go into their table, (zero - K0 scale) stays in registers until the rings are free.
  if constexpr (W3) {  // the first unit of weights whole; the groups below bring the following ones part by part
#pragma unroll
    for (int part = 0; part < 3; ++part)
#pragma unroll
      for (int q = 0; q < NDMA; ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcW, (lds_ptr_t)(wring + part * WSTAGE + (th * NDMA + q) * 1024), 16,
                                                 voffW[q] + (unsigned)(3 * u0 + part) * 128u, 0, 0, 0);
  }
#pragma unroll
  for (int j = 0; j < QT_NS - 1; ++j) issue_dma(j);
  float4 bzrows[QT_ROWQ];
  {
    float4 srows[QT_ROWQ];
    load_rows(rsrcS, srows);
    load_rows(rsrcZ, bzrows);
    store_rows(srows, sl);
#pragma unroll
    for (int q = 0; q < QT_ROWQ; ++q) {
      bzrows[q].x -= K0 * srows[q].x; bzrows[q].y -= K0 * srows[q].y;
      bzrows[q].z -= K0 * srows[q].z; bzrows[q].w -= K0 * srows[q].w;
    }
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(0));  // these stages and the table loads have landed
  __builtin_amdgcn_sched_barrier(0);
  // From here on the only vector-memory operations are the DMA loads: after the DMA of stage j + 1, by the end of
  // stage j, the DMA of stages j + 2 .. j + QT_NS - 1 has been issued.
  static_assert((QT_NS - 2) * LOADS <= 63, "vmcnt is a 6-bit counter");
  for (int j = 0; j < nst; j += 2) {
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_lgkm0());
    __builtin_amdgcn_s_barrier();  // stage j is complete for every wave; every wave is done with stage j - 1
    __builtin_amdgcn_sched_barrier(0);
    issue_dma(j + QT_NS - 1);
    __builtin_amdgcn_sched_barrier(0);
    consume(j);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm((QT_NS - 2) * LOADS));  // stage j + 1 has landed
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_lgkm0());
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    issue_dma(j + QT_NS);
    __builtin_amdgcn_sched_barrier(0);
    consume(j + 1);  // with an odd stage count this is a stage of zeros: it adds nothing
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm((QT_NS - 2) * LOADS));  // stage j + 2 has landed
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_vm(0));
  __syncthreads();  // the sum table is complete and the rings are free

  // (zero - K0 scale) of the workgroup's 64 rows into the ring space, rows padded to an odd pitch
  float* bzl = reinterpret_cast<float*>(tlds);
  const int bz_pitch = sx_pitch;
  store_rows(bzrows, bzl);
  __syncthreads();

  // zero-point term and store: register e of this wave's token block tb is token 16 (th TBW + tb) + 4 kg + e of row p
  const float* bzrow = bzl + (rt * 16 + ln) * bz_pitch;
#pragma unroll 4
  for (int grp = 0; grp < groups; ++grp) {
    const float bz = bzrow[grp];
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        acc[tb][e] = fmaf(bz, sx[((th * TBW + tb) * 16 + M::token(e, kg)) * sx_pitch + grp], acc[tb][e]);
  }
#pragma unroll
  for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int tl = (th * TBW + tb) * 16 + M::token(e, kg), t = t0 + tl;
      if (t < T && p < o) {
        if (part == nullptr) Y[(int64_t)t * o + p] = f32_to_bf16(acc[tb][e]);
        else part[((int64_t)slice * n_pass + tl) * o + p] = acc[tb][e];  // [slice][token of the pass][row]
      }
    }
#endif
}

// Weights resident in registers, activations streamed: the form for a few tokens to a few token blocks.
// The compute units' register files are the largest fast memory of the chip (512 KB each, against 160 KB of LDS), and a
// layer's packed codes divided over the units are small (22.5 MB / 256 = 88 KB).  One workgroup of 16 waves takes NT
// 16-row tiles (tiles blockIdx.x + n gridDim.x) and the whole of k, cut into chunks of 256 k-values: wave w owns chunks
// w, w + 16, ... (CPW of them) of every tile of the workgroup, i.e. NT x CPW units of 16 rows x 256 codes.  Every load of
// the kernel's weight stream - a unit is BITS x 2 dwords per lane - is issued in the first instructions, straight into
// registers: no ring, no stage barriers, and the whole matrix is in flight at once over the chip.  Lane (row r, group
// kq) of a unit holds the two 32-code pieces at k = 128 h + 32 kq (h = 0, 1) of its row; matrix op d of half h takes
// dword-sized fragment d of that piece, so one op covers k = 128 h + {32 kq + 8 d + j}: groups of 128 and more are
// whole numbers of halves.  The activations of a token block (16 tokens x the wave's chunks) are loaded with the same
// k assignment, 16 bytes per lane and op, from the L2; their sums per (token, half) come from ops against ones.  Each
// token block ends with the partial sums of the 16 waves meeting in LDS (double-buffered: one barrier per block) and
// 256 outputs per tile written by 256 threads.  With more than one token block the codes are converted again for
// each block (the registers hold the packed codes, not the operands).  4 bits: the codes of a dword are paired
// (j, j + 4), one shift and one mask-or per pair, and the activation fragment is permuted to match.
// (Exchanging the dwords of a piece over the four lane groups of a row, so that the four lanes of a token read 64
// contiguous bytes per load and the activation loads touch half as many cache lines, changed no time: dropped.)
// Two shapes of workgroup: WV = 16 waves with one token block per pass (TBP = 1; 128 registers per lane: up to 4 units per
// wave), and WV = 8 waves with twice the chunks each and two token blocks per pass (TBP = 2; 256 registers: the codes
// are converted once for 32 tokens, which is what the time per block is made of beyond one block).
constexpr int WR_WAVES = 16;
constexpr int WR_UNITS_MAX = 4;  // units (tiles x chunks) per wave that fit 128 registers

template <int BITS, int NT, int CPW, int WV = WR_WAVES, int TBP = 1>
__global__ __launch_bounds__(WV * 64) void qgemm_wreg_kernel(const bf16_t* __restrict__ X,
                                                                    const uint32_t* __restrict__ packed,
                                                                    const float* __restrict__ scale,
                                                                    const float* __restrict__ zero,
                                                                    bf16_t* __restrict__ Y, float* __restrict__ part,
                                                                    int T, int o, int i, int g) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char wlds[];
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(BITS == 2 || BITS == 3 || BITS == 4 || BITS == 8, "bits");
  static_assert(NT * CPW <= (WV == WR_WAVES ? WR_UNITS_MAX : 6), "units per wave");
  static_assert((WV == 16 && TBP == 1) || (WV == 8 && TBP == 2), "workgroup shapes");
  typedef QsMfma<16> M;
  typedef typename M::acc_t acc_t;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
  constexpr float K0 = BITS == 8 ? 0.f : 128.f + (float)(1 << (BITS - 1));
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 15, kq = lane >> 4;
  const int rb = i / 8 * BITS, G = i / g;
  const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, ones_bits);
  // k-slices (gridDim.y > 1: layers with long rows and few row tiles, whose units would otherwise each read the whole
  // of X for 16 rows): slice s takes chunks s WV CPW .. + WV CPW - 1 and writes binary32 partial sums
  // part[slice][token][row], which qgemm_slices_sum_kernel adds in slice order
  const int chunk0 = (int)blockIdx.y * (WV * CPW) + wave;  // this wave's first chunk; the others follow at WV apart
  const int grp0 = (int)blockIdx.y * (WV * CPW) * 256 / g;  // first group the slice meets; the tables start there
  int Gs = (((int)blockIdx.y + 1) * (WV * CPW) * 256 + g - 1) / g;
  Gs = (Gs < G ? Gs : G) - grp0;
  if (Gs < 1) Gs = 1;

  const __amdgpu_buffer_rsrc_t rsrcW = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(packed), 0, (int)((int64_t)o * rb), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcX = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(X), 0, (int)((int64_t)T * i * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcS = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(scale), 0, (int)((int64_t)o * G * 4), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcZ = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(zero), 0, (int)((int64_t)o * G * 4), 0x00020000);

  // The scale and zero values of the workgroup's rows (NT x 16 rows x G groups each): one 16-byte piece of either table
  // per thread, requested ahead of everything else, and passed on through LDS in rows of odd pitch (a lane reading its
  // row's value of a group per unit straight from memory would touch 16 cache lines per wave-wide load, and the
  // kernel would spend more time on those loads than on the weight stream).  zero is stored as zero - K0 scale.
  const int ppr = (Gs + 3) / 4, pitch = Gs | 1;
  float* tab = reinterpret_cast<float*>(wlds) + 2 * NT * TBP * WV * 256;  // [NT * 16][pitch][scale, zero - K0 scale]
  const bool tab_thread = (int)threadIdx.x < NT * 16 * ppr;
  const int tab_nr = (int)threadIdx.x / ppr, tab_c = (int)threadIdx.x - tab_nr * ppr;
  float tab_sv[4], tab_zv[4];
  {
    const int row = ((int)blockIdx.x + (tab_nr >> 4) * (int)gridDim.x) * 16 + (tab_nr & 15);
    const unsigned off = tab_thread && row < o ? (unsigned)((row * G + grp0 + 4 * tab_c) * 4) : gemm::OOB_OFFSET;
    const float4 sv = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsrcS, off, 0, 0));
    const float4 zv = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsrcZ, off, 0, 0));
    tab_sv[0] = sv.x; tab_sv[1] = sv.y; tab_sv[2] = sv.z; tab_sv[3] = sv.w;
    tab_zv[0] = zv.x; tab_zv[1] = zv.y; tab_zv[2] = zv.z; tab_zv[3] = zv.w;
  }

  // Steps of a token block: the wave's half-chunks (q, h) in order, S = 2 CPW of them.  The activations of a step (four
  // fragments per lane) sit in a ring of D buffers over the steps of all blocks: the step that frees a buffer requests
  // the one D steps ahead into it.
  constexpr int S = 2 * CPW;
  constexpr int D = TBP == 2 ? 2 : CPW == 3 ? 3 : (CPW == 2 && NT == 1) ? 4 : 2;  // (what the registers hold)
  constexpr int WW = BITS == 8 ? 8 : 4;
  // steps whose weights are requested ahead of the tables' barrier: all of them where a wave has two loads only
  // ([4096 x 4096]: 4.4 against 4.7 us at one token), none otherwise ([11008 x 4096]: 6.9 against 7.7 with one step)
  constexpr int PRE = NT * S <= 2 ? S : 0;
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  // (x & mask) | bias as one v_and_or_b32 needs the two constants in registers (one scalar, one vector): they are
  // made opaque so that the compiler keeps them there instead of folding them into two ops with literals.  (The op
  // itself is left to the compiler: written as inline assembly it would hide from the compiler that a vector op
  // wrote the register, and the two wait states a matrix op needs before it reads such a register would be missing.)
  uint32_t pair_mask = 0x000F000Fu, pair_bias = 0x43004300u;
  asm volatile("" : "+s"(pair_mask));
  asm volatile("" : "+v"(pair_bias));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  unsigned xoff[CPW][2];  // token ln of a block, k = chunk 256 + 128 h + 32 kq (+ 8 d: 16 bytes each); halves past i: off
#pragma unroll
  for (int q = 0; q < CPW; ++q)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = (chunk0 + WV * q) * 256 + h * 128;
      xoff[q][h] = k0 < i ? (unsigned)((ln * i + k0 + kq * 32) * 2) : gemm::OOB_OFFSET;
    }
  bf16x8_t xb[D][TBP][4];
  // (The block's first token goes into the per-lane offset, not the scalar one: the range check that makes tokens
  // past T read as zero - and keeps the loads inside X - looks at the per-lane offset only.)
  auto load_x = [&](int buf, int q, int h, int pass) {
#pragma unroll
    for (int t = 0; t < TBP; ++t) {
      const unsigned voff = xoff[q][h] + (unsigned)((pass * TBP + t) * 16 * i * 2);
#pragma unroll
      for (int d = 0; d < 4; ++d)
        xb[buf][t][d] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(rsrcX, voff, d * 16, 0));
    }
  };
#pragma unroll
  for (int st = 0; st < D; ++st) load_x(st, st / 2, st % 2, 0);

  // the weight stream: everything this wave will ever read of it, requested now, in the order of the steps (loads
  // return in order: a step waits for exactly what it needs)
  uint32_t w[NT][CPW][2][WW];
  auto load_w = [&](int st_from, int st_to) {
#pragma unroll
  for (int st = st_from; st < st_to; ++st) {
      const int q = st / 2, h = st % 2;
      const int k0 = (chunk0 + WV * q) * 256 + h * 128;
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        const int row = ((int)blockIdx.x + n * (int)gridDim.x) * 16 + ln;
        const bool live = row < o && k0 < i;
        const unsigned off = live ? (unsigned)(row * rb + (k0 + kq * 32) / 8 * BITS) : gemm::OOB_OFFSET;
        if constexpr (BITS == 4) {
          const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off, 0, 0);
#pragma unroll
          for (int c = 0; c < 4; ++c) w[n][q][h][c] = v[c];
        } else if constexpr (BITS == 3) {
          const u32x3 v = __builtin_amdgcn_raw_buffer_load_b96(rsrcW, off, 0, 0);
#pragma unroll
          for (int c = 0; c < 3; ++c) w[n][q][h][c] = v[c];
          w[n][q][h][3] = 0u;
        } else if constexpr (BITS == 2) {
          const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrcW, off, 0, 0);
          w[n][q][h][0] = v[0]; w[n][q][h][1] = v[1]; w[n][q][h][2] = 0u; w[n][q][h][3] = 0u;
        } else {
          const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off, 0, 0);
          const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off, 16, 0);
#pragma unroll
          for (int c = 0; c < 4; ++c) { w[n][q][h][c] = v0[c]; w[n][q][h][4 + c] = v1[c]; }
        }
      }
    }
  };
  // The tables: written once the two pieces are here (the oldest loads in flight), visible after one barrier - which
  // every wave reaches before it requests its weights: a wave cannot issue its whole stream at once (the memory
  // pipeline of the compute unit takes so many requests), and behind the stream the barrier would complete only when
  // most of it had arrived (3 us into a 6.5 us kernel), with all the arithmetic still to do.
  load_w(0, PRE);
  if (tab_thread) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (4 * tab_c + c < Gs) {
        *reinterpret_cast<float2*>(tab + (tab_nr * pitch + 4 * tab_c + c) * 2) =
            make_float2(tab_sv[c], tab_zv[c] - K0 * tab_sv[c]);
      }
  }
  __syncthreads();
  load_w(PRE, S);
  const float* tab_row = tab + ln * pitch * 2;  // this lane's row of the first tile
  int grp[CPW][2];  // group of each step, capped to the table
#pragma unroll
  for (int q = 0; q < CPW; ++q)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = (chunk0 + WV * q) * 256 + h * 128;
      grp[q][h] = k0 < i ? k0 / g - grp0 : 0;
    }

  float* red = reinterpret_cast<float*>(wlds);  // [2][NT][TBP][WV waves][64 lanes][4]
  const int ntb = (T + 16 * TBP - 1) / (16 * TBP);  // passes of TBP token blocks
  // one token block; par: the block's position in the ring's period (S steps per block, D buffers)
  auto block = [&](auto par, int tb) {
    constexpr int P = decltype(par)::value;
    acc_t acc[NT][TBP];
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int t = 0; t < TBP; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[n][t][e] = 0.f;
#pragma unroll
    for (int st = 0; st < S; ++st) {
      const int q = st / 2, h = st % 2, buf = (P * S + st) % D;
      acc_t xs[TBP];
#pragma unroll
      for (int t = 0; t < TBP; ++t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) xs[t][e] = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d) xs[t] = M::mma(xb[buf][t][d], ones, xs[t]);
        if constexpr (BITS == 4) {
          // 4 bits: the codes of a dword are paired (j, j + 4) - one shift and one mask-or per pair instead of three
          // ops for the pair (2 j, 2 j + 1) - and the activations follow: elements (0 4 1 5 2 6 3 7) of each fragment
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const u32x4 x = __builtin_bit_cast(u32x4, xb[buf][t][d]);
            const u32x4 y = {__builtin_amdgcn_perm(x[2], x[0], 0x05040100u), __builtin_amdgcn_perm(x[2], x[0], 0x07060302u),
                             __builtin_amdgcn_perm(x[3], x[1], 0x05040100u), __builtin_amdgcn_perm(x[3], x[1], 0x07060302u)};
            xb[buf][t][d] = __builtin_bit_cast(bf16x8_t, y);
          }
        }
      }
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        // (the packed codes are made opaque here, so that their conversion is not hoisted out of the loop over the
        // token blocks: the converted operands of every unit would not fit the registers)
#pragma unroll
        for (int c = 0; c < (BITS == 8 ? 8 : BITS); ++c) asm volatile("" : "+v"(w[n][q][h][c]));
        acc_t tw[TBP];
#pragma unroll
        for (int t = 0; t < TBP; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) tw[t][e] = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          bf16x8_t wf;
          if constexpr (BITS == 8) {
            const u32x4 c = {w[n][q][h][4 * (d >> 1)], w[n][q][h][4 * (d >> 1) + 1], w[n][q][h][4 * (d >> 1) + 2],
                             w[n][q][h][4 * (d >> 1) + 3]};
            wf = code_fragment<8>(c, d & 1);
          } else {
            const u32x4 c = {w[n][q][h][0], w[n][q][h][1], w[n][q][h][2], w[n][q][h][3]};
            if constexpr (BITS == 4) {
              u32x4 f;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                f[e] = ((c[d] >> (4 * e)) & pair_mask) | pair_bias;
              }
              wf = __builtin_bit_cast(bf16x8_t, f);
            } else {
              wf = code_fragment<BITS>(c, d);
            }
          }
#pragma unroll
          for (int t = 0; t < TBP; ++t) tw[t] = M::mma(xb[buf][t][d], wf, tw[t]);
        }
        const int gofs = grp[q][h];
        const float2 sz = *reinterpret_cast<const float2*>(tab_row + n * 16 * pitch * 2 + gofs * 2);
#pragma unroll
        for (int t = 0; t < TBP; ++t) {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[n][t][e] = fmaf(sz.x, tw[t][e], fmaf(sz.y, xs[t][e], acc[n][t][e]));
          // units one after the other (their operands do not all fit the registers), each one's sums folded into
          // the outputs before the next starts
          asm volatile("" : "+v"(acc[n][t][0]), "+v"(acc[n][t][1]), "+v"(acc[n][t][2]), "+v"(acc[n][t][3]));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // the buffer is free: the step D ahead goes into it
      const int st2 = (st + D) % S, dtb = (st + D) / S;
      if (tb + dtb < ntb) load_x(buf, st2 / 2, st2 % 2, tb + dtb);
    }
    float* buf = red + (tb & 1) * (NT * TBP * WV * 256);
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int t = 0; t < TBP; ++t)
        *reinterpret_cast<float4*>(buf + (((n * TBP + t) * WV + wave) * 64 + lane) * 4) =
            make_float4(acc[n][t][0], acc[n][t][1], acc[n][t][2], acc[n][t][3]);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < (NT * TBP * 256 + WV * 64 - 1) / (WV * 64); ++it) {
      // thread -> (tile n, block t of the pass, token te of the block, row r): 16 consecutive threads = 16
      // consecutive rows of one token
      const int u = it * (WV / 4) + ((int)threadIdx.x >> 8), idx = (int)threadIdx.x & 255;
      const int r = idx & 15, te = idx >> 4;
      if (u < NT * TBP) {
        const int n = u / TBP, t = u - n * TBP;
        const float* src = buf + u * WV * 256 + ((te >> 2) * 16 + r) * 4 + (te & 3);
        float v = src[0];
#pragma unroll
        for (int wv = 1; wv < WV; ++wv) v += src[wv * 256];
        const int row = ((int)blockIdx.x + n * (int)gridDim.x) * 16 + r, tok = (tb * TBP + t) * 16 + te;
        if (tok < T && row < o) {
          if (part == nullptr) Y[(int64_t)tok * o + row] = f32_to_bf16(v);
          else part[((int64_t)blockIdx.y * T + tok) * o + row] = v;
        }
      }
    }
  };
  if constexpr (S % D == 0) {
    for (int tb = 0; tb < ntb; ++tb) block(std::integral_constant<int, 0>(), tb);
  } else {
    static_assert((2 * S) % D == 0, "the ring's period is two blocks");
    for (int tb = 0; tb < ntb; tb += 2) {
      block(std::integral_constant<int, 0>(), tb);
      if (tb + 1 < ntb) block(std::integral_constant<int, 1>(), tb + 1);
    }
  }
#endif
}

// Y[t0 + tl][p] = sum over the k-slices, in slice order, of part[slice][tl][p]; four rows per thread.
__global__ __launch_bounds__(256) void qgemm_slices_sum_kernel(const float* __restrict__ part, bf16_t* __restrict__ Y,
                                                               int slices, int n_pass, int t0, int o) {
  const int64_t quads = (int64_t)n_pass * o / 4;  // o is a multiple of 8
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= quads) return;
  float4 v = reinterpret_cast<const float4*>(part)[q];
  float4 w[QT_SLICES_MAX];  // every slice requested before the first is added
#pragma unroll
  for (int sl = 1; sl < QT_SLICES_MAX; ++sl)
    if (sl < slices) w[sl] = reinterpret_cast<const float4*>(part)[(int64_t)sl * quads + q];
#pragma unroll
  for (int sl = 1; sl < QT_SLICES_MAX; ++sl)
    if (sl < slices) { v.x += w[sl].x; v.y += w[sl].y; v.z += w[sl].z; v.w += w[sl].w; }
  uint2 out;
  out.x = pack_bf16x2(v.x, v.y);
  out.y = pack_bf16x2(v.z, v.w);
  reinterpret_cast<uint2*>(Y + (int64_t)t0 * o)[q] = out;
}

// rows per workgroup the streaming kernel can use for this layer (0: not at all)
int qgemm_stream_rows(const LayerDims& d, int tokens_in_pass) {
  if (d.bits != 4 && d.bits != 8) return 0;
  const int64_t rb = d.i / 8 * d.bits;
  if (d.i % 8 != 0 || rb % 128 != 0 || d.o * rb >= (1ll << 31)) return 0;
  const int ch = 128 / d.bits;
  if (tokens_in_pass <= 16 && d.g % (4 * ch) == 0) return 16;
  if (d.g % (2 * ch) == 0) return 32;
  return 0;
}

// Whether qgemm_decode_kernel can run this layer (any token count it has LDS for): 2 / 4 / 8 bits, packed rows whose
// 16-byte pieces are aligned, a group a whole number of sub-steps (128 codes; 64 at 8 bits).
bool qgemm_decode_ok(const LayerDims& d) {
  if (d.bits != 2 && d.bits != 4 && d.bits != 8) return false;
  const int64_t rb = d.i / 8 * d.bits;
  if (d.i % 8 != 0 || rb % 16 != 0 || (d.o + 16) * rb >= (1ll << 31) || 16 * d.i * 2 >= (1ll << 31)) return false;
  return d.g % (d.bits == 8 ? 64 : 128) == 0;
}

// How the 64-row tile kernel would run this layer: token blocks per pass (0: not at all), k-slices per row tile,
// the pitch of its tables in LDS (groups a slice can meet, made odd) and the LDS of a pass of tb token blocks (rings,
// sum table, scale table; the zero-point table reuses the rings; 0 where that does not fit).
// One workgroup per compute unit at a time: with one slice it is worth it when the tiles keep most units busy over
// the rounds they need.  Measured at [11008 x 4096] (172 tiles on 256 units) against the k-split streaming kernel:
// 17 vs 23 us at 16 tokens, 23 vs 31 at 32, 33 vs 59 at 64; at [8192 x 8192] (128 tiles) 29 vs 29, 40 vs 30, 59 vs 59.
// With fewer tiles, as many k-slices as fill the units, each at least four stages long.
struct TilePlan {
  int tb_max, slices;
  int pitch[5];
  int64_t lds[5];
};
TilePlan qgemm_tile_plan(const LayerDims& d) {
  TilePlan plan = {0, 1, {1, 1, 1, 1, 1}, {0, 0, 0, 0, 0}};
  // 3 bits: activation stages of 256 k-values, weights in units of three 128-byte stages = four activation stages
  const bool w3 = d.bits == 3 && d.i % 256 == 0 && d.g % 128 == 0 && d.o * (d.i / 8 * 3) < (1ll << 31);
  if (!w3 && qgemm_stream_rows(d, 16) != 16) return plan;
  const int64_t tiles = (d.o + 63) / 64, cus = device_compute_units();
  const int64_t rounds = (tiles + cus - 1) / cus;
  const int64_t ks = w3 ? 256 : 8 * (128 / d.bits), G = d.i / d.g;
  const int64_t nst = d.i / ks;  // activation stages of a row
  if (8 * tiles < 5 * rounds * cus) {
    int64_t want = cus / tiles;
    if (want > nst / 4) want = nst / 4;
    if (want > QT_SLICES_MAX) want = QT_SLICES_MAX;
    if (want < 2) return plan;
    plan.slices = (int)want;
  }
  // stages of the longest slice (3 bits: slices are whole units of four stages)
  const int64_t stages = w3 ? 4 * (((nst + 3) / 4 + plan.slices - 1) / plan.slices) : (nst + plan.slices - 1) / plan.slices;
  int64_t groups = (stages * ks - 1) / d.g + 2;                   // groups it can meet, wherever it starts
  if (groups > G) groups = G;
  if (groups > 4 * (QT_ROWQ * 256 / 64)) return plan;  // table rows longer than a thread's pieces cover
  const int xrow = (int)ks * 2;
  for (int tb = 1; tb <= 4; ++tb) {
    const int64_t rings = w3 ? 4 * (2 * 3 * 2048) + 3 * (int64_t)tb * 16 * xrow
                             : (int64_t)qt_ring_stages(tb) * (4 * 2048 + (int64_t)tb * 16 * xrow);
    // table rows of odd pitch (the 16 rows of a tile read one group together: no bank conflicts); where only the
    // even pitch fits (3 bits, four token blocks, 32 groups: by 512 bytes) that read is serialised instead
    for (int64_t pitch = groups | 1; pitch >= groups; --pitch) {
      const int64_t lds = rings + (int64_t)(tb * 16 + 64) * pitch * 4;
      if (lds <= QD_LDS_MAX && 64 * pitch * 4 <= rings) {  // (the ring depth is not monotonic in tb)
        plan.lds[tb] = lds;
        plan.pitch[tb] = (int)pitch;
        plan.tb_max = tb;
        break;
      }
    }
  }
  return plan;
}

// How the weights-in-registers kernel would run this layer: tiles per workgroup and chunks per wave (nt = 0: not at
// all, or not faster than the streaming forms).  Measured against those (us; T = 1 / 5 / 16 / 33 / 64):
//   4 bits [11008 x 4096] (3 tiles, 1 chunk): 6.9 / 7.6 / 9.9 / 18.2 / 23.9 against 7.2 / 12.6 / 16.9 / 27.1 / 28.1;
//          [16384 x 4096] (4, 1): 8.5 / 9.5 / 11.7 / 21.7 / 28.3 against 9.6 / 17.1 / 22.5 / 27.9 / 29.6;
//          [4096 x 4096] (1, 1): 4.7 / 5.6 / 6.9 / 12.1 / 17.8 against 4.7 / 5.3 / 6.4 / 12.9 / 14.2;
//          [8192 x 8192] (2, 2): 10.2 / 11.0 / 15.0 / 27.5 / 38.6 against 10.0 / 14.6 / 28.6 / 30.1 / 31.5;
//          [4096 x 11008] (1, 3): 9.0 / 10.4 / 15.4 / 30.1 / 45.1 against 8.6 / 9.9 / 15.6 / 24.1 / 25.3 (every
//          compute unit reads the whole of X for its 16 rows: the time per token block grows with the chunks per wave);
//   3 bits [11008 x 4096]: 7.5 / 8.2 / 10.5 / 20.2 / 26.0 against 9.7 / 15.2 / 22.2 / 33.0 / 35.8;
//          [4096 x 11008]: 9.0 / 10.1 / 14.9 / 29.8 / 44.7 against 11.6 / 19.9 / 20.1 / 28.5 / 27.4;
//   2 bits [11008 x 4096]: 7.3 / 8.2 / 10.2 / 20.1 / 25.7 against 7.7 / 13.8 / 18.3 / 43.6 / 54.0;
//          [4096 x 11008]: 8.6 / 9.9 / 14.7 / 29.7 / 44.8 against 10.0 / 11.3 / 25.5 / 40.0 / 55.0;
//   8 bits [4096 x 4096]: 5.7 / 6.2 / 8.3 / 13.8 / 19.1 against 7.3 / 8.2 / 8.6 / 14.5 / 15.0;
//          [8192 x 4096] (2, 1): 7.5 / 8.0 / 10.1 / 19.9 / 25.8 against 9.0 / 13.0 / 16.1 / 22.8 / 22.8.
struct WregPlan {
  int nt, cpw;
  unsigned grid;
  int wv, tbp;  // waves per workgroup, token blocks per pass
  int slices;   // k-slices (partial sums through the caller's workspace)
};
constexpr int WR_SLICE_T_MIN = 8, WR_SLICE_T_MAX = 32;  // token counts the k-sliced form takes
inline int64_t plan_grid_rounds(int64_t tiles, int64_t nt, int64_t cus) { return ((tiles + nt - 1) / nt + cus - 1) / cus; }
// Build-time switches for measurements (the in-register form off; any token count; the 16-wave shape only).
#ifndef L4Q_WREG_SWITCH
#define L4Q_WREG_SWITCH true
#endif
#ifndef L4Q_WREG_ANY
#define L4Q_WREG_ANY false
#endif
#ifndef L4Q_WREG_TWO_BLOCKS
#define L4Q_WREG_TWO_BLOCKS true
#endif
// k-slices the in-register kernel would use for this layer if it had a workspace (1: none): rows of more than 16
// chunks on layers whose row tiles do not fill the compute units more than once
int qgemm_wreg_slices(const LayerDims& d) {
  if (d.bits != 2 && d.bits != 3 && d.bits != 4) return 1;
  const int64_t tiles = (d.o + 15) / 16, chunks = (d.i + 255) / 256, cus = device_compute_units();
  const int64_t slices = (chunks + WR_WAVES - 1) / WR_WAVES;
  if (slices < 2 || slices > WR_UNITS_MAX || tiles > cus || 2 * tiles < cus) return 1;
  return (int)slices;
}

WregPlan qgemm_wreg_plan(const LayerDims& d, bool any_size = false, bool have_workspace = false) {
  WregPlan plan = {0, 0, 0, WR_WAVES, 1, 1};
  if (d.bits != 2 && d.bits != 3 && d.bits != 4 && d.bits != 8) return plan;
  const int64_t rb = d.i / 8 * d.bits;
  if (d.i % 128 != 0 || d.g % 128 != 0 || d.o * rb >= (1ll << 31) || d.T * d.i * 2 >= (1ll << 31) ||
      d.o * (d.i / d.g) * 4 >= (1ll << 31))
    return plan;
  const int64_t tiles = (d.o + 15) / 16, chunks = (d.i + 255) / 256, cus = device_compute_units();
  // Long rows, few row tiles, a workspace: k-slices of 16 chunks, so that a unit holds 2 - 4 tiles x a 16th of their
  // slice and reads a half to a quarter of X, plus one summing launch (4 bits, 8 / 16 tokens: [4096 x 11008] 11.6 / 13.4
  // us against 12.8 / 16.0 for the streaming forms; [4096 x 8192] 9.4 / 10.9 against 8.4 / 15.8 (12.7 in one piece);
  // [2400 x 14336] 10.6 / 12.0 against 17.9 / 22.4; at 17 .. 32 tokens in the 8-wave shape where three tiles do:
  // [4096 x 8192] 11.9 - 14.6 against 14.4 - 15.0, [2400 x 14336] 13.3 - 15.6 against 17.2).
  const int slices = have_workspace ? qgemm_wreg_slices(d) : 1;
  if (slices > 1 && !any_size && d.T >= WR_SLICE_T_MIN && d.T <= WR_SLICE_T_MAX && d.i % d.g == 0) {
    // tiles per workgroup: the fewest with which all slices' workgroups run at once (a second round for a few
    // left-over workgroups would double the time: [4096 x 11008] in 3 slices of 86 x 3 tiles = 258 workgroups)
    int64_t nt = (tiles * slices + cus - 1) / cus;
    while ((tiles + nt - 1) / nt * slices > cus) ++nt;
    const bool two = L4Q_WREG_TWO_BLOCKS && d.T > 16 && nt <= 3;  // 8 waves: a slice is 16 chunks = two per wave
    if (nt <= (d.T > 16 && !two ? 0 : WR_UNITS_MAX) && nt * 16 * (((two ? 16 : WR_WAVES) * 256 / d.g + 1 + 3) / 4) <= (two ? 512 : 1024)) {
      plan.nt = (int)nt;
      plan.cpw = two ? 2 : 1;
      plan.wv = two ? 8 : WR_WAVES;
      plan.tbp = two ? 2 : 1;
      plan.slices = slices;
      plan.grid = (unsigned)((tiles + nt - 1) / nt);
      return plan;
    }
  }
  const int64_t cpw = (chunks + WR_WAVES - 1) / WR_WAVES;
  if (cpw > WR_UNITS_MAX || (d.bits == 4 && cpw == 3)) return plan;  // (4 bits, three chunks: not instantiated)
  int64_t nt = (tiles + cus - 1) / cus;
  if (nt > WR_UNITS_MAX / cpw) nt = WR_UNITS_MAX / cpw;
  if (d.bits == 8) {  // twice the registers per unit: one chunk per wave, two tiles at most
    if (cpw > 1) return plan;
    if (nt > 2) nt = 2;
  }
  if (!any_size) {
    const int64_t T = d.T;
    const bool few_tiles = 2 * tiles < cus;  // (the streaming forms split k further over the idle units)
    // More workgroups than compute units (13B / 70B-class projections; us at 4 / 16 / 24 / 40 tokens): the later rounds
    // do not overlap the first one's latency, and the streaming forms catch up beyond a token block -
    // 4 bits [28672 x 8192] 39.5 / 55.9 / 76.8 / 105 against 46.6 / 67.4 / 76.0 / 98.7, [13824 x 5120] 18.0 / 22.8 /
    // 31.5 / 42.7 against 18.9 / 23.1 / 26.0 / 33.6, [5120 x 13824] (4 chunks per wave) 23.3 / 36.2 against 20.7 / 37.7;
    // 3 bits [13824 x 5120] 19.6 / 24.3 / 34.6 / 46.5 against 26.8 / 26.9 / 28.8 / 40.0;
    // 2 bits [5120 x 13824] 22.7 / 35.0 / 51.4 / 76.2 against 22.8 / 36.1 / 39.7 / 57.4, one token 17 - 37 against 12 - 30.
    const bool many = plan_grid_rounds(tiles, nt, cus) > 1;
    int64_t lo = 1, hi = 0;
    if (d.bits == 4) {
      if (cpw == 1) { lo = nt == 1 ? 17 : 1; hi = nt >= 3 ? 64 : nt == 2 ? 48 : 40; }
      else if (cpw == 2) { lo = nt == 2 ? 3 : 6; hi = nt == 2 ? 40 : 16; }
      else { lo = 3; hi = 16; }
      if (few_tiles) { lo = 17; hi = cpw == 1 ? 64 : 0; }
      if (many) hi = cpw >= 3 ? 0 : hi < 16 ? hi : 16;
    } else if (d.bits == 3) {
      if (cpw == 1) hi = nt >= 3 ? 64 : nt == 2 ? 48 : 40;
      else if (cpw == 2) hi = nt == 2 ? 64 : 16;
      else hi = 16;
      if (few_tiles && cpw == 1) hi = 64;
      if (many) hi = cpw >= 3 ? 8 : hi < 16 ? hi : 16;
    } else if (d.bits == 2) {
      lo = nt == 1 && cpw == 1 ? 3 : 1;
      hi = 64;
      if (few_tiles) lo = 17;
      if (many) { lo = 2; if (cpw >= 3) hi = 16; }
    } else {
      lo = (int64_t)plan_grid_rounds(tiles, nt, cus) > 1 ? 2 : 1;
      hi = lo > 1 ? 16 : 32;
      if (few_tiles) { lo = 17; hi = 48; }
    }
    if (T < lo || T > hi) return plan;
    // Whole passes of two token blocks (17 .. 32 and 49 .. 64 tokens) on layers of up to 16 chunks: 8 waves with two
    // chunks each convert the codes once for both blocks (4 bits: [11008 x 4096] 11.1 / 13.6 us at 17 / 32 tokens
    // against 13.0 / 15.5, 22.7 against 24.3 at 64; [8192 x 4096] 9.3 / 11.9 against 10.9 / 13.1; [4096 x 4096]
    // 7.7 / 10.3 against 8.3 / 10.7; 2 bits [11008 x 4096] at 64 tokens: 22.9 against 25.7).
    const int64_t cpw8 = (chunks + 7) / 8;
    if (L4Q_WREG_TWO_BLOCKS && d.bits != 8 && T > 16 && (T <= 32 || T > 48) && cpw8 <= 2 && nt <= 3 && nt * 16 * ((d.i / d.g + 3) / 4) <= 512) {
      plan.wv = 8;
      plan.tbp = 2;
      plan.nt = (int)nt;
      plan.cpw = (int)cpw8;
      plan.grid = (unsigned)((tiles + nt - 1) / nt);
      return plan;
    }
  }
  plan.nt = (int)nt;
  plan.cpw = (int)cpw;
  plan.grid = (unsigned)((tiles + nt - 1) / nt);
  return plan;
}

template <int BITS>
void launch_qgemm_wreg(const WregPlan& plan, const LayerDims& d, const bf16_t* X, const uint32_t* packed,
                       const float* scale, const float* zero, bf16_t* Y, float* partial, hipStream_t stream) {
  int64_t G = d.i / d.g;  // groups a workgroup's tables hold: all of a row's, or those a k-slice can meet
  if (plan.slices > 1 && (int64_t)plan.wv * plan.cpw * 256 / d.g + 2 < G) G = (int64_t)plan.wv * plan.cpw * 256 / d.g + 2;
  const size_t lds_bytes =
      ((size_t)2 * plan.nt * plan.tbp * plan.wv * 256 + (size_t)2 * plan.nt * 16 * (G | 1)) * sizeof(float);
  float* part = plan.slices > 1 ? partial : nullptr;
#define L4Q_WR(N, C, W, P)                                                                                          \
  do {                                                                                                               \
    if (lds_bytes > 64 * 1024)                                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_wreg_kernel<BITS, N, C, W, P>),                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, QD_LDS_MAX);                             \
    hipLaunchKernelGGL((qgemm_wreg_kernel<BITS, N, C, W, P>), dim3(plan.grid, plan.slices), dim3(W * 64), lds_bytes, \
                       stream, X, packed, scale, zero, Y, part, (int)d.T, (int)d.o, (int)d.i, d.g);                  \
  } while (0)
  const int key = plan.nt * 10 + plan.cpw;
  // (every combination qgemm_wreg_plan can return, and no other)
  if (plan.wv == 8) {
    if constexpr (BITS != 8) {
      if (key == 11) L4Q_WR(1, 1, 8, 2); else if (key == 21) L4Q_WR(2, 1, 8, 2); else if (key == 31) L4Q_WR(3, 1, 8, 2);
      else if (key == 12) L4Q_WR(1, 2, 8, 2); else if (key == 22) L4Q_WR(2, 2, 8, 2); else L4Q_WR(3, 2, 8, 2);
    }
  } else if constexpr (BITS == 8) {
    if (key == 11) L4Q_WR(1, 1, 16, 1); else L4Q_WR(2, 1, 16, 1);
  } else {
    if (key == 11) L4Q_WR(1, 1, 16, 1); else if (key == 21) L4Q_WR(2, 1, 16, 1); else if (key == 31) L4Q_WR(3, 1, 16, 1);
    else if (key == 41) L4Q_WR(4, 1, 16, 1); else if (key == 12) L4Q_WR(1, 2, 16, 1); else if (key == 22) L4Q_WR(2, 2, 16, 1);
    else if (key == 14) L4Q_WR(1, 4, 16, 1);
    else if constexpr (BITS != 4) L4Q_WR(1, 3, 16, 1);  // (4 bits: one register too many, and no faster than the streaming forms)
  }
#undef L4Q_WR
  if (plan.slices > 1) {
    const int64_t quads = d.T * d.o / 4;
    hipLaunchKernelGGL(qgemm_slices_sum_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, partial, Y,
                       plan.slices, (int)d.T, 0, (int)d.o);
  }
}

}  // namespace

void launch_pack_codes(const int8_t* codes, int64_t o, int64_t i, int bits, uint32_t* packed, hipStream_t stream) {
  const int64_t n = o * (bits * i / 32);
  hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, codes, o, i, bits,
                     -(1 << (bits - 1)), packed);
}

bool qgemm_supported(const LayerDims& d) { return (d.bits == 2 || d.bits == 3 || d.bits == 4 || d.bits == 8) && d.i % 64 == 0 && d.g >= 8; }

size_t qgemm_workspace_bytes(const LayerDims& d) {
  const TilePlan plan = qgemm_tile_plan(d);
  size_t tile_bytes = 0, wreg_bytes = 0;
  if (plan.tb_max > 0 && plan.slices > 1)
    tile_bytes = (size_t)plan.slices * 16 * plan.tb_max * (size_t)d.o * sizeof(float);  // [slice][token of a pass][row]
  const int ws = qgemm_wreg_slices(d);
  if (ws > 1) wreg_bytes = (size_t)ws * WR_SLICE_T_MAX * (size_t)d.o * sizeof(float);  // [slice][token][row]
  return tile_bytes > wreg_bytes ? tile_bytes : wreg_bytes;
}

void launch_qgemm(const LayerDims& d, const bf16_t* X, const uint32_t* packed, const float* scale, const float* zero,
                  bf16_t* Y, float* partial, size_t partial_bytes, hipStream_t stream) {
  dim3 grid((unsigned)((d.o + 31) / 32));
  // a few token blocks at most, groups of 128 and more: the packed codes resident in registers
  if (L4Q_WREG_SWITCH) {
    const WregPlan wr =
        qgemm_wreg_plan(d, L4Q_WREG_ANY, partial != nullptr && partial_bytes >= qgemm_workspace_bytes(d));
    if (wr.nt > 0) {
      if (d.bits == 2) launch_qgemm_wreg<2>(wr, d, X, packed, scale, zero, Y, partial, stream);
      else if (d.bits == 3) launch_qgemm_wreg<3>(wr, d, X, packed, scale, zero, Y, partial, stream);
      else if (d.bits == 4) launch_qgemm_wreg<4>(wr, d, X, packed, scale, zero, Y, partial, stream);
      else launch_qgemm_wreg<8>(wr, d, X, packed, scale, zero, Y, partial, stream);
      return;
    }
  }
  // more than 32 tokens: the general kernel reads the weights once per 64 tokens, the streaming form once per 32
  // smallest batches: activations and the tile's scale / zero in LDS
  if (d.T <= 16 && qgemm_decode_ok(d)) {
    const int64_t rb = d.i / 8 * d.bits, ks = 128 * 8 / d.bits, nst = (rb + 127) / 128;
    const int64_t xpitch = (nst * ks * 2 + 1023) / 1024 * 1024 + 16;  // a token's row up to the end of its last stage
    const int64_t xb = d.T * xpitch;
    const int64_t Gp = (nst * ks + d.g - 1) / d.g, pitch = 64 * ((Gp + 63) / 64) + 1;  // whole 64-lane loads per row, odd: no bank conflicts
    const int64_t sbb = 2 * 16 * pitch * 4;
    const int64_t tiles = (d.o + 15) / 16;
    int nsw = tiles <= device_compute_units() ? 8 : 4;
    if (4 * nsw * 16 * 128 + xb + sbb > QD_LDS_MAX) nsw = 4;
    if (4 * nsw * 16 * 128 + xb + sbb > QD_LDS_MAX) nsw = 2;  // (16 tokens of a 4096-wide layer: 17.0 against 18.3 us in 64-row tiles)
    if (xb <= QD_X_MAX && sbb <= QD_SB_MAX && 4 * nsw * 16 * 128 + xb + sbb <= QD_LDS_MAX) {
      const size_t lds_bytes = (size_t)(4 * nsw * 16 * 128 + xb + sbb);
      dim3 sgrid((unsigned)tiles);
      // more than 64 KiB of dynamic LDS has to be allowed per function and device
#define L4Q_QD(B, N)                                                                                                \
  do {                                                                                                              \
    if (lds_bytes > 64 * 1024)                                                                                      \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_decode_kernel<B, N>),                          \
                                hipFuncAttributeMaxDynamicSharedMemorySize, QD_LDS_MAX);                                   \
    hipLaunchKernelGGL((qgemm_decode_kernel<B, N>), sgrid, dim3(256), lds_bytes, stream, X, packed, scale, zero, Y, \
                       (int)d.T, (int)d.o, (int)d.i, d.g, (int)xpitch, (int)pitch);                                 \
  } while (0)
      if (d.bits == 2 && nsw == 2) L4Q_QD(2, 2);
      else if (d.bits == 2 && nsw == 4) L4Q_QD(2, 4);
      else if (d.bits == 2) L4Q_QD(2, 8);
      else if (d.bits == 4 && nsw == 2) L4Q_QD(4, 2);
      else if (d.bits == 4 && nsw == 4) L4Q_QD(4, 4);
      else if (d.bits == 4) L4Q_QD(4, 8);
      else if (nsw == 2) L4Q_QD(8, 2);
      else if (nsw == 4) L4Q_QD(8, 4);
      else L4Q_QD(8, 8);
#undef L4Q_QD
      return;
    }
  }
  // larger batches: 64-row tiles that share each activation stage through LDS, up to 64 tokens per pass
  {
    const TilePlan plan = qgemm_tile_plan(d);
    int tb_max = plan.tb_max, slices = 1;
    if (plan.slices > 1) {  // too few row tiles for one k-slice each: split, if the caller gave room for the partial sums
      // (at 16 tokens or fewer the k-split inside a workgroup wins where it exists: 4 and 8 bits)
      if ((d.T > 16 || d.bits == 3) && partial != nullptr && partial_bytes >= qgemm_workspace_bytes(d)) slices = plan.slices;
      else tb_max = 0;
    }
    if (tb_max > 0) {
      dim3 tgrid((unsigned)((d.o + 63) / 64), (unsigned)slices);
      float* part = slices > 1 ? partial : nullptr;
      for (int t0 = 0; t0 < d.T; t0 += 16 * tb_max) {
        const int n = (int)d.T - t0 < 16 * tb_max ? (int)d.T - t0 : 16 * tb_max;
        int tb = (n + 15) / 16;
        while (plan.lds[tb] == 0) ++tb;  // a form that does not fit: the next larger one (tb_max fits) masks the tokens
        const size_t lds_bytes = (size_t)plan.lds[tb];
        const int pitch = plan.pitch[tb];
#define L4Q_QT(B, N, W)                                                                                               \
  do {                                                                                                               \
    if (lds_bytes > 64 * 1024)                                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_tile_kernel<B, N, W>),                          \
                                hipFuncAttributeMaxDynamicSharedMemorySize, QD_LDS_MAX);                             \
    hipLaunchKernelGGL((qgemm_tile_kernel<B, N, W>), tgrid, dim3(W * 64), lds_bytes, stream, X, packed, scale, zero, \
                       Y, part, (int)d.T, t0, (int)d.o, (int)d.i, d.g, pitch);                                       \
  } while (0)
        if (d.bits == 3) {
          if (tb == 1) L4Q_QT(3, 1, 4); else if (tb == 2) L4Q_QT(3, 2, 8); else if (tb == 3) L4Q_QT(3, 3, 4); else L4Q_QT(3, 4, 8);
        } else if (d.bits == 4) {
          if (tb == 1) L4Q_QT(4, 1, 4); else if (tb == 2) L4Q_QT(4, 2, 8); else if (tb == 3) L4Q_QT(4, 3, 4); else L4Q_QT(4, 4, 8);
        } else {
          if (tb == 1) L4Q_QT(8, 1, 4); else if (tb == 2) L4Q_QT(8, 2, 8); else if (tb == 3) L4Q_QT(8, 3, 4); else L4Q_QT(8, 4, 8);
        }
#undef L4Q_QT
        if (slices > 1) {  // the next pass reuses the partial sums' memory: stream order keeps the two apart
          const int64_t quads = (int64_t)n * d.o / 4;
          hipLaunchKernelGGL(qgemm_slices_sum_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream,
                             partial, Y, slices, n, t0, (int)d.o);
        }
      }
      return;
    }
  }
  if (qgemm_stream_rows(d, 32) != 0 && (d.T <= 32 || d.g < 64)) {
    const int step = d.T <= 16 && qgemm_stream_rows(d, 16) == 16 ? 16 : 32;
    for (int t0 = 0; t0 < d.T; t0 += step) {  // the weight stream is read once per pass
      const int rows = qgemm_stream_rows(d, (int)d.T - t0 < step ? (int)d.T - t0 : step);
      dim3 sgrid((unsigned)((d.o + rows - 1) / rows));
#define L4Q_QS(B, R)                                                                                              \
  hipLaunchKernelGGL((qgemm_stream_kernel<B, R>), sgrid, dim3(256), 0, stream, X, packed, scale, zero, Y, (int)d.T, \
                     t0, (int)d.o, (int)d.i, d.g)
      if (d.bits == 4 && rows == 16) L4Q_QS(4, 16);
      else if (d.bits == 4) L4Q_QS(4, 32);
      else if (rows == 16) L4Q_QS(8, 16);
      else L4Q_QS(8, 32);
#undef L4Q_QS
    }
    return;
  }
#define L4Q_QGEMM(B, N, F)                                                                                  \
  hipLaunchKernelGGL((qgemm_kernel<B, N, F>), grid, dim3(QG_WAVES * 64), 0, stream, X, packed, scale, zero, Y, \
                     (int)d.T, (int)d.o, (int)d.i, d.g, d.qn)
#define L4Q_QGEMM_B(B)                                  \
  do {                                                  \
    if (d.g < 64) L4Q_QGEMM(B, 1, true);                \
    else if (d.T <= 32) L4Q_QGEMM(B, 1, false);         \
    else L4Q_QGEMM(B, 2, false);                        \
  } while (0)
  if (d.bits == 2) L4Q_QGEMM_B(2);
  else if (d.bits == 3) L4Q_QGEMM_B(3);
  else if (d.bits == 4) L4Q_QGEMM_B(4);
  else L4Q_QGEMM_B(8);
#undef L4Q_QGEMM_B
#undef L4Q_QGEMM
}

}  // namespace l4q
