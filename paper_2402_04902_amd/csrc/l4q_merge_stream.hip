// Merge + quantize pass, streaming form for bfloat16 storage (Sec. 3.2, Eqs. l4q_Wcombine, l4q_Wquant,
// l4q_Wdequant; the backward form also leaves what the fused weight-gradient kernel needs: Wq^T, the
// d(Wq)/d(scale) factor of Eq. quant_lsq_s with the straight-through mask of Eq. appen_ste in its magnitude, B^T).
//
// Bound: HBM (2 bytes read + 2 written per weight forward, 2 + 4 backward) with a vector-ALU load close behind it,
// so the kernel is built to keep both busy at once:
//  * a wavefront is the unit of work and shares nothing with the other wavefronts of its workgroup (no workgroup
//    barrier anywhere): four wavefronts per SIMD sit in different phases and overlap their loads, matrix ops, LDS
//    round trips, vector arithmetic and stores.  A wavefront owns 64 columns of the weight and walks a run of row
//    blocks of 32 down them (forward: one resident round of wavefronts covers the matrix), with the loads of the next row
//    block in flight while it works on the current one; it has 9 KiB of LDS.
//  * rank sums sum_k B[p,k] A[k,j] on the matrix core as a chain of K = 1 binary32 ops, one per k in ascending order:
//    each step is RN(acc + b a) with the bfloat16 product exact, i.e. the stated sequential order bit for bit.
//    The accumulators come out one column per lane and pass through LDS once to become 4 consecutive columns of 8
//    rows per lane: 16 lanes then cover 128 contiguous bytes of a weight row, a cache line, in every load.
//  * Wq and Wq^T leave in the blocked layout the GEMM reads (32 k-values of all rows together): the forward form
//    stores 256-byte runs, the backward form turns the row block over in LDS and stores 1 KiB runs.
//  * the division w = (Wc - b) / s is not the 11-instruction IEEE expansion per weight.  One lane per (row, group)
//    loads s and b, forms the correctly rounded reciprocal r = RN(1 / s) (hardware estimate, one Newton step, then the
//    choice among the result and its two neighbours by the exact residual 1 - s r), and parks (s, b, r, 1024 s) in
//    LDS; per weight the quotient is  q = x r;  t = fma(-s, q, x);  w = fma(t, r, q)  after clamping x to +-1024 s.
//    With r correctly rounded, q is within one unit of x / s and the corrected w is the correctly rounded quotient
//    (Markstein's theorem on division by multiplication with the reciprocal and one exact-remainder correction), so codes
//    and mask are those of the stated arithmetic.  |x| > 1024 s lies beyond every code grid, where code, mask and
//    factor depend on the sign of x alone.  Scales outside [2^-60, 2^60] take the IEEE divide instead (wave-uniform
//    branch).  l4q_check_fast_divide compares the sequence with the IEEE divide on the GPU for every significand of s.
//  * gamma a power of two (alpha = 2 r, the usual choice): gamma acc is exact, and W0 + gamma acc is one fused
//    multiply-add with the same bits.
// Shapes: bfloat16, rank a multiple of 8, group size >= 32; anything else runs merge_quant_tile_kernel.
#include <type_traits>

#include "l4q_device.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

constexpr int MS_COLS = 256;                     // columns per workgroup: 4 wavefronts x 64
constexpr int MS_THREADS = 256;
#ifndef MS_BWD_WAVES
#define MS_BWD_WAVES 3                           // wavefronts per SIMD of the backward form
#endif
constexpr int MS_SPITCH = 72;                    // floats per row of the sums tile: 64 + 8, and 4 rows = 32 banks
constexpr int MS_WAVE_LDS = 32 * MS_SPITCH * 4;  // 9216; the transposed tile of the backward form (5 KiB) aliases it

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x32_t __attribute__((ext_vector_type(32)));

// RN(1 / s) for a normal s > 0 whose reciprocal is normal: the hardware estimate is within one unit in the last
// place, a Newton step brings it to the correctly rounded value or a neighbour, and the exact residuals 1 - s r
// (a fused multiply-add each; exact where it matters, |residual| <= 2^-24) pick the nearest of the three.
__device__ __forceinline__ float exact_reciprocal(float s) {
  const float r0 = __builtin_amdgcn_rcpf(s);
  const float e = fmaf(-s, r0, 1.f);
  float r = fmaf(e, r0, r0);
  const float e0 = fabsf(fmaf(-s, r, 1.f));
  const float rp = __uint_as_float(__float_as_uint(r) + 1u), rm = __uint_as_float(__float_as_uint(r) - 1u);
  const float ep = fabsf(fmaf(-s, rp, 1.f)), em = fabsf(fmaf(-s, rm, 1.f));
  r = ep < e0 ? rp : r;  // at most one neighbour is closer than r
  r = em < e0 ? rm : r;
  return r;
}

// s for which the reciprocal path is used: 2^-60 <= s <= 2^60 (everything in it then stays a normal number)
__device__ __forceinline__ bool scale_in_fast_range(float s) {
  return __float_as_uint(s) - 0x21800000u <= 0x5D800000u - 0x21800000u;
}

// fl(x / s) from the group's (s, r = RN(1 / s), hi = 1024 s); see the top of the file
__device__ __forceinline__ float fast_quotient(float x, float s, float r, float hi) {
  const float xc = __builtin_amdgcn_fmed3f(x, -hi, hi);
  const float q = xc * r;
  const float t = fmaf(-s, q, xc);
  return fmaf(t, r, q);
}

// What one row block (32 rows x 64 columns) needs from memory.  The weight rows are requested a whole row block
// ahead of their use (two register sets); the factors and the quantizer parameters of the next row block are
// requested as soon as the current one has consumed its own (one set), before its streaming phase.
struct FactorLoads {
  u32x4 bq0, bq1;   // B[p0 + lane % 32, 0 .. 15] (first rank chunk)
  float s, b;       // table role: scale / zero of (row lane % 32, group lane / 32)
};
struct WeightLoads {
  u32x2 w0[8];      // streaming role: W0[p0 + 8 (lane / 16) + rr, 4 columns]
};

// MODE 1: forward (dequantized Wq, [ld_wq / 32][o][32]).  MODE 2: backward (Wq^T, [ld_wqT / 32][i][32]; optionally the
// factor [o, i] and B^T).  MODE 3: export (any of int8 codes, binary32 merged weight, mask; all [o, i]).
// Grid: x = 256-column strips, y = partitions of the row blocks; wavefront w of a workgroup walks the row blocks
// [nrb y / gridDim.y, nrb (y + 1) / gridDim.y) of its 64 columns (forward / export: one resident round of workgroups
// covers the matrix; backward: four rounds' worth of shorter runs).
// Transposed tile of the backward form (64 columns x 32 rows of bf16, column-major): pitch 80 bytes; it takes the place
// of the sums tile once the row block has been streamed
constexpr int MS_TPITCH = 80;
static_assert(64 * MS_TPITCH <= MS_WAVE_LDS, "transposed tile aliases the sums tile");
template <int MODE> constexpr int ms_wave_lds() { return MS_WAVE_LDS; }

// ACH: 16-k chunks of the rank whose A values a wavefront keeps in registers for its whole run (1: ranks up to 16;
// 4: ranks up to 64, further chunks are loaded where they are used).
template <int MODE, bool GAMMA_POW2, int ACH>
__device__ __forceinline__ void merge_quant_stream_body(const LayerDims& d, const bf16_t* __restrict__ W0,
                                                        const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                        const float* __restrict__ scale,
                                                        const float* __restrict__ zero,
                                                        const MergeQuantOut<bf16_t>& out, int nrb,
                                                        unsigned char* lds_all) {
#if defined(__HIP_DEVICE_COMPILE__)
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char* lds = lds_all + wave * ms_wave_lds<MODE>();
  float* S = reinterpret_cast<float*>(lds);
  unsigned char* Tt = lds;  // backward form: the transposed tile, in place of the sums tile
  const int jw = blockIdx.x * MS_COLS + wave * 64;  // first column of this wavefront
  const int i = (int)d.i, o = (int)d.o, r = d.r, g = d.g;
  const int G = i / g;
  const int rb_begin = (int)((int64_t)nrb * blockIdx.y / gridDim.y);
  const int rb_end = (int)((int64_t)nrb * (blockIdx.y + 1) / gridDim.y);
  if constexpr (MODE == 2) {
    // the first column strip also leaves B^T for its rows (zeros from o to the padded width)
    if (blockIdx.x == 0 && out.bT) {
      const int ld = (int)out.ld_wqT;
      const int pa = rb_begin * 32, pe = rb_end * 32 < ld ? rb_end * 32 : ld;
      const int np = pe - pa;
      for (int idx = threadIdx.x; idx < r * np; idx += MS_THREADS) {
        const int k = idx / np;
        const int p2 = pa + idx % np;
        out.bT[(int64_t)k * ld + p2] = p2 < o ? B[(int64_t)p2 * r + k] : (bf16_t)0;
      }
    }
  }
  if (jw >= i) return;  // a whole wavefront past the last column (no workgroup barrier exists to miss)

  // streaming role: 4 consecutive columns and 8 rows of the row block.  Forward: rows 4 rr + lane / 16, so that one
  // store instruction covers 4 consecutive rows (Wq is written in blocks of 32 columns, [j / 32][p][j % 32]: 4 rows of a
  // block are 256 contiguous bytes).  Backward / export: rows 8 (lane / 16) + rr, 8 consecutive rows per lane (a lane's
  // column of the transposed tile is then 16 contiguous bytes).
  constexpr int ROW_G = MODE == 1 ? 1 : 8, ROW_R = MODE == 1 ? 4 : 1;  // row = ROW_G (lane / 16) + ROW_R rr
  const int g16 = lane >> 4, c16 = lane & 15;
  const int j0 = jw + 4 * c16;
  const bool col_ok = j0 < i;
  const int grp_lane = g == 32 ? (c16 >> 3) : 0;  // group of the lane's columns within the wavefront's 64
  // matrix role: lane = column jw + lane of the A operand, row p0 + lane % 32 of the B operand
  const int jm = jw + lane;
  const int l32 = lane & 31;
  // table role: lane = (row lane % 32, group lane / 32) of the row block
  const bool tab_lane = lane < (g == 32 ? 64 : 32);
  const int qtab = jw / g + (lane >> 5);

  const __amdgpu_buffer_rsrc_t rsW0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W0), 0, o * i * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, r * i * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(B), 0, o * r * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(scale), 0, o * G * 4, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsZ = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(zero), 0, o * G * 4, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;
  // outputs of the streaming layout
  const int ld_out = MODE == 1 ? (int)out.ld_wq : i;
  // forward: byte offset of the lane's 4 columns in row 0 of their 32-column block of Wq
  const unsigned wq_col_off = j0 < ld_out ? (unsigned)((((jw >> 5) + (c16 >> 3)) * o * 32 + 4 * (c16 & 7)) * 2) : OOB;
  const __amdgpu_buffer_rsrc_t rsOut = __builtin_amdgcn_make_buffer_rsrc(
      MODE == 1 ? (void*)out.wq : MODE == 2 ? (void*)out.fgrad : (void*)out.codes, 0,
      MODE == 3 ? o * i : o * ld_out * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsMask = __builtin_amdgcn_make_buffer_rsrc(out.mask, 0, o * i, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsWc = __builtin_amdgcn_make_buffer_rsrc(out.wcomb, 0, o * i * 4, 0x00020000);
  const bool want_f = MODE == 2 && out.fgrad != nullptr;

  // A[k, jm] of the first ACH rank chunks, two bfloat16 per register: loaded once per wavefront
  uint32_t apk[8 * ACH];
  const unsigned voffA = jm < i ? (unsigned)(jm * 2) : OOB;
#pragma unroll
  for (int c = 0; c < ACH; ++c) {
    uint32_t araw[16];
#pragma unroll
    for (int k = 0; k < 16; ++k)  // steps past the rank: a valid row is read; the B factor of that step is zero
      araw[k] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsA, (int)voffA, (16 * c + k < r ? 16 * c + k : r - 1) * i * 2, 0);
#pragma unroll
    for (int k = 0; k < 8; ++k) apk[8 * c + k] = araw[2 * k] | (araw[2 * k + 1] << 16);
  }

  // every load of row block rb; past the wavefront's range (or the matrix) the offsets are out of range: nothing moves
  auto request_factors = [&](FactorLoads& F, int rb) {
    const int p0 = rb * 32;
    const bool row_m = rb < rb_end && p0 + l32 < o;
    const unsigned voffB = row_m ? (unsigned)((p0 + l32) * r * 2) : OOB;
    F.bq0 = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)voffB, 0, 0);
    F.bq1 = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)(r > 8 ? voffB + 16u : voffB), 0, 0);
    const unsigned vt = tab_lane && row_m ? (unsigned)(((p0 + l32) * G + qtab) * 4) : OOB;
    F.s = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsS, (int)vt, 0, 0));
    F.b = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsZ, (int)vt, 0, 0));
  };
  auto request_weights = [&](WeightLoads& L, int rb) {
    const int p0 = rb * 32;
    // rows are valid in blocks of 8 (o % 8 == 0).  Backward / export: this lane's 8 rows are all inside or all outside.
    // Forward: rows 4 rr .. 4 rr + 3 of the block are inside or outside together (uniform in the wave): rows past o
    // re-read the block's first rows, and nothing is stored for them.
    const bool lane_rows_ok = MODE == 1 ? true : p0 + 8 * g16 < o;
    const unsigned vw = rb < rb_end && lane_rows_ok && col_ok ? (unsigned)(((p0 + ROW_G * g16) * i + j0) * 2) : OOB;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
      const int rsel = MODE == 1 && p0 + ROW_R * rr >= o ? 0 : ROW_R * rr;
      L.w0[rr] = __builtin_amdgcn_raw_buffer_load_b64(rsW0, (int)vw, rsel * i * 2, 0);
    }
  };

  FactorLoads F;
  auto compute = [&](WeightLoads& L, int rb) {
    const int p0 = rb * 32;
    const bool rows_ok = MODE == 1 ? true : p0 + 8 * g16 < o;  // (forward: decided per row, uniformly)
    // ---- rank sums on the matrix core, k ascending
    f32x32_t sum;
#pragma unroll
    for (int e = 0; e < 32; ++e) sum[e] = 0.f;
    // B[p0 + lane % 32, 16 c .. 16 c + 15] of the chunks 1 .. ACH - 1, requested before the first chunk's matrix ops
    u32x4 bx[ACH > 1 ? ACH - 1 : 1][2];
    if constexpr (ACH > 1) {
#pragma unroll
      for (int c = 1; c < ACH; ++c) {
        const unsigned vb = p0 + l32 < o && 16 * c < r ? (unsigned)((p0 + l32) * r * 2 + 32 * c) : OOB;
        bx[c - 1][0] = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)vb, 0, 0);
        bx[c - 1][1] = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)(16 * c + 8 < r ? vb + 16u : vb), 0, 0);
      }
    }
    {
      const uint32_t bw[8] = {F.bq0[0], F.bq0[1], F.bq0[2], F.bq0[3], F.bq1[0], F.bq1[1], F.bq1[2], F.bq1[3]};
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        // a row of B ends at r: what follows in memory is the next row, not a zero
        const float bk = k < r ? __uint_as_float(k & 1 ? bw[k >> 1] & 0xFFFF0000u : bw[k >> 1] << 16) : 0.f;
        const float ak = __uint_as_float(k & 1 ? apk[k >> 1] & 0xFFFF0000u : apk[k >> 1] << 16);
        sum = __builtin_amdgcn_mfma_f32_32x32x1f32(bk, ak, sum, 0, 0, 0);
      }
    }
    if constexpr (ACH > 1) {
#pragma unroll
      for (int c = 1; c < ACH; ++c) {
        if (16 * c < r) {  // (uniform)
          const uint32_t bw[8] = {bx[c - 1][0][0], bx[c - 1][0][1], bx[c - 1][0][2], bx[c - 1][0][3],
                                  bx[c - 1][1][0], bx[c - 1][1][1], bx[c - 1][1][2], bx[c - 1][1][3]};
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            const float bk = 16 * c + k < r ? __uint_as_float(k & 1 ? bw[k >> 1] & 0xFFFF0000u : bw[k >> 1] << 16) : 0.f;
            const float ak = __uint_as_float(k & 1 ? apk[8 * c + (k >> 1)] & 0xFFFF0000u : apk[8 * c + (k >> 1)] << 16);
            sum = __builtin_amdgcn_mfma_f32_32x32x1f32(bk, ak, sum, 0, 0, 0);
          }
        }
      }
    }
    for (int k0 = 16 * ACH; k0 < r; k0 += 16) {  // chunks beyond those in registers: loaded where they are used
      const unsigned voffB = p0 + l32 < o ? (unsigned)((p0 + l32) * r * 2 + 2 * k0) : OOB;
      const u32x4 q0 = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)voffB, 0, 0);
      const u32x4 q1 = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)(k0 + 8 < r ? voffB + 16u : voffB), 0, 0);
      float af[16];
#pragma unroll
      for (int k = 0; k < 16; ++k)
        af[k] = bf16_to_f32((uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
            rsA, (int)voffA, (k0 + k < r ? k0 + k : r - 1) * i * 2, 0));
      const uint32_t bw[8] = {q0[0], q0[1], q0[2], q0[3], q1[0], q1[1], q1[2], q1[3]};
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const float bk = k0 + k < r ? __uint_as_float(k & 1 ? bw[k >> 1] & 0xFFFF0000u : bw[k >> 1] << 16) : 0.f;
        sum = __builtin_amdgcn_mfma_f32_32x32x1f32(bk, af[k], sum, 0, 0, 0);
      }
    }

    // ---- (row, group) table into the padding of the sums tile: s, b, RN(1 / s), 1024 s
    const bool bad_scale = tab_lane && p0 + l32 < o && !scale_in_fast_range(F.s);
    const bool slow = __builtin_amdgcn_ballot_w64(bad_scale) != 0;  // wave-uniform
    if (tab_lane) {
      const float rc = exact_reciprocal(F.s);
      *reinterpret_cast<float4*>(S + l32 * MS_SPITCH + 64 + 4 * (lane >> 5)) = make_float4(F.s, F.b, rc, F.s * 1024.f);
    }
    request_factors(F, rb + 1);  // this row block has consumed its own
    // ---- sums to the streaming layout: register e of lane l is row 8 ((e % 16) / 4) + 4 (l / 32) + e % 4,
    //      column 32 (e / 16) + l % 32
#pragma unroll
    for (int e = 0; e < 32; ++e)
      S[(8 * ((e & 15) >> 2) + 4 * (lane >> 5) + (e & 3)) * MS_SPITCH + 32 * (e >> 4) + l32] = sum[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- stream: 8 rows x 4 columns per lane.  Forward: the padding columns i .. ld_wq - 1 are written as zeros.
    const unsigned vo_out = MODE == 1 ? (wq_col_off == OOB ? OOB : wq_col_off + (unsigned)((p0 + g16) * 64))
                            : rows_ok && j0 < ld_out ? (unsigned)(((p0 + 8 * g16) * ld_out + j0) * (MODE == 3 ? 1 : 2)) : OOB;
    const int row_bytes = MODE == 1 ? ROW_R * 64 : ld_out * (MODE == 3 ? 1 : 2);
    uint32_t wqpack[4][4];  // backward form: dequantized weights of the row block, [column][row pair]
    // (the padding columns are zeroed with a mask, not a select: a select over the whole quantizer chain is compiled
    // into a branch per row, which cuts the eight rows into pieces that cannot be scheduled together; for the same
    // reason the row guard of the forward form exists only in the instance for the matrix's last, partial row block)
    const uint32_t colmask = col_ok ? 0xFFFFFFFFu : 0u;
    auto stream_rows = [&](auto fast_tag, auto guard_tag) {
      constexpr bool FAST = decltype(fast_tag)::value;
      constexpr bool GUARD_ROWS = decltype(guard_tag)::value;
      float wqprev[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) {
        const int row = ROW_G * g16 + ROW_R * rr;
        const float4 acc = *reinterpret_cast<const float4*>(S + row * MS_SPITCH + 4 * c16);
        const float4 tab = *reinterpret_cast<const float4*>(S + row * MS_SPITCH + 64 + 4 * grp_lane);
        const float s = tab.x, b = tab.y, rc = tab.z, hi = tab.w;
        const float av[4] = {acc.x, acc.y, acc.z, acc.w};
        const float w0[4] = {__uint_as_float(L.w0[rr][0] << 16), __uint_as_float(L.w0[rr][0] & 0xFFFF0000u),
                             __uint_as_float(L.w0[rr][1] << 16), __uint_as_float(L.w0[rr][1] & 0xFFFF0000u)};
        float wc[4], wq[4], fg[4];
        uint32_t cpack = 0, mpack = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          wc[c] = GAMMA_POW2 ? fmaf(d.gamma, av[c], w0[c]) : w0[c] + d.gamma * av[c];
          const float x = wc[c] - b;
          const float w = FAST ? fast_quotient(x, s, rc, hi) : __fdiv_rn(x, s);
          const float cl = __builtin_amdgcn_fmed3f(w, d.qn, d.qp);
          const float code = rintf(cl);
          if (MODE != 3) wq[c] = fmaf(code, s, b);
          if (MODE == 2) fg[c] = cl == w ? code - w : code;  // in range = the clamp changed nothing
          if (MODE == 3) {
            cpack |= ((uint32_t)(uint8_t)(int8_t)(int)code) << (8 * c);
            mpack |= (cl == w ? 1u : 0u) << (8 * c);
          }
        }
        if (MODE == 1) {
          const u32x2 v = {pack_bf16x2(wq[0], wq[1]) & colmask, pack_bf16x2(wq[2], wq[3]) & colmask};
          if (!GUARD_ROWS || p0 + ROW_R * rr < o)  // uniform
            __builtin_amdgcn_raw_buffer_store_b64(v, rsOut, (int)vo_out, rr * row_bytes, 0);
        } else if (MODE == 2) {
          if (want_f) {
            typedef _Float16 h4 __attribute__((ext_vector_type(4)));
            const h4 h = {(_Float16)fg[0], (_Float16)fg[1], (_Float16)fg[2], (_Float16)fg[3]};
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsOut, (int)vo_out, rr * row_bytes, 0);
          }
          // rows 2 h, 2 h + 1 of this lane's 8 share a register per column; rows past o (the zero padding of Wq^T up
          // to its leading dimension) are kept as zeros
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if ((rr & 1) == 0) wqprev[c] = wq[c];
            else wqpack[c][rr >> 1] = rows_ok ? pack_bf16x2(wqprev[c], wq[c]) : 0u;
          }
        } else {
          if (out.codes) __builtin_amdgcn_raw_buffer_store_b32(cpack, rsOut, (int)vo_out, rr * row_bytes, 0);
          if (out.mask) __builtin_amdgcn_raw_buffer_store_b32(mpack, rsMask, (int)vo_out, rr * row_bytes, 0);
          if (out.wcomb) {
            const u32x4 v = {__float_as_uint(wc[0]), __float_as_uint(wc[1]), __float_as_uint(wc[2]), __float_as_uint(wc[3])};
            __builtin_amdgcn_raw_buffer_store_b128(v, rsWc, (int)(vo_out == OOB ? OOB : vo_out * 4u), rr * row_bytes * 4, 0);
          }
        }
      }
    };
    if (MODE == 1 && p0 + 32 > o) {  // last, partial row block of the forward form
      if (!slow) stream_rows(std::true_type{}, std::true_type{});
      else stream_rows(std::false_type{}, std::true_type{});
    } else {
      if (!slow) stream_rows(std::true_type{}, std::false_type{});
      else stream_rows(std::false_type{}, std::false_type{});
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // every lane's reads of the sums tile are done: it may be overwritten
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    if constexpr (MODE == 2) {
      // ---- Wq^T in blocks of 32 rows, [p / 32][j][p % 32]: this row block's 64 columns are 4 KiB of consecutive
      //      addresses.  Through LDS, column-major, then 16 bytes per lane, 1 KiB per store instruction.
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const u32x4 v = {wqpack[c][0], wqpack[c][1], wqpack[c][2], wqpack[c][3]};
        *reinterpret_cast<u32x4*>(Tt + (4 * c16 + c) * MS_TPITCH + 16 * g16) = v;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const int ld = (int)out.ld_wqT;
      const __amdgpu_buffer_rsrc_t rsT = __builtin_amdgcn_make_buffer_rsrc(out.wqT, 0, i * ld * 2, 0x00020000);
      const int ch = lane & 3;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int col = it * 16 + (lane >> 2);
        const u32x4 v = *reinterpret_cast<const u32x4*>(Tt + col * MS_TPITCH + ch * 16);
        const unsigned vo = jw + col < i ? (unsigned)(((rb * i + jw + col) * 32 + 8 * ch) * 2) : OOB;
        __builtin_amdgcn_raw_buffer_store_b128(v, rsT, (int)vo, 0, 0);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();  // the tile is read out: the next row block's sums may overwrite it
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  };

  // Row blocks alternate between two register sets, so that the weight rows of the next row block are in flight while
  // this one is worked on.
  int rb = rb_begin;
  request_factors(F, rb);
  WeightLoads L0, L1;
  request_weights(L0, rb);
  while (rb < rb_end) {
    request_weights(L1, rb + 1);
    compute(L0, rb);
    if (++rb >= rb_end) break;
    request_weights(L0, rb + 1);
    compute(L1, rb);
    ++rb;
  }
#endif
}

// Forward and export: 4 workgroups (16 wavefronts, 144 KiB of LDS) per compute unit.  Backward: MS_BWD_WAVES (the
// dequantized weights of a row block wait in registers for the transposition: 152 registers per lane).
template <bool GAMMA_POW2, int ACH = 1>
__global__ __launch_bounds__(MS_THREADS) __attribute__((amdgpu_waves_per_eu(ACH == 1 ? 4 : 3, ACH == 1 ? 4 : 3)))
void merge_quant_stream_fwd_kernel(LayerDims d, const bf16_t* __restrict__ W0, const bf16_t* __restrict__ A,
                                   const bf16_t* __restrict__ B, const float* __restrict__ scale,
                                   const float* __restrict__ zero, MergeQuantOut<bf16_t> out, int nrb) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * ms_wave_lds<1>()];
  merge_quant_stream_body<1, GAMMA_POW2, ACH>(d, W0, A, B, scale, zero, out, nrb, lds_all);
}
template <bool GAMMA_POW2>
__global__ __launch_bounds__(MS_THREADS) __attribute__((amdgpu_waves_per_eu(MS_BWD_WAVES, MS_BWD_WAVES)))
void merge_quant_stream_bwd_kernel(LayerDims d, const bf16_t* __restrict__ W0, const bf16_t* __restrict__ A,
                                   const bf16_t* __restrict__ B, const float* __restrict__ scale,
                                   const float* __restrict__ zero, MergeQuantOut<bf16_t> out, int nrb) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * ms_wave_lds<2>()];
  merge_quant_stream_body<2, GAMMA_POW2, 1>(d, W0, A, B, scale, zero, out, nrb, lds_all);
}
template <bool GAMMA_POW2>
__global__ __launch_bounds__(MS_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4)))
void merge_quant_stream_export_kernel(LayerDims d, const bf16_t* __restrict__ W0, const bf16_t* __restrict__ A,
                                      const bf16_t* __restrict__ B, const float* __restrict__ scale,
                                      const float* __restrict__ zero, MergeQuantOut<bf16_t> out, int nrb) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * ms_wave_lds<3>()];
  merge_quant_stream_body<3, GAMMA_POW2, 1>(d, W0, A, B, scale, zero, out, nrb, lds_all);
}

// ------------------------------------------------------------------ check of the reciprocal-based quotient
// For significand m of s (bits 0 .. 22) and three exponents, compares exact_reciprocal(s) with the IEEE 1 / s and
// fast_quotient with the IEEE x / s for x = s t pushed -5 .. +5 units in the last place, t every rounding tie k + 1/2
// (-128 <= k < 128) and every grid end of 2 .. 8 bits.  counts[0] += wrong reciprocals, counts[1] += wrong quotients,
// counts[2] += quotients compared.
__global__ __launch_bounds__(256) void check_fast_divide_kernel(uint32_t first, uint32_t count,
                                                                unsigned long long* __restrict__ counts) {
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  unsigned long long bad_r = 0, bad_q = 0, n = 0;
  if (idx < count) {
    const uint32_t m = (first + idx) & 0x7FFFFFu;
    const int expos[3] = {127 - 9, 127, 127 + 6};
    for (int ei = 0; ei < 3; ++ei) {
      const float s = __uint_as_float(((uint32_t)expos[ei] << 23) | m);
      const float rc = exact_reciprocal(s);
      if (__float_as_uint(rc) != __float_as_uint(__fdiv_rn(1.f, s))) ++bad_r;
      const float hi = s * 1024.f;
      for (int t2 = -256; t2 < 256 + 14; ++t2) {
        float t;
        if (t2 < 256) {
          if ((t2 & 1) == 0) continue;  // odd halves: k + 1/2
          t = 0.5f * (float)t2;
        } else {
          const int n2 = 2 + (t2 - 256) / 2;
          t = (t2 - 256) & 1 ? (float)((1 << (n2 - 1)) - 1) : -(float)(1 << (n2 - 1));
        }
        const float x0 = s * t;
        for (int u = -5; u <= 5; ++u) {
          const float x = __uint_as_float(__float_as_uint(x0) + (uint32_t)u);  // sign-magnitude: +-u ulps in magnitude
          const float want = __fdiv_rn(x, s);
          const float got = fast_quotient(x, s, rc, hi);
          if (__float_as_uint(want) != __float_as_uint(got)) ++bad_q;
          ++n;
        }
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) {
    bad_r += __shfl_xor(bad_r, off, 64);
    bad_q += __shfl_xor(bad_q, off, 64);
    n += __shfl_xor(n, off, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(&counts[0], bad_r);
    atomicAdd(&counts[1], bad_q);
    atomicAdd(&counts[2], n);
  }
}

}  // namespace

bool merge_quant_stream_supported(const LayerDims& d, const MergeQuantOut<bf16_t>& out) {
  const bool misc = out.codes || out.wcomb || out.mask;
  const bool fwd = out.wq && !out.wqT && !out.fgrad && !misc;
  const bool bwd = !out.wq && out.wqT && !misc;
  const bool exp = !out.wq && !out.wqT && !out.fgrad && misc;
  const bool blocks = (!out.wq || out.ld_wq % 32 == 0) && (!out.wqT || out.ld_wqT % 32 == 0);
  return (fwd || bwd || exp) && blocks && d.r % 8 == 0 && d.g >= 32;
}

void launch_merge_quant_stream(const LayerDims& d, const bf16_t* W0, const bf16_t* A, const bf16_t* B,
                               const float* scale, const float* zero, const MergeQuantOut<bf16_t>& out,
                               hipStream_t stream) {
  const int mode = out.wq ? 1 : out.wqT ? 2 : 3;
  const int64_t rows = mode == 2 && out.ld_wqT > d.o ? out.ld_wqT : d.o;
  const int nrb = (int)((rows + 31) / 32);
  // one resident round: 4 (backward: 3) workgroups per compute unit, each wavefront walking a run of row blocks
  const int strips = (int)((d.i + MS_COLS - 1) / MS_COLS);
  // Forward form at ranks above 16: A for four chunks in registers, 3 wavefronts per SIMD (rank 64: 111 against 134 us;
  // the backward form, which would be down to 2 wavefronts per SIMD, does not gain: 124 against 120 us)
  const bool wide = d.r > 16 && mode == 1;
  int parts = (mode == 2 ? MS_BWD_WAVES : wide ? 3 : 4) * device_compute_units() / strips;
  // backward: four times as many, shorter runs (about two row blocks each), handed out as workgroups finish: its
  // wavefronts are fewer and their phases longer, and one round of 5-or-6-block runs ends ragged (stand-alone 62-65
  // against 68-75 us; inside a training step 65 against 66)
  if (mode == 2) parts *= 4;
  if (parts < 1) parts = 1;
  if (parts > nrb) parts = nrb;
  dim3 grid((unsigned)strips, (unsigned)parts);
  // gamma acc is exact when gamma is a power of two >= 1 (no underflow of the product)
  const uint32_t gb = __builtin_bit_cast(uint32_t, d.gamma);
  const bool pow2 = (gb & 0x807FFFFFu) == 0 && d.gamma >= 1.f && d.gamma <= 1048576.f;
#define L4Q_MS_LAUNCH(K, ...) \
  hipLaunchKernelGGL((K<__VA_ARGS__>), grid, dim3(MS_THREADS), 0, stream, d, W0, A, B, scale, zero, out, nrb)
  if (mode == 1 && wide) { if (pow2) L4Q_MS_LAUNCH(merge_quant_stream_fwd_kernel, true, 4); else L4Q_MS_LAUNCH(merge_quant_stream_fwd_kernel, false, 4); }
  else if (mode == 1) { if (pow2) L4Q_MS_LAUNCH(merge_quant_stream_fwd_kernel, true); else L4Q_MS_LAUNCH(merge_quant_stream_fwd_kernel, false); }
  else if (mode == 2) { if (pow2) L4Q_MS_LAUNCH(merge_quant_stream_bwd_kernel, true); else L4Q_MS_LAUNCH(merge_quant_stream_bwd_kernel, false); }
  else { if (pow2) L4Q_MS_LAUNCH(merge_quant_stream_export_kernel, true); else L4Q_MS_LAUNCH(merge_quant_stream_export_kernel, false); }
#undef L4Q_MS_LAUNCH
}

void launch_check_fast_divide(uint32_t first, uint32_t count, unsigned long long* counts, hipStream_t stream) {
  hipLaunchKernelGGL(check_fast_divide_kernel, dim3((count + 255u) / 256u), dim3(256), 0, stream, first, count, counts);
}

}  // namespace l4q
