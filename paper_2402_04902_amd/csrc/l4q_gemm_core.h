// Main loop of the bf16 MFMA GEMM for gfx950:  acc[M,N] += A[M,K] . B[N,K]^T  (binary32 accumulate).
//
// One workgroup = 2 x WAVES_N wavefronts (2 x 2 for the weight gradient, 2 x 4 = two per SIMD for the forward and
// dX products) computes a BM x BN macro tile; each wavefront owns a (BM/2) x (BN/WAVES_N) block of 32 x 32
// accumulator tiles fed by v_mfma_f32_32x32x16_bf16.
//
// Operand path.  Both operands are K-contiguous in memory.  Tiles of BK k-values travel
// HBM/L2 -> LDS with buffer_load_dwordx4 ... lds (no VGPR staging): one wave instruction fills
// 1 KiB of LDS, lane l writing bytes [16 l, 16 l + 16).  Rows past the matrix edge are given an
// out-of-range buffer offset, for which the hardware returns zeros, so the loop has no branches.
// LDS holds a ring of NS stages; loads run D = NS - 1 stages ahead of the MFMAs and are waited
// for with a partial s_waitcnt vmcnt(), so HBM latency is covered by D stages of matrix work.
//
// LDS layout.  A stage is BM + BN rows of BK bf16 (64 or 128 bytes).  The 16-byte chunk c of
// row r is stored at chunk position c ^ ((r / RW) % CPR) with CPR chunks per row and RW rows per
// 256 bytes (one sweep over the 64 banks).  The DMA writes (consecutive lanes = consecutive
// positions of a row) and the MFMA fragment reads (consecutive lanes = consecutive rows, same
// logical chunk) both cover all 64 banks once per 16 lanes.
//
// Operand order.  The MFMA is issued as D = Bfrag . Afrag^T, i.e. the accumulator tile holds
// C^T: lane l owns column m = l % 32 of C^T (a row of C) and its 16 registers hold
// n = 8 (e / 4) + 4 (l / 32) + (e % 4).  Four consecutive registers are four consecutive
// n (contiguous in memory for row-major C), which gives 8/16-byte stores and, for the weight
// gradient, makes a lane the owner of one weight row.
#pragma once

#include <type_traits>

#include "l4q_device.h"

namespace l4q {
namespace gemm {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 4;
// Operands are below 1 GiB.  A row outside the matrix gets OOB_OFFSET; a stage past the end of K adds
// PAST_END_OFFSET.  Either one, or both together, lands beyond num_records without wrapping 32 bits.
constexpr unsigned OOB_OFFSET = 0x80000000u;
constexpr unsigned PAST_END_OFFSET = 0x40000000u;

// gfx9 s_waitcnt immediate for "vmcnt(n)" only
constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }
constexpr int waitcnt_lgkm0() { return 15 | (3 << 14) | (7 << 4) | (0 << 8); }

// Hardware workgroup id -> tile.  Ids go round-robin over the 8 XCDs; XCD x gets the x-th
// contiguous band of tile ids, and ids walk GROUP_M tile rows at a time.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  const int xcd = pid % NUM_XCD;
  const int local = pid / NUM_XCD;
  const int per = (total + NUM_XCD - 1) / NUM_XCD;
  const int tall = total % NUM_XCD;
  int id;
  if (tall == 0 || xcd < tall) id = xcd * per + local;
  else id = tall * per + (xcd - tall) * (per - 1) + local;
  const int in_group = GROUP_M * tiles_n;
  const int group = id / in_group;
  const int first_m = group * GROUP_M;
  const int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int rem = id - group * in_group;
  tm = first_m + rem % gsz;
  tn = rem / gsz;
}

template <int BM_, int BN_, int BK_, int NS_, bool PAIR_ = false, int WAVES_N_ = 2>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, NS = NS_;
  static constexpr bool PAIR = PAIR_;                 // stages are loaded two at a time (see mainloop)
  static constexpr int WAVES_M = 2, WAVES_N = WAVES_N_;  // wavefronts: 2 x 2, or 2 x 4 (two per SIMD)
  static constexpr int NW = WAVES_M * WAVES_N;
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;  // 32 x 32 accumulator tiles per wave
  static constexpr int CPR = BK / 8;                  // 16-byte chunks per LDS row
  static constexpr int ROWB = BK * 2;                 // bytes per LDS row
  static constexpr int RW = 256 / ROWB;               // rows per 256 bytes
  static constexpr int RPI = 64 / CPR;                // rows filled by one wave-wide load
  static constexpr int A_INSTR = BM / RPI / NW;       // loads per wave per stage, operand A
  static constexpr int B_INSTR = BN / RPI / NW;
  static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int KK = BK / 16;                  // MFMA k-steps per stage
  static constexpr int D = NS - 1;                    // prefetch distance in stages
  static constexpr int LDS_BYTES = NS * STAGE;
  static_assert(BK == 32 || BK == 64, "BK");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "load split");
  static_assert(KK % 2 == 0, "fragment double buffering assumes an even number of k-steps");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  static_assert(NS >= 3, "the last part of a stage's loads is issued after the wait for the next stage");
  static_assert(!PAIR || (BK == 32 && NS == 5), "paired loading: 64-byte LDS rows, ring of five stages");
};

template <class T>
struct Accum {
  f32x16_t v[T::TM][T::TN];
};

// Runs the whole K loop for the tile (m0, n0) and leaves C^T tiles in `acc`.
//
// Operand forms.  The MFMA wants, per lane, 8 consecutive k of one row.
//  * K-contiguous operand (A_KM / B_KM = false): P[rows, ld] with k along the contiguous axis.  A stage
//    is `rows` LDS rows of BK bf16, XOR-swizzled as described at the top; one ds_read_b128 per fragment.
//  * K-major operand (true): P[k, ld] with the tile's 256 rows along the contiguous axis (dY and X
//    in dWq = dY^T X, Wq in dX = dY Wq).  A stage is BK LDS rows of 512 B exactly as they lie in
//    memory (each wave-wide load brings two full 512 B rows), and the transposition happens on
//    the way to the registers with ds_read_b64_tr_b16: within 16 lanes, lane j supplies the address of
//    4 consecutive elements of row k0 + j / 4 at column 4 (j % 4), and receives column j of rows
//    k0 .. k0 + 3.  Two such reads fill the 8 k-slots of a lane.  The 16-byte chunk c of LDS row k sits
//    at chunk position c ^ 4 (k % 4), which puts the 4 x 32 B a 16-lane group reads, and the two
//    groups of a half-wave, on all 64 banks once.
// Ranges.  rows_a / rows_b: valid tile-axis extent of the operand (M, N).  K: number of k values.
// Anything outside reads as zero through the buffer range check for K-major operands (their row
// axis is k, so num_records ends the matrix in k; out-of-range columns get an out-of-bounds offset).
// A K-contiguous operand reads zeros for rows past its extent but, when K is not a multiple of BK,
// whatever follows in memory for k >= K: the caller pairs it with an operand that is exactly zero there
// (K-major, or zero-padded storage).
// On return every wave has passed a barrier after its last LDS read, so LDS may be reused.
//
// Tail loads (non-paired loop).  The loop keeps issuing loads for the D stages past the end of K so that its wait
// arithmetic stays uniform; by default they carry an out-of-range offset and move nothing.  A caller whose epilogue
// needs a block of memory right after the loop can have those D x (A_INSTR + B_INSTR) loads per wave fetch it
// instead: tail stage q = 0 .. D - 1 lands in ring slot (nk + q) % NS, load c of the A part at byte
// (wave A_INSTR + c) 1024 + 16 lane of the slot, load c of the B part A_BYTES further on, each lane reading 16 bytes
// at byte offset voff_a[c] / voff_b[c] + q * stage_bytes of the buffer (out-of-range offsets read as zero).
struct NoTailLoads {
  static constexpr bool ENABLED = false;
};
template <int NA, int NB>
struct TailLoads {
  static constexpr bool ENABLED = true;
  const void* base;                 // the buffer the tail loads read: base address and size in bytes (< 2 GiB)
  int bytes;
  unsigned voff_a[NA], voff_b[NB];  // per lane
  unsigned stage_bytes;             // added once per tail stage
};

// MASK_A_K (paired loop only): operand A is valid for k < K_a only (K_a a multiple of 8, K - 32 < K_a <= K) and what
// follows a row in memory is the next row, not padding: the 16-byte chunks of the last stage that start at k >= K_a
// get an out-of-range offset and read as zero, so that a NaN or Inf in row m + 1 cannot reach row m of the product
// through 0 x Inf.
// B_BLK (K-contiguous B only): operand B lies in memory in blocks of 32 k-values, B[k / 32][row][k % 32] with all N rows
// of a k-block contiguous (ldb is not used): a stage of the tile is then 256 x 64 contiguous bytes and every wave-wide
// load reads 1 KiB of consecutive addresses, eight whole cache lines, instead of sixteen separate half lines (measured:
// 0.5 .. 1 % of the GEMM; what pays is that the merge + quantize pass, which writes Wq and Wq^T this way, stores whole
// 1 KiB / 4 KiB runs).
template <class T, bool A_KM = false, bool B_KM = false, class Tail = NoTailLoads, bool MASK_A_K = false,
          bool B_BLK = false>
__device__ __forceinline__ void mainloop(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                         int64_t ldb, int M, int N, int K, int m0, int n0, unsigned char* lds,
                                         Accum<T>& acc, const Tail& tail = Tail(), int K_a = 0) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the declaration
  static_assert((!A_KM || T::BM == 256) && (!B_KM || T::BN == 256), "K-major staging is written for 256-wide tiles");
  typedef short s16x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr_t;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS bases in SGPRs
  const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
  static_assert((!A_KM && !B_KM) || T::NW == 4, "K-major staging is written for 2 x 2 waves");

  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(A), 0, (int)((int64_t)(A_KM ? K : M) * lda * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(B), 0, (int)((int64_t)(B_KM ? K : N) * (B_BLK ? (int64_t)K : ldb) * 2), 0x00020000);

  // per-lane source offsets (bytes) of the loads this wave issues each stage
  unsigned voffA[T::A_INSTR], voffB[T::B_INSTR];
  auto setup_voff = [&](auto km, unsigned* voff, int ninstr, int64_t ld, int origin, int extent) {
#pragma unroll
    for (int c = 0; c < ninstr; ++c) {
      const int q = wave * ninstr + c;
      if constexpr (decltype(km)::value) {
        const int kr = q * 2 + (lane >> 5);                    // LDS row = k within the stage
        const int col = origin + (((lane & 31) ^ (4 * (kr & 3))) << 3);
        voff[c] = col < extent ? (unsigned)(((int64_t)kr * ld + col) * 2) : OOB_OFFSET;
      } else {
        const int row = q * T::RPI + lane / T::CPR;
        const int ch = (lane % T::CPR) ^ ((row / T::RW) % T::CPR);
        voff[c] = origin + row < extent ? (unsigned)(((int64_t)(origin + row) * ld + ch * 8) * 2) : OOB_OFFSET;
      }
    }
  };
  static_assert(!B_BLK || (!B_KM && T::BK == 32), "blocked B: K-contiguous, 32-k stages");
  setup_voff(std::integral_constant<bool, A_KM>(), voffA, T::A_INSTR, lda, m0, M);
  // blocked B: a row is T::BK elements long inside its k-block, and a stage further is N rows further
  setup_voff(std::integral_constant<bool, B_KM>(), voffB, T::B_INSTR, B_BLK ? (int64_t)T::BK : ldb, n0, N);
  const unsigned stage_bytes_a = A_KM ? (unsigned)(T::BK * lda * 2) : (unsigned)(T::BK * 2);
  const unsigned stage_bytes_b = B_KM    ? (unsigned)(T::BK * ldb * 2)
                                 : B_BLK ? (unsigned)N * (T::BK * 2)
                                         : (unsigned)(T::BK * 2);

  // per-lane LDS offsets of the MFMA fragments.
  // K-contiguous: row (lane % 32) of a 32-row block, logical chunk 2 kk + lane / 32; block bases are
  // multiples of 16 rows, so the swizzle term depends on the lane only (one offset per k-step).
  unsigned frag_off[T::KK];
  {
    const int r = lane & 31;
    const int sw = (r / T::RW) % T::CPR;
#pragma unroll
    for (int kk = 0; kk < T::KK; ++kk) frag_off[kk] = r * T::ROWB + (((kk * 2 + (lane >> 5)) ^ sw) << 4);
  }
  // K-major: one offset per 32-column block; k-steps and the second half add constants.
  unsigned km_off_a[T::TM], km_off_b[T::TN];
  auto setup_km = [&](unsigned* off, int nblk, int wave_col0) {
    const int j = lane & 15, g16 = lane >> 4;
    const int kr = 8 * (lane >> 5) + (j >> 2);
#pragma unroll
    for (int blk = 0; blk < nblk; ++blk) {
      const int chunk = (wave_col0 + blk * 32) / 8 + 2 * (g16 & 1) + ((j & 3) >> 1);
      off[blk] = kr * 512 + ((chunk ^ (4 * (j >> 2))) << 4) + ((j & 1) << 3);
    }
  };
  if constexpr (A_KM) setup_km(km_off_a, T::TM, wm * T::WTM);
  if constexpr (B_KM) setup_km(km_off_b, T::TN, wn * T::WTN);

  // part `part` of `nparts` of the loads of stage `stage` < nk into ring slot `slot`
  auto issue_loads = [&](int stage, int slot, int part, int nparts) {
    const unsigned ka = (unsigned)stage * stage_bytes_a, kb = (unsigned)stage * stage_bytes_b;
    unsigned char* base = lds + slot * T::STAGE;
#pragma unroll
    for (int c = 0; c < T::A_INSTR; ++c)
      if (c * nparts / T::A_INSTR == part)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)(base + (wave * T::A_INSTR + c) * 1024), 16,
                                                 voffA[c] + ka, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < T::B_INSTR; ++c)
      if (c * nparts / T::B_INSTR == part)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrcB, (lds_ptr_t)(base + T::A_BYTES + (wave * T::B_INSTR + c) * 1024), 16, voffB[c] + kb, 0, 0, 0);
  };
  // the same number of loads for tail stage q (stage nk + q): the caller's block, or nothing (out-of-range offsets)
  auto issue_tail = [&](int q, int slot, int part, int nparts) {
    unsigned char* base = lds + slot * T::STAGE;
    __amdgpu_buffer_rsrc_t rt = rsrcA;
    unsigned kq = PAST_END_OFFSET;
    if constexpr (Tail::ENABLED) {
      rt = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(tail.base), 0, tail.bytes, 0x00020000);
      kq = (unsigned)q * tail.stage_bytes;
    }
#pragma unroll
    for (int c = 0; c < T::A_INSTR; ++c)
      if (c * nparts / T::A_INSTR == part) {
        unsigned v = voffA[c];
        if constexpr (Tail::ENABLED) v = tail.voff_a[c];
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_ptr_t)(base + (wave * T::A_INSTR + c) * 1024), 16, v + kq,
                                                 0, 0, 0);
      }
#pragma unroll
    for (int c = 0; c < T::B_INSTR; ++c)
      if (c * nparts / T::B_INSTR == part) {
        unsigned v = voffB[c];
        if constexpr (Tail::ENABLED) v = tail.voff_b[c];
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_ptr_t)(base + T::A_BYTES + (wave * T::B_INSTR + c) * 1024),
                                                 16, v + kq, 0, 0, 0);
      }
  };

  bf16x8_t fa[2][T::TM], fb[2][T::TN];
  auto read_km = [&](const unsigned char* region, unsigned off, int kk) -> bf16x8_t {
    const unsigned char* p0 = region + off + kk * (16 * 512);
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)p0);
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(p0 + 4 * 512));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  };
  auto read_frags_a = [&](int slot, int kk, int set) {
    const unsigned char* region = lds + slot * T::STAGE;
#pragma unroll
    for (int a = 0; a < T::TM; ++a) {
      if constexpr (A_KM) fa[set][a] = read_km(region, km_off_a[a], kk);
      else fa[set][a] = *reinterpret_cast<const bf16x8_t*>(region + wm * T::WTM * T::ROWB + frag_off[kk] + a * 32 * T::ROWB);
    }
  };
  auto read_frags_b = [&](int slot, int kk, int set) {
    const unsigned char* region = lds + slot * T::STAGE + T::A_BYTES;
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
      if constexpr (B_KM) fb[set][b] = read_km(region, km_off_b[b], kk);
      else fb[set][b] = *reinterpret_cast<const bf16x8_t*>(region + wn * T::WTN * T::ROWB + frag_off[kk] + b * 32 * T::ROWB);
    }
  };
  auto mfma_block = [&](int set) {
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
      for (int b = 0; b < T::TN; ++b)
        acc.v[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][b], fa[set][a], acc.v[a][b], 0, 0, 0);
  };

  const int nk = (K + T::BK - 1) / T::BK;
  constexpr int LOADS = T::A_INSTR + T::B_INSTR;
  static_assert(T::A_INSTR % T::KK == 0 && T::B_INSTR % T::KK == 0, "loads are spread evenly over the k-steps");
  constexpr int LPK = LOADS / T::KK;                 // loads issued per k-step
  constexpr int NDA = T::TM * (A_KM ? 2 : 1);        // LDS read instructions per k-step
  constexpr int NDB = T::TN * (B_KM ? 2 : 1);
  constexpr int NMF = T::TM * T::TN;
  constexpr int EXTRA = NDA + NDB + LPK > NMF ? NDA + NDB + LPK - NMF : 0;  // reads that share a matrix op
  static_assert(2 * EXTRA <= NDA + NDB, "too many LDS reads per matrix op");
  static_assert(!Tail::ENABLED || !T::PAIR, "tail loads are wired into the non-paired loop");
  static_assert(!MASK_A_K || T::PAIR, "k-masking of operand A is wired into the paired loop");
  if constexpr (T::PAIR) {
    // Paired loading for K-contiguous operands.  A stage takes 64 bytes of every operand row, half a 128-byte
    // cache line; when the second half is requested a stage later the line has already left the 32 KiB vector
    // cache, and the L2 delivers every line twice (measured: twice the read sectors of a 64-k stage).  Here the
    // two stages that share a line, 2 j and 2 j + 1, are requested by back-to-back instructions, so the second
    // request meets the line while it is still being filled.  Ring of five stages: while stage s (even) and
    // s + 1 are consumed, pair (s + 2, s + 3) has landed or is landing, and pair (s + 4, s + 5) is issued from the
    // middle of stage s on, as soon as every wave has left stage s, into the slots that stages s - 1 and s vacated.
    // Each pair is therefore issued two and a half stages before its first use.  An odd stage count is rounded up:
    // the extra stage is loaded as zeros.
    static_assert(!T::PAIR || (!A_KM && !B_KM && T::KK == 2), "paired loading is for K-contiguous operands");
    unsigned voffA_last[MASK_A_K ? T::A_INSTR : 1];  // offsets of operand A in the last stage: chunks past K_a masked
    if constexpr (MASK_A_K) {
#pragma unroll
      for (int c = 0; c < T::A_INSTR; ++c) {
        const int row = (wave * T::A_INSTR + c) * T::RPI + lane / T::CPR;
        const int ch = (lane % T::CPR) ^ ((row / T::RW) % T::CPR);
        voffA_last[c] = (nk - 1) * T::BK + ch * 8 < K_a ? voffA[c] : OOB_OFFSET;
      }
    }
    auto issue_pair = [&](int stage0, int slot0, int slot1, int part) {
      const unsigned sb = part == 0 ? stage_bytes_a : stage_bytes_b;
      const unsigned k0 = stage0 < nk ? (unsigned)stage0 * sb : PAST_END_OFFSET;
      const unsigned k1 = stage0 + 1 < nk ? (unsigned)(stage0 + 1) * sb : PAST_END_OFFSET;
      unsigned char* base0 = lds + slot0 * T::STAGE;
      unsigned char* base1 = lds + slot1 * T::STAGE;
      if (part == 0) {
#pragma unroll
        for (int c = 0; c < T::A_INSTR; ++c) {
          const int o = (wave * T::A_INSTR + c) * 1024;
          unsigned v0 = voffA[c], v1 = voffA[c];
          if constexpr (MASK_A_K) {
            v0 = stage0 == nk - 1 ? voffA_last[c] : v0;
            v1 = stage0 + 1 == nk - 1 ? voffA_last[c] : v1;
          }
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)(base0 + o), 16, v0 + k0, 0, 0, 0);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)(base1 + o), 16, v1 + k1, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int c = 0; c < T::B_INSTR; ++c) {
          const int o = T::A_BYTES + (wave * T::B_INSTR + c) * 1024;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)(base0 + o), 16, voffB[c] + k0, 0, 0, 0);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)(base1 + o), 16, voffB[c] + k1, 0, 0, 0);
        }
      }
    };
    constexpr int PAIR_A = 2 * T::A_INSTR, PAIR_B = 2 * T::B_INSTR;  // loads of a pair's two parts
    // the matrix ops of a k-step that are not paired with an LDS read share the loads issued in that k-step
    constexpr int AVAIL = NMF - NDA - NDB;
    static_assert(AVAIL > 0 && (PAIR_A <= AVAIL || PAIR_A == 2 * AVAIL) && (PAIR_B <= AVAIL || PAIR_B == 2 * AVAIL),
                  "one or two loads per remaining matrix op");
    auto spread_loads = [](auto n) {
      constexpr int NL = decltype(n)::value;
      if constexpr (NL <= AVAIL) {
#pragma unroll
        for (int q = 0; q < NL; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        if constexpr (AVAIL > NL) __builtin_amdgcn_sched_group_barrier(0x008, AVAIL - NL, 0);
      } else {
#pragma unroll
        for (int q = 0; q < AVAIL; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
        }
      }
    };
    issue_pair(0, 0, 1, 0);
    issue_pair(0, 0, 1, 1);
    issue_pair(2, 2, 3, 0);
    issue_pair(2, 2, 3, 1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(PAIR_A + PAIR_B));  // the first pair has landed
    __builtin_amdgcn_s_barrier();
    read_frags_a(0, 0, 0);
    read_frags_b(0, 0, 0);
    const int nk2 = (nk + 1) & ~1;
    int slot = 0;
    for (int s = 0; s < nk2; s += 2) {
      int n1 = slot + 1;
      if (n1 == T::NS) n1 = 0;
      int n2 = n1 + 1;
      if (n2 == T::NS) n2 = 0;
      int p0 = slot + 4;
      if (p0 >= T::NS) p0 -= T::NS;
      // stage s, first half: no loads.  Its partner stage landed together with it.
      read_frags_a(slot, 1, 1);
      read_frags_b(slot, 1, 1);
      mfma_block(0);
#pragma unroll
      for (int q = 0; q < NDA + NDB; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMF - NDA - NDB, 0);
      __builtin_amdgcn_sched_barrier(0);  // the matrix ops above stay ahead of the wait: they cover the LDS latency
      __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
      __builtin_amdgcn_s_barrier();  // every wave is done reading `slot`: the pair issued below may refill it
      // stage s, second half, and stage s + 1, first half: the two parts of pair (s + 4, s + 5) go into the slots
      // of stages s - 1 and s as early as those are free (the operands come from the L2 of another XCD or from the
      // memory side more often than not, and every k-step of lead counts: issuing half a stage later costs 1-2 %,
      // a whole stage later 8 %)
      read_frags_a(n1, 0, 0);
      read_frags_b(n1, 0, 0);
      issue_pair(s + 4, p0, slot, 0);
      mfma_block(1);
#pragma unroll
      for (int q = 0; q < NDA + NDB; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      spread_loads(std::integral_constant<int, PAIR_A>{});
      read_frags_a(n1, 1, 1);
      read_frags_b(n1, 1, 1);
      issue_pair(s + 4, p0, slot, 1);
      mfma_block(0);
#pragma unroll
      for (int q = 0; q < NDA + NDB; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      spread_loads(std::integral_constant<int, PAIR_B>{});
      // pair (s + 2, s + 3) was issued an iteration ago; only the pair issued above may still be in flight
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(waitcnt_vm(PAIR_A + PAIR_B));
      __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
      __builtin_amdgcn_s_barrier();
      // stage s + 1, second half: no loads
      read_frags_a(n2, 0, 0);
      read_frags_b(n2, 0, 0);
      mfma_block(1);
#pragma unroll
      for (int q = 0; q < NDA + NDB; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMF - NDA - NDB, 0);
      slot = n2;
    }
  } else {
#pragma unroll
    for (int s = 0; s < T::D; ++s) {
      if (s < nk) issue_loads(s, s, 0, 1);
      else issue_tail(s - nk, s, 0, 1);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    read_frags_a(0, 0, 0);
    read_frags_b(0, 0, 0);

    // Steady state.  Per k-step: the LDS reads of the next k-step, 1/KK of the global loads for stage
    // s + D (stages past the end get an out-of-range offset: no memory traffic, and the vmcnt arithmetic
    // stays uniform), and TM x TN matrix ops, interleaved so that the other two kinds issue in the
    // shadow of the matrix pipeline and the global loads of the four waves do not arrive in one burst.
    // The LDS reads come first and the matrix ops left over come last, so that the wait for the reads
    // at the next stage boundary finds them complete.  Program order is reads, then DMA loads: the DMA
    // loads write LDS and the compiler keeps them behind the reads before them.
    constexpr int REST = NMF - (NDA + NDB - EXTRA + LPK);
    static_assert(REST >= 0, "more LDS reads and loads than matrix ops to hide them behind");
    int slot = 0;
    // one stage; `load_part(kk)` issues part kk of the loads of stage s + D into the slot stage s - 1 has left
    auto stage = [&](auto&& load_part) {
      int pslot = slot + T::D;
      if (pslot >= T::NS) pslot -= T::NS;
      int nslot = slot + 1;
      if (nslot == T::NS) nslot = 0;
#pragma unroll
      for (int kk = 0; kk < T::KK; ++kk) {
        const bool last = kk + 1 == T::KK;
        if (last) {
          // Stage s + 1 must have landed for every wave: all but the loads of stages s + 2 .. s + D issued
          // so far, i.e. (D - 2) whole stages plus this stage's first KK - 1 parts, may still be in flight.
          // All of this wave's LDS reads have returned, so the slot refilled next is free once every wave is here.
          __builtin_amdgcn_sched_barrier(0);  // the matrix ops of the previous k-step are issued before the wait
          __builtin_amdgcn_s_waitcnt(waitcnt_vm((T::D - 2) * LOADS + (T::KK - 1) * LPK));
          __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
          __builtin_amdgcn_s_barrier();
        }
        // after the last stage the reads below fetch stale LDS; the values are never used
        read_frags_a(last ? nslot : slot, last ? 0 : kk + 1, (kk + 1) & 1);
        read_frags_b(last ? nslot : slot, last ? 0 : kk + 1, (kk + 1) & 1);
        load_part(pslot, kk);
        mfma_block(kk & 1);
#pragma unroll
        for (int q = 0; q < EXTRA; ++q) {  // where reads outnumber matrix ops, two reads per matrix op
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
#pragma unroll
        for (int q = 0; q < NDA + NDB - 2 * EXTRA; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int q = 0; q < LPK; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        if constexpr (REST > 0) __builtin_amdgcn_sched_group_barrier(0x008, REST, 0);
      }
      slot = nslot;
    };
    // The stages whose look-ahead stage still lies inside K, then the last D whose loads are the tail loads: two
    // copies of the same straight-line body, no selection inside it.
    const int n_inside = nk > T::D ? nk - T::D : 0;
    int s = 0;
    for (; s < n_inside; ++s) stage([&](int pslot, int kk) { issue_loads(s + T::D, pslot, kk, T::KK); });
    for (; s < nk; ++s) stage([&](int pslot, int kk) { issue_tail(s + T::D - nk, pslot, kk, T::KK); });
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
  __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
  __builtin_amdgcn_s_barrier();
#endif
}

// Row m and first column n of the 4 consecutive outputs held in registers 4 eg .. 4 eg + 3 of
// accumulator tile (a, b), relative to the macro tile origin.
template <class T>
__device__ __forceinline__ void acc_coords(int a, int b, int eg, int& m, int& n) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  m = (wave / T::WAVES_N) * T::WTM + a * 32 + (lane & 31);
  n = (wave % T::WAVES_N) * T::WTN + b * 32 + 8 * eg + 4 * (lane >> 5);
}

}  // namespace gemm
}  // namespace l4q
