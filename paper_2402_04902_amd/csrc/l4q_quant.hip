// Merge + quantize pass, integer-code export, min/max initialisation.
//
// merge_quant_tile_kernel is the HBM-streaming prologue of both passes: it reads W0 once with
// coalesced 8/16-byte loads, adds the rank-r update from registers, applies the group-wise
// quantizer and writes whichever outputs were asked for (dequantized Wq, its transpose, the
// per-element d(Wq)/d(scale) factor, int8 codes, the binary32 merged weight, the mask).
#include <type_traits>

#include "l4q_device.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------ merge + quantize, tiled
// Block tile: MQ_ROWS weight rows x 256 columns, 8 waves.  A thread owns 4 consecutive columns (one
// 8- or 16-byte load of W0 per row, 512 B / 1 KiB contiguous per wave) and its wave walks MQ_RPW
// rows.  The rank loop runs k-outer: A[k, 4 columns] is unpacked once and used for all rows, B[p, k]
// is wave-uniform and comes through scalar loads, and the running sums of all rows stay
// in registers, which keeps the k-ascending summation order for any rank.
// Every load is unconditional (clamped address, value discarded where out of range) so that the
// W0 / scale / zero loads of all rows are in flight while the rank loop runs.
constexpr int MQ_ROWS = 64;
constexpr int MQ_COLS = 256;
constexpr int MQ_THREADS = 512;
constexpr int MQ_RPW = MQ_ROWS / (MQ_THREADS / 64);  // rows per wave = 8
constexpr int MQ_KC = 16;                            // rank chunk
constexpr int MQ_TROW = 144;                         // bytes per row of the transposed LDS tile: 64 bf16 + 16 B pad

template <class T> struct Raw4;
template <> struct Raw4<float> { typedef float4 type; };
template <> struct Raw4<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ void unpack4(const float4& r, float (&v)[4]) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
__device__ __forceinline__ void unpack4(const uint2& r, float (&v)[4]) {
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
}

// acc[rr][c] = sum_k B[pw + rr, k] * A[k, jc + c], k ascending, for the MQ_RPW rows of a wave and the 4 columns
// of a lane (binary32 storage; bfloat16 storage takes lora_rows_mfma).  Rows past o are clamped (their sums are
// never used).  A row of B is wave-uniform: it is fetched with scalar loads and each B[p, k] reaches the
// multiply-add as a scalar operand.
template <class T> struct BWord;
template <> struct BWord<float> { static constexpr int PER = 1; };   // B values per 32-bit word
template <> struct BWord<bf16_t> { static constexpr int PER = 2; };
__device__ __forceinline__ float bword_value(const float*, uint32_t w, int) { return __uint_as_float(w); }
__device__ __forceinline__ float bword_value(const bf16_t*, uint32_t w, int half) {
  return __uint_as_float(half ? (w & 0xFFFF0000u) : (w << 16));
}

template <class T>
__device__ __forceinline__ void lora_rows(const LayerDims& d, const T* __restrict__ A, const T* __restrict__ B,
                                          unsigned jc, int64_t pw, int lane, float (&acc)[MQ_RPW][4]) {
  typedef typename Raw4<T>::type raw4_t;
  constexpr int PER = BWord<T>::PER;
#pragma unroll
  for (int rr = 0; rr < MQ_RPW; ++rr)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[rr][c] = 0.f;
  {  // rows of B are whole 32-bit words (binary32 storage; bfloat16 rows with an even rank): scalar path, any rank
    const int nw = d.r / PER;
    const uint32_t* Bw = reinterpret_cast<const uint32_t*>(B);
    const uint32_t* brow[MQ_RPW];
#pragma unroll
    for (int rr = 0; rr < MQ_RPW; ++rr) brow[rr] = Bw + (pw + rr < d.o ? pw + rr : d.o - 1) * nw;
    const T* ak = A + jc;
#pragma unroll 2
    for (int w = 0; w < nw; ++w) {
      uint32_t bw[MQ_RPW];
#pragma unroll
      for (int rr = 0; rr < MQ_RPW; ++rr) bw[rr] = brow[rr][w];
#pragma unroll
      for (int h = 0; h < PER; ++h) {
        float a[4];
        unpack4(*reinterpret_cast<const raw4_t*>(ak), a);
        ak += d.i;
#pragma unroll
        for (int rr = 0; rr < MQ_RPW; ++rr) {
          const float bk = bword_value((const T*)nullptr, bw[rr], h);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[rr][c] = lora_mac<T>(acc[rr][c], bk, a[c]);
        }
      }
    }
  }
}

// The same sums on the matrix core (bfloat16 storage only).  A product of two bfloat16 values is exact in
// binary32, so step k of the stated chain is acc = RN(acc + B[p,k] A[k,j]): exactly what one
// v_mfma_f32_32x32x1_2b_f32 does for 2 x 32 x 32 outputs (K = 1: there is nothing else to add and nothing to
// reorder; checked bit for bit against fmaf chains on 8.4 M sums).  r such instructions in k order give the
// stated sums for a 32-row x 64-column block per wave; a rank that does not fill a chunk of 16 is padded with
// zero factors, which leave the sums unchanged.  The accumulators come out one column per lane, so they pass
// through LDS once to reach the 4-columns-of-a-row layout of the streaming code below.
// f32_tile: MQ_ROWS x MQ_FPITCH floats of LDS.  Contains two barriers; every wave must call it.
constexpr int MQ_FPITCH = MQ_COLS + 8;  // 4 rows further = 32 banks further: the two half-waves write different banks
constexpr int MQ_F32_TILE = MQ_ROWS * MQ_FPITCH * 4 + MQ_KC * MQ_COLS * 2;  // sums + the A panel of a chunk

// `after_first_loads` runs once, right after the first chunk's factor loads have been issued: the caller requests
// its row data there.  Loads complete in issue order, so requesting the HBM stream first would make the matrix ops
// wait for it.
template <class F>
__device__ __forceinline__ void lora_rows_mfma(const LayerDims& d, const bf16_t* __restrict__ A,
                                               const bf16_t* __restrict__ B, int64_t jblk, int64_t pblk, int lane,
                                               int wave, float* f32_tile, float (&acc)[MQ_RPW][4],
                                               F&& after_first_loads) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef float f32x32_t __attribute__((ext_vector_type(32)));
  static_assert(MQ_ROWS == 64 && MQ_COLS == 256 && MQ_THREADS == 512, "8 waves = 2 row blocks x 4 column blocks");
  const int rb = wave >> 2, cb = wave & 3;
  const int64_t p = pblk + 32 * rb + (lane & 31);
  const bf16_t* brow = B + (p < d.o ? p : d.o - 1) * d.r;
  f32x32_t sum;
#pragma unroll
  for (int e = 0; e < 32; ++e) sum[e] = 0.f;
  // Few, wide loads: the 16 ranks of a row of B are contiguous (two 16-byte loads per lane where rows are 16-byte
  // aligned); the A panel of the chunk (16 ranks x 256 columns) is fetched once per workgroup, 16 bytes per
  // thread, and handed to the column-per-lane layout through LDS.
  bf16_t* a_lds = reinterpret_cast<bf16_t*>(f32_tile + MQ_ROWS * MQ_FPITCH);  // [MQ_KC][MQ_COLS]
  const int tid = threadIdx.x;
  const int ak = tid >> 5, acols = 8 * (tid & 31);
  const bool b_vec = (d.r & 7) == 0;
  auto chunk = [&](int k0, auto&& between) {
    uint4 apanel = make_uint4(0u, 0u, 0u, 0u);
    {
      const int kc = k0 + ak < d.r ? k0 + ak : d.r - 1;
      const int64_t jc8 = jblk + acols < d.i ? jblk + acols : 0;
      apanel = *reinterpret_cast<const uint4*>(A + (int64_t)kc * d.i + jc8);
    }
    uint4 bq[2];
    bf16_t braw[MQ_KC];
    if (b_vec) {
      bq[0] = *reinterpret_cast<const uint4*>(brow + k0);
      bq[1] = *reinterpret_cast<const uint4*>(brow + (k0 + 8 < d.r ? k0 + 8 : k0));
    } else {
#pragma unroll
      for (int k = 0; k < MQ_KC; ++k) braw[k] = brow[k0 + k < d.r ? k0 + k : d.r - 1];
    }
    __builtin_amdgcn_sched_barrier(0);  // the factor loads are in flight before anything waits for one of them
    between();                          // the caller's row data: issued behind them
    __builtin_amdgcn_sched_barrier(0);
    *reinterpret_cast<uint4*>(a_lds + ak * MQ_COLS + acols) = apanel;
    __syncthreads();
    if (b_vec) {
      const uint32_t w[8] = {bq[0].x, bq[0].y, bq[0].z, bq[0].w, bq[1].x, bq[1].y, bq[1].z, bq[1].w};
#pragma unroll
      for (int k = 0; k < MQ_KC; ++k) braw[k] = (bf16_t)(k & 1 ? w[k >> 1] >> 16 : w[k >> 1] & 0xFFFFu);
    }
#pragma unroll
    for (int k = 0; k < MQ_KC; ++k) {
      const bf16_t araw = a_lds[k * MQ_COLS + 64 * cb + lane];
      const float b = k0 + k < d.r ? bf16_to_f32(braw[k]) : 0.f, a = k0 + k < d.r ? bf16_to_f32(araw) : 0.f;
      sum = __builtin_amdgcn_mfma_f32_32x32x1f32(b, a, sum, 0, 0, 0);
    }
    __syncthreads();  // the panel may be overwritten by the next chunk
  };
  chunk(0, after_first_loads);  // straight-line code: the waits of this chunk then count the row loads behind it
  for (int k0 = MQ_KC; k0 < d.r; k0 += MQ_KC) chunk(k0, [] {});
  // register e of lane l: block e / 16 (columns 32 (e / 16) + l % 32), row 8 ((e % 16) / 4) + 4 (l / 32) + e % 4
#pragma unroll
  for (int e = 0; e < 32; ++e) {
    const int row = 32 * rb + 8 * ((e & 15) >> 2) + 4 * (lane >> 5) + (e & 3);
    const int col = 64 * cb + 32 * (e >> 4) + (lane & 31);
    f32_tile[row * MQ_FPITCH + col] = sum[e];
  }
  __syncthreads();
#pragma unroll
  for (int rr = 0; rr < MQ_RPW; ++rr) {
    const float4 v = *reinterpret_cast<const float4*>(f32_tile + (wave * MQ_RPW + rr) * MQ_FPITCH + 4 * lane);
    acc[rr][0] = v.x; acc[rr][1] = v.y; acc[rr][2] = v.z; acc[rr][3] = v.w;
  }
  __syncthreads();  // the tile may be reused (transposed output) once every wave has its sums
#endif
}

template <class T, class F>
__device__ __forceinline__ void lora_sums(const LayerDims& d, const T* __restrict__ A, const T* __restrict__ B,
                                          unsigned jc, int64_t jblk, int64_t pblk, int64_t pw, int lane, int wave,
                                          unsigned char* lds, float (&acc)[MQ_RPW][4], F&& request_row_data) {
  if constexpr (std::is_same<T, bf16_t>::value) {
    lora_rows_mfma(d, A, B, jblk, pblk, lane, wave, reinterpret_cast<float*>(lds), acc, request_row_data);
  } else {
    request_row_data();
    lora_rows<T>(d, A, B, jc, pw, lane, acc);
  }
}

// Eq. quant / l4q_Wquant on one element, in the operation order of quantize_elem(); the clamp is one median
// instruction and "in range" is "the clamp changed nothing" (the same decision for every non-NaN w).
struct QuantFast {
  float w, code;
  bool in_range;
};
__device__ __forceinline__ QuantFast quantize_fast(float wc, float s, float b, float qn, float qp) {
  QuantFast q;
  q.w = __fdiv_rn(wc - b, s);
  const float cl = __builtin_amdgcn_fmed3f(q.w, qn, qp);
  q.code = rintf(cl);
  q.in_range = cl == q.w;
  return q;
}

// MODE 0: any combination of outputs.  MODE 1: the forward pass (dequantized Wq only).  MODE 2: the fused
// backward pass (Wq^T and the d(Wq)/d(scale) factor only).  The specialisations drop the arithmetic of the
// outputs they do not write; all three compute w, the code and the mask with the same instructions.
template <class T, int MODE>
__global__ __launch_bounds__(MQ_THREADS) void merge_quant_tile_kernel(LayerDims d, const T* __restrict__ W0,
                                                                       const T* __restrict__ A,
                                                                       const T* __restrict__ B,
                                                                       const float* __restrict__ scale,
                                                                       const float* __restrict__ zero,
                                                                       MergeQuantOut<T> out) {
  typedef typename Raw4<T>::type raw4_t;
  constexpr int LDS_T = MODE == 1 ? 16 : MQ_COLS * MQ_TROW;                        // transposed output staging
  constexpr int LDS_F = std::is_same<T, bf16_t>::value ? MQ_F32_TILE : 16;        // LoRA sums from the matrix core
  __shared__ __attribute__((aligned(16))) unsigned char tile[LDS_T > LDS_F ? LDS_T : LDS_F];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t jblk = (int64_t)blockIdx.x * MQ_COLS;
  const int64_t j0 = jblk + lane * 4;
  const bool col_ok = j0 < d.i;
  const unsigned jc = col_ok ? (unsigned)j0 : 0u;                      // clamped column for loads (32-bit lane offset)
  const unsigned j32 = (unsigned)j0;
  const int64_t pw = (int64_t)blockIdx.y * MQ_ROWS + wave * MQ_RPW;    // first row of this wave
  const int64_t G = d.i / d.g;
  const unsigned q = jc / (unsigned)d.g;  // 4 consecutive columns lie in one group because g % 4 == 0
  const float zero4[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr bool want_wq = MODE != 2, want_t = MODE != 1, want_f = MODE != 1, want_misc = MODE == 0;

  // bf16 operands are below 1 GiB (checked by the caller): rows are addressed through buffer descriptors, 32-bit lane
  // offset plus a wave-uniform row offset in a scalar register, which takes the 64-bit address arithmetic off the
  // vector unit (a fifth of this kernel's vector instructions before)
  constexpr bool BUF = std::is_same<T, bf16_t>::value;
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const __amdgpu_buffer_rsrc_t rsrcW0 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<T*>(W0), 0, BUF ? (int)(d.o * d.i * 2) : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcS = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(scale), 0, BUF ? (int)(d.o * G * 4) : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcZ = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(zero), 0, BUF ? (int)(d.o * G * 4) : 0, 0x00020000);

  // row data: every load is requested before the rank sums are consumed
  raw4_t w0raw[MQ_RPW];
  float sv[MQ_RPW], bv[MQ_RPW];
  auto request_row_data = [&]() {
#pragma unroll
    for (int rr = 0; rr < MQ_RPW; ++rr) {
      const int64_t pc = pw + rr < d.o ? pw + rr : d.o - 1;
      if constexpr (BUF) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rsrcW0, (int)(jc * 2), (int)(pc * d.i * 2), 0);
        w0raw[rr] = make_uint2(w[0], w[1]);
        sv[rr] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrcS, (int)(q * 4), (int)(pc * G * 4), 0));
        bv[rr] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrcZ, (int)(q * 4), (int)(pc * G * 4), 0));
      } else {
        // wave-uniform row base first, lane offset second: the loads take a scalar base register
        w0raw[rr] = *reinterpret_cast<const raw4_t*>((W0 + pc * d.i) + jc);
        sv[rr] = (scale + pc * G)[q];
        bv[rr] = (zero + pc * G)[q];
      }
    }
  };

  float acc[MQ_RPW][4];
  lora_sums<T>(d, A, B, jc, jblk, (int64_t)blockIdx.y * MQ_ROWS, pw, lane, wave, tile, acc, request_row_data);

  float wqkeep[want_t ? MQ_RPW : 1][4];  // dequantized values of all rows, for the transposed output
#pragma unroll
  for (int rr = 0; rr < MQ_RPW; ++rr) {
    const int64_t p = pw + rr;
    const bool ok = col_ok && p < d.o;
    float w0[4], wc[4], fg[4], wqv[4];
    unpack4(w0raw[rr], w0);
    const float s = sv[rr], b = bv[rr];
    uint32_t cpack = 0, mpack = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wc[c] = w0[c] + d.gamma * acc[rr][c];
      const QuantFast qo = quantize_fast(wc[c], s, b, d.qn, d.qp);
      wqv[c] = dequant_elem(qo.code, s, b);
      if (want_f) fg[c] = qo.in_range ? qo.code - qo.w : qo.code;
      if (want_misc) {
        cpack |= ((uint32_t)(uint8_t)(int8_t)(int)qo.code) << (8 * c);
        mpack |= (qo.in_range ? 1u : 0u) << (8 * c);
      }
      if (want_t) wqkeep[want_t ? rr : 0][c] = wqv[c];
    }
    const int64_t rowoff = p * d.i;  // wave-uniform
    if (want_wq && (MODE == 1 || out.wq) && p < d.o) {
      // the dequantized weight is zero-padded up to its leading dimension (k-step of the GEMM)
      if constexpr (BUF) {  // one store per lane: the values, zeros in the padding, dropped (offset out of range) past it
        // bf16: Wq lies in blocks of 32 columns, [j / 32][p][j % 32] (the GEMM's blocked B operand; ld_wq % 32 == 0)
        const __amdgpu_buffer_rsrc_t rsrcWq = __builtin_amdgcn_make_buffer_rsrc(
            out.wq, 0, (int)(d.o * out.ld_wq * 2), 0x00020000);
        const u32x2 v = {col_ok ? pack_bf16x2(wqv[0], wqv[1]) : 0u, col_ok ? pack_bf16x2(wqv[2], wqv[3]) : 0u};
        const unsigned voff = j0 < out.ld_wq ? ((j32 >> 5) * (unsigned)d.o * 32u + (j32 & 31u)) * 2u : 0x80000000u;
        __builtin_amdgcn_raw_buffer_store_b64(v, rsrcWq, (int)voff, (int)(p * 64), 0);
      } else {
        if (col_ok) store4((out.wq + p * out.ld_wq) + j32, wqv);
        else if (j0 < out.ld_wq) store4((out.wq + p * out.ld_wq) + j32, zero4);
      }
    }
    if (ok) {
      if (want_misc) {
        if (out.codes) *reinterpret_cast<uint32_t*>((out.codes + rowoff) + j32) = cpack;
        if (out.mask) *reinterpret_cast<uint32_t*>((out.mask + rowoff) + j32) = mpack;
        if (out.wcomb) store4((out.wcomb + rowoff) + j32, wc);
      }
      if (!BUF && want_f && (MODE == 2 || out.fgrad)) {
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        h4 h = {(_Float16)fg[0], (_Float16)fg[1], (_Float16)fg[2], (_Float16)fg[3]};
        *reinterpret_cast<h4*>((out.fgrad + rowoff) + j32) = h;
      }
    }
    if constexpr (BUF) {
      if (want_f && (MODE == 2 || out.fgrad) && p < d.o) {  // (uniform) lanes past the last column: offset out of range
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        const h4 h = {(_Float16)fg[0], (_Float16)fg[1], (_Float16)fg[2], (_Float16)fg[3]};
        const __amdgpu_buffer_rsrc_t rsrcF = __builtin_amdgcn_make_buffer_rsrc(
            out.fgrad, 0, (int)(d.o * d.i * 2), 0x00020000);
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsrcF, (int)(col_ok ? j32 * 2u : 0x80000000u),
                                              (int)(rowoff * 2), 0);
      }
    }
  }

  if constexpr (MODE == 2 && std::is_same<T, bf16_t>::value) {
    // The first column tile of every row block also leaves B^T for its 64 rows (the fused weight-gradient kernel's
    // dA product reads B that way): r x 64 elements, zeros past o up to the padded width.
    if (blockIdx.x == 0 && out.bT) {
      const int64_t pblk = (int64_t)blockIdx.y * MQ_ROWS;
      for (int idx = threadIdx.x; idx < d.r * MQ_ROWS; idx += MQ_THREADS) {
        const int k = idx / MQ_ROWS;
        const int64_t p = pblk + idx % MQ_ROWS;
        if (p < out.ld_wqT) out.bT[(int64_t)k * out.ld_wqT + p] = p < d.o ? B[p * d.r + k] : (bf16_t)0;
      }
    }
  }

  if (want_t && (MODE == 2 || out.wqT)) {  // uniform: transpose the 64 x 256 tile through LDS
    // column c of this lane, rows of this wave: 8 bf16 = one 16-byte LDS write
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint32_t tp[MQ_RPW / 2];
#pragma unroll
      for (int h = 0; h < MQ_RPW / 2; ++h) tp[h] = pack_bf16x2(wqkeep[want_t ? 2 * h : 0][c], wqkeep[want_t ? 2 * h + 1 : 0][c]);
      unsigned char* dst = tile + (lane * 4 + c) * MQ_TROW + wave * (MQ_RPW * 2);
      *reinterpret_cast<uint4*>(dst) = make_uint4(tp[0], tp[1], tp[2], tp[3]);
    }
    __syncthreads();
    // rows past o (o % 8 == 0 in bf16 mode, so whole 16-byte pieces) and the padding up to ld_wqT are zeros
    const int64_t pblk = (int64_t)blockIdx.y * MQ_ROWS;
#pragma unroll
    for (int it = 0; it < MQ_COLS * 8 / MQ_THREADS; ++it) {
      const int idx = threadIdx.x + it * MQ_THREADS;
      const int jr = idx >> 3, ch = idx & 7;
      const int64_t j = jblk + jr, p = pblk + ch * 8;
      if (j < d.i && p < out.ld_wqT) {
        uint4 v = *reinterpret_cast<const uint4*>(tile + jr * MQ_TROW + ch * 16);
        if (p >= d.o) v = make_uint4(0u, 0u, 0u, 0u);
        // Wq^T lies in blocks of 32 rows of Wq, [p / 32][j][p % 32] (the GEMM's blocked B operand; ld_wqT % 32 == 0)
        *reinterpret_cast<uint4*>(out.wqT + ((p >> 5) * d.i + j) * 32 + (p & 31)) = v;
      }
    }
  }
}

// ------------------------------------------------------------------ per-group statistics of the merged weight
// Same tile mapping as the merge pass.  mode 0..3: initialisation schemes of App. B (asymmetric, symmetric,
// L4Q_init, LSQ+_init) for group sizes up to 256 (a group then lies inside one wave's 256 columns);
// mode 4: per-row, per-column-block sums of |Wc - Wq| and |Wc - (clamp(w) s + b)| (E_quant, E_clip).
constexpr int STAT_ERRORS = 4;

template <class T>
__global__ __launch_bounds__(MQ_THREADS) void weight_stats_tile_kernel(LayerDims d, const T* __restrict__ W0,
                                                                        const T* __restrict__ A,
                                                                        const T* __restrict__ B, int mode,
                                                                        float* __restrict__ scale,
                                                                        float* __restrict__ zero,
                                                                        float* __restrict__ err_part) {
  typedef typename Raw4<T>::type raw4_t;
  __shared__ __attribute__((aligned(16))) unsigned char lds[std::is_same<T, bf16_t>::value ? MQ_F32_TILE : 16];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t j0 = (int64_t)blockIdx.x * MQ_COLS + lane * 4;
  const bool col_ok = j0 < d.i;
  const unsigned jc = col_ok ? (unsigned)j0 : 0u;
  const int64_t pw = (int64_t)blockIdx.y * MQ_ROWS + wave * MQ_RPW;
  const int64_t G = d.i / d.g;
  const unsigned q = jc / (unsigned)d.g;
  const int width = d.g / 4 < 64 ? d.g / 4 : 64;  // lanes per group (power of two)
  const float inf = __builtin_huge_valf();

  raw4_t w0raw[MQ_RPW];
  float sv[MQ_RPW], bv[MQ_RPW];
  auto request_row_data = [&]() {
#pragma unroll
    for (int rr = 0; rr < MQ_RPW; ++rr) {
      const int64_t pc = pw + rr < d.o ? pw + rr : d.o - 1;
      w0raw[rr] = *reinterpret_cast<const raw4_t*>((W0 + pc * d.i) + jc);
      sv[rr] = mode == STAT_ERRORS ? (scale + pc * G)[q] : 1.f;
      bv[rr] = mode == STAT_ERRORS ? (zero + pc * G)[q] : 0.f;
    }
  };
  float acc[MQ_RPW][4];
  lora_sums<T>(d, A, B, jc, (int64_t)blockIdx.x * MQ_COLS, (int64_t)blockIdx.y * MQ_ROWS, pw, lane, wave, lds, acc,
               request_row_data);

#pragma unroll
  for (int rr = 0; rr < MQ_RPW; ++rr) {
    const int64_t p = pw + rr;
    const bool ok = col_ok && p < d.o;
    float w0[4], wc[4];
    unpack4(w0raw[rr], w0);
#pragma unroll
    for (int c = 0; c < 4; ++c) wc[c] = w0[c] + d.gamma * acc[rr][c];
    if (mode == STAT_ERRORS) {
      float eq = 0.f, ec = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const QuantOut qo = quantize_elem(wc[c], sv[rr], bv[rr], d.qn, d.qp);
        const float clamped = fminf(fmaxf(qo.w, d.qn), d.qp);
        eq += ok ? fabsf(wc[c] - dequant_elem(qo.code, sv[rr], bv[rr])) : 0.f;
        ec += ok ? fabsf(wc[c] - dequant_elem(clamped, sv[rr], bv[rr])) : 0.f;
      }
      eq = wave_sum_width(eq, 64);
      ec = wave_sum_width(ec, 64);
      if (lane == 0 && p < d.o) {
        float* dst = err_part + (p * gridDim.x + blockIdx.x) * 2;
        dst[0] = eq;
        dst[1] = ec;
      }
    } else {
      float lo = inf, hi = -inf, sum = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        lo = ok ? fminf(lo, wc[c]) : lo;
        hi = ok ? fmaxf(hi, wc[c]) : hi;
        sum += ok ? wc[c] : 0.f;
      }
      for (int off = width >> 1; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
        sum += __shfl_xor(sum, off, 64);
      }
      float s = 0.f, b = 0.f;
      if (mode == 0) {  // asymmetric min/max
        s = __fdiv_rn(hi - lo, d.qp - d.qn);
        b = lo - s * d.qn;
      } else if (mode == 1) {  // symmetric
        s = __fdiv_rn(fmaxf(fabsf(lo), fabsf(hi)), -d.qn);
      } else if (mode == 2) {  // L4Q_init (Eq. l4q_quant_init)
        s = fmaxf(fabsf(__fdiv_rn(lo, d.qn)), fabsf(__fdiv_rn(hi, d.qp)));
      } else {  // LSQ+_init: mean and (population) standard deviation of the group, two passes in registers
        const float mu = sum / (float)d.g;
        float ss = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) ss += ok ? (wc[c] - mu) * (wc[c] - mu) : 0.f;
        for (int off = width >> 1; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
        const float sd = sqrtf(ss / (float)d.g);
        s = fmaxf(fabsf(mu - 3.f * sd), fabsf(mu + 3.f * sd)) / -d.qn;
      }
      if (ok && (lane & (width - 1)) == 0) {
        scale[p * G + q] = s;
        zero[p * G + q] = b;
      }
    }
  }
}

// sums err_part [rows * 2] pairs into out[0] (E_quant) and out[1] (E_clip); one block, fixed order
__global__ __launch_bounds__(256) void sum_error_pairs_kernel(const float* __restrict__ part, int64_t npairs,
                                                               float* __restrict__ out) {
  __shared__ double sh[2][256];
  double a = 0.0, b = 0.0;
  for (int64_t e = threadIdx.x; e < npairs; e += 256) {
    a += part[2 * e];
    b += part[2 * e + 1];
  }
  sh[0][threadIdx.x] = a;
  sh[1][threadIdx.x] = b;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if ((int)threadIdx.x < st) {
      sh[0][threadIdx.x] += sh[0][threadIdx.x + st];
      sh[1][threadIdx.x] += sh[1][threadIdx.x + st];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    out[0] = (float)sh[0][0];
    out[1] = (float)sh[1][0];
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

}  // namespace

template <class T>
void launch_merge_quant(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                        const float* zero, const MergeQuantOut<T>& out, hipStream_t stream) {
  if constexpr (std::is_same<T, bf16_t>::value) {
    if (merge_quant_stream_supported(d, out)) {
      launch_merge_quant_stream(d, W0, A, B, scale, zero, out, stream);
      return;
    }
  }
  const int64_t rows = out.wqT && out.ld_wqT > d.o ? out.ld_wqT : d.o;
  dim3 grid((unsigned)((d.i + MQ_COLS - 1) / MQ_COLS), (unsigned)((rows + MQ_ROWS - 1) / MQ_ROWS));
  const bool misc = out.codes || out.wcomb || out.mask;
  if (out.wq && !out.wqT && !out.fgrad && !misc)
    hipLaunchKernelGGL((merge_quant_tile_kernel<T, 1>), grid, dim3(MQ_THREADS), 0, stream, d, W0, A, B, scale, zero, out);
  else if (!out.wq && out.wqT && out.fgrad && !misc)
    hipLaunchKernelGGL((merge_quant_tile_kernel<T, 2>), grid, dim3(MQ_THREADS), 0, stream, d, W0, A, B, scale, zero, out);
  else
    hipLaunchKernelGGL((merge_quant_tile_kernel<T, 0>), grid, dim3(MQ_THREADS), 0, stream, d, W0, A, B, scale, zero, out);
}

template <class T>
void launch_init_qparams(const LayerDims& d, const T* W0, const T* A, const T* B, int method, float* scale,
                         float* zero, hipStream_t stream) {
  if (d.g <= 256) {
    dim3 grid((unsigned)((d.i + MQ_COLS - 1) / MQ_COLS), (unsigned)((d.o + MQ_ROWS - 1) / MQ_ROWS));
    hipLaunchKernelGGL(weight_stats_tile_kernel<T>, grid, dim3(MQ_THREADS), 0, stream, d, W0, A, B, method, scale,
                       zero, (float*)nullptr);
    return;
  }
  const int rows_per_block = kThreads / 64;
  dim3 grid((unsigned)((d.o + rows_per_block - 1) / rows_per_block));
  hipLaunchKernelGGL(init_qparams_kernel<T>, grid, dim3(kThreads), 0, stream, d, W0, A, B, method, scale, zero);
}

template <class T>
void launch_quant_errors(const LayerDims& d, const T* W0, const T* A, const T* B, const float* scale,
                         const float* zero, float* partial, float* out2, hipStream_t stream) {
  dim3 grid((unsigned)((d.i + MQ_COLS - 1) / MQ_COLS), (unsigned)((d.o + MQ_ROWS - 1) / MQ_ROWS));
  hipLaunchKernelGGL(weight_stats_tile_kernel<T>, grid, dim3(MQ_THREADS), 0, stream, d, W0, A, B, STAT_ERRORS,
                     const_cast<float*>(scale), const_cast<float*>(zero), partial);
  hipLaunchKernelGGL(sum_error_pairs_kernel, dim3(1), dim3(256), 0, stream, partial, d.o * (int64_t)grid.x, out2);
}


template void launch_merge_quant<float>(const LayerDims&, const float*, const float*, const float*, const float*,
                                        const float*, const MergeQuantOut<float>&, hipStream_t);
template void launch_merge_quant<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*,
                                         const float*, const float*, const MergeQuantOut<bf16_t>&, hipStream_t);
template void launch_quant_errors<float>(const LayerDims&, const float*, const float*, const float*, const float*,
                                         const float*, float*, float*, hipStream_t);
template void launch_quant_errors<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*,
                                          const float*, const float*, float*, float*, hipStream_t);
template void launch_init_qparams<float>(const LayerDims&, const float*, const float*, const float*, int, float*,
                                         float*, hipStream_t);
template void launch_init_qparams<bf16_t>(const LayerDims&, const bf16_t*, const bf16_t*, const bf16_t*, int,
                                          float*, float*, hipStream_t);

}  // namespace l4q
