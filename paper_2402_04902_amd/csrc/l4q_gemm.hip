// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] . B[N,K]^T  with binary32 accumulation.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants per lane
// (8 consecutive k of one row).  The three GEMMs of the layer are all brought to this form:
//   forward   Y  [T,o] = X  [T,i] . Wq  [o,i]^T
//   dX        dX [T,i] = dY [T,o] . WqT [i,o]^T
//   dWq       dWq[o,i] = dYT[o,T] . XT  [i,T]^T
//
// Tiling: BM x BN x 64 macro tile per workgroup, double-buffered in LDS (2 x (BM + BN) x 128 B),
// waves arranged WAVES_M x WAVES_N, each owning a (BM/WAVES_M) x (BN/WAVES_N) block of 32 x 32
// accumulator tiles.  LDS rows are 128 B (64 bf16); the 16-byte chunk index is XOR-swizzled with
// (row >> 1) & 7 so that both the 16-byte writes (8 lanes per row) and the MFMA fragment reads
// (consecutive rows, same chunk) touch all 64 banks evenly.
// Workgroup ids are remapped so that each of the 8 XCDs (which receive ids round-robin) works
// on a contiguous band of tiles, and inside a band tiles are walked in groups of GROUP_M rows
// so that concurrently running workgroups share A and B panels in their XCD's L2.
#include "l4q_device.h"
#include "l4q_gemm_core.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

// ---------------------------------------------------------------------------------------------
// Fast path: direct-to-LDS ring pipeline (l4q_gemm_core.h) + plain store epilogue.
// Needs K % BK == 0 and operands below 2 GiB; anything else takes the generic kernel below.
// ---------------------------------------------------------------------------------------------
template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT) void gemm_bf16_nt_fast_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                   const bf16_t* __restrict__ B, int64_t ldb, int M,
                                                                   int N, int K, void* __restrict__ Cout,
                                                                   int64_t ldc, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
  int tile_m, tile_n;
  gemm::tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * T::BM, n0 = tile_n * T::BN;
  gemm::Accum<T> acc;
#pragma unroll
  for (int a = 0; a < T::TM; ++a)
#pragma unroll
    for (int b = 0; b < T::TN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc.v[a][b][e] = 0.f;
  gemm::mainloop<T>(A, lda, B, ldb, M, N, K, m0, n0, lds, acc);
#pragma unroll
  for (int a = 0; a < T::TM; ++a) {
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        int m, n;
        gemm::acc_coords<T>(a, b, eg, m, n);
        m += m0;
        n += n0;
        if (m < M && n < N) {  // N % 4 == 0: the 4 consecutive columns are all inside
          const float v[4] = {acc.v[a][b][4 * eg], acc.v[a][b][4 * eg + 1], acc.v[a][b][4 * eg + 2],
                              acc.v[a][b][4 * eg + 3]};
          if (OUT_BF16) store4(reinterpret_cast<bf16_t*>(Cout) + (int64_t)m * ldc + n, v);
          else store4(reinterpret_cast<float*>(Cout) + (int64_t)m * ldc + n, v);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Generic kernel: register-staged, bounds-checked loads; any K % 8 == 0.
// ---------------------------------------------------------------------------------------------

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 64;            // k extent of one LDS stage (bf16 elements)
constexpr int ROW_BYTES = BK * 2; // 128

__device__ __forceinline__ int swizzled_offset(int row, int chunk) {
  return row * ROW_BYTES + ((chunk ^ ((row >> 1) & 7)) << 4);
}

using gemm::tile_of_block;

template <int BM, int BN, int WAVES_M, int WAVES_N>
struct Cfg {
  static constexpr int NT = WAVES_M * WAVES_N * 64;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static constexpr int A_CHUNKS = BM * 8 / NT, B_CHUNKS = BN * 8 / NT;  // 16-byte chunks per thread per stage
  static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static_assert(BM % (WAVES_M * 32) == 0 && BN % (WAVES_N * 32) == 0, "wave tile must be a multiple of 32");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "chunks must divide evenly");
};

template <class C, bool OUT_BF16>
__global__ __launch_bounds__(C::NT) void gemm_bf16_nt_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                              const bf16_t* __restrict__ B, int64_t ldb, int M,
                                                              int N, int K, void* __restrict__ Cout, int64_t ldc,
                                                              int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * C::STAGE_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / C::WAVES_N_, wn = wave % C::WAVES_N_;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * C::BM_, n0 = tile_n * C::BN_;

  f32x16_t acc[C::TM][C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
#pragma unroll
    for (int b = 0; b < C::TN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  uint4 ra[C::A_CHUNKS], rb[C::B_CHUNKS];

  auto gload = [&](int k0) {
#pragma unroll
    for (int c = 0; c < C::A_CHUNKS; ++c) {
      const int idx = tid + c * C::NT;
      const int row = idx >> 3, ch = idx & 7;
      const int m = m0 + row, k = k0 + ch * 8;
      ra[c] = (m < M && k < K) ? *reinterpret_cast<const uint4*>(A + (int64_t)m * lda + k) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < C::B_CHUNKS; ++c) {
      const int idx = tid + c * C::NT;
      const int row = idx >> 3, ch = idx & 7;
      const int n = n0 + row, k = k0 + ch * 8;
      rb[c] = (n < N && k < K) ? *reinterpret_cast<const uint4*>(B + (int64_t)n * ldb + k) : make_uint4(0, 0, 0, 0);
    }
  };
  auto lstore = [&](int stage) {
    unsigned char* as = lds + stage * C::STAGE_BYTES;
    unsigned char* bs = as + C::A_BYTES;
#pragma unroll
    for (int c = 0; c < C::A_CHUNKS; ++c) {
      const int idx = tid + c * C::NT;
      *reinterpret_cast<uint4*>(as + swizzled_offset(idx >> 3, idx & 7)) = ra[c];
    }
#pragma unroll
    for (int c = 0; c < C::B_CHUNKS; ++c) {
      const int idx = tid + c * C::NT;
      *reinterpret_cast<uint4*>(bs + swizzled_offset(idx >> 3, idx & 7)) = rb[c];
    }
  };
  auto compute = [&](int stage) {
    const unsigned char* as = lds + stage * C::STAGE_BYTES;
    const unsigned char* bs = as + C::A_BYTES;
    const int frow = lane & 31, fch = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t fa[C::TM], fb[C::TN];
#pragma unroll
      for (int a = 0; a < C::TM; ++a)
        fa[a] = *reinterpret_cast<const bf16x8_t*>(as + swizzled_offset(wm * C::WTM + a * 32 + frow, kk * 2 + fch));
#pragma unroll
      for (int b = 0; b < C::TN; ++b)
        fb[b] = *reinterpret_cast<const bf16x8_t*>(bs + swizzled_offset(wn * C::WTN + b * 32 + frow, kk * 2 + fch));
#pragma unroll
      for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
  };

  const int nk = (K + BK - 1) / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
    compute(cur);
    if (kt + 1 < nk) lstore(cur ^ 1);
    __syncthreads();
  }

  // accumulator tile layout of the 32x32 MFMA: lane -> column (lane & 31); register e -> row
  // 8 * (e / 4) + 4 * (lane / 32) + (e % 4).
#pragma unroll
  for (int a = 0; a < C::TM; ++a) {
#pragma unroll
    for (int b = 0; b < C::TN; ++b) {
      const int n = n0 + wn * C::WTN + b * 32 + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * C::WTM + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (m < M && n < N) {
          if (OUT_BF16) reinterpret_cast<bf16_t*>(Cout)[(int64_t)m * ldc + n] = f32_to_bf16(acc[a][b][e]);
          else reinterpret_cast<float*>(Cout)[(int64_t)m * ldc + n] = acc[a][b][e];
        }
      }
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
struct CfgT : Cfg<BM, BN, WAVES_M, WAVES_N> {
  static constexpr int BM_ = BM, BN_ = BN, WAVES_M_ = WAVES_M, WAVES_N_ = WAVES_N;
};

}  // namespace

void launch_gemm_bf16_nt(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                         int64_t K, bf16_t* C_bf16, float* C_f32, int64_t ldc, hipStream_t stream) {
  typedef gemm::Tile<256, 256, 32, 4> F;
  const bool fast = K % F::BK == 0 && N % 4 == 0 && ldc % 4 == 0 && M * lda * 2 < (1ll << 30) &&
                    N * ldb * 2 < (1ll << 30);
  if (fast) {
    const int tiles_m = (int)((M + F::BM - 1) / F::BM), tiles_n = (int)((N + F::BN - 1) / F::BN);
    dim3 grid((unsigned)(tiles_m * tiles_n));
    if (C_bf16)
      hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<F, true>), grid, dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M,
                         (int)N, (int)K, (void*)C_bf16, ldc, tiles_m, tiles_n);
    else
      hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<F, false>), grid, dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M,
                         (int)N, (int)K, (void*)C_f32, ldc, tiles_m, tiles_n);
    return;
  }
  typedef CfgT<256, 256, 2, 2> C;
  const int tiles_m = (int)((M + C::BM_ - 1) / C::BM_), tiles_n = (int)((N + C::BN_ - 1) / C::BN_);
  dim3 grid((unsigned)(tiles_m * tiles_n));
  if (C_bf16)
    hipLaunchKernelGGL((gemm_bf16_nt_kernel<C, true>), grid, dim3(C::NT), 0, stream, A, lda, B, ldb, (int)M, (int)N,
                       (int)K, (void*)C_bf16, ldc, tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemm_bf16_nt_kernel<C, false>), grid, dim3(C::NT), 0, stream, A, lda, B, ldb, (int)M, (int)N,
                       (int)K, (void*)C_f32, ldc, tiles_m, tiles_n);
}

}  // namespace l4q
