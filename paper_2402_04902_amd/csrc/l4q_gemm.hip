// bf16 MFMA GEMMs of the layer with a plain store epilogue (main loop: l4q_gemm_core.h).
//
//   forward   Y  [T,o] = X  [T,i] . Wq  [o,ipad]^T      both operands K-contiguous; Wq in blocks of 32 k-values
//   dX        dX [T,i] = dY [T,o] . WqT [i,opad]^T      both operands K-contiguous; WqT likewise
//   dWq       dWq[o,i] = dY [T,o]^T . X [T,i]           both operands K-major (unfused backward only;
//                                                       the fused form lives in l4q_bwd_fused.hip)
// The workspace operand (Wq, WqT) is zero-padded along k to the 32-wide k-step; the caller's operand is
// not: its 16-byte chunks past the row end are masked (read as zeros) in the last stage.
#include "l4q_device.h"
#include "l4q_gemm_core.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS ring pipeline (l4q_gemm_core.h) + plain store epilogue.  Operands below 1 GiB.
// ---------------------------------------------------------------------------------------------
// Store epilogue of a macro tile; `LDS_BYTES` of LDS at `lds` are free.
template <class T, bool OUT_BF16, int LDS_BYTES>
__device__ __forceinline__ void store_tile(gemm::Accum<T>& acc, int M, int N, void* __restrict__ Cout, int64_t ldc,
                                           int m0, int n0, unsigned char* lds) {
  // bf16 output through LDS (free after the main loop): a lane holds 4 consecutive columns of 64 different
  // rows, which as direct stores are 16-byte pieces of 32 cache lines per instruction.  Each wave instead
  // parks its 128 x 128 block in its own LDS region (rows padded to 272 bytes) and writes it out as 16 bytes
  // per lane, 16 lanes per 256-byte row segment.  Needs 16-byte aligned rows: ldc % 8 == 0 and N % 8 == 0.
  constexpr int EP_ROW = T::WTN * 2 + 16;
  constexpr int EP_LPR = T::WTN / 8;  // lanes that cover a row of the wave's block with 16 bytes each
  constexpr bool EP_FITS = OUT_BF16 && (T::WTN == 128 || T::WTN == 64) && T::NW * T::WTM * EP_ROW <= LDS_BYTES;
  if (EP_FITS && (ldc & 7) == 0 && (N & 7) == 0) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned char* region = lds + wave * (T::WTM * EP_ROW);
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
      for (int b = 0; b < T::TN; ++b)
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          uint2 v;
          v.x = pack_bf16x2(acc.v[a][b][4 * eg], acc.v[a][b][4 * eg + 1]);
          v.y = pack_bf16x2(acc.v[a][b][4 * eg + 2], acc.v[a][b][4 * eg + 3]);
          *reinterpret_cast<uint2*>(region + (a * 32 + (lane & 31)) * EP_ROW + (b * 32 + 8 * eg + 4 * (lane >> 5)) * 2) = v;
        }
    bf16_t* C = reinterpret_cast<bf16_t*>(Cout);
    const int mw = m0 + (wave / T::WAVES_N) * T::WTM;
    const int nw = n0 + (wave % T::WAVES_N) * T::WTN + (lane % EP_LPR) * 8;
#pragma unroll 8
    for (int it = 0; it < T::WTM * EP_LPR / 64; ++it) {
      const int row = it * (64 / EP_LPR) + lane / EP_LPR;
      const uint4 v = *reinterpret_cast<const uint4*>(region + row * EP_ROW + (lane % EP_LPR) * 16);
      if (mw + row < M && nw < N) *reinterpret_cast<uint4*>(C + (int64_t)(mw + row) * ldc + nw) = v;
    }
    return;
  }
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

// One macro tile: main loop, then the store epilogue.
template <class T, bool OUT_BF16, bool A_KM, bool B_KM, bool MASK_A_K, bool B_BLK>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                                          int64_t ldb, int M, int N, int K, int K_a, void* __restrict__ Cout,
                                          int64_t ldc, int m0, int n0, unsigned char* lds) {
  gemm::Accum<T> acc;
#pragma unroll
  for (int a = 0; a < T::TM; ++a)
#pragma unroll
    for (int b = 0; b < T::TN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc.v[a][b][e] = 0.f;
  gemm::mainloop<T, A_KM, B_KM, gemm::NoTailLoads, MASK_A_K, B_BLK>(A, lda, B, ldb, M, N, K, m0, n0, lds, acc,
                                                                   gemm::NoTailLoads(), K_a);
  store_tile<T, OUT_BF16, T::LDS_BYTES>(acc, M, N, Cout, ldc, m0, n0, lds);
}

template <class T, bool OUT_BF16, bool A_KM = false, bool B_KM = false, bool MASK_A_K = false, bool B_BLK = false>
__global__ __launch_bounds__(T::NT) void gemm_bf16_nt_fast_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                   const bf16_t* __restrict__ B, int64_t ldb, int M,
                                                                   int N, int K, int K_a, void* __restrict__ Cout,
                                                                   int64_t ldc, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
  int tile_m, tile_n;
  gemm::tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  gemm_tile<T, OUT_BF16, A_KM, B_KM, MASK_A_K, B_BLK>(A, lda, B, ldb, M, N, K, K_a, Cout, ldc, tile_m * T::BM,
                                                      tile_n * T::BN, lds);
}

// One (tile, k-slice) of a product with few tiles: slice blockIdx.y of gridDim.y takes a run of whole stage pairs of
// the k range and leaves its binary32 tile in part[slice][M][N].  K-contiguous operands; B row-major (ldb) or, B_BLK, in
// blocks of 32 k-values.
template <class T, bool MASK_A_K, bool B_BLK>
__global__ __launch_bounds__(T::NT) void gemm_bf16_nt_splitk_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                     const bf16_t* __restrict__ B, int64_t ldb, int M,
                                                                     int N, int K, int K_a, float* __restrict__ part,
                                                                     int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
  int tile_m, tile_n;
  gemm::tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int slices = gridDim.y, slice = blockIdx.y;
  const int pairs = ((K + T::BK - 1) / T::BK + 1) / 2;
  const int k0 = (int)((int64_t)pairs * slice / slices) * (2 * T::BK);
  int k1 = (int)((int64_t)pairs * (slice + 1) / slices) * (2 * T::BK);
  if (k1 > K) k1 = K;
  // rows of A end at K_a: inside the last slice, at or past the end of every other
  const int ka = (K_a < k1 ? K_a : k1) - k0;
  const bf16_t* Bs = B_BLK ? B + (int64_t)(k0 / T::BK) * N * T::BK : B + k0;
  gemm_tile<T, false, false, false, MASK_A_K, B_BLK>(A + k0, lda, Bs, ldb, M, N, k1 - k0, ka,
                                                     part + (int64_t)slice * M * N, N, tile_m * T::BM, tile_n * T::BN, lds);
}

// The same for K-major operands (rows = k): slice blockIdx.y takes a run of whole stages.
template <class T>
__global__ __launch_bounds__(T::NT) void gemm_bf16_kmajor_splitk_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                         const bf16_t* __restrict__ B, int64_t ldb,
                                                                         int M, int N, int K, float* __restrict__ part,
                                                                         int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
  int tile_m, tile_n;
  gemm::tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int slices = gridDim.y, slice = blockIdx.y;
  const int nk = (K + T::BK - 1) / T::BK;
  const int k0 = (int)((int64_t)nk * slice / slices) * T::BK;
  int k1 = (int)((int64_t)nk * (slice + 1) / slices) * T::BK;
  if (k1 > K) k1 = K;
  gemm_tile<T, false, true, true, false, false>(A + (int64_t)k0 * lda, lda, B + (int64_t)k0 * ldb, ldb, M, N, k1 - k0,
                                                k1 - k0, part + (int64_t)slice * M * N, N, tile_m * T::BM,
                                                tile_n * T::BN, lds);
}

// C[m, n] = bf16(sum over the slices, in slice order, of part[slice][m][n]); N % 4 == 0, four columns per thread.
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float* __restrict__ part, int slices, int64_t M, int64_t N,
                                                         bf16_t* __restrict__ C, int64_t ldc) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= M * N / 4) return;
  float4 v = reinterpret_cast<const float4*>(part)[q];
  for (int s = 1; s < slices; ++s) {
    const float4 w = reinterpret_cast<const float4*>(part + (int64_t)s * M * N)[q];
    v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
  }
  const int64_t m = q * 4 / N, n = q * 4 - m * N;
  const float f[4] = {v.x, v.y, v.z, v.w};
  store4(C + m * ldc + n, f);
}

// Matrix-core-only loop with the GEMM's register shape (4 x 4 accumulator tiles, 8 fragments per wave) and
// no memory traffic inside the loop: what the matrix pipeline sustains on this chip for the given data.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const bf16_t* __restrict__ data, int iterations,
                                                         float* __restrict__ sink) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef gemm::bf16x8_t bf16x8_t;
  typedef gemm::f32x16_t f32x16_t;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16x8_t fa[4], fb[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {  // 8 fragments of 16 bytes per lane out of the first 64 KiB of data
    fa[q] = *reinterpret_cast<const bf16x8_t*>(data + ((wave * 8 + q) * 64 + lane) * 8);
    fb[q] = *reinterpret_cast<const bf16x8_t*>(data + ((wave * 8 + 4 + q) * 64 + lane) * 8);
  }
  f32x16_t acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
  for (int it = 0; it < iterations; ++it) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[b], fa[a], acc[a][b], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[a][b][e];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
#endif
}

}  // namespace

double launch_mfma_probe(const bf16_t* data, int iterations, int workgroups, float* sink, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, data, iterations, sink);
  return (double)workgroups * 4.0 * (double)iterations * 16.0 * (2.0 * 32 * 32 * 16);
}

int device_compute_units() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// Slices of the k range for a product with few tiles: as many as put a workgroup on every compute unit, each at
// least four stage pairs (256 k) long, at most 8, and no more than keep the partial tiles (slices x M x N x 4 bytes,
// written and read once) within the size of operand B (N x K x 2 bytes).
int gemm_nt_splitk_slices(int64_t M, int64_t N, int64_t K) {
  typedef gemm::Tile<256, 256, 32, 5, true, 4> F;
  const int64_t tiles = ((M + F::BM - 1) / F::BM) * ((N + F::BN - 1) / F::BN);
  const int64_t cus = device_compute_units();
  if (tiles <= 0 || 2 * tiles > cus) return 1;
  const int64_t pairs = ((K + F::BK - 1) / F::BK + 1) / 2;
  int64_t s = cus / tiles;
  if (s > pairs / 4) s = pairs / 4;
  if (s > 8) s = 8;
  if (s > K / (2 * M)) s = K / (2 * M);
  return s < 1 ? 1 : (int)s;
}

void launch_gemm_bf16_nt(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                         int64_t K, int64_t K_a, bf16_t* C, int64_t ldc, hipStream_t stream, float* partial) {
  // K-contiguous operands: stages loaded in cache-line pairs; 8 waves (2 x 4, two per SIMD, 128 x 64 each): a second
  // wave on the SIMD keeps the matrix pipe busy while the first waits for a barrier or for operands (1.5 % over 2 x 2)
  typedef gemm::Tile<256, 256, 32, 5, true, 4> F;
  const int tiles_m = (int)((M + F::BM - 1) / F::BM), tiles_n = (int)((N + F::BN - 1) / F::BN);
  const int slices = partial ? gemm_nt_splitk_slices(M, N, K) : 1;
  if (slices > 1) {
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)slices);
    if (K_a == K)
      hipLaunchKernelGGL((gemm_bf16_nt_splitk_kernel<F, false, true>), grid, dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M,
                         (int)N, (int)K, (int)K_a, partial, tiles_m, tiles_n);
    else
      hipLaunchKernelGGL((gemm_bf16_nt_splitk_kernel<F, true, true>), grid, dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M,
                         (int)N, (int)K, (int)K_a, partial, tiles_m, tiles_n);
    const int64_t quads = M * N / 4;
    hipLaunchKernelGGL(splitk_sum_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, partial, slices,
                       M, N, C, ldc);
    return;
  }
  // rows of A end at K_a: where that is short of the k-step, the chunks past it are masked (a second instance, so
  // that the usual shapes do not pay for the selection)
  if (K_a == K)
    hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<F, true, false, false, false, true>),
                       dim3((unsigned)(tiles_m * tiles_n)), dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M, (int)N, (int)K,
                       (int)K_a, (void*)C, ldc, tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<F, true, false, false, true, true>),
                       dim3((unsigned)(tiles_m * tiles_n)), dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M, (int)N, (int)K,
                       (int)K_a, (void*)C, ldc, tiles_m, tiles_n);
}

void launch_gemm_bf16_kmajor_f32(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N,
                                 int64_t K, float* C, int64_t ldc, hipStream_t stream) {
  typedef gemm::Tile<256, 256, 32, 4> F;
  const int tiles_m = (int)((M + F::BM - 1) / F::BM), tiles_n = (int)((N + F::BN - 1) / F::BN);
  hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<F, false, true, true>), dim3((unsigned)(tiles_m * tiles_n)),
                     dim3(F::NT), 0, stream, A, lda, B, ldb, (int)M, (int)N, (int)K, (int)K, (void*)C, ldc, tiles_m,
                     tiles_n);
}

// k-slices of the two thin products of the masked form (dB = dWm A^T: [o, r], k = i; dA = B^T dWm: [r, i], k = o): each
// has o / 256 or i / 256 tiles only, one tile row or column, and a long k range; as many slices as put a workgroup on
// every compute unit, each at least 8 stages long, at most 8 (and 32 MiB of partial results).
void dw_masked_product_slices(const LayerDims& d, int* slices_a, int* slices_b) {
  const int64_t cus = device_compute_units();
  auto pick = [&](int64_t tiles, int64_t stages, int64_t out_elems) {
    int64_t s = cus / (tiles > 0 ? tiles : 1);
    if (s > stages / 8) s = stages / 8;
    if (s > 8) s = 8;
    while (s > 1 && s * out_elems * 4 > (32ll << 20)) --s;
    return (int)(s < 1 ? 1 : s);
  };
  const int64_t tr = (d.r + 255) / 256;
  *slices_b = pick(((d.o + 255) / 256) * tr, (d.i + 31) / 32, d.o * d.r);
  *slices_a = pick(tr * ((d.i + 255) / 256), (d.o + 31) / 32, (int64_t)d.r * d.i);
}

void launch_dw_masked_products(const LayerDims& d, const bf16_t* dWm, const bf16_t* A, const bf16_t* B, float* rawA,
                               float* rawB, hipStream_t stream) {
  int sa = 1, sb = 1;
  dw_masked_product_slices(d, &sa, &sb);
  // rawB [sb][o, r] = dWm [o, i] . A [r, i]^T: both K-contiguous, k = i (a multiple of 32: nothing to pad or mask)
  {
    typedef gemm::Tile<256, 256, 32, 5, true, 4> F;
    const int tiles_m = (int)((d.o + F::BM - 1) / F::BM), tiles_n = (d.r + F::BN - 1) / F::BN;
    hipLaunchKernelGGL((gemm_bf16_nt_splitk_kernel<F, false, false>), dim3((unsigned)(tiles_m * tiles_n), (unsigned)sb),
                       dim3(F::NT), 0, stream, dWm, d.i, A, d.i, (int)d.o, d.r, (int)d.i, (int)d.i, rawB, tiles_m, tiles_n);
  }
  // rawA [sa][r, i] = B [o, r]^T . dWm [o, i]: both K-major, k = o
  {
    typedef gemm::Tile<256, 256, 32, 4> F;
    const int tiles_m = (d.r + F::BM - 1) / F::BM, tiles_n = (int)((d.i + F::BN - 1) / F::BN);
    hipLaunchKernelGGL((gemm_bf16_kmajor_splitk_kernel<F>), dim3((unsigned)(tiles_m * tiles_n), (unsigned)sa), dim3(F::NT),
                       0, stream, B, (int64_t)d.r, dWm, d.i, d.r, (int)d.i, (int)d.o, rawA, tiles_m, tiles_n);
  }
}

}  // namespace l4q
