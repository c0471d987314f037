// Weight-gradient GEMM with the quantizer backward fused into its epilogue (bf16 mode).
//
//   dWq[o,i] = dY[T,o]^T . X[T,i]              (App. A.1, Eq. appen_wq)   -- stays in registers;
//                                              dY and X are read as they lie in memory (K-major operands)
//   dscale[p,q] = sum_{j in group q} dWq[p,j] * f[p,j]                    (Eq. quant_lsq_s + case list)
//   dzero [p,q] = sum_{j in group q} dWq[p,j] * (1 - m[p,j])              (Eq. appen_lsq_b)
//   dB[p,k]     = gamma * sum_j (m * dWq)[p,j] A[k,j]                     (Eq. appen_l4q_b)
//   dA[k,j]     = gamma * sum_p B[p,k] (m * dWq)[p,j]                     (Eq. appen_l4q_a)
//
// f = d(Wq)/d(scale) is what the merge+quantize pass of this same backward call left in the
// workspace as binary16: code - w (|f| <= 1/2) where the element is in range, Q_N or Q_P
// (|f| >= 1) where it is clipped; the straight-through mask m is read off its magnitude.
// dWq itself is never written to memory.
//
// Accumulator layout (see l4q_gemm_core.h): a lane owns weight row p = 32 a + lane % 32 of its
// wave's 128 rows and, per 32-column tile b, the 16 columns 8 (e/4) + 4 (lane/32) + e%4.
//  * group sums over j are in-lane adds plus one exchange with lane ^ 32;
//  * dB is a second MFMA straight from the registers: the masked gradient is the row operand and
//    the 8 k-slots of a lane are loaded from A with the same column pattern;
//  * dA contracts over p, the lane axis, so the masked tile goes through LDS once (row-major, 8-byte writes of what a
//    lane holds; the transposing LDS read turns it into operand fragments) and is multiplied with B^T.
// Partial results per tile row / tile column go to the workspace and are summed by a second,
// tiny kernel in a fixed order, so the result does not depend on scheduling.
//
// Ranks above 32.  The volume of those partial sums grows with the rank (o i r / 32 bytes: at r = 64 as much as the
// masked gradient itself in bfloat16, at r = 128 as much as dWq in binary32), so from rank 33 on the kernel runs in a
// second form: group sums as above, and the masked tile m * dWq, which the epilogue has in LDS anyway, leaves as
// bfloat16 [o, i] (half of what a stored binary32 dWq would take); dA and dB are then two thin products on the matrix
// core (launch_dw_masked_products).
#include "l4q_device.h"
#include "l4q_gemm_core.h"
#include "l4q_kernels.h"

namespace l4q {

namespace {

typedef gemm::Tile<256, 256, 32, 5> T;
static_assert(T::WTM == 128 && T::WTN == 128 && T::TM == 4 && T::TN == 4, "epilogue is written for 128 x 128 wave tiles");

constexpr int EP_ROWB = 256 * 2 + 16;             // bytes per row p of the masked tile in LDS: 256 columns + pad
constexpr int EP_TILE = 256 * EP_ROWB;            // 135168
constexpr int EP_SCRATCH = 2 * 128 * 2 * 4;       // per wave-row pair: 128 rows x (dscale, dzero)
constexpr int EP_LDS = EP_TILE + EP_SCRATCH;
constexpr int FUSED_LDS = EP_LDS > T::LDS_BYTES ? EP_LDS : T::LDS_BYTES;

typedef gemm::bf16x8_t bf16x8_t;
typedef gemm::f32x16_t f32x16_t;

struct FusedArgs {
  const bf16_t* dY;                   // [T, o]
  const bf16_t* X;                    // [T, i]
  int K;                              // T
  int o, i, r, g;
  const uint16_t* fgrad;              // [o, i] binary16
  const bf16_t* A;                    // [r, i]
  const bf16_t* BT; int64_t ld_bt;    // [r, ld_bt], zero beyond o
  float* dscale; float* dzero;        // [o, i/g]
  float* dA_part;                     // [tiles_m, r, i]
  float* dB_part;                     // [2 * tiles_n, o, r]
  bf16_t* dWm;                        // [o, i]: the masked gradient (second form only); may be the fgrad array itself
  int tiles_m, tiles_n;
  int accumulate;                     // add dscale / dzero to what the outputs hold
};

__device__ __forceinline__ bf16x8_t as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 v = {a, b, c, d};
  return __builtin_bit_cast(bf16x8_t, v);
}

// STORE_MASKED = false: dA / dB partial sums in the epilogue (rank <= 32).  true: the masked tile is written out.
template <bool STORE_MASKED>
__global__ __launch_bounds__(T::NT) void dw_fused_kernel(FusedArgs p) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[FUSED_LDS];
#if defined(__HIP_DEVICE_COMPILE__)
  int tile_m, tile_n;
  gemm::tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * T::BM, n0 = tile_n * T::BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  gemm::Accum<T> acc;
#pragma unroll
  for (int a = 0; a < T::TM; ++a)
#pragma unroll
    for (int b = 0; b < T::TN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc.v[a][b][e] = 0.f;
  // The d(Wq)/d(scale) factors of the tile (128 KiB of a weight-sized array streamed once from HBM) are needed right
  // after the main loop.  They ride on the loads the loop issues for the four stages past the
  // end of K: tail stage q brings the factor rows of row block a = q (32 rows of the upper and of the lower wave
  // row) into the ring slot that stage would have used, 512 bytes per row, the 16-byte chunk c of row l at position
  // c ^ l so that the 32 rows a wave reads together spread over the banks.  Rows past the matrix lie beyond the
  // buffer and read as zero; columns past it get an out-of-range offset.
  typedef gemm::TailLoads<T::A_INSTR, T::B_INSTR> FTail;
  static_assert(T::D == 4 && T::A_INSTR == 4 && T::B_INSTR == 4 && T::STAGE == 64 * 512, "factor rows per tail stage");
  FTail ftail;
  ftail.base = p.fgrad;
  ftail.bytes = (int)((int64_t)p.o * p.i * 2);
  ftail.stage_bytes = (unsigned)(32 * p.i * 2);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int lr = (wave * 4 + c) * 2 + (lane >> 5);  // row inside the 32-row block
    const int col = n0 + (((lane & 31) ^ lr) << 3);   // first of the 8 columns this lane fetches
    const bool ok = col < p.i && m0 + lr < p.o;
    ftail.voff_a[c] = ok ? (unsigned)(((int64_t)(m0 + lr) * p.i + col) * 2) : gemm::OOB_OFFSET;
    ftail.voff_b[c] = ok && m0 + 128 + lr < p.o ? (unsigned)(((int64_t)(m0 + 128 + lr) * p.i + col) * 2)
                                                 : gemm::OOB_OFFSET;
  }
  gemm::mainloop<T, true, true, FTail>(p.dY, p.o, p.X, p.i, p.o, p.i, p.K, m0, n0, lds, acc, ftail);
  // the operand stages are consumed (mainloop ends with a barrier after the last fragment read); slots
  // (nk + q) % NS, q = 0 .. 3, hold the factor rows

  // ---- fragments of the LoRA factor A for the dB product: lane = rank index, 8 k-slots = the same
  //      column pattern the accumulator registers 8h .. 8h+7 of a lane group have
  bf16x8_t afrag[T::TN][2];
#pragma unroll
  for (int b = 0; b < T::TN; ++b) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = n0 + wn * 128 + b * 32 + 16 * h + 4 * lh;
      uint2 lo = make_uint2(0, 0), hi = make_uint2(0, 0);
      if (!STORE_MASKED && l32 < p.r && j < p.i) {  // i is a multiple of 32 here (g >= 32), so a 32-column tile is inside or outside as a whole
        lo = *reinterpret_cast<const uint2*>(p.A + (int64_t)l32 * p.i + j);
        hi = *reinterpret_cast<const uint2*>(p.A + (int64_t)l32 * p.i + j + 8);
      }
      afrag[b][h] = as_bf16x8(lo.x, lo.y, hi.x, hi.y);
    }
  }

  // The factors this lane needs: 64 pieces of 4 consecutive columns, one per (row block, column tile, register
  // group), all four row blocks read out of the ring slots (nk + a) % NS, after which the LDS is free for the
  // epilogue.  Rows and columns past the matrix: the LDS pieces are zeros, and so are their accumulators.
  typedef _Float16 h4 __attribute__((ext_vector_type(4)));
  h4 fpre[T::TM][T::TN][4];
  {
    const int nk = (p.K + T::BK - 1) / T::BK;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const unsigned char* rowp = lds + ((nk + a) % T::NS) * T::STAGE + wm * (32 * 512) + l32 * 512 + lh * 8;
#pragma unroll
      for (int b = 0; b < T::TN; ++b)
#pragma unroll
        for (int eg = 0; eg < 4; ++eg)
          fpre[a][b][eg] = *reinterpret_cast<const h4*>(rowp + (((wn * 16 + b * 4 + eg) ^ l32) << 4));
    }
  }
  __builtin_amdgcn_s_waitcnt(gemm::waitcnt_lgkm0());
  __builtin_amdgcn_s_barrier();  // every wave has its factors in registers: the LDS is free from here on

  const int G = p.i / p.g;
  auto put = [&](float* dst, float v) { *dst = p.accumulate ? *dst + v : v; };  // each element has one writer
  float keep_ds[T::TM], keep_db[T::TM];  // g == 256: this wave's half of the group, per row block
  f32x16_t accB[T::TM];

#pragma unroll
  for (int a = 0; a < T::TM; ++a) {
    const int row = m0 + wm * 128 + a * 32 + l32;  // the weight row this lane owns in block a
    const bool row_ok = row < p.o;
    float ds_b[T::TN], db_b[T::TN];
    uint32_t pk[T::TN][8];
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
      ds_b[b] = 0.f;
      db_b[b] = 0.f;
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        const h4 fh = fpre[a][b][eg];
        float xm[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = acc.v[a][b][4 * eg + e];
          const float f = (float)fh[e];
          // one use of the comparison (a second one keeps 64 lane masks alive in scalar registers and spills them):
          // x - xm is exactly x where the element is clipped and 0 elsewhere
          xm[e] = __builtin_fabsf16(fh[e]) > (_Float16)0.75f ? 0.f : x;  // decided on the stored binary16 value
          ds_b[b] = fmaf(x, f, ds_b[b]);
          db_b[b] += x - xm[e];
        }
        pk[b][2 * eg] = pack_bf16x2(xm[0], xm[1]);
        pk[b][2 * eg + 1] = pack_bf16x2(xm[2], xm[3]);
      }
    }

    // ---- group sums: the other half of every 8-column run lives in lane ^ 32
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
      ds_b[b] += __shfl_xor(ds_b[b], 32, 64);
      db_b[b] += __shfl_xor(db_b[b], 32, 64);
    }
    const int col0 = n0 + wn * 128;
    if (p.g == 32) {
#pragma unroll
      for (int b = 0; b < T::TN; ++b) {
        const int q = (col0 + b * 32) / 32;
        if (lh == 0 && row_ok && q < G) {
          put(p.dscale + (int64_t)row * G + q, ds_b[b]);
          put(p.dzero + (int64_t)row * G + q, db_b[b]);
        }
      }
    } else if (p.g == 64) {
#pragma unroll
      for (int b = 0; b < T::TN; b += 2) {
        const int q = (col0 + b * 32) / 64;
        if (lh == 0 && row_ok && q < G) {
          put(p.dscale + (int64_t)row * G + q, ds_b[b] + ds_b[b + 1]);
          put(p.dzero + (int64_t)row * G + q, db_b[b] + db_b[b + 1]);
        }
      }
    } else {
      const float ds = (ds_b[0] + ds_b[1]) + (ds_b[2] + ds_b[3]);
      const float db = (db_b[0] + db_b[1]) + (db_b[2] + db_b[3]);
      keep_ds[a] = ds;
      keep_db[a] = db;
      if (p.g == 128) {
        const int q = col0 / 128;
        if (lh == 0 && row_ok && q < G) {
          put(p.dscale + (int64_t)row * G + q, ds);
          put(p.dzero + (int64_t)row * G + q, db);
        }
      } else if (wn == 1 && lh == 0) {  // g == 256: hand the right half to the left wave
        float* sc = reinterpret_cast<float*>(lds + EP_TILE) + (wm * 128 + a * 32 + l32) * 2;
        sc[0] = ds;
        sc[1] = db;
      }
    }

    // ---- dB: (masked gradient) x A^T on the matrix core, 2 k-steps of 16 columns per 32-column tile
    if constexpr (!STORE_MASKED) {
      f32x16_t cb;
#pragma unroll
      for (int e = 0; e < 16; ++e) cb[e] = 0.f;
#pragma unroll
      for (int b = 0; b < T::TN; ++b) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const bf16x8_t gfrag = as_bf16x8(pk[b][4 * h], pk[b][4 * h + 1], pk[b][4 * h + 2], pk[b][4 * h + 3]);
          cb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gfrag, afrag[b][h], cb, 0, 0, 0);
        }
      }
      accB[a] = cb;
    }

    // ---- masked gradient to LDS as it lies in the registers: row p, 4 consecutive columns per 8-byte write
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        const int jl = wn * 128 + b * 32 + 8 * eg + 4 * lh;
        const int pl = wm * 128 + a * 32 + l32;
        *reinterpret_cast<uint2*>(lds + pl * EP_ROWB + jl * 2) = make_uint2(pk[b][2 * eg], pk[b][2 * eg + 1]);
      }
    }
  }

  if constexpr (STORE_MASKED) {
    __syncthreads();
    if (p.g == 256 && wn == 0 && lh == 0) {
      const int q = n0 / 256;
#pragma unroll
      for (int a = 0; a < T::TM; ++a) {
        const int row = m0 + wm * 128 + a * 32 + l32;
        const float* sc = reinterpret_cast<const float*>(lds + EP_TILE) + (wm * 128 + a * 32 + l32) * 2;
        if (row < p.o && q < G) {
          put(p.dscale + (int64_t)row * G + q, keep_ds[a] + sc[0]);
          put(p.dzero + (int64_t)row * G + q, keep_db[a] + sc[1]);
        }
      }
    }
    // ---- the masked tile leaves as it lies in LDS: 16 bytes per lane, a 512-byte row per 32 lanes; rows past o and
    //      columns past i (whole 16-byte pieces: i % 8 == 0) get an out-of-range offset
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(p.dWm, 0, (int)((int64_t)p.o * p.i * 2),
                                                                         0x00020000);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int ch = threadIdx.x & 31;
#pragma unroll 4
    for (int it = 0; it < 256 / 8; ++it) {
      const int row = it * 8 + (threadIdx.x >> 5);
      const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * EP_ROWB + ch * 16);
      const bool ok = m0 + row < p.o && n0 + ch * 8 < p.i;
      const unsigned vo = ok ? (unsigned)(((int64_t)(m0 + row) * p.i + n0 + ch * 8) * 2) : gemm::OOB_OFFSET;
      __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)vo, 0, 0);
    }
    return;
  }

  // ---- dB partials: register e of lane l is (row 8 (e/4) + 4 (l/32) + e%4 of the block, rank l % 32)
  //      Stored through a buffer descriptor of this partial's [o, r] block: rows past o fall beyond its range and are
  //      dropped by the hardware, lanes past the rank get an out-of-range offset, so the 64 stores carry no branches.
  {
    float* dst = p.dB_part + (int64_t)(tile_n * 2 + wn) * p.o * p.r;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(dst, 0, p.o * p.r * 4, 0x00020000);
    const unsigned lane_off = l32 < p.r ? (unsigned)(((m0 + wm * 128 + 4 * lh) * p.r + l32) * 4) : gemm::OOB_OFFSET;
#pragma unroll
    for (int a = 0; a < T::TM; ++a) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const unsigned row_off = (unsigned)((a * 32 + 8 * (e >> 2) + (e & 3)) * p.r * 4);  // uniform
        const float v = accB[a][e];
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rsrc, lane_off + row_off, 0, 0);
      }
    }
  }

  // B^T fragments of the dA product (lane = rank index, 8 consecutive rows): all 16 k-steps requested before the
  // barrier, so the product below does not wait for them one batch at a time
  uint4 bt_all[16];
#pragma unroll
  for (int ks = 0; ks < 16; ++ks) {
    const int64_t prow = (int64_t)m0 + ks * 16 + lh * 8;
    const bool live = l32 < p.r && prow < p.ld_bt;
    const uint4 v = *reinterpret_cast<const uint4*>(p.BT + (int64_t)(live ? l32 : 0) * p.ld_bt + (live ? prow : 0));
    bt_all[ks] = live ? v : make_uint4(0, 0, 0, 0);
  }

  __syncthreads();

  if (p.g == 256 && wn == 0 && lh == 0) {
    const int q = n0 / 256;
#pragma unroll
    for (int a = 0; a < T::TM; ++a) {
      const int row = m0 + wm * 128 + a * 32 + l32;
      const float* sc = reinterpret_cast<const float*>(lds + EP_TILE) + (wm * 128 + a * 32 + l32) * 2;
      if (row < p.o && q < G) {
        put(p.dscale + (int64_t)row * G + q, keep_ds[a] + sc[0]);
        put(p.dzero + (int64_t)row * G + q, keep_db[a] + sc[1]);
      }
    }
  }

  // ---- dA: B^T x (masked gradient); this wave takes the 64 columns 64 wave .. 64 wave + 63, all 256 rows
  f32x16_t ca[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int e = 0; e < 16; ++e) ca[nb][e] = 0.f;
  // The operand wants, per lane, 8 consecutive rows p of one column: the transposing LDS read delivers that from the
  // row-major tile.  Lane (g16, j16) of a read fetches 4 columns of row 8 (g16 / 2) + j16 / 4 (and of the row 4 below
  // for the second half); the hardware exchanges them within each group of 16 lanes.
  typedef short s16x4_t __attribute__((ext_vector_type(4)));
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr_t;
  const int j16 = lane & 15, g16 = lane >> 4;
  const unsigned tr_off = (unsigned)((8 * (g16 >> 1) + (j16 >> 2)) * EP_ROWB + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2);
#pragma unroll
  for (int ks = 0; ks < 16; ++ks) {
    const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bt_all[ks]);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const unsigned char* p0 = lds + tr_off + ks * 16 * EP_ROWB + (wave * 64 + nb * 32) * 2;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)p0);
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(p0 + 4 * EP_ROWB));
      const s16x8_t gv = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      ca[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, __builtin_bit_cast(bf16x8_t, gv), ca[nb], 0, 0, 0);
    }
  }
  {  // this tile row's [r, i] block through a buffer descriptor: rank indices past r fall beyond its range
    float* dst = p.dA_part + (int64_t)tile_m * p.r * p.i;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(dst, 0, p.r * p.i * 4, 0x00020000);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int j = n0 + wave * 64 + nb * 32 + l32;
      const unsigned lane_off = j < p.i ? (unsigned)((4 * lh * p.i + j) * 4) : gemm::OOB_OFFSET;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const unsigned k_off = (unsigned)((8 * (e >> 2) + (e & 3)) * p.i * 4);  // uniform
        const float v = ca[nb][e];
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rsrc, lane_off + k_off, 0, 0);
      }
    }
  }
#endif
}

}  // namespace

bool dw_fused_supported(const LayerDims& d) {
  const bool g_ok = d.g == 32 || d.g == 64 || d.g == 128 || d.g == 256;
  return g_ok && d.r <= 32 && d.i < (1 << 22);  // 32-bit offsets of factor rows up to 255 past the last one
}

// The second form (masked gradient stored as bfloat16, dA / dB as thin products): ranks 33 .. 256 that are multiples
// of 8 (16-byte rows of B and of the binary32 results), in-features a multiple of the 32-wide k-step of the dB product.
bool dw_masked_supported(const LayerDims& d) {
  const bool g_ok = d.g == 32 || d.g == 64 || d.g == 128 || d.g == 256;
  return g_ok && d.r > 32 && d.r <= 256 && d.r % 8 == 0 && d.i % 32 == 0 && d.i < (1 << 22);
}

void dw_fused_tiles(const LayerDims& d, int* tiles_m, int* tiles_n) {
  *tiles_m = (int)((d.o + T::BM - 1) / T::BM);
  *tiles_n = (int)((d.i + T::BN - 1) / T::BN);
}

void launch_dw_fused(const LayerDims& d, const bf16_t* dY, const bf16_t* X, const uint16_t* fgrad, const bf16_t* A,
                     const bf16_t* BT, int64_t ld_bt, float* dscale, float* dzero, float* dA_part, float* dB_part,
                     hipStream_t stream) {
  FusedArgs p;
  p.dY = dY;
  p.X = X;
  p.K = (int)d.T;
  p.o = (int)d.o; p.i = (int)d.i; p.r = d.r; p.g = d.g;
  p.fgrad = fgrad; p.A = A; p.BT = BT; p.ld_bt = ld_bt;
  p.dscale = dscale; p.dzero = dzero; p.dA_part = dA_part; p.dB_part = dB_part;
  p.dWm = nullptr;
  dw_fused_tiles(d, &p.tiles_m, &p.tiles_n);
  p.accumulate = d.accumulate ? 1 : 0;
  hipLaunchKernelGGL(dw_fused_kernel<false>, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(T::NT), 0, stream, p);
}

void launch_dw_masked(const LayerDims& d, const bf16_t* dY, const bf16_t* X, const uint16_t* fgrad, float* dscale,
                      float* dzero, bf16_t* dWm, hipStream_t stream) {
  FusedArgs p = {};
  p.dY = dY;
  p.X = X;
  p.K = (int)d.T;
  p.o = (int)d.o; p.i = (int)d.i; p.r = d.r; p.g = d.g;
  p.fgrad = fgrad;
  p.dscale = dscale; p.dzero = dzero;
  p.dWm = dWm;
  dw_fused_tiles(d, &p.tiles_m, &p.tiles_n);
  p.accumulate = d.accumulate ? 1 : 0;
  hipLaunchKernelGGL(dw_fused_kernel<true>, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(T::NT), 0, stream, p);
}

}  // namespace l4q
