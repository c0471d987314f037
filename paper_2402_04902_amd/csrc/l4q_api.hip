// C ABI of the library: argument validation, workspace carving and kernel sequencing.
// See include/l4q.h for the contract of every entry point.
#include "../../include/l4q.h"

#include "l4q_kernels.h"

#include <cmath>
#include <mutex>
#include <utility>
#include <vector>

namespace {

using l4q::bf16_t;
using l4q::LayerDims;

constexpr size_t kWsAlign = 256;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

int check_desc(const l4q_desc* d, bool need_tokens) {
  if (!d) return L4Q_ERR_NULL;
  if (d->dtype != L4Q_DTYPE_F32 && d->dtype != L4Q_DTYPE_BF16) return L4Q_ERR_DTYPE;
  if (d->flags & ~(int32_t)(L4Q_FLAG_UNFUSED_BACKWARD | L4Q_FLAG_ACCUMULATE_GRADS)) return L4Q_ERR_DTYPE;
  if (d->bits < 2 || d->bits > 8) return L4Q_ERR_BITS;
  if (d->in_features < 1 || d->out_features < 1 || d->rank < 1 || d->rank > 256) return L4Q_ERR_SHAPE;
  if (need_tokens && d->tokens < 1) return L4Q_ERR_SHAPE;
  if (d->in_features >= (1ll << 30) || d->out_features >= (1ll << 30) || d->tokens >= (1ll << 30)) return L4Q_ERR_SHAPE;
  if (d->group_size < 4 || !is_pow2(d->group_size) || d->in_features % d->group_size != 0) return L4Q_ERR_SHAPE;
  if (d->dtype == L4Q_DTYPE_BF16) {
    if (d->group_size % 8 != 0 || d->out_features % 8 != 0) return L4Q_ERR_SHAPE;
    // the matrix-core kernels address each operand with 32-bit byte offsets below 1 GiB
    const int64_t lim = (1ll << 29) - (1ll << 20);  // elements
    const int64_t t = need_tokens ? d->tokens : 1;
    // the workspace copies are padded: Wq is [o, i rounded up to 32], Wq^T is [i, o rounded up to 32]
    const int64_t ipad = (d->in_features + 31) / 32 * 32, opad = (d->out_features + 31) / 32 * 32;
    if (t * d->in_features >= lim || t * d->out_features >= lim || d->out_features * ipad >= lim ||
        d->in_features * opad >= lim)
      return L4Q_ERR_SHAPE;
  }
  if (!(d->alpha == d->alpha)) return L4Q_ERR_SHAPE;
  return L4Q_OK;
}

LayerDims dims_of(const l4q_desc* d) {
  LayerDims L;
  L.T = d->tokens;
  L.i = d->in_features;
  L.o = d->out_features;
  L.r = d->rank;
  L.bits = d->bits;
  L.g = d->group_size;
  L.gamma = d->alpha / (float)d->rank;
  L.qn = -(float)(1 << (d->bits - 1));
  L.qp = (float)((1 << (d->bits - 1)) - 1);
  L.accumulate = (d->flags & L4Q_FLAG_ACCUMULATE_GRADS) != 0;
  return L;
}

struct Carver {
  unsigned char* base;
  size_t used = 0;
  explicit Carver(void* p) : base(static_cast<unsigned char*>(p)) {}
  template <class T> T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
    used += align_up(count * sizeof(T), kWsAlign);
    return p;
  }
};

struct FwdWs {
  void* wq;      // [o,ipad] storage type; ipad = i rounded up to the GEMM k-step in bf16 mode (bf16: in blocks of 32 columns)
  float* splitk;  // [slices][T][o] binary32 tiles of the forward product's k-slices (bf16, few tokens), else null
  int64_t ipad;
  size_t bytes;
};
struct BwdWs {
  bool fused;        // bf16: weight-gradient GEMM with the fused quantizer epilogue
  bool masked;       // bf16, ranks above 32: its second form (masked gradient stored as bf16, thin dA / dB products);
                     // the masked gradient takes the place of the factor array, tile by tile
  float* rawA;       // [slices_a][r,i]            (bf16 masked)
  float* rawB;       // [slices_b][o,r]            (bf16 masked)
  int slices_a, slices_b;
  float* wq32;       // [o,i]                      (binary32 mode)
  bf16_t* wqT;       // [i,opad], in blocks of 32  (bf16)
  uint16_t* fgrad;   // [o,i] binary16             (bf16 fused)
  bf16_t* bT;        // [r,opad]                   (bf16 fused)
  float* dB_part;    // [2 tiles_n, o, r]          (bf16 fused)
  float* dwq;        // [o,i]                      (binary32 mode, bf16 unfused)
  float* dA_part;    // [tiles_m or ceil(o/kDaRowBlock), r, i]
  float* splitk;     // [slices][T][i] binary32 tiles of the dX product's k-slices (bf16, few tokens), else null
  int64_t opad;
  int tiles_m, tiles_n;
  size_t bytes;
};

FwdWs carve_fwd(const l4q_desc* d, void* ws) {
  Carver c(ws);
  FwdWs w;
  w.ipad = d->dtype == L4Q_DTYPE_BF16 ? (int64_t)align_up((size_t)d->in_features, 32) : d->in_features;
  const size_t n = (size_t)d->out_features * (size_t)w.ipad;
  w.wq = d->dtype == L4Q_DTYPE_BF16 ? (void*)c.take<bf16_t>(n) : (void*)c.take<float>(n);
  w.splitk = nullptr;
  if (d->dtype == L4Q_DTYPE_BF16) {
    const int slices = l4q::gemm_nt_splitk_slices(d->tokens, d->out_features, w.ipad);
    if (slices > 1) w.splitk = c.take<float>((size_t)slices * (size_t)d->tokens * (size_t)d->out_features);
  }
  w.bytes = c.used;
  return w;
}

BwdWs carve_bwd(const l4q_desc* d, void* ws) {
  Carver c(ws);
  BwdWs w = {};
  const size_t o = (size_t)d->out_features, i = (size_t)d->in_features, r = (size_t)d->rank;
  const size_t n = o * i;
  // Wq^T is zero-padded along its out-feature axis to the k-step of the matrix-core kernels
  w.opad = (int64_t)align_up(o, 32);
  const LayerDims L = dims_of(d);
  const size_t nrb = (o + l4q::kDaRowBlock - 1) / l4q::kDaRowBlock;
  if (d->dtype == L4Q_DTYPE_BF16) {
    w.fused = !(d->flags & L4Q_FLAG_UNFUSED_BACKWARD) && l4q::dw_fused_supported(L);
    w.masked = !(d->flags & L4Q_FLAG_UNFUSED_BACKWARD) && l4q::dw_masked_supported(L);
    w.wqT = c.take<bf16_t>(i * (size_t)w.opad);
    if (w.masked) {
      w.fgrad = c.take<uint16_t>(n);
      l4q::dw_masked_product_slices(L, &w.slices_a, &w.slices_b);
      w.rawA = c.take<float>((size_t)w.slices_a * r * i);
      w.rawB = c.take<float>((size_t)w.slices_b * o * r);
    } else if (w.fused) {
      l4q::dw_fused_tiles(L, &w.tiles_m, &w.tiles_n);
      w.fgrad = c.take<uint16_t>(n);
      w.bT = c.take<bf16_t>(r * (size_t)w.opad);
      w.dB_part = c.take<float>(2 * (size_t)w.tiles_n * o * r);
      w.dA_part = c.take<float>((size_t)w.tiles_m * r * i);
    } else {
      w.dwq = c.take<float>(n);
      w.dA_part = c.take<float>(nrb * r * i);
    }
  } else {
    w.wq32 = c.take<float>(n);
    w.dwq = c.take<float>(n);
    w.dA_part = c.take<float>(nrb * r * i);
  }
  if (d->dtype == L4Q_DTYPE_BF16) {  // (last: the arrays above keep their places whatever the token count)
    const int slices = l4q::gemm_nt_splitk_slices(d->tokens, d->in_features, w.opad);
    if (slices > 1) w.splitk = c.take<float>((size_t)slices * (size_t)d->tokens * i);
  }
  w.bytes = c.used;
  return w;
}

int launch_status() { return hipGetLastError() == hipSuccess ? L4Q_OK : L4Q_ERR_LAUNCH; }

// ---- device-resident scratch of l4q_quant_errors_static ----
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: the device address is asked for once per device and kept in g_static_scratch.
constexpr size_t kStaticScratchBytes = L4Q_STATIC_SCRATCH_BYTES;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
struct StaticScratch {
  std::mutex mu;
  void* ptr[kMaxDevices] = {};
} g_static_scratch;

// Device address of `scratch` on the current device (null on failure).
void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_static_scratch.mu);
  if (!g_static_scratch.ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_static_scratch.ptr[dev] = p;
  }
  return g_static_scratch.ptr[dev];
}

// ---- opt-in timing of the GEMM and merge + quantize launches (l4q_profile_gemm) ----
enum { kKindGemm = 0, kKindMergeFwd = 1, kKindMergeBwd = 2, kKinds = 3 };
struct Profile {
  std::mutex mu;
  bool on = false;
  struct Rec { hipEvent_t e0, e1; int kind; };
  std::vector<Rec> events;
  double work[kKinds] = {0.0, 0.0, 0.0};  // FLOPs (GEMM) or algorithmic bytes (merge + quantize)
} g_prof;

// Brackets what is enqueued between construction and destruction with two events on `stream` while profiling is on.
struct Timed {
  hipStream_t stream;
  int kind;
  double work;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool timed = false;
  Timed(hipStream_t s, int k, double w) : stream(s), kind(k), work(w) {
    {
      std::lock_guard<std::mutex> lk(g_prof.mu);
      if (g_prof.on && hipEventCreate(&e0) == hipSuccess) {
        if (hipEventCreate(&e1) == hipSuccess) timed = true;
        else (void)hipEventDestroy(e0);
      }
    }
    if (timed) (void)hipEventRecord(e0, stream);
  }
  ~Timed() {
    if (!timed) return;
    (void)hipEventRecord(e1, stream);
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.events.push_back({e0, e1, kind});
    g_prof.work[kind] += work;
  }
};

// Enqueue one bf16 GEMM (rows of A end at K_algorithmic, the padded operand B at K).
// `splitk`: room for the k-slices' tiles where the product has too few tiles for the chip (or null: one pass).
void gemm_nt(const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
             int64_t K_algorithmic, bf16_t* C, int64_t ldc, hipStream_t stream, float* splitk = nullptr) {
  Timed t(stream, kKindGemm, 2.0 * (double)M * (double)N * (double)K_algorithmic);
  l4q::launch_gemm_bf16_nt(A, lda, B, ldb, M, N, K, K_algorithmic, C, ldc, stream, splitk);
}

// The fused weight-gradient kernel is a GEMM launch too: time it the same way.
void dw_fused(const LayerDims& d, const BwdWs& w, const bf16_t* dY, const bf16_t* X, const bf16_t* A, float* dscale,
              float* dzero, hipStream_t stream) {
  Timed t(stream, kKindGemm, 2.0 * (double)d.o * (double)d.i * (double)d.T);
  l4q::launch_dw_fused(d, dY, X, w.fgrad, A, w.bT, w.opad, dscale, dzero, w.dA_part, w.dB_part, stream);
}

// The merge + quantize pass of the bf16 layer.  Algorithmic bytes: the frozen weight read once, scale and zero, and
// what the pass must hand on: Wq (forward), or Wq^T and the gradient factor (fused backward).
void merge_quant_bf16(const LayerDims& d, const bf16_t* W0, const bf16_t* A, const bf16_t* B, const float* scale,
                      const float* zero, const l4q::MergeQuantOut<bf16_t>& mq, hipStream_t stream) {
  const double oi = (double)d.o * (double)d.i;
  const double bytes = 2.0 * oi + 8.0 * (double)d.o * (double)d.G() + (mq.wq ? 2.0 * oi : 0.0) +
                       (mq.wqT ? 2.0 * oi : 0.0) + (mq.fgrad ? 2.0 * oi : 0.0);
  Timed t(stream, mq.wq ? kKindMergeFwd : kKindMergeBwd, bytes);
  l4q::launch_merge_quant<bf16_t>(d, W0, A, B, scale, zero, mq, stream);
}

struct QlFwdWs {
  void* wq;       // [o, ipad] storage type (bf16: in blocks of 32 columns)
  float* xa;      // [T, r]
  int64_t ipad;
  size_t bytes;
};
struct QlBwdWs {
  float* wq32;    // [o, i]      (binary32 mode)
  bf16_t* wqT;    // [i, opad], in blocks of 32   (bf16)
  float* dwq;     // [o, i]      the stored weight gradient
  float* dyb;     // [T, r]
  float* xa;      // [T, r]
  float* part;    // [token blocks, r, max(i, o)]
  int64_t opad;
  size_t bytes;
};

QlFwdWs carve_ql_fwd(const l4q_desc* d, void* ws) {
  Carver c(ws);
  QlFwdWs w;
  w.ipad = d->dtype == L4Q_DTYPE_BF16 ? (int64_t)align_up((size_t)d->in_features, 32) : d->in_features;
  const size_t n = (size_t)d->out_features * (size_t)w.ipad;
  w.wq = d->dtype == L4Q_DTYPE_BF16 ? (void*)c.take<bf16_t>(n) : (void*)c.take<float>(n);
  w.xa = c.take<float>((size_t)d->tokens * (size_t)d->rank);
  w.bytes = c.used;
  return w;
}

QlBwdWs carve_ql_bwd(const l4q_desc* d, void* ws) {
  Carver c(ws);
  QlBwdWs w = {};
  const size_t o = (size_t)d->out_features, i = (size_t)d->in_features, r = (size_t)d->rank, T = (size_t)d->tokens;
  w.opad = (int64_t)align_up(o, 32);
  if (d->dtype == L4Q_DTYPE_BF16) w.wqT = c.take<bf16_t>(i * (size_t)w.opad);
  else w.wq32 = c.take<float>(o * i);
  w.dwq = c.take<float>(o * i);
  w.dyb = c.take<float>(T * r);
  w.xa = c.take<float>(T * r);
  w.part = c.take<float>((size_t)l4q::lora_tn_blocks((int64_t)T) * r * (i > o ? i : o));
  w.bytes = c.used;
  return w;
}

}  // namespace

extern "C" {

int l4q_version(void) { return L4Q_VERSION; }

const char* l4q_status_string(int status) {
  switch (status) {
    case L4Q_OK: return "ok";
    case L4Q_ERR_NULL: return "a required pointer is NULL";
    case L4Q_ERR_SHAPE: return "invalid shape (dimension, group size or divisibility rule)";
    case L4Q_ERR_BITS: return "bits must be in 2..8";
    case L4Q_ERR_DTYPE: return "unknown dtype or flags";
    case L4Q_ERR_ALIGN: return "pointer not sufficiently aligned";
    case L4Q_ERR_WORKSPACE: return "workspace missing or too small";
    case L4Q_ERR_LAUNCH: return "kernel launch failed";
    case L4Q_ERR_METHOD: return "unknown initialisation method";
    case L4Q_ERR_TOO_LARGE: return "problem needs more scratch than this entry point's fixed device array holds";
    default: return "unknown status";
  }
}

int l4q_workspace_bytes(const l4q_desc* desc, size_t* forward_bytes, size_t* backward_bytes) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (forward_bytes) *forward_bytes = carve_fwd(desc, nullptr).bytes;
  if (backward_bytes) *backward_bytes = carve_bwd(desc, nullptr).bytes;
  return L4Q_OK;
}

int l4q_forward(const l4q_desc* desc, const void* X, const void* W0, const void* A, const void* B,
                const float* scale, const float* zero, void* Y, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (!X || !W0 || !A || !B || !scale || !zero || !Y) return L4Q_ERR_NULL;
  if (!aligned(X, 16) || !aligned(W0, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(scale, 16) ||
      !aligned(zero, 16) || !aligned(Y, 16))
    return L4Q_ERR_ALIGN;
  const FwdWs w = carve_fwd(desc, workspace);
  if (!workspace || workspace_bytes < w.bytes) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    bf16_t* wq = static_cast<bf16_t*>(w.wq);
    l4q::MergeQuantOut<bf16_t> mq;
    mq.wq = wq;
    mq.ld_wq = w.ipad;
    merge_quant_bf16(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero, mq, stream);
    gemm_nt((const bf16_t*)X, d.i, wq, w.ipad, d.T, d.o, w.ipad, d.i, (bf16_t*)Y, d.o, stream, w.splitk);
  } else {
    float* wq = static_cast<float*>(w.wq);
    l4q::MergeQuantOut<float> mq;
    mq.wq = wq;
    mq.ld_wq = d.i;
    l4q::launch_merge_quant<float>(d, (const float*)W0, (const float*)A, (const float*)B, scale, zero, mq, stream);
    // Y[t,p] = sum_j X[t,j] Wq[p,j]
    l4q::launch_sgemm((const float*)X, d.i, 1, wq, 1, d.i, (float*)Y, d.o, d.T, d.o, d.i, 1.f, stream);
  }
  return launch_status();
}

int l4q_backward(const l4q_desc* desc, const void* X, const void* dY, const void* W0, const void* A,
                 const void* B, const float* scale, const float* zero, void* dX, float* dA, float* dB,
                 float* dscale, float* dzero, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (!X || !dY || !W0 || !A || !B || !scale || !zero || !dX || !dA || !dB || !dscale || !dzero) return L4Q_ERR_NULL;
  const void* ptrs[] = {X, dY, W0, A, B, scale, zero, dX, dA, dB, dscale, dzero};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const BwdWs w = carve_bwd(desc, workspace);
  if (!workspace || workspace_bytes < w.bytes) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    const bf16_t* W0b = (const bf16_t*)W0;
    const bf16_t* Ab = (const bf16_t*)A;
    const bf16_t* Bb = (const bf16_t*)B;
    // recompute the quantizer (nothing was kept from the forward pass): Wq^T for dX = dY . Wq and,
    // for the fused epilogue, the per-element d(Wq)/d(scale) factor
    l4q::MergeQuantOut<bf16_t> mq;
    mq.wqT = w.wqT;
    mq.ld_wqT = w.opad;
    mq.fgrad = w.fgrad;  // null when unfused
    mq.bT = w.fused ? w.bT : nullptr;  // (the masked form reads B as it lies)
    merge_quant_bf16(d, W0b, Ab, Bb, scale, zero, mq, stream);
    // dWq = dY^T . X, both operands read as they lie in memory.  The fused kernel goes first: the factor array the
    // merge pass has just written is then still in the memory-side cache when the epilogues ask for it.
    if (w.fused) {
      dw_fused(d, w, (const bf16_t*)dY, (const bf16_t*)X, Ab, dscale, dzero, stream);
      l4q::launch_reduce_two_partials(w.dA_part, w.tiles_m, (int64_t)d.r * d.i, dA, w.dB_part, 2 * w.tiles_n,
                                      d.o * d.r, dB, d.gamma, d.accumulate, stream);
    }
    if (w.masked) {
      {
        Timed t(stream, kKindGemm, 2.0 * (double)d.o * (double)d.i * (double)d.T);
        // in place: a workgroup has its tile of the factors in LDS before it writes the tile's masked gradient, and no
        // other workgroup touches that tile
        l4q::launch_dw_masked(d, (const bf16_t*)dY, (const bf16_t*)X, w.fgrad, dscale, dzero, (bf16_t*)w.fgrad, stream);
      }
      l4q::launch_dw_masked_products(d, (const bf16_t*)w.fgrad, Ab, Bb, w.rawA, w.rawB, stream);
      l4q::launch_reduce_two_partials(w.rawA, w.slices_a, (int64_t)d.r * d.i, dA, w.rawB, w.slices_b, d.o * d.r, dB, d.gamma,
                                      d.accumulate, stream);
    }
    gemm_nt((const bf16_t*)dY, d.o, w.wqT, w.opad, d.T, d.i, w.opad, d.o, (bf16_t*)dX, d.i, stream, w.splitk);
    if (!w.fused && !w.masked) {
      l4q::launch_gemm_bf16_kmajor_f32((const bf16_t*)dY, d.o, (const bf16_t*)X, d.i, d.o, d.i, d.T, w.dwq, d.i, stream);
      l4q::launch_quant_grads<bf16_t>(d, W0b, Ab, Bb, scale, zero, w.dwq, dscale, dzero, dB, stream);
      l4q::launch_dA<bf16_t>(d, Bb, w.dwq, w.dA_part, dA, stream);
    }
  } else {
    const float* W0f = (const float*)W0;
    const float* Af = (const float*)A;
    const float* Bf = (const float*)B;
    float* wq = w.wq32;
    l4q::MergeQuantOut<float> mq;
    mq.wq = wq;
    mq.ld_wq = d.i;
    l4q::launch_merge_quant<float>(d, W0f, Af, Bf, scale, zero, mq, stream);
    // dX[t,j] = sum_p dY[t,p] Wq[p,j]
    l4q::launch_sgemm((const float*)dY, d.o, 1, wq, d.i, 1, (float*)dX, d.i, d.T, d.i, d.o, 1.f, stream);
    // dWq[p,j] = sum_t dY[t,p] X[t,j]
    l4q::launch_sgemm((const float*)dY, 1, d.o, (const float*)X, d.i, 1, w.dwq, d.i, d.o, d.i, d.T, 1.f, stream);
    l4q::launch_quant_grads<float>(d, W0f, Af, Bf, scale, zero, w.dwq, dscale, dzero, dB, stream);
    l4q::launch_dA<float>(d, Bf, w.dwq, w.dA_part, dA, stream);
  }
  return launch_status();
}

int l4q_export_codes(const l4q_desc* desc, const void* W0, const void* A, const void* B, const float* scale,
                     const float* zero, int8_t* codes, float* wcomb, uint8_t* mask, void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (!W0 || !A || !B || !scale || !zero) return L4Q_ERR_NULL;
  const void* ptrs[] = {W0, A, B, scale, zero, codes, wcomb, mask};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    l4q::MergeQuantOut<bf16_t> mq;
    mq.codes = codes;
    mq.wcomb = wcomb;
    mq.mask = mask;
    l4q::launch_merge_quant<bf16_t>(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero, mq, stream);
  } else {
    l4q::MergeQuantOut<float> mq;
    mq.codes = codes;
    mq.wcomb = wcomb;
    mq.mask = mask;
    l4q::launch_merge_quant<float>(d, (const float*)W0, (const float*)A, (const float*)B, scale, zero, mq, stream);
  }
  return launch_status();
}

int l4q_init_qparams(const l4q_desc* desc, const void* W0, const void* A, const void* B, int method, float* scale,
                     float* zero, void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (method != L4Q_INIT_ASYMM && method != L4Q_INIT_SYMM && method != L4Q_INIT_L4Q && method != L4Q_INIT_LSQPLUS)
    return L4Q_ERR_METHOD;
  if (method == L4Q_INIT_LSQPLUS && desc->group_size > 256) return L4Q_ERR_METHOD;
  if (!W0 || !A || !B || !scale || !zero) return L4Q_ERR_NULL;
  const void* ptrs[] = {W0, A, B, scale, zero};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16)
    l4q::launch_init_qparams<bf16_t>(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, method, scale, zero,
                                     stream);
  else
    l4q::launch_init_qparams<float>(d, (const float*)W0, (const float*)A, (const float*)B, method, scale, zero,
                                    stream);
  return launch_status();
}

int l4q_export_packed(const l4q_desc* desc, const void* W0, const void* A, const void* B, const float* scale,
                      const float* zero, uint32_t* packed, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (desc->in_features % 32 != 0) return L4Q_ERR_SHAPE;
  if (!W0 || !A || !B || !scale || !zero || !packed) return L4Q_ERR_NULL;
  const void* ptrs[] = {W0, A, B, scale, zero, packed};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const size_t need = (size_t)desc->out_features * (size_t)desc->in_features;
  if (!workspace || workspace_bytes < need) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  int8_t* codes = static_cast<int8_t*>(workspace);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    l4q::MergeQuantOut<bf16_t> mq;
    mq.codes = codes;
    l4q::launch_merge_quant<bf16_t>(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero, mq, stream);
  } else {
    l4q::MergeQuantOut<float> mq;
    mq.codes = codes;
    l4q::launch_merge_quant<float>(d, (const float*)W0, (const float*)A, (const float*)B, scale, zero, mq, stream);
  }
  l4q::launch_pack_codes(codes, d.o, d.i, d.bits, packed, stream);
  return launch_status();
}

int l4q_quantized_forward(const l4q_desc* desc, const void* X, const uint32_t* packed, const float* scale,
                          const float* zero, void* Y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (desc->dtype != L4Q_DTYPE_BF16) return L4Q_ERR_DTYPE;
  const LayerDims d = dims_of(desc);
  if (!l4q::qgemm_supported(d)) return (d.bits == 2 || d.bits == 3 || d.bits == 4 || d.bits == 8) ? L4Q_ERR_SHAPE : L4Q_ERR_BITS;
  if (!X || !packed || !scale || !zero || !Y) return L4Q_ERR_NULL;
  const void* ptrs[] = {X, packed, scale, zero, Y};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  if (workspace && !aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  (void)hipGetLastError();
  l4q::launch_qgemm(d, (const bf16_t*)X, packed, scale, zero, (bf16_t*)Y, static_cast<float*>(workspace),
                    workspace ? workspace_bytes : 0, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int l4q_quantized_forward_workspace_bytes(const l4q_desc* desc, size_t* bytes) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (!bytes) return L4Q_ERR_NULL;
  const LayerDims d = dims_of(desc);
  *bytes = desc->dtype == L4Q_DTYPE_BF16 && l4q::qgemm_supported(d) ? l4q::qgemm_workspace_bytes(d) : 0;
  return L4Q_OK;
}

int l4q_qatlora_workspace_bytes(const l4q_desc* desc, size_t* forward_bytes, size_t* backward_bytes) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (forward_bytes) *forward_bytes = carve_ql_fwd(desc, nullptr).bytes;
  if (backward_bytes) *backward_bytes = carve_ql_bwd(desc, nullptr).bytes;
  return L4Q_OK;
}

int l4q_qatlora_forward(const l4q_desc* desc, const void* X, const void* W0, const void* A, const void* B,
                        const float* scale, const float* zero, void* Y, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (!X || !W0 || !A || !B || !scale || !zero || !Y) return L4Q_ERR_NULL;
  if (!aligned(X, 16) || !aligned(W0, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(scale, 16) ||
      !aligned(zero, 16) || !aligned(Y, 16))
    return L4Q_ERR_ALIGN;
  const QlFwdWs w = carve_ql_fwd(desc, workspace);
  if (!workspace || workspace_bytes < w.bytes) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  LayerDims dq = d;   // the quantizer sees the frozen weight alone
  dq.gamma = 0.f;
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    bf16_t* wq = static_cast<bf16_t*>(w.wq);
    l4q::MergeQuantOut<bf16_t> mq;
    mq.wq = wq;
    mq.ld_wq = w.ipad;
    l4q::launch_merge_quant<bf16_t>(dq, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero, mq, stream);
    gemm_nt((const bf16_t*)X, d.i, wq, w.ipad, d.T, d.o, w.ipad, d.i, (bf16_t*)Y, d.o, stream);
    l4q::launch_lora_down<bf16_t>((const bf16_t*)X, d.T, d.i, (const bf16_t*)A, d.r, false, w.xa, stream);
    l4q::launch_lora_up<bf16_t>((bf16_t*)Y, d.T, d.o, w.xa, (const bf16_t*)B, d.r, true, d.gamma, stream);
  } else {
    float* wq = static_cast<float*>(w.wq);
    l4q::MergeQuantOut<float> mq;
    mq.wq = wq;
    mq.ld_wq = d.i;
    l4q::launch_merge_quant<float>(dq, (const float*)W0, (const float*)A, (const float*)B, scale, zero, mq, stream);
    l4q::launch_sgemm((const float*)X, d.i, 1, wq, 1, d.i, (float*)Y, d.o, d.T, d.o, d.i, 1.f, stream);
    l4q::launch_lora_down<float>((const float*)X, d.T, d.i, (const float*)A, d.r, false, w.xa, stream);
    l4q::launch_lora_up<float>((float*)Y, d.T, d.o, w.xa, (const float*)B, d.r, true, d.gamma, stream);
  }
  return launch_status();
}

int l4q_qatlora_backward(const l4q_desc* desc, const void* X, const void* dY, const void* W0, const void* A,
                         const void* B, const float* scale, const float* zero, void* dX, float* dA, float* dB,
                         float* dscale, float* dzero, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_desc(desc, true);
  if (st != L4Q_OK) return st;
  if (!X || !dY || !W0 || !A || !B || !scale || !zero || !dX || !dA || !dB || !dscale || !dzero) return L4Q_ERR_NULL;
  const void* ptrs[] = {X, dY, W0, A, B, scale, zero, dX, dA, dB, dscale, dzero};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const QlBwdWs w = carve_ql_bwd(desc, workspace);
  if (!workspace || workspace_bytes < w.bytes) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  LayerDims dq = d;
  dq.gamma = 0.f;
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16) {
    const bf16_t *Xb = (const bf16_t*)X, *dYb = (const bf16_t*)dY, *W0b = (const bf16_t*)W0, *Ab = (const bf16_t*)A,
                 *Bb = (const bf16_t*)B;
    l4q::MergeQuantOut<bf16_t> mq;
    mq.wqT = w.wqT;
    mq.ld_wqT = w.opad;
    l4q::launch_merge_quant<bf16_t>(dq, W0b, Ab, Bb, scale, zero, mq, stream);
    gemm_nt(dYb, d.o, w.wqT, w.opad, d.T, d.i, w.opad, d.o, (bf16_t*)dX, d.i, stream);
    l4q::launch_lora_down<bf16_t>(dYb, d.T, d.o, Bb, d.r, true, w.dyb, stream);
    l4q::launch_lora_up<bf16_t>((bf16_t*)dX, d.T, d.i, w.dyb, Ab, d.r, false, d.gamma, stream);
    // the weight gradient is materialised: scale and zero are updated from it
    l4q::launch_gemm_bf16_kmajor_f32(dYb, d.o, Xb, d.i, d.o, d.i, d.T, w.dwq, d.i, stream);
    l4q::launch_quant_grads<bf16_t>(dq, W0b, Ab, Bb, scale, zero, w.dwq, dscale, dzero, dB, stream);  // its dB term is gamma = 0
    l4q::launch_lora_down<bf16_t>(Xb, d.T, d.i, Ab, d.r, false, w.xa, stream);
    l4q::launch_lora_tn<bf16_t>(w.dyb, Xb, d.T, d.i, d.r, false, w.part, d.gamma, dA, d.accumulate, stream);
    l4q::launch_lora_tn<bf16_t>(w.xa, dYb, d.T, d.o, d.r, true, w.part, d.gamma, dB, d.accumulate, stream);
  } else {
    const float *Xf = (const float*)X, *dYf = (const float*)dY, *W0f = (const float*)W0, *Af = (const float*)A,
                *Bf = (const float*)B;
    l4q::MergeQuantOut<float> mq;
    mq.wq = w.wq32;
    mq.ld_wq = d.i;
    l4q::launch_merge_quant<float>(dq, W0f, Af, Bf, scale, zero, mq, stream);
    l4q::launch_sgemm(dYf, d.o, 1, w.wq32, d.i, 1, (float*)dX, d.i, d.T, d.i, d.o, 1.f, stream);
    l4q::launch_lora_down<float>(dYf, d.T, d.o, Bf, d.r, true, w.dyb, stream);
    l4q::launch_lora_up<float>((float*)dX, d.T, d.i, w.dyb, Af, d.r, false, d.gamma, stream);
    l4q::launch_sgemm(dYf, 1, d.o, Xf, d.i, 1, w.dwq, d.i, d.o, d.i, d.T, 1.f, stream);
    l4q::launch_quant_grads<float>(dq, W0f, Af, Bf, scale, zero, w.dwq, dscale, dzero, dB, stream);
    l4q::launch_lora_down<float>(Xf, d.T, d.i, Af, d.r, false, w.xa, stream);
    l4q::launch_lora_tn<float>(w.dyb, Xf, d.T, d.i, d.r, false, w.part, d.gamma, dA, d.accumulate, stream);
    l4q::launch_lora_tn<float>(w.xa, dYf, d.T, d.o, d.r, true, w.part, d.gamma, dB, d.accumulate, stream);
  }
  return launch_status();
}

int l4q_quant_errors(const l4q_desc* desc, const void* W0, const void* A, const void* B, const float* scale,
                     const float* zero, float* errors, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (!W0 || !A || !B || !scale || !zero || !errors) return L4Q_ERR_NULL;
  const void* ptrs[] = {W0, A, B, scale, zero, errors};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const size_t need = (size_t)desc->out_features * (size_t)((desc->in_features + 255) / 256) * 2 * sizeof(float);
  if (!workspace || workspace_bytes < need) return L4Q_ERR_WORKSPACE;
  if (!aligned(workspace, kWsAlign)) return L4Q_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  if (desc->dtype == L4Q_DTYPE_BF16)
    l4q::launch_quant_errors<bf16_t>(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero,
                                     (float*)workspace, errors, stream);
  else
    l4q::launch_quant_errors<float>(d, (const float*)W0, (const float*)A, (const float*)B, scale, zero,
                                    (float*)workspace, errors, stream);
  return launch_status();
}

int l4q_quant_errors_static(const l4q_desc* desc, const void* W0, const void* A, const void* B, const float* scale,
                            const float* zero, float* errors, void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (!W0 || !A || !B || !scale || !zero || !errors) return L4Q_ERR_NULL;
  const void* ptrs[] = {W0, A, B, scale, zero, errors};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const size_t need = (size_t)desc->out_features * (size_t)((desc->in_features + 255) / 256) * 2 * sizeof(float);
  if (need > kStaticScratchBytes) return L4Q_ERR_TOO_LARGE;
  float* partial = static_cast<float*>(static_scratch_ptr());
  if (!partial) return L4Q_ERR_LAUNCH;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const LayerDims d = dims_of(desc);
  (void)hipGetLastError();
  // every pair the sum kernel reads is written by the error kernel of this same call: nothing needs clearing
  if (desc->dtype == L4Q_DTYPE_BF16)
    l4q::launch_quant_errors<bf16_t>(d, (const bf16_t*)W0, (const bf16_t*)A, (const bf16_t*)B, scale, zero, partial,
                                     errors, stream);
  else
    l4q::launch_quant_errors<float>(d, (const float*)W0, (const float*)A, (const float*)B, scale, zero, partial,
                                    errors, stream);
  return launch_status();
}

int l4q_adamw_step(const l4q_desc* desc, const l4q_adamw* hp, float* A32, float* B32, float* scale, float* zero,
                   const float* dA, const float* dB, const float* dscale, const float* dzero, float* m, float* v,
                   void* A_copy, void* B_copy, void* hip_stream) {
  const int st = check_desc(desc, false);
  if (st != L4Q_OK) return st;
  if (!hp || !A32 || !B32 || !scale || !zero || !dA || !dB || !dscale || !dzero || !m || !v) return L4Q_ERR_NULL;
  if (hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f)) return L4Q_ERR_SHAPE;
  if ((A_copy || B_copy) && desc->dtype != L4Q_DTYPE_BF16) return L4Q_ERR_DTYPE;
  const void* ptrs[] = {A32, B32, scale, zero, dA, dB, dscale, dzero, m, v, A_copy, B_copy};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return L4Q_ERR_ALIGN;
  const LayerDims d = dims_of(desc);
  l4q::AdamwArgs a;
  a.param[0] = A32; a.param[1] = B32; a.param[2] = scale; a.param[3] = zero;
  a.grad[0] = dA; a.grad[1] = dB; a.grad[2] = dscale; a.grad[3] = dzero;
  a.n[0] = (int64_t)d.r * d.i; a.n[1] = d.o * d.r; a.n[2] = d.o * d.G(); a.n[3] = d.o * d.G();
  a.m = m; a.v = v;
  a.copy_bf16[0] = static_cast<bf16_t*>(A_copy); a.copy_bf16[1] = static_cast<bf16_t*>(B_copy);
  a.lr = hp->lr; a.beta1 = hp->beta1; a.beta2 = hp->beta2; a.eps = hp->eps; a.weight_decay = hp->weight_decay;
  a.bias1 = (float)(1.0 - std::pow((double)hp->beta1, (double)hp->step));
  a.bias2 = (float)(1.0 - std::pow((double)hp->beta2, (double)hp->step));
  (void)hipGetLastError();
  l4q::launch_adamw(a, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

float l4q_cosine_lr(int64_t step, int64_t total_steps, double lr_max, double warmup_fraction) {
  if (total_steps <= 0 || step < 0) return 0.f;
  const int64_t w = (int64_t)std::ceil(warmup_fraction * (double)total_steps);
  if (step < w) return (float)(lr_max * (double)(step + 1) / (double)w);
  if (step >= total_steps) return 0.f;
  const double pi = 3.14159265358979323846;
  return (float)(lr_max * 0.5 * (1.0 + std::cos(pi * (double)(step - w) / (double)(total_steps - w))));
}

int l4q_mfma_probe(const void* data, int iterations, int workgroups, float* sink, double* flops, void* hip_stream) {
  if (!data || !sink) return L4Q_ERR_NULL;
  if (iterations < 1 || workgroups < 1 || workgroups > (1 << 20)) return L4Q_ERR_SHAPE;
  if (!aligned(data, 16) || !aligned(sink, 16)) return L4Q_ERR_ALIGN;
  (void)hipGetLastError();
  const double f = l4q::launch_mfma_probe((const bf16_t*)data, iterations, workgroups, sink,
                                          static_cast<hipStream_t>(hip_stream));
  if (flops) *flops = f;
  return launch_status();
}

int l4q_profile_gemm(int enable) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (auto& ev : g_prof.events) {
    (void)hipEventDestroy(ev.e0);
    (void)hipEventDestroy(ev.e1);
  }
  g_prof.events.clear();
  for (double& w : g_prof.work) w = 0.0;
  g_prof.on = enable != 0;
  return L4Q_OK;
}

int l4q_profile_read(int kind, double* total_ms, int64_t* launches, double* total_work) {
  if (kind < 0 || kind >= kKinds) return L4Q_ERR_SHAPE;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  double ms = 0.0;
  int64_t n = 0;
  for (auto& ev : g_prof.events) {
    if (ev.kind != kind) continue;
    if (hipEventSynchronize(ev.e1) != hipSuccess) return L4Q_ERR_LAUNCH;
    float t = 0.f;
    if (hipEventElapsedTime(&t, ev.e0, ev.e1) != hipSuccess) return L4Q_ERR_LAUNCH;
    ms += t;
    ++n;
  }
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  if (total_work) *total_work = g_prof.work[kind];
  return L4Q_OK;
}

int l4q_profile_gemm_read(double* total_ms, int64_t* launches, double* total_flops) {
  return l4q_profile_read(kKindGemm, total_ms, launches, total_flops);
}

int l4q_check_fast_divide(uint32_t first_significand, uint32_t count, uint64_t* counts, void* hip_stream) {
  if (!counts) return L4Q_ERR_NULL;
  if (!aligned(counts, 16)) return L4Q_ERR_ALIGN;
  if (count == 0 || count > (1u << 23)) return L4Q_ERR_SHAPE;
  (void)hipGetLastError();
  l4q::launch_check_fast_divide(first_significand, count, reinterpret_cast<unsigned long long*>(counts),
                                static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

}  // extern "C"
