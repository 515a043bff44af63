// C ABI of the library (declared in include/qlora.h): argument validation on the host,
// then kernel launches on the caller's stream.  No allocation, no synchronisation, no state
// apart from the thread-local code of the last failed launch.
#include "qlora.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <mutex>

#include "common.hpp"
#include "launch.hpp"

namespace {

// ---- optional event bracket around the main GEMM launches (benchmark aid) ----
// A fixed pool of event pairs, created on first use while the aid is enabled and reused after every read; a mutex
// makes enabling, recording and reading safe from several host threads.  Launches beyond the pool's capacity between
// two reads run unbracketed and are counted as dropped.
struct GemmProfile {
  static constexpr int kCap = 4096;
  struct Rec { hipEvent_t start, stop; double flops; };
  std::mutex mu;
  bool enabled = false;
  int created = 0, used = 0;
  int64_t dropped = 0;
  Rec recs[kCap];
} g_prof;

template <class Launch>
hipError_t timed_launch(double flops, hipStream_t st, Launch&& launch) {
  GemmProfile::Rec* r = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.enabled) {
      if (g_prof.used == g_prof.created && g_prof.created < GemmProfile::kCap) {
        GemmProfile::Rec n{};
        // timing-only events: no system-scope fence (and the cache write-back it implies) when they complete
        if (hipError_t e = hipEventCreateWithFlags(&n.start, hipEventDisableSystemFence)) return e;
        if (hipError_t e = hipEventCreateWithFlags(&n.stop, hipEventDisableSystemFence)) { (void)hipEventDestroy(n.start); return e; }
        g_prof.recs[g_prof.created++] = n;
      }
      if (g_prof.used < g_prof.created) { r = &g_prof.recs[g_prof.used++]; r->flops = flops; }
      else ++g_prof.dropped;
    }
  }
  if (!r) return launch();
  (void)hipEventRecord(r->start, st);
  const hipError_t e = launch();
  (void)hipEventRecord(r->stop, st);
  return e;
}

hipError_t gemm_nt_timed(const uint16_t* A0, const uint16_t* B0, int64_t lda0, int64_t ldb0, int K0,
                         const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                         uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  return timed_launch(2.0 * (double)M * (double)N * (double)(K0 + K1), st, [&] {
    return qlora::launch_gemm_nt(A0, B0, lda0, ldb0, K0, A1, B1, lda1, ldb1, K1, C, ldc, M, N, st);
  });
}

thread_local int g_last_hip_error = 0;

// Whether the large-token backward decodes the weight inside the product (qlora_bwd_fused_dequant).
std::atomic<int> g_bwd_fused{0};

// The fused form of gemm_nt_timed's product (weight-side operand of segment 0 as codes + constants), timed alike.
hipError_t gemm_nt_fused_timed(const uint16_t* A0, const uint8_t* Bq, const float* Bc, const float* tab16, int64_t lda0,
                               int K0, const uint16_t* A1, const uint16_t* B1, int64_t lda1, int64_t ldb1, int K1,
                               uint16_t* C, int64_t ldc, int M, int N, hipStream_t st) {
  return timed_launch(2.0 * (double)M * (double)N * (double)(K0 + K1), st, [&] {
    return qlora::launch_gemm_nt_fused(A0, Bq, Bc, tab16, lda0, K0, A1, B1, lda1, ldb1, K1, C, ldc, M, N, st);
  });
}

// Tag of a work-list launch (1 .. 255): arrival words in the counter header carry it, so words left behind by
// another call are told from this call's own.  Consecutive calls get different tags.
std::atomic<unsigned> g_nonce{0};
inline unsigned next_nonce() { return 1u + g_nonce.fetch_add(1u, std::memory_order_relaxed) % 255u; }
std::atomic<int> g_poll_limit{64};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline qlora_status hip_status(hipError_t e) {
  if (e == hipSuccess) return QLORA_OK;
  g_last_hip_error = (int)e;
  return QLORA_ERR_HIP;
}

// Shape rules common to everything that touches a quantised tensor.
qlora_status check_quant_shape(int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize) {
  if (rows <= 0 || cols <= 0 || blocksize <= 0 || dq_blocksize < 0) return QLORA_ERR_SHAPE;
  if (blocksize != 64 || (dq_blocksize != 256 && dq_blocksize != 0)) return QLORA_ERR_UNSUPPORTED;   // 0: no Double Quantization
  if (cols % blocksize != 0) return QLORA_ERR_SHAPE;       // a block never straddles two rows
  if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31) return QLORA_ERR_SHAPE;
  if ((rows * cols) / blocksize >= (int64_t)1 << 32) return QLORA_ERR_SHAPE;
  return QLORA_OK;
}

qlora_status check_view(const qlora_nf4_view* v) {
  if (!v) return QLORA_ERR_NULL;
  const bool dq = v->dq_blocksize != 0;                    // without Double Quantization only packed and c1 (= c2) are read
  if (!v->packed || !v->c1 || (dq && (!v->c2_code || !v->c2_mean))) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(v->rows, v->cols, v->blocksize, v->dq_blocksize)) return st;
  if (!aligned16(v->packed) || !aligned16(v->c1) || (dq && (!aligned16(v->c2_code) || ((uintptr_t)v->c2_mean & 3u))))
    return QLORA_ERR_ALIGN;
  if (v->dtype < 0 || v->dtype >= qlora::kNumTypes) return QLORA_ERR_UNSUPPORTED;
  return QLORA_OK;
}

// The few-token streaming kernels read 4-bit indices and double-quantised constants; every other storage goes
// through dequantise + GEMM whatever the token count.
inline bool streams_few(const qlora_nf4_view* v) { return v->dq_blocksize != 0 && v->dtype != qlora::kTypeInt8; }

inline qlora::NF4Dev to_dev(const qlora_nf4_view* v) {
  return qlora::NF4Dev{v->packed, v->c2_code, v->c1, v->c2_mean, v->rows, v->cols, v->dtype, v->dq_blocksize != 0};
}

qlora_status check_linear(int64_t M, int64_t h, int64_t o, int32_t r) {
  if (M <= 0 || h <= 0 || o <= 0 || r < 0) return QLORA_ERR_SHAPE;
  if (M > (int64_t)1 << 30) return QLORA_ERR_SHAPE;
  if (h % 64 != 0 || o % 64 != 0) return QLORA_ERR_UNSUPPORTED;
  if (r % 16 != 0 || r > 256) return QLORA_ERR_UNSUPPORTED;
  return QLORA_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Bump allocator over the caller's workspace; the same walk computes the size query.  Every plan starts
// behind the counter header, which only the few-token kernels touch (and leave zero).
struct Carver {
  char* base; size_t off = qlora::kWorkspaceHeaderBytes;
  explicit Carver(void* b) : base((char*)b) {}
  template <class T> T* take(size_t count) {
    T* p = base ? (T*)(base + off) : nullptr;
    off = align_up(off + count * sizeof(T), 256);
    return p;
  }
};

struct FwdPlan {
  uint16_t* Wt;      // o x (h + rp)   dequantised weight, transposed (K-contiguous for the forward), and behind it in
                     //                every row L2^T with the rank zero-padded to a multiple of 64: both K segments
  uint16_t* Ts;      // M x rp    bf16(s * X L1)
  float* part;       // split-K partials of X L1
  float* fpart;      // few-token path: split partials of X What
  float* lpart;      // few-token path: partials of X L1
  int rp, splits, fsplits, n_lparts;
  bool few;
  size_t bytes;
};
FwdPlan plan_fwd(void* ws, int64_t M, int64_t h, int64_t o, int32_t r, bool allow_few = true) {
  FwdPlan p{};
  Carver c(ws);
  p.rp = (r + 63) / 64 * 64;
  p.few = allow_few && M <= qlora::kFewTokens && qlora::fewtok_fwd_slabs((int)o) <= qlora::kFewMaxSlabs;
  if (p.few) {
    p.fsplits = qlora::fewtok_fwd_splits((int)h, (int)o);
    p.fpart = c.take<float>((size_t)p.fsplits * M * o);
    p.n_lparts = qlora::fewtok_fwd_lparts((int)h, r);
    p.lpart = c.take<float>((size_t)p.n_lparts * M * r + 4);
    p.bytes = c.off;
    return p;
  }
  p.Wt = c.take<uint16_t>((size_t)(h + (r > 0 ? p.rp : 0)) * o);
  if (r > 0) {
    p.splits = qlora::small_gemm_splits((int)M, r, (int)h);
    p.Ts = c.take<uint16_t>((size_t)M * p.rp);
    p.part = c.take<float>((size_t)p.splits * M * r);
  }
  p.bytes = c.off;
  return p;
}

struct BwdPlan {
  uint16_t* Wd;      // h x o     dequantised weight (K-contiguous for the backward)
  uint16_t* L1p;     // h x rp    L1 with the rank zero-padded (only when r % 64 != 0)
  uint16_t* Us;      // M x rp    bf16(s * dY L2^T)
  uint16_t* Uhl;     // M x 2r    dY L2^T as a [hi | lo] bf16 pair
  uint16_t* Thl;     // M x 2r    X L1 as a [hi | lo] pair, recomputed when the caller saved none
  float* part;       // split-K partials, reused by the four skinny products
  float* fpart;      // few-token path: split partials of dY What^T
  float* lpart;      // few-token path: partials of dY L2^T
  int rp, sU, sT, sL1, sL2, fsplits, n_lparts;
  bool few;
  size_t bytes;
};
BwdPlan plan_bwd(void* ws, int64_t M, int64_t h, int64_t o, int32_t r, bool allow_few = true) {
  BwdPlan p{};
  Carver c(ws);
  p.rp = (r + 63) / 64 * 64;
  p.few = allow_few && M <= qlora::kFewTokens && qlora::fewtok_bwd_slabs((int)h) <= qlora::kFewMaxSlabs;
  if (p.few) {
    p.fsplits = qlora::fewtok_bwd_splits((int)h, (int)o);
    p.fpart = c.take<float>((size_t)p.fsplits * M * h);
    p.n_lparts = qlora::fewtok_bwd_lparts((int)o, r);
    p.lpart = c.take<float>((size_t)p.n_lparts * M * r + 4);
  } else {
    p.Wd = c.take<uint16_t>((size_t)h * o);
  }
  if (r > 0) {
    p.sU = qlora::small_gemm_splits((int)M, r, (int)o);
    p.sT = qlora::small_gemm_splits((int)M, r, (int)h);
    p.sL1 = qlora::small_gemm_splits((int)h, r, (int)M);
    p.sL2 = qlora::small_gemm_splits(r, (int)o, (int)M);
    size_t pe = (size_t)p.sU * M * r;
    if ((size_t)p.sT * M * r > pe) pe = (size_t)p.sT * M * r;
    if ((size_t)p.sL1 * h * r > pe) pe = (size_t)p.sL1 * h * r;
    if ((size_t)p.sL2 * r * o > pe) pe = (size_t)p.sL2 * r * o;
    p.L1p = (r % 64 && !p.few) ? c.take<uint16_t>((size_t)h * p.rp) : nullptr;
    p.Us = c.take<uint16_t>((size_t)M * p.rp);
    p.Uhl = c.take<uint16_t>((size_t)M * 2 * r);
    p.Thl = c.take<uint16_t>((size_t)M * 2 * r);
    p.part = c.take<float>(pe);
  }
  p.bytes = c.off;
  return p;
}

// Several layers on one X.  Few tokens: one launch, every layer with its own partial buffers.  Otherwise the layers
// run one after the other through the single-layer path, sharing one workspace of the largest size.
static_assert(QLORA_MULTI_MAX == qlora::kFewMaxLayers, "the header's limit is the kernel's");
struct MultiPlan {
  float* fpart[qlora::kFewMaxLayers];
  float* lpart[qlora::kFewMaxLayers];
  int splits;
  bool few;
  size_t bytes;
};
MultiPlan plan_fwd_multi(void* ws, int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r) {
  MultiPlan p{};
  int slabs = 0, r_max = 0, oi[qlora::kFewMaxLayers];
  for (int l = 0; l < n; ++l) {
    slabs += qlora::fewtok_fwd_slabs((int)o[l]);
    if (r[l] > r_max) r_max = r[l];
    oi[l] = (int)o[l];
  }
  p.few = M <= qlora::kFewTokens && slabs <= qlora::kFewMaxSlabs;
  if (p.few) {
    Carver c(ws);
    p.splits = qlora::fewtok_multi_splits(n, (int)h, oi, r_max);
    for (int l = 0; l < n; ++l) {
      p.fpart[l] = c.take<float>((size_t)p.splits * M * o[l]);
      p.lpart[l] = c.take<float>((size_t)qlora::fewtok_fwd_lparts((int)h, r[l]) * M * r[l] + 4);
    }
    p.bytes = c.off;
  } else {
    for (int l = 0; l < n; ++l) {
      const size_t b = plan_fwd(nullptr, M, h, o[l], r[l]).bytes;
      if (b > p.bytes) p.bytes = b;
    }
  }
  return p;
}

// A list of independent layers at a few tokens: one persistent launch; every layer with its own partial buffers.
// At more tokens the layers run one after the other through the single-layer path, sharing one workspace.
static_assert(QLORA_LIST_MAX == qlora::kListMax, "the header's limit is the kernel's");
static_assert(QLORA_STATIC_QUANT_MAX_WEIGHTS == qlora::kStaticQuantBlocks * 64, "the header's limit is the kernel's");
struct ListWs {
  qlora::ListPlan plan;
  float* part[qlora::kListMax];
  float* lpart[qlora::kListMax];
  bool few;
  size_t bytes;
};
ListWs plan_list(void* ws, bool bwd, int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r) {
  ListWs p{};
  int hi[qlora::kListMax], oi[qlora::kListMax];
  for (int l = 0; l < n; ++l) { hi[l] = (int)h[l]; oi[l] = (int)o[l]; }
  if (M <= qlora::kFewTokens) p.plan = qlora::fewlist_plan(bwd, (int)M, n, hi, oi, r);
  p.few = p.plan.ok;
  if (p.few) {
    Carver c(ws);
    for (int l = 0; l < n; ++l) {
      p.part[l] = c.take<float>(p.plan.part_floats[l]);
      p.lpart[l] = c.take<float>(p.plan.lpart_floats[l]);
    }
    p.bytes = c.off;
  } else {
    for (int l = 0; l < n; ++l) {
      const size_t b = bwd ? plan_bwd(nullptr, M, h[l], o[l], r[l]).bytes : plan_fwd(nullptr, M, h[l], o[l], r[l]).bytes;
      if (b > p.bytes) p.bytes = b;
    }
  }
  return p;
}

}  // namespace

extern "C" {

const char* qlora_status_string(qlora_status st) {
  switch (st) {
    case QLORA_OK: return "QLORA_OK";
    case QLORA_ERR_NULL: return "QLORA_ERR_NULL: a required pointer is NULL";
    case QLORA_ERR_SHAPE: return "QLORA_ERR_SHAPE: bad size (non-positive, or cols not a multiple of blocksize)";
    case QLORA_ERR_UNSUPPORTED: return "QLORA_ERR_UNSUPPORTED: blocksize must be 64, dq_blocksize 256, r a multiple of 16 up to 256";
    case QLORA_ERR_WORKSPACE: return "QLORA_ERR_WORKSPACE: workspace or scratch too small";
    case QLORA_ERR_ALIGN: return "QLORA_ERR_ALIGN: pointer not 16-byte aligned";
    case QLORA_ERR_HIP: return "QLORA_ERR_HIP: kernel launch failed";
    case QLORA_ERR_STATE: return "QLORA_ERR_STATE: the workspace's counter header was not zero when a few-token kernel used it";
    default: return "QLORA: unknown status";
  }
}

int qlora_last_hip_error(void) { return g_last_hip_error; }

void qlora_profile_gemm(int enable) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  g_prof.enabled = enable != 0;
}

qlora_status qlora_profile_gemm_read(double* total_ms, int64_t* launches, double* total_flops) {
  if (!total_ms || !launches || !total_flops) return QLORA_ERR_NULL;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  double ms = 0.0, fl = 0.0;
  hipError_t bad = hipSuccess;
  for (int i = 0; i < g_prof.used; ++i) {
    GemmProfile::Rec& r = g_prof.recs[i];
    float t = 0.0f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
    if (e != hipSuccess) bad = e;
    ms += t; fl += r.flops;
  }
  *total_ms = ms; *launches = (int64_t)g_prof.used; *total_flops = fl;
  g_prof.used = 0;                                           // the events stay for the next measurement
  g_prof.dropped = 0;
  return hip_status(bad);
}

qlora_status qlora_nf4_sizes(int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize,
                             size_t* packed_bytes, size_t* code_bytes, size_t* c1_bytes,
                             size_t* scratch_bytes) {
  return qlora_quant_sizes(rows, cols, blocksize, dq_blocksize, QLORA_NF4, packed_bytes, code_bytes, c1_bytes,
                           scratch_bytes);
}

qlora_status qlora_quant_sizes(int64_t rows, int64_t cols, int32_t blocksize, int32_t dq_blocksize, int32_t dtype,
                               size_t* packed_bytes, size_t* code_bytes, size_t* c1_bytes,
                               size_t* scratch_bytes) {
  if (qlora_status st = check_quant_shape(rows, cols, blocksize, dq_blocksize)) return st;
  if (dtype < 0 || dtype >= qlora::kNumTypes) return QLORA_ERR_UNSUPPORTED;
  const int64_t P = rows * cols, n = P / blocksize;
  const int64_t n1 = dq_blocksize ? (n + dq_blocksize - 1) / dq_blocksize : n;   // without DQ the c1 buffer holds the n constants c2
  if (packed_bytes) *packed_bytes = dtype == qlora::kTypeInt8 ? (size_t)P : (size_t)(P / 2);
  if (code_bytes) *code_bytes = dq_blocksize ? (size_t)n : 0;
  if (c1_bytes) *c1_bytes = (size_t)n1 * sizeof(float);
  if (scratch_bytes) *scratch_bytes = qlora::kQuantBinsBytes + (dq_blocksize ? (size_t)n * sizeof(float) : 0);
  return QLORA_OK;
}

qlora_status qlora_nf4_quantize(const float* W, int64_t rows, int64_t cols,
                                int32_t blocksize, int32_t dq_blocksize,
                                uint8_t* packed, uint8_t* c2_code, float* c1, float* c2_mean,
                                void* scratch, size_t scratch_bytes, void* hip_stream) {
  return qlora_quantize_4bit(W, rows, cols, blocksize, dq_blocksize, QLORA_NF4, packed, c2_code, c1, c2_mean, scratch,
                             scratch_bytes, hip_stream);
}

qlora_status qlora_codebook_4bit(int32_t dtype, float* values16) {
  if (!values16) return QLORA_ERR_NULL;
  if (!qlora::is_table_type(dtype)) return QLORA_ERR_UNSUPPORTED;
  const qlora::Table4 t = qlora::table4_host(dtype);
  for (int i = 0; i < 16; ++i) values16[i] = t.v[i];
  return QLORA_OK;
}

qlora_status qlora_quantize_4bit(const float* W, int64_t rows, int64_t cols,
                                 int32_t blocksize, int32_t dq_blocksize, int32_t dtype,
                                 uint8_t* packed, uint8_t* c2_code, float* c1, float* c2_mean,
                                 void* scratch, size_t scratch_bytes, void* hip_stream) {
  const bool dq = dq_blocksize != 0;
  if (!W || !packed || !c1 || !scratch || (dq && (!c2_code || !c2_mean))) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, blocksize, dq_blocksize)) return st;
  if (!qlora::is_table_type(dtype)) return QLORA_ERR_UNSUPPORTED;
  size_t need = 0;
  qlora_nf4_sizes(rows, cols, blocksize, dq_blocksize, nullptr, nullptr, nullptr, &need);
  if (scratch_bytes < need) return QLORA_ERR_WORKSPACE;
  if (!aligned16(W) || !aligned16(packed) || !aligned16(c1) || !aligned16(scratch) ||
      (dq && (!aligned16(c2_code) || ((uintptr_t)c2_mean & 3u))))
    return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_quantize(W, rows, cols, packed, c2_code, c1, c2_mean, scratch,
                                           (hipStream_t)hip_stream, dtype, dq));
}

qlora_status qlora_nf4_quantize_static(const float* W, int64_t rows, int64_t cols, int32_t blocksize,
                                       int32_t dq_blocksize, uint8_t* packed, uint8_t* c2_code, float* c1,
                                       float* c2_mean, void* hip_stream) {
  const bool dq = dq_blocksize != 0;
  if (!W || !packed || !c1 || (dq && (!c2_code || !c2_mean))) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, blocksize, dq_blocksize)) return st;
  if (rows * cols > (int64_t)QLORA_STATIC_QUANT_MAX_WEIGHTS) return QLORA_ERR_WORKSPACE;
  if (!aligned16(W) || !aligned16(packed) || !aligned16(c1) ||
      (dq && (!aligned16(c2_code) || ((uintptr_t)c2_mean & 3u))))
    return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_quantize_static(W, rows, cols, packed, c2_code, c1, c2_mean,
                                                  (hipStream_t)hip_stream, QLORA_NF4, dq));
}

qlora_status qlora_quantize_int8(const float* W, int64_t rows, int64_t cols,
                                 int32_t blocksize, int32_t dq_blocksize,
                                 int8_t* q8, uint8_t* c2_code, float* c1, float* c2_mean,
                                 void* scratch, size_t scratch_bytes, void* hip_stream) {
  const bool dq = dq_blocksize != 0;
  if (!W || !q8 || !c1 || !scratch || (dq && (!c2_code || !c2_mean))) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, blocksize, dq_blocksize)) return st;
  size_t need = 0;
  qlora_quant_sizes(rows, cols, blocksize, dq_blocksize, QLORA_INT8, nullptr, nullptr, nullptr, &need);
  if (scratch_bytes < need) return QLORA_ERR_WORKSPACE;
  if (!aligned16(W) || !aligned16(q8) || !aligned16(c1) || !aligned16(scratch) ||
      (dq && (!aligned16(c2_code) || ((uintptr_t)c2_mean & 3u))))
    return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_quantize(W, rows, cols, (uint8_t*)q8, c2_code, c1, c2_mean, scratch,
                                           (hipStream_t)hip_stream, qlora::kTypeInt8, dq));
}

qlora_status qlora_nf4_dequant(const qlora_nf4_view* Wq, uint16_t* W_bf16, void* hip_stream) {
  if (qlora_status st = check_view(Wq)) return st;
  if (!W_bf16) return QLORA_ERR_NULL;
  if (!aligned16(W_bf16)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_dequant(to_dev(Wq), W_bf16, (hipStream_t)hip_stream));
}

// --- linear layer -----------------------------------------------------------------------------------
qlora_status qlora_linear_fwd_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* workspace_bytes) {
  if (qlora_status st = check_linear(M, h, o, r)) return st;
  if (!workspace_bytes) return QLORA_ERR_NULL;
  // no view here: few tokens stream 4-bit, double-quantised weights, every other weight takes the dequantise + GEMM
  // plan at any M, so the size that serves both is reported
  *workspace_bytes = std::max(plan_fwd(nullptr, M, h, o, r, true).bytes, plan_fwd(nullptr, M, h, o, r, false).bytes);
  return QLORA_OK;
}

qlora_status qlora_linear_bwd_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* workspace_bytes) {
  if (qlora_status st = check_linear(M, h, o, r)) return st;
  if (!workspace_bytes) return QLORA_ERR_NULL;
  *workspace_bytes = std::max(plan_bwd(nullptr, M, h, o, r, true).bytes, plan_bwd(nullptr, M, h, o, r, false).bytes);
  return QLORA_OK;
}

qlora_status qlora_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace) return QLORA_ERR_NULL;
  if (workspace_bytes < qlora::kWorkspaceHeaderBytes) return QLORA_ERR_WORKSPACE;
  if (!aligned16(workspace)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_workspace_init(workspace, (hipStream_t)hip_stream));
}

#define QL_TRY(expr) do { if (hipError_t e_ = (expr)) return hip_status(e_); } while (0)

}  // extern "C"

namespace {
// LoRA dropout: the kept elements' 1/(1-p) goes into the adapter's scale, the mask into the operand loads.
inline float dropout_scale(float s, float p) { return (float)((double)s / (1.0 - (double)p)); }

// The forward pass; keep_mask != NULL: LoRA dropout on the adapter's input (large-GEMM path whatever M).
qlora_status linear_fwd_impl(const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1, const uint16_t* L2,
                             float s, int64_t M, int32_t r, const uint8_t* keep_mask, uint16_t* Y, uint16_t* T_save,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (qlora_status st = check_view(Wq)) return st;
  const int64_t h = Wq->rows, o = Wq->cols;
  if (qlora_status st = check_linear(M, h, o, r)) return st;
  if (!X || !Y || !workspace) return QLORA_ERR_NULL;
  if (r > 0 && (!L1 || !L2)) return QLORA_ERR_NULL;
  const FwdPlan p = plan_fwd(workspace, M, h, o, r, keep_mask == nullptr && streams_few(Wq));
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  if (!aligned16(X) || !aligned16(Y) || !aligned16(workspace) || !aligned16(L1) || !aligned16(L2) ||
      !aligned16(T_save))
    return QLORA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  const qlora::NF4Dev W = to_dev(Wq);

  if (p.few) {
    // few tokens: one launch streams the packed weight once and dequantises in registers; the adapter's
    // T = X L1 comes from a few extra workgroups and is applied (and saved) by each slab's last arriver
    QL_TRY(qlora::launch_fewtok_fwd(X, (int)M, W, p.fpart, p.fsplits, L1, L2, r, s, p.lpart, (unsigned*)workspace, Y,
                                    T_save, st));
    return QLORA_OK;
  }
  if (r > 0) {
    // T = X L1 (Eq. 3): split-K partials, then Ts = bf16(s T) (rank zero-padded) and T_save = [hi | lo] of T
    QL_TRY(qlora::launch_small_gemm(X, h, false, L1, r, true, 0, 0, (int)M, r, (int)h, p.part, p.splits, st, keep_mask));
    QL_TRY(qlora::launch_small_finalize(p.part, p.splits, (int)M, r, p.Ts, p.rp, p.rp, s, T_save, nullptr, st));
  }
  const int64_t ldw = h + (r > 0 ? p.rp : 0);               // one row of Wt: What^T[n][0 .. h), then L2^T[n][0 .. rp)
  QL_TRY(qlora::launch_dequant_t(W, p.Wt, ldw, st, r > 0 ? L2 : nullptr, r, r > 0 ? p.rp : 0));
  // Y = X What + Ts L2 (Eq. 5): the adapter term is the second K segment of the same accumulators
  QL_TRY(gemm_nt_timed(X, p.Wt, h, ldw, (int)h, p.Ts, p.Wt + h, p.rp, ldw, r > 0 ? p.rp : 0, Y, o, (int)M, (int)o,
                               st));
  return QLORA_OK;
}
}  // namespace

extern "C" {

qlora_status qlora_linear_fwd(const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1, const uint16_t* L2,
                              float s, int64_t M, int32_t r, uint16_t* Y, uint16_t* T_save, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  return linear_fwd_impl(X, Wq, L1, L2, s, M, r, nullptr, Y, T_save, workspace, workspace_bytes, hip_stream);
}

qlora_status qlora_linear_dropout_sizes(int64_t M, int64_t h, int64_t o, int32_t r, size_t* fwd_bytes,
                                        size_t* bwd_bytes) {
  if (qlora_status st = check_linear(M, h, o, r)) return st;
  // without an adapter there is nothing to drop and the calls are the plain ones, few-token path included
  if (fwd_bytes) *fwd_bytes = plan_fwd(nullptr, M, h, o, r, r == 0).bytes;
  if (bwd_bytes) *bwd_bytes = plan_bwd(nullptr, M, h, o, r, r == 0).bytes;
  return QLORA_OK;
}

qlora_status qlora_linear_fwd_dropout(const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1,
                                      const uint16_t* L2, float s, int64_t M, int32_t r, const uint8_t* keep_mask,
                                      float p, uint16_t* Y, uint16_t* T_save, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (!(p >= 0.0f && p < 1.0f)) return QLORA_ERR_SHAPE;
  if (r > 0 && !keep_mask) return QLORA_ERR_NULL;
  return linear_fwd_impl(X, Wq, L1, L2, r > 0 ? dropout_scale(s, p) : s, M, r, r > 0 ? keep_mask : nullptr, Y, T_save,
                         workspace, workspace_bytes, hip_stream);
}

qlora_status qlora_linear_fwd_multi_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                          size_t* workspace_bytes) {
  if (!o || !r || !workspace_bytes) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  for (int l = 0; l < n; ++l)
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
  *workspace_bytes = plan_fwd_multi(nullptr, M, n, h, o, r).bytes;
  return QLORA_OK;
}

qlora_status qlora_linear_fwd_multi(const uint16_t* X, int32_t n, const qlora_nf4_view* Wq, const uint16_t* const* L1,
                                    const uint16_t* const* L2, const float* s, int64_t M, const int32_t* r,
                                    uint16_t* const* Y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!X || !Wq || !s || !r || !Y || !workspace) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  int64_t o[QLORA_MULTI_MAX];
  const int64_t h = Wq[0].rows;
  for (int l = 0; l < n; ++l) {
    if (qlora_status st = check_view(&Wq[l])) return st;
    if (Wq[l].rows != h) return QLORA_ERR_SHAPE;              // every layer reads the same X
    o[l] = Wq[l].cols;
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
    if (!Y[l]) return QLORA_ERR_NULL;
    if (r[l] > 0 && (!L1 || !L2 || !L1[l] || !L2[l])) return QLORA_ERR_NULL;
    if (!aligned16(Y[l]) || (r[l] > 0 && (!aligned16(L1[l]) || !aligned16(L2[l])))) return QLORA_ERR_ALIGN;
  }
  if (!aligned16(X) || !aligned16(workspace)) return QLORA_ERR_ALIGN;
  if (M <= qlora::kFewTokens)
    for (int l = 0; l < n; ++l)
      if (!streams_few(&Wq[l])) return QLORA_ERR_UNSUPPORTED;      // the streaming kernels read 4-bit indices and double-quantised constants
  const MultiPlan p = plan_fwd_multi(workspace, M, n, h, o, r);
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  if (!p.few) {
    for (int l = 0; l < n; ++l)
      if (qlora_status st = qlora_linear_fwd(X, &Wq[l], r[l] > 0 ? L1[l] : nullptr, r[l] > 0 ? L2[l] : nullptr, s[l], M,
                                             r[l], Y[l], nullptr, workspace, workspace_bytes, hip_stream))
        return st;
    return QLORA_OK;
  }
  qlora::FewLayer layers[QLORA_MULTI_MAX];
  for (int l = 0; l < n; ++l)
    layers[l] = qlora::FewLayer{to_dev(&Wq[l]), r[l] > 0 ? L1[l] : nullptr, r[l] > 0 ? L2[l] : nullptr, r[l], s[l],
                                p.fpart[l], p.lpart[l], Y[l]};
  QL_TRY(qlora::launch_fewtok_fwd_multi(X, (int)M, n, layers, p.splits, (unsigned*)workspace, (hipStream_t)hip_stream));
  return QLORA_OK;
}

// Several layers on one X at training token counts: the dequantised weights stacked along n, the adapters
// block-diagonal in the second K segment, one product for all outputs.
namespace {
struct StackPlan {
  uint16_t* Wt;      // (sum o) x (h + Rp): row n of layer l = What_l^T[n], then L2_l^T[n] in the layer's rank columns
  uint16_t* Ts;      // M x Rp: [s_0 X L1_0 | s_1 X L1_1 | ...], every layer's rank zero-padded to a multiple of 64
  float* part;       // split-K partials of one X L1 at a time
  int Rp, off[QLORA_MULTI_MAX], rp[QLORA_MULTI_MAX], splits[QLORA_MULTI_MAX];
  int64_t N;
  size_t bytes;
};
StackPlan plan_fwd_stacked(void* ws, int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r) {
  StackPlan p{};
  Carver c(ws);
  size_t pe = 0;
  for (int l = 0; l < n; ++l) {
    p.N += o[l];
    p.off[l] = p.Rp;
    p.rp[l] = r[l] > 0 ? (r[l] + 63) / 64 * 64 : 0;
    p.Rp += p.rp[l];
    if (r[l] > 0) {
      p.splits[l] = qlora::small_gemm_splits((int)M, r[l], (int)h);
      pe = std::max(pe, (size_t)p.splits[l] * M * r[l]);
    }
  }
  p.Wt = c.take<uint16_t>((size_t)(h + p.Rp) * p.N);
  if (p.Rp > 0) {
    p.Ts = c.take<uint16_t>((size_t)M * p.Rp);
    p.part = c.take<float>(pe);
  }
  p.bytes = c.off;
  return p;
}
}  // namespace

qlora_status qlora_linear_fwd_stacked_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                            size_t* workspace_bytes) {
  if (!o || !r || !workspace_bytes) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  for (int l = 0; l < n; ++l)
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
  *workspace_bytes = plan_fwd_stacked(nullptr, M, n, h, o, r).bytes;
  return QLORA_OK;
}

qlora_status qlora_linear_fwd_stacked(const uint16_t* X, int32_t n, const qlora_nf4_view* Wq, const uint16_t* const* L1,
                                      const uint16_t* const* L2, const float* s, int64_t M, const int32_t* r,
                                      uint16_t* Y, uint16_t* const* T_save, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
  if (!X || !Wq || !s || !r || !Y || !workspace) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  int64_t o[QLORA_MULTI_MAX];
  const int64_t h = Wq[0].rows;
  for (int l = 0; l < n; ++l) {
    if (qlora_status st = check_view(&Wq[l])) return st;
    if (Wq[l].rows != h) return QLORA_ERR_SHAPE;              // every layer reads the same X
    o[l] = Wq[l].cols;
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
    if (r[l] > 0 && (!L1 || !L2 || !L1[l] || !L2[l])) return QLORA_ERR_NULL;
    if (r[l] > 0 && (!aligned16(L1[l]) || !aligned16(L2[l]))) return QLORA_ERR_ALIGN;
    if (T_save && !aligned16(T_save[l])) return QLORA_ERR_ALIGN;
  }
  if (!aligned16(X) || !aligned16(Y) || !aligned16(workspace)) return QLORA_ERR_ALIGN;
  const StackPlan p = plan_fwd_stacked(workspace, M, n, h, o, r);
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t ldw = h + p.Rp;
  int64_t n0 = 0;
  for (int l = 0; l < n; ++l) {
    if (r[l] > 0) {
      // T_l = X L1_l (Eq. 3), scaled and rounded into its rank columns of Ts
      QL_TRY(qlora::launch_small_gemm(X, h, false, L1[l], r[l], true, 0, 0, (int)M, r[l], (int)h, p.part, p.splits[l], st,
                                      nullptr));
      QL_TRY(qlora::launch_small_finalize(p.part, p.splits[l], (int)M, r[l], p.Ts + p.off[l], p.Rp, p.rp[l], s[l],
                                          T_save ? T_save[l] : nullptr, nullptr, st));
    }
    QL_TRY(qlora::launch_dequant_t(to_dev(&Wq[l]), p.Wt + n0 * ldw, ldw, st, r[l] > 0 ? L2[l] : nullptr, r[l], p.Rp,
                                   p.off[l]));
    n0 += o[l];
  }
  // Y[:, layer l's columns] = X What_l + s_l (X L1_l) L2_l (Eq. 5 per layer)
  QL_TRY(gemm_nt_timed(X, p.Wt, h, ldw, (int)h, p.Ts, p.Wt + h, p.Rp, ldw, p.Rp, Y, p.N, (int)M, (int)p.N, st));
  return QLORA_OK;
}

}  // extern "C"

namespace {
// The backward pass; the adapter gradients go to bf16 matrices (dL1, dL2) or are added to fp32 ones (aL1, aL2).
qlora_status linear_bwd_impl(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1,
                             const uint16_t* L2, float s, int64_t M, int32_t r, const uint8_t* keep_mask,
                             const uint16_t* T_saved, uint16_t* dX, uint16_t* dL1, uint16_t* dL2, float* aL1,
                             float* aL2, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (qlora_status st = check_view(Wq)) return st;
  const int64_t h = Wq->rows, o = Wq->cols;
  if (qlora_status st = check_linear(M, h, o, r)) return st;
  if (!dY || !workspace) return QLORA_ERR_NULL;
  if (r == 0) { dL1 = nullptr; dL2 = nullptr; aL1 = nullptr; aL2 = nullptr; }
  if (r > 0 && (!L1 || !L2)) return QLORA_ERR_NULL;
  const bool want1 = dL1 || aL1, want2 = dL2 || aL2;
  if ((want1 || want2) && !X) return QLORA_ERR_NULL;
  const BwdPlan p = plan_bwd(workspace, M, h, o, r, keep_mask == nullptr && streams_few(Wq));
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  if (!aligned16(dY) || !aligned16(X) || !aligned16(workspace) || !aligned16(L1) || !aligned16(L2) ||
      !aligned16(T_saved) || !aligned16(dX) || !aligned16(dL1) || !aligned16(dL2) || !aligned16(aL1) || !aligned16(aL2))
    return QLORA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  const qlora::NF4Dev W = to_dev(Wq);

  if (p.few && dX) {
    // few tokens: one launch streams the packed weight once; U = dY L2^T comes from extra workgroups, is applied
    // by each slab's last arriver and left as a [hi | lo] pair for dL1
    QL_TRY(qlora::launch_fewtok_bwd(dY, (int)M, W, p.fpart, p.fsplits, L1, L2, r, s, p.lpart, (unsigned*)workspace, dX,
                                    (r > 0 && want1) ? p.Uhl : nullptr, st));
  } else if (r > 0 && (dX || want1)) {
    // U = dY L2^T: Us = bf16(s U) feeds the adapter segment of dX, the [hi | lo] pair of U feeds dL1
    QL_TRY(qlora::launch_small_gemm(dY, o, false, L2, o, false, 0, 0, (int)M, r, (int)o, p.part, p.sU, st));
    QL_TRY(qlora::launch_small_finalize(p.part, p.sU, (int)M, r, p.Us, p.rp, p.rp, s, p.Uhl, nullptr, st));
  }
  if (!p.few && dX) {
    const uint16_t* B1 = L1;
    if (r > 0 && p.L1p) { QL_TRY(qlora::launch_copy_pad(L1, (int)h, r, p.L1p, p.rp, st)); B1 = p.L1p; }
    const int K1 = r > 0 ? p.rp : 0;
    if (g_bwd_fused.load(std::memory_order_relaxed) && W.dtype != qlora::kTypeInt8 && o % 64 == 0 &&
        qlora::gemm_nt_fused_fits((int)o, K1, (int)h)) {
      // dX = Us L1^T + dY What^T with What decoded tile by tile inside the product: the workspace that would hold
      // What takes the h x o / 64 block constants and the 16 values of the data type instead
      float* consts = (float*)p.Wd;
      float* tab16 = consts + ((size_t)h * (o / 64) + 15) / 16 * 16;
      QL_TRY(qlora::launch_block_consts(W, consts, tab16, st));
      QL_TRY(gemm_nt_fused_timed(dY, W.packed, W.dq ? consts : W.c1, tab16, o, (int)o, p.Us, B1, p.rp, p.rp, K1, dX, h,
                                 (int)M, (int)h, st));
    } else {
      QL_TRY(qlora::launch_dequant(W, p.Wd, st));
      // dX = dY What^T + Us L1^T
      QL_TRY(gemm_nt_timed(dY, p.Wd, o, o, (int)o, p.Us, B1, p.rp, p.rp, K1, dX, h, (int)M, (int)h, st));
    }
    // LoRA dropout: a dropped input element gets no gradient through the adapter
    if (r > 0 && keep_mask) QL_TRY(qlora::launch_dropout_dx_fix(dX, (int)M, (int)h, keep_mask, p.Us, p.rp, L1, r, st));
  }
  if (want1) {
    // dL1 = s X^T U: contraction over the tokens, both operands stored token-major; U enters as hi + lo
    QL_TRY(qlora::launch_small_gemm(X, h, true, p.Uhl, 2 * r, true, 2, r, (int)h, r, (int)M, p.part, p.sL1, st, keep_mask));
    QL_TRY(qlora::launch_small_finalize(p.part, p.sL1, (int)h, r, dL1, r, r, s, nullptr, aL1, st));
  }
  if (want2) {
    const uint16_t* T = T_saved;
    if (!T) {                                               // gradient checkpointing: recompute T = X L1
      QL_TRY(qlora::launch_small_gemm(X, h, false, L1, r, true, 0, 0, (int)M, r, (int)h, p.part, p.sT, st, keep_mask));
      QL_TRY(qlora::launch_small_finalize(p.part, p.sT, (int)M, r, nullptr, 0, 0, 0.0f, p.Thl, nullptr, st));
      T = p.Thl;
    }
    // dL2 = s T^T dY with T as hi + lo rows
    QL_TRY(qlora::launch_small_gemm(T, 2 * r, true, dY, o, true, 1, r, r, (int)o, (int)M, p.part, p.sL2, st));
    QL_TRY(qlora::launch_small_finalize(p.part, p.sL2, r, (int)o, dL2, o, (int)o, s, nullptr, aL2, st));
  }
  return QLORA_OK;
}
}  // namespace

extern "C" {

qlora_status qlora_linear_bwd(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1,
                              const uint16_t* L2, float s, int64_t M, int32_t r, const uint16_t* T_saved,
                              uint16_t* dX, uint16_t* dL1, uint16_t* dL2, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  return linear_bwd_impl(dY, X, Wq, L1, L2, s, M, r, nullptr, T_saved, dX, dL1, dL2, nullptr, nullptr, workspace,
                         workspace_bytes, hip_stream);
}

qlora_status qlora_linear_bwd_acc(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq, const uint16_t* L1,
                                  const uint16_t* L2, float s, int64_t M, int32_t r, const uint16_t* T_saved,
                                  uint16_t* dX, float* dL1_acc, float* dL2_acc, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  return linear_bwd_impl(dY, X, Wq, L1, L2, s, M, r, nullptr, T_saved, dX, nullptr, nullptr, dL1_acc, dL2_acc,
                         workspace, workspace_bytes, hip_stream);
}

qlora_status qlora_linear_bwd_dropout(const uint16_t* dY, const uint16_t* X, const qlora_nf4_view* Wq,
                                      const uint16_t* L1, const uint16_t* L2, float s, int64_t M, int32_t r,
                                      const uint8_t* keep_mask, float p, const uint16_t* T_saved, uint16_t* dX,
                                      uint16_t* dL1, uint16_t* dL2, float* dL1_acc, float* dL2_acc, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (!(p >= 0.0f && p < 1.0f)) return QLORA_ERR_SHAPE;
  if (r > 0 && !keep_mask) return QLORA_ERR_NULL;
  return linear_bwd_impl(dY, X, Wq, L1, L2, r > 0 ? dropout_scale(s, p) : s, M, r, r > 0 ? keep_mask : nullptr, T_saved,
                         dX, dL1, dL2, dL1_acc, dL2_acc, workspace, workspace_bytes, hip_stream);
}

// The input gradient of several layers that read one input is the SUM of their input gradients; with the outputs
// side by side (the layout qlora_linear_fwd_stacked writes) that sum is one product whose contraction runs over all
// layers' outputs, then over all layers' ranks:  dX = [dY_0 | dY_1 ...] [What_0 | What_1 ...]^T + [Us_0 | ...] [L1_0 | ...]^T.
namespace {
struct StackBwdPlan {
  uint16_t* Wd;      // h x (sum o): the dequantised weights side by side
  uint16_t* L1s;     // h x Rp: the layers' L1, every rank zero-padded to a multiple of 64
  uint16_t* Us;      // M x Rp: bf16(s_l dY_l L2_l^T) in layer l's rank columns
  uint16_t* Uhl;     // M x 2 r_max: one layer's dY L2^T as a [hi | lo] pair, for its dL1
  uint16_t* Thl;     // M x 2 r_max: one layer's X L1, recomputed when the caller saved none
  float* part;       // split-K partials, reused by every skinny product
  int Rp, off[QLORA_MULTI_MAX], rp[QLORA_MULTI_MAX];
  int64_t N;
  size_t bytes;
};
StackBwdPlan plan_bwd_stacked(void* ws, int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r) {
  StackBwdPlan p{};
  Carver c(ws);
  size_t pe = 0;
  int r_max = 0;
  for (int l = 0; l < n; ++l) {
    p.N += o[l];
    p.off[l] = p.Rp;
    p.rp[l] = r[l] > 0 ? (r[l] + 63) / 64 * 64 : 0;
    p.Rp += p.rp[l];
    r_max = std::max(r_max, (int)r[l]);
    if (r[l] > 0) {
      pe = std::max(pe, (size_t)qlora::small_gemm_splits((int)M, r[l], (int)o[l]) * M * r[l]);
      pe = std::max(pe, (size_t)qlora::small_gemm_splits((int)M, r[l], (int)h) * M * r[l]);
      pe = std::max(pe, (size_t)qlora::small_gemm_splits((int)h, r[l], (int)M) * h * r[l]);
      pe = std::max(pe, (size_t)qlora::small_gemm_splits(r[l], (int)o[l], (int)M) * r[l] * o[l]);
    }
  }
  p.Wd = c.take<uint16_t>((size_t)h * p.N);
  if (p.Rp > 0) {
    p.L1s = c.take<uint16_t>((size_t)h * p.Rp);
    p.Us = c.take<uint16_t>((size_t)M * p.Rp);
    p.Uhl = c.take<uint16_t>((size_t)M * 2 * r_max);
    p.Thl = c.take<uint16_t>((size_t)M * 2 * r_max);
    p.part = c.take<float>(pe);
  }
  p.bytes = c.off;
  return p;
}
}  // namespace

qlora_status qlora_linear_bwd_stacked_sizes(int64_t M, int32_t n, int64_t h, const int64_t* o, const int32_t* r,
                                            size_t* workspace_bytes) {
  if (!o || !r || !workspace_bytes) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  for (int l = 0; l < n; ++l)
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
  *workspace_bytes = plan_bwd_stacked(nullptr, M, n, h, o, r).bytes;
  return QLORA_OK;
}

qlora_status qlora_linear_bwd_stacked(const uint16_t* dY, const uint16_t* X, int32_t n, const qlora_nf4_view* Wq,
                                      const uint16_t* const* L1, const uint16_t* const* L2, const float* s, int64_t M,
                                      const int32_t* r, const uint16_t* const* T_saved, uint16_t* dX,
                                      uint16_t* const* dL1, uint16_t* const* dL2, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (!dY || !Wq || !s || !r || !dX || !workspace) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_MULTI_MAX) return QLORA_ERR_SHAPE;
  int64_t o[QLORA_MULTI_MAX];
  const int64_t h = Wq[0].rows;
  bool want_dl = false;
  for (int l = 0; l < n; ++l) {
    if (qlora_status st = check_view(&Wq[l])) return st;
    if (Wq[l].rows != h) return QLORA_ERR_SHAPE;              // one input, one input gradient
    o[l] = Wq[l].cols;
    if (qlora_status st = check_linear(M, h, o[l], r[l])) return st;
    if (r[l] > 0 && (!L1 || !L2 || !L1[l] || !L2[l])) return QLORA_ERR_NULL;
    if (r[l] > 0 && (!aligned16(L1[l]) || !aligned16(L2[l]))) return QLORA_ERR_ALIGN;
    if ((T_saved && !aligned16(T_saved[l])) || (dL1 && !aligned16(dL1[l])) || (dL2 && !aligned16(dL2[l])))
      return QLORA_ERR_ALIGN;
    if (r[l] > 0 && ((dL1 && dL1[l]) || (dL2 && dL2[l]))) want_dl = true;
  }
  if (want_dl && !X) return QLORA_ERR_NULL;
  if (!aligned16(dY) || !aligned16(X) || !aligned16(dX) || !aligned16(workspace)) return QLORA_ERR_ALIGN;
  const StackBwdPlan p = plan_bwd_stacked(workspace, M, n, h, o, r);
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t N = p.N;
  int64_t n0 = 0;
  for (int l = 0; l < n; ++l) {
    const uint16_t* dYl = dY + n0;                           // layer l's columns of dY, row stride N
    const int rl = r[l];
    if (rl > 0) {
      // U_l = dY_l L2_l^T: bf16(s_l U_l) into the layer's rank columns of Us, the [hi | lo] pair for dL1
      const int sU = qlora::small_gemm_splits((int)M, rl, (int)o[l]);
      QL_TRY(qlora::launch_small_gemm(dYl, N, false, L2[l], o[l], false, 0, 0, (int)M, rl, (int)o[l], p.part, sU, st));
      QL_TRY(qlora::launch_small_finalize(p.part, sU, (int)M, rl, p.Us + p.off[l], p.Rp, p.rp[l], s[l], p.Uhl, nullptr, st));
      QL_TRY(qlora::launch_copy_pad(L1[l], (int)h, rl, p.L1s + p.off[l], p.rp[l], st, p.Rp));
      if (dL1 && dL1[l]) {                                   // dL1_l = s_l X^T U_l
        const int sL1 = qlora::small_gemm_splits((int)h, rl, (int)M);
        QL_TRY(qlora::launch_small_gemm(X, h, true, p.Uhl, 2 * rl, true, 2, rl, (int)h, rl, (int)M, p.part, sL1, st));
        QL_TRY(qlora::launch_small_finalize(p.part, sL1, (int)h, rl, dL1[l], rl, rl, s[l], nullptr, nullptr, st));
      }
      if (dL2 && dL2[l]) {                                   // dL2_l = s_l T_l^T dY_l
        const uint16_t* T = T_saved ? T_saved[l] : nullptr;
        if (!T) {
          const int sT = qlora::small_gemm_splits((int)M, rl, (int)h);
          QL_TRY(qlora::launch_small_gemm(X, h, false, L1[l], rl, true, 0, 0, (int)M, rl, (int)h, p.part, sT, st));
          QL_TRY(qlora::launch_small_finalize(p.part, sT, (int)M, rl, nullptr, 0, 0, 0.0f, p.Thl, nullptr, st));
          T = p.Thl;
        }
        const int sL2 = qlora::small_gemm_splits(rl, (int)o[l], (int)M);
        QL_TRY(qlora::launch_small_gemm(T, 2 * rl, true, dYl, N, true, 1, rl, rl, (int)o[l], (int)M, p.part, sL2, st));
        QL_TRY(qlora::launch_small_finalize(p.part, sL2, rl, (int)o[l], dL2[l], o[l], (int)o[l], s[l], nullptr, nullptr, st));
      }
    }
    QL_TRY(qlora::launch_dequant(to_dev(&Wq[l]), p.Wd + n0, st, N));
    n0 += o[l];
  }
  // dX = sum over the layers of dY_l What_l^T + Us_l L1_l^T: one product, contraction over all outputs, then all ranks
  QL_TRY(gemm_nt_timed(dY, p.Wd, N, N, (int)N, p.Us, p.L1s, p.Rp, p.Rp, p.Rp, dX, h, (int)M, (int)h, st));
  return QLORA_OK;
}

}  // extern "C"

// --- lists of layers at a few tokens ------------------------------------------------------------------
namespace {
qlora_status list_impl(bool bwd, int32_t n, const uint16_t* const* In, const qlora_nf4_view* Wq, const uint16_t* const* L1,
                       const uint16_t* const* L2, const float* s, int64_t M, const int32_t* r, uint16_t* const* Out,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!In || !Wq || !s || !r || !Out || !workspace) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_LIST_MAX) return QLORA_ERR_SHAPE;
  int64_t h[QLORA_LIST_MAX], o[QLORA_LIST_MAX];
  for (int l = 0; l < n; ++l) {
    if (qlora_status st = check_view(&Wq[l])) return st;
    h[l] = Wq[l].rows; o[l] = Wq[l].cols;
    if (qlora_status st = check_linear(M, h[l], o[l], r[l])) return st;
    if (!In[l] || !Out[l]) return QLORA_ERR_NULL;
    if (r[l] > 0 && (!L1 || !L2 || !L1[l] || !L2[l])) return QLORA_ERR_NULL;
    if (!aligned16(In[l]) || !aligned16(Out[l]) || (r[l] > 0 && (!aligned16(L1[l]) || !aligned16(L2[l])))) return QLORA_ERR_ALIGN;
  }
  if (!aligned16(workspace)) return QLORA_ERR_ALIGN;
  if (M <= qlora::kFewTokens)
    for (int l = 0; l < n; ++l)
      if (!streams_few(&Wq[l]) || Wq[l].dtype != Wq[0].dtype) return QLORA_ERR_UNSUPPORTED;   // one decode table per launch
  const ListWs p = plan_list(workspace, bwd, M, n, h, o, r);
  if (M <= qlora::kFewTokens && !p.few) return QLORA_ERR_UNSUPPORTED;
  if (workspace_bytes < p.bytes) return QLORA_ERR_WORKSPACE;
  if (!p.few) {
    for (int l = 0; l < n; ++l) {
      const uint16_t* l1 = r[l] > 0 ? L1[l] : nullptr;
      const uint16_t* l2 = r[l] > 0 ? L2[l] : nullptr;
      const qlora_status st =
          bwd ? qlora_linear_bwd(In[l], nullptr, &Wq[l], l1, l2, s[l], M, r[l], nullptr, Out[l], nullptr, nullptr, workspace,
                                 workspace_bytes, hip_stream)
              : qlora_linear_fwd(In[l], &Wq[l], l1, l2, s[l], M, r[l], Out[l], nullptr, workspace, workspace_bytes, hip_stream);
      if (st) return st;
    }
    return QLORA_OK;
  }
  qlora::ListLayerDesc layers[QLORA_LIST_MAX];
  for (int l = 0; l < n; ++l)
    layers[l] = qlora::ListLayerDesc{to_dev(&Wq[l]), In[l], r[l] > 0 ? L1[l] : nullptr, r[l] > 0 ? L2[l] : nullptr, r[l], s[l],
                                     p.part[l], p.lpart[l], Out[l], nullptr};
  QL_TRY(qlora::launch_fewlist(bwd, (int)M, n, layers, p.plan, (unsigned*)workspace, next_nonce(),
                               g_poll_limit.load(std::memory_order_relaxed), (hipStream_t)hip_stream));
  return QLORA_OK;
}

qlora_status list_sizes_impl(bool bwd, int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r,
                             size_t* workspace_bytes) {
  if (!h || !o || !r || !workspace_bytes) return QLORA_ERR_NULL;
  if (n < 1 || n > QLORA_LIST_MAX) return QLORA_ERR_SHAPE;
  for (int l = 0; l < n; ++l)
    if (qlora_status st = check_linear(M, h[l], o[l], r[l])) return st;
  const ListWs p = plan_list(nullptr, bwd, M, n, h, o, r);
  if (M <= qlora::kFewTokens && !p.few) return QLORA_ERR_UNSUPPORTED;
  *workspace_bytes = p.bytes;
  return QLORA_OK;
}
}  // namespace

extern "C" {

qlora_status qlora_linear_fwd_list_sizes(int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r,
                                         size_t* workspace_bytes) {
  return list_sizes_impl(false, M, n, h, o, r, workspace_bytes);
}
qlora_status qlora_linear_bwd_list_sizes(int64_t M, int32_t n, const int64_t* h, const int64_t* o, const int32_t* r,
                                         size_t* workspace_bytes) {
  return list_sizes_impl(true, M, n, h, o, r, workspace_bytes);
}

qlora_status qlora_linear_fwd_list(int32_t n, const uint16_t* const* X, const qlora_nf4_view* Wq, const uint16_t* const* L1,
                                   const uint16_t* const* L2, const float* s, int64_t M, const int32_t* r,
                                   uint16_t* const* Y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return list_impl(false, n, X, Wq, L1, L2, s, M, r, Y, workspace, workspace_bytes, hip_stream);
}
qlora_status qlora_linear_bwd_list(int32_t n, const uint16_t* const* dY, const qlora_nf4_view* Wq, const uint16_t* const* L1,
                                   const uint16_t* const* L2, const float* s, int64_t M, const int32_t* r,
                                   uint16_t* const* dX, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return list_impl(true, n, dY, Wq, L1, L2, s, M, r, dX, workspace, workspace_bytes, hip_stream);
}

qlora_status qlora_workspace_check(const void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace) return QLORA_ERR_NULL;
  if (workspace_bytes < qlora::kWorkspaceHeaderBytes) return QLORA_ERR_WORKSPACE;
  unsigned status = 0;
  QL_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
  QL_TRY(hipMemcpy(&status, (const unsigned*)workspace + qlora::kHeaderStatusWord, sizeof(status), hipMemcpyDeviceToHost));
  return status ? QLORA_ERR_STATE : QLORA_OK;
}

qlora_status qlora_kbit_sizes(int64_t rows, int64_t cols, int32_t k, size_t* stream_bytes) {
  if (!stream_bytes) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, 64, 256)) return st;
  if (k != 2 && k != 3) return QLORA_ERR_UNSUPPORTED;
  *stream_bytes = (size_t)(rows * cols / 8 * k);
  return QLORA_OK;
}

qlora_status qlora_kbit_pack(const uint8_t* packed4, int64_t rows, int64_t cols, int32_t k, uint8_t* stream,
                             void* hip_stream) {
  if (!packed4 || !stream) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, 64, 256)) return st;
  if (k != 2 && k != 3) return QLORA_ERR_UNSUPPORTED;
  if (!aligned16(packed4) || !aligned16(stream)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_kbit_pack(packed4, rows * cols, k, stream, (hipStream_t)hip_stream));
}

qlora_status qlora_kbit_unpack(const uint8_t* stream, int64_t rows, int64_t cols, int32_t k, uint8_t* packed4,
                               void* hip_stream) {
  if (!packed4 || !stream) return QLORA_ERR_NULL;
  if (qlora_status st = check_quant_shape(rows, cols, 64, 256)) return st;
  if (k != 2 && k != 3) return QLORA_ERR_UNSUPPORTED;
  if (!aligned16(packed4) || !aligned16(stream)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_kbit_unpack(stream, rows * cols, k, packed4, (hipStream_t)hip_stream));
}

qlora_status qlora_grad_sqnorm(const float* grad, int64_t n, double* sqnorm_accum, void* hip_stream) {
  if (n < 0) return QLORA_ERR_SHAPE;
  if (n == 0) return QLORA_OK;                               // an empty buffer adds nothing
  if (!grad || !sqnorm_accum) return QLORA_ERR_NULL;
  if (!aligned16(grad) || ((uintptr_t)sqnorm_accum & 7u)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_grad_sqnorm(grad, n, sqnorm_accum, (hipStream_t)hip_stream));
}

qlora_status qlora_adam_step(float* param, float* m, float* v, float* grad, uint16_t* param_bf16, int64_t n,
                             const qlora_adam_config* cfg, const double* sqnorm, void* hip_stream) {
  if (!cfg) return QLORA_ERR_NULL;
  if (n < 0 || cfg->step < 1) return QLORA_ERR_SHAPE;
  if (!(cfg->beta1 >= 0.0 && cfg->beta1 < 1.0) || !(cfg->beta2 >= 0.0 && cfg->beta2 < 1.0) || !(cfg->eps >= 0.0) ||
      !(cfg->lr == cfg->lr) || !(cfg->weight_decay == cfg->weight_decay) || !(cfg->grad_scale == cfg->grad_scale) ||
      cfg->reserved != 0)
    return QLORA_ERR_UNSUPPORTED;
  if (n == 0) return QLORA_OK;                               // no parameters: nothing to do
  if (!param || !m || !v || !grad) return QLORA_ERR_NULL;
  if (!aligned16(param) || !aligned16(m) || !aligned16(v) || !aligned16(grad) || ((uintptr_t)param_bf16 & 7u) ||
      ((uintptr_t)sqnorm & 7u))
    return QLORA_ERR_ALIGN;
  qlora::AdamConsts c{};
  c.b1 = (float)cfg->beta1; c.b2 = (float)cfg->beta2;
  c.omb1 = (float)(1.0 - cfg->beta1); c.omb2 = (float)(1.0 - cfg->beta2);
  c.bc1 = (float)(1.0 - std::pow(cfg->beta1, (double)cfg->step));
  c.bc2 = (float)(1.0 - std::pow(cfg->beta2, (double)cfg->step));
  c.eps = (float)cfg->eps; c.lr = (float)cfg->lr;
  c.lrwd = cfg->weight_decay != 0.0 ? (float)(cfg->lr * cfg->weight_decay) : 0.0f;
  c.zero_grad = cfg->zero_grad != 0;
  c.grad_scale = cfg->grad_scale; c.max_norm = cfg->max_grad_norm;
  c.sqnorm = cfg->max_grad_norm > 0.0 ? sqnorm : nullptr;
  return hip_status(qlora::launch_adam(param, m, v, grad, param_bf16, n, c, (hipStream_t)hip_stream));
}

qlora_status qlora_hbm_probe(int32_t mode, const void* src, void* dst, int64_t bytes, uint32_t* sink, int32_t wgs_per_cu,
                             void* hip_stream) {
  if (mode < 0 || mode > 2 || bytes <= 0 || bytes % 16 != 0 || wgs_per_cu < 1 || wgs_per_cu > 64) return QLORA_ERR_SHAPE;
  if ((mode != 1 && !src) || (mode != 0 && !dst) || (mode == 0 && !sink)) return QLORA_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return QLORA_ERR_ALIGN;
  return hip_status(qlora::launch_hbm_probe(mode, src, dst, bytes, sink, wgs_per_cu, (hipStream_t)hip_stream));
}

qlora_status qlora_mfma_probe(int32_t lds_traffic, int32_t iters, float* out, size_t out_bytes, void* hip_stream) {
  if (!out) return QLORA_ERR_NULL;
  if (lds_traffic < 0 || lds_traffic > 2 || iters <= 0 || iters > (1 << 20) ||
      out_bytes < (size_t)256 * 256 * sizeof(float))
    return QLORA_ERR_SHAPE;
  return hip_status(qlora::launch_mfma_probe(lds_traffic, iters, out, (hipStream_t)hip_stream));
}

int32_t qlora_bwd_fused_dequant(int32_t mode) {
  if (mode < 0) return g_bwd_fused.load(std::memory_order_relaxed);
  return g_bwd_fused.exchange(mode != 0 ? 1 : 0, std::memory_order_relaxed);
}

void qlora_fewtok_poll_limit(int32_t polls) { g_poll_limit.store(polls < 0 ? 0 : polls, std::memory_order_relaxed); }

}  // extern "C"
