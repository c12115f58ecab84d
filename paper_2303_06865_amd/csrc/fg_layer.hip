// Host side of the library: argument validation, the linear dispatcher, one transformer layer in
// its prefill and decode forms (Section 3), and the block-schedule driver (Section 4.2,
// Algorithm 1) that generates n tokens for a block of GPU batches.
#include <math.h>
#include <string.h>

#include <string>
#include <vector>

#include "fg_common.h"

namespace fg {

// ---------------------------------------------------------------- errors, profile
static thread_local std::string g_dev_err;

void set_device_error(hipError_t e, const char* what) {
  g_dev_err = std::string(hipGetErrorString(e)) + " in " + what;
}

struct ProfRec {
  int k;
  hipEvent_t e0, e1;
};
static bool g_prof_on = false;
static uint32_t g_prof_mask = 0xffffffffu;   // bit k set: launches of kernel class k are timed
static std::vector<ProfRec> g_prof_open;
static double g_prof_ms[FG_K_COUNT];
static int64_t g_prof_n[FG_K_COUNT];

bool profile_enabled() { return g_prof_on; }

void profile_mark(int kclass, hipStream_t stream, bool begin) {
  if (!((g_prof_mask >> kclass) & 1u)) return;
  if (begin) {
    ProfRec r;
    r.k = kclass;
    if (hipEventCreate(&r.e0) != hipSuccess) return;
    if (hipEventCreate(&r.e1) != hipSuccess) {
      (void)hipEventDestroy(r.e0);
      return;
    }
    (void)hipEventRecord(r.e0, stream);
    g_prof_open.push_back(r);
  } else {
    // scopes never nest across kernel classes: the most recent open record of this class
    for (size_t i = g_prof_open.size(); i-- > 0;) {
      if (g_prof_open[i].k == kclass) {
        (void)hipEventRecord(g_prof_open[i].e1, stream);
        break;
      }
    }
  }
}

// ---------------------------------------------------------------- validation
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_cfg(const fg_model_cfg* c) {
  if (c->h1 <= 0 || c->nh <= 0 || c->h2 <= 0 || c->vocab <= 0 || c->max_pos <= 0) return FG_ERR_SHAPE;
  if (c->h1 % c->nh != 0) return FG_ERR_SHAPE;
  const int dh = c->h1 / c->nh;
  if (dh != 64 && dh != 128) return FG_ERR_UNSUPPORTED;
  if (c->h1 % kGroup != 0 || c->h2 % kGroup != 0) return FG_ERR_SHAPE;
  if (!(c->ln_eps > 0.f)) return FG_ERR_SHAPE;
  return FG_OK;
}

// for_pack: also accept the canonical FP16-pair form, which only fg_pack_weights consumes
int check_mat(const fg_mat* w, bool for_pack) {
  const bool tiled = w->dtype == FG_Q4G64_TILED || w->dtype == FG_Q4G64_H16_TILED;
  if (w->dtype != FG_F16 && w->dtype != FG_Q4G64 && !tiled && !(for_pack && w->dtype == FG_Q4G64_H16))
    return FG_ERR_UNSUPPORTED;
  if (w->rows <= 0 || w->cols <= 0 || w->cols % kGroup != 0 || w->rows % 8 != 0) return FG_ERR_SHAPE;
  if (tiled && w->rows % 32 != 0) return FG_ERR_SHAPE;
  if (w->rows > 0x7fffffff || w->cols > 0x7fffffff) return FG_ERR_SHAPE;
  if (!w->data) return FG_ERR_NULL;
  if (w->dtype != FG_F16 && !w->meta) return FG_ERR_NULL;
  if (!aligned16(w->data) || (w->meta && !aligned16(w->meta))) return FG_ERR_SHAPE;
  return FG_OK;
}

int check_kv(const fg_model_cfg* cfg, const fg_kv_cache* kv) {
  (void)cfg;
  const bool q4 = kv->dtype == FG_Q4G64 || kv->dtype == FG_Q4G64_H16;
  if (kv->dtype != FG_F16 && !q4) return FG_ERR_UNSUPPORTED;
  if (kv->batch <= 0 || kv->cap <= 0) return FG_ERR_SHAPE;
  if (!kv->k_codes || !kv->v_codes) return FG_ERR_NULL;
  if (q4 && (!kv->k_meta || !kv->v_meta)) return FG_ERR_NULL;
  if (!aligned16(kv->k_codes) || !aligned16(kv->v_codes)) return FG_ERR_SHAPE;
  if (q4 && (!aligned16(kv->k_meta) || !aligned16(kv->v_meta))) return FG_ERR_SHAPE;
  return FG_OK;
}

int check_pages(const fg_model_cfg* cfg, const fg_kv_pages* pages, const fg_ragged* seqs) {
  (void)cfg;
  if (!pages || !seqs) return FG_ERR_NULL;
  const bool q4 = pages->dtype == FG_Q4G64 || pages->dtype == FG_Q4G64_H16;
  if (!q4 && pages->dtype != FG_F16) return FG_ERR_UNSUPPORTED;
  if (pages->n_pages <= 0 || seqs->table_stride <= 0 || seqs->n_seqs <= 0) return FG_ERR_SHAPE;
  if ((int64_t)seqs->table_stride * FG_PAGE_ROWS > 0x7fffffff) return FG_ERR_SHAPE;
  if (!pages->k_codes || !pages->v_codes || !seqs->page_table) return FG_ERR_NULL;
  if (q4 && (!pages->k_meta || !pages->v_meta)) return FG_ERR_NULL;
  if (!aligned16(pages->k_codes) || !aligned16(pages->v_codes)) return FG_ERR_SHAPE;
  if (q4 && (!aligned16(pages->k_meta) || !aligned16(pages->v_meta))) return FG_ERR_SHAPE;
  return FG_OK;
}

static int check_layer(const fg_model_cfg* cfg, const fg_layer_weights* w) {
  int rc;
  if ((rc = check_mat(&w->wqkv)) || (rc = check_mat(&w->wo)) || (rc = check_mat(&w->w1)) ||
      (rc = check_mat(&w->w2)))
    return rc;
  const int64_t h1 = cfg->h1, h2 = cfg->h2;
  if (w->wqkv.rows != 3 * h1 || w->wqkv.cols != h1 || w->wo.rows != h1 || w->wo.cols != h1 ||
      w->w1.rows != h2 || w->w1.cols != h1 || w->w2.rows != h1 || w->w2.cols != h2)
    return FG_ERR_SHAPE;
  if (!w->ln1_g || !w->ln1_b || !w->ln2_g || !w->ln2_b) return FG_ERR_NULL;
  return FG_OK;
}

// ---------------------------------------------------------------- linear dispatch
static const int64_t kSmallMLimit = 512;   // rows up to which the weight-streaming kernel is used

// Tiled 4-bit weights always take the stream kernels, and so do row-major FP16 weights whose row count
// (output columns) is a multiple of 32: the decode phase and the LM head as a pure weight streamer, the
// prefill phase on 256 x 256 tiles (measured on the OPT-6.7B prefill shapes in one run: 0.94-1.15 PFLOP/s
// against 0.74-0.91 for gemm_large_m_kernel).
static bool use_stream(int dtype, int64_t n, int64_t m) {
  (void)m;
  if (dtype == FG_Q4G64_TILED || dtype == FG_Q4G64_H16_TILED) return true;
  return dtype == FG_F16 && n % 32 == 0;
}

// Row-major FP16 weights with up to 128 rows: the narrow-tile weight streamer, where it takes the shape.
static bool use_f16w(int dtype, int64_t n, int64_t k, int64_t m) {
  return dtype == FG_F16 && use_stream(dtype, n, m) && gemm_f16w_pick_cols(n, k, m) != 0;
}

size_t linear_workspace_bytes(int dtype, int64_t n, int64_t k, int64_t m) {
  if (use_f16w(dtype, n, k, m)) return gemm_f16w_workspace(n, k, m);
  if (use_stream(dtype, n, m)) return gemm_stream_workspace(n, k, m);
  if (m > kSmallMLimit) return 0;
  return gemm_small_m_workspace(dtype, n, k, m);
}

int linear_launch(const LinearArgs& a, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (use_f16w(a.dtype, a.n, a.k, a.m)) return gemm_f16w_launch(a, ws, ws_bytes, stream);
  if (use_stream(a.dtype, a.n, a.m)) return gemm_stream_launch(a, ws, ws_bytes, stream);
  if (a.m > kSmallMLimit) return gemm_large_m_launch(a, stream);
  return gemm_small_m_launch(a, ws, ws_bytes, stream);
}

static LinearArgs make_linear(const fg_mat& w, const void* bias, const half_t* x, int64_t ldx, int64_t m,
                              const half_t* residual, int64_t ldr, int relu, half_t* out, int64_t ldo) {
  LinearArgs a;
  a.w_data = w.data;
  a.w_meta = w.meta;
  a.dtype = w.dtype;
  a.n = w.rows;
  a.k = w.cols;
  a.x = x;
  a.ldx = ldx;
  a.m = m;
  a.bias = reinterpret_cast<const half_t*>(bias);
  a.residual = residual;
  a.ldr = ldr;
  a.relu = relu;
  a.out_f16 = out;
  a.out_f32 = nullptr;
  a.ldo = ldo;
  return a;
}

// ---------------------------------------------------------------- one layer
// Row stride of the FFN hidden buffer: h2 plus one 128-byte line.  With rows exactly h2 * 2 bytes apart
// (96 KiB at h2 = 49152) the 256 rows of an activation tile that a K step of the second FFN projection
// fetches fall on few memory channels; one line of padding spreads them (measured 3.6 to 3.9 % on that
// projection at 18432 rows; other pads up to 1 KiB gain less, strides of 24 KiB gain nothing).
static inline int64_t act_stride(const fg_model_cfg& c) { return (int64_t)c.h2 + 64; }

struct LayerWs {
  half_t *y, *qkv, *o, *x1, *act;
  void* gemm;
  size_t gemm_bytes;
  size_t total;
};

static size_t layer_gemm_ws(const fg_model_cfg& c, const fg_layer_weights& w, int64_t rows) {
  size_t g = linear_workspace_bytes(w.wqkv.dtype, 3 * (int64_t)c.h1, c.h1, rows);
  size_t t = linear_workspace_bytes(w.wo.dtype, c.h1, c.h1, rows);
  g = t > g ? t : g;
  t = linear_workspace_bytes(w.w1.dtype, c.h2, c.h1, rows);
  g = t > g ? t : g;
  t = linear_workspace_bytes(w.w2.dtype, c.h1, c.h2, rows);
  return t > g ? t : g;
}

static LayerWs carve_layer_ws(const fg_model_cfg& c, const fg_layer_weights& w, int64_t rows, void* base) {
  LayerWs L;
  unsigned char* p = reinterpret_cast<unsigned char*>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    unsigned char* r = p ? p + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  };
  L.y = reinterpret_cast<half_t*>(take((size_t)rows * c.h1 * 2));
  L.qkv = reinterpret_cast<half_t*>(take((size_t)rows * 3 * c.h1 * 2));
  L.o = reinterpret_cast<half_t*>(take((size_t)rows * c.h1 * 2));
  L.x1 = reinterpret_cast<half_t*>(take((size_t)rows * c.h1 * 2));
  L.act = reinterpret_cast<half_t*>(take((size_t)rows * act_stride(c) * 2));
  L.gemm_bytes = layer_gemm_ws(c, w, rows);
  L.gemm = take(L.gemm_bytes);
  L.total = off;
  return L;
}

// Section 3 with OPT's pre-LayerNorm placement.  prefill: s > 0 rows per sequence, causal attention
// over the fresh K/V, rows stored at 0..s-1.  decode: one row per sequence, K/V appended at row t,
// attention over rows 0..t read back from the cache.
// paged != nullptr: the cache is *paged / *seqs instead of kv (rows of sequences at their own positions).
struct PagedKv {
  const fg_kv_pages* pages;
  const fg_ragged* seqs;
};
static int run_layer(const fg_model_cfg& c, const fg_layer_weights& w, const half_t* x_in, int32_t b, int32_t s,
                     bool prefill, int32_t t, const fg_kv_cache& kv, int32_t batch_offset, half_t* x_out,
                     void* ws, size_t ws_bytes, hipStream_t st, const PagedKv* paged = nullptr, int32_t topk = 0) {
  const int64_t rows = (int64_t)b * (prefill ? s : 1);
  const int64_t h1 = c.h1;
  LayerWs L = carve_layer_ws(c, w, rows, ws);
  // the scratch is carved for THIS row count; the size of the GEMMs' partial-sum area is not monotone in
  // the row count, so a buffer sized for more rows need not be large enough
  if (L.total > ws_bytes) return FG_ERR_WORKSPACE;
  int rc;
  if ((rc = layernorm_launch(x_in, h1, reinterpret_cast<const half_t*>(w.ln1_g),
                             reinterpret_cast<const half_t*>(w.ln1_b), rows, h1, c.ln_eps, L.y, h1, st)))
    return rc;
  if ((rc = linear_launch(make_linear(w.wqkv, w.bqkv, L.y, h1, rows, nullptr, 0, 0, L.qkv, 3 * h1), L.gemm,
                          L.gemm_bytes, st)))
    return rc;
  if (paged) {
    if (prefill) {
      if ((rc = prefill_attention_launch(c, L.qkv, b, s, L.o, st))) return rc;
      if ((rc = kv_append_paged_launch(c, L.qkv + h1, L.qkv + 2 * h1, 3 * h1, b, s, *paged->pages, *paged->seqs,
                                       false, st)))
        return rc;
    } else {
      if ((rc = kv_append_paged_launch(c, L.qkv + h1, L.qkv + 2 * h1, 3 * h1, b, 1, *paged->pages, *paged->seqs,
                                       true, st)))
        return rc;
      // Section 5, sparse attention: every row keeps its min(topk, rows) highest-weighted V rows
      if (topk > 0)
        rc = decode_attention_topk_paged_launch(c, L.qkv, 3 * h1, b, topk, *paged->pages, *paged->seqs, 1, L.o,
                                                nullptr, st);
      else
        rc = decode_attention_paged_launch(c, L.qkv, 3 * h1, b, *paged->pages, *paged->seqs, 1, L.o, st);
      if (rc) return rc;
    }
  } else if (prefill) {
    if ((rc = prefill_attention_launch(c, L.qkv, b, s, L.o, st))) return rc;
    if ((rc = kv_append_launch(c, L.qkv + h1, L.qkv + 2 * h1, 3 * h1, b, s, kv, batch_offset, 0, st))) return rc;
  } else {
    if ((rc = kv_append_launch(c, L.qkv + h1, L.qkv + 2 * h1, 3 * h1, b, 1, kv, batch_offset, t, st))) return rc;
    if (topk > 0 && topk < t + 1)   // Section 5, sparse attention (with topk >= rows it IS the dense one)
      rc = decode_attention_topk_launch(c, L.qkv, 3 * h1, b, t + 1, topk, kv, batch_offset, L.o, nullptr, st);
    else
      rc = decode_attention_launch(c, L.qkv, 3 * h1, b, t + 1, kv, batch_offset, L.o, st);
    if (rc) return rc;
  }
  if ((rc = linear_launch(make_linear(w.wo, w.bo, L.o, h1, rows, x_in, h1, 0, L.x1, h1), L.gemm, L.gemm_bytes,
                          st)))
    return rc;
  if ((rc = layernorm_launch(L.x1, h1, reinterpret_cast<const half_t*>(w.ln2_g),
                             reinterpret_cast<const half_t*>(w.ln2_b), rows, h1, c.ln_eps, L.y, h1, st)))
    return rc;
  if ((rc = linear_launch(make_linear(w.w1, w.b1, L.y, h1, rows, nullptr, 0, 1, L.act, act_stride(c)), L.gemm,
                          L.gemm_bytes, st)))
    return rc;
  return linear_launch(make_linear(w.w2, w.b2, L.act, act_stride(c), rows, L.x1, h1, 0, x_out, h1), L.gemm, L.gemm_bytes,
                       st);
}

// ---------------------------------------------------------------- LM head
struct HeadWs {
  half_t* y;
  void* gemm;
  size_t gemm_bytes;
  size_t total;
};
static HeadWs carve_head_ws(const fg_model_cfg& c, int64_t rows, void* base) {
  HeadWs H;
  unsigned char* p = reinterpret_cast<unsigned char*>(base);
  const size_t ybytes = align_up((size_t)rows * c.h1 * 2, 256);
  H.y = reinterpret_cast<half_t*>(p);
  H.gemm_bytes = linear_workspace_bytes(FG_F16, c.vocab, c.h1, rows);
  H.gemm = p ? p + ybytes : nullptr;
  H.total = ybytes + align_up(H.gemm_bytes, 256);
  return H;
}

static int run_lm_head(const fg_model_cfg& c, const half_t* x, int64_t ldx, int64_t rows, const half_t* g,
                       const half_t* bta, const half_t* emb, int32_t* out_ids, int64_t out_stride, float* logits,
                       void* ws, size_t ws_bytes, hipStream_t st, const int32_t* out_index = nullptr) {
  HeadWs H = carve_head_ws(c, rows, ws);
  if (H.total > ws_bytes) return FG_ERR_WORKSPACE;
  int rc;
  if ((rc = layernorm_launch(x, ldx, g, bta, rows, c.h1, c.ln_eps, H.y, c.h1, st))) return rc;
  LinearArgs a;
  a.w_data = emb;
  a.w_meta = nullptr;
  a.dtype = FG_F16;
  a.n = c.vocab;
  a.k = c.h1;
  a.x = H.y;
  a.ldx = c.h1;
  a.m = rows;
  a.bias = nullptr;
  a.residual = nullptr;
  a.ldr = 0;
  a.relu = 0;
  a.out_f16 = nullptr;
  a.out_f32 = logits;
  a.ldo = c.vocab;
  if ((rc = linear_launch(a, H.gemm, H.gemm_bytes, st))) return rc;
  return argmax_launch(logits, rows, c.vocab, out_ids, out_stride, st, out_index);
}

}  // namespace fg

using namespace fg;

// ================================================================ C ABI
extern "C" const char* fg_error_string(int status) {
  switch (status) {
    case FG_OK: return "ok";
    case FG_ERR_NULL: return "a required pointer is NULL";
    case FG_ERR_SHAPE: return "bad shape, size or alignment";
    case FG_ERR_UNSUPPORTED: return "unsupported format (only 4-bit codes, groups of 64, head size 64 or 128)";
    case FG_ERR_WORKSPACE: return "workspace missing or too small";
    case FG_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" const char* fg_last_device_error(void) { return g_dev_err.c_str(); }

extern "C" int fg_version(void) { return 100; }

extern "C" const char* fg_kernel_class_name(int k) {
  static const char* names[FG_K_COUNT] = {"quantize",      "dequantize",          "layernorm",    "gemm_small_m",
                                          "gemm_small_m_finish", "gemm_large_m",  "kv_append",    "attn_decode",
                                          "attn_prefill",  "embed",               "argmax"};
  return (k >= 0 && k < FG_K_COUNT) ? names[k] : "?";
}

extern "C" int fg_profile_begin_classes(uint32_t class_mask) {
  for (auto& r : g_prof_open) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  g_prof_open.clear();
  memset(g_prof_ms, 0, sizeof(g_prof_ms));
  memset(g_prof_n, 0, sizeof(g_prof_n));
  g_prof_mask = class_mask;
  g_prof_on = class_mask != 0;
  return FG_OK;
}

extern "C" int fg_profile_begin(void) { return fg_profile_begin_classes(0xffffffffu); }

extern "C" int fg_profile_end(void) {
  g_prof_on = false;
  int rc = FG_OK;
  for (auto& r : g_prof_open) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
      g_prof_ms[r.k] += ms;
      g_prof_n[r.k] += 1;
    } else {
      rc = FG_ERR_DEVICE;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  g_prof_open.clear();
  return rc;
}

extern "C" int fg_profile_read(int k, double* total_ms, int64_t* launches) {
  if (k < 0 || k >= FG_K_COUNT) return FG_ERR_SHAPE;
  if (total_ms) *total_ms = g_prof_ms[k];
  if (launches) *launches = g_prof_n[k];
  return FG_OK;
}

extern "C" int fg_pack_weights(const fg_mat* src, void* data_out, void* meta_out, void* stream) {
  if (!src) return FG_ERR_NULL;
  int rc = check_mat(src, true);
  if (rc) return rc;
  if (src->dtype != FG_Q4G64 && src->dtype != FG_Q4G64_H16) return FG_ERR_UNSUPPORTED;
  if (src->rows % 32 != 0) return FG_ERR_SHAPE;
  if (!data_out || !meta_out) return FG_ERR_NULL;
  if (!aligned16(data_out) || !aligned16(meta_out)) return FG_ERR_SHAPE;
  return pack_weights_launch(src->data, src->meta, src->dtype == FG_Q4G64_H16, src->rows, src->cols, data_out,
                             meta_out, as_stream(stream));
}

extern "C" size_t fg_linear_workspace_bytes(const fg_mat* w, int64_t m) {
  if (!w || m <= 0) return 0;
  return linear_workspace_bytes(w->dtype, w->rows, w->cols, m);
}

extern "C" int fg_linear(const fg_mat* w, const void* bias_f16, const void* x_f16, int64_t m,
                         const void* residual_f16, int relu, void* out_f16, void* ws, size_t ws_bytes,
                         void* stream) {
  if (!w) return FG_ERR_NULL;
  int rc = check_mat(w);
  if (rc) return rc;
  if (m < 0 || m > 0x7fffffff) return FG_ERR_SHAPE;
  if (m == 0) return FG_OK;
  if (!x_f16 || !out_f16) return FG_ERR_NULL;
  if (!aligned16(x_f16) || !aligned16(out_f16)) return FG_ERR_SHAPE;
  const size_t need = linear_workspace_bytes(w->dtype, w->rows, w->cols, m);
  if (need && (!ws || ws_bytes < need)) return FG_ERR_WORKSPACE;
  return linear_launch(make_linear(*w, bias_f16, reinterpret_cast<const half_t*>(x_f16), w->cols, m,
                                   reinterpret_cast<const half_t*>(residual_f16), w->rows, relu,
                                   reinterpret_cast<half_t*>(out_f16), w->rows),
                       ws, ws_bytes, as_stream(stream));
}

// ---------------------------------------------------------------- fg_linear without a workspace argument
// For callers that can neither allocate device memory nor carry a workspace through their call chain
// (code under HIP graph capture, tight serving loops): the partial sums of the split contraction go
// to a fixed array in device memory that belongs to the library.  Every GPU the library runs on holds
// its own copy of the array, at its own address, from the moment the code object is loaded until the
// process ends.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)80 << 20;   // the decode-shape projections (up to 320 rows) need at most this
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, looked up once per device
bool g_scratch_known[kMaxDevices];

// In host code the array's name is only a handle for the runtime, not a device address: the address is
// asked for once per device, with that device current, and that is what the kernels are given.
int static_scratch(void** ptr) {
  int dev = -1;
  FG_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return FG_ERR_UNSUPPORTED;
  if (!g_scratch_known[dev]) {
    void* p = nullptr;
    FG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return FG_ERR_DEVICE;
    g_scratch_ptr[dev] = p;
    g_scratch_known[dev] = true;
  }
  *ptr = g_scratch_ptr[dev];
  return FG_OK;
}
}  // namespace

extern "C" size_t fg_linear_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int fg_linear_static(const fg_mat* w, const void* bias_f16, const void* x_f16, int64_t m,
                                const void* residual_f16, int relu, void* out_f16, void* stream) {
  if (!w) return FG_ERR_NULL;
  int rc = check_mat(w);
  if (rc) return rc;
  if (m < 0 || m > 0x7fffffff) return FG_ERR_SHAPE;
  if (m == 0) return FG_OK;
  if (!x_f16 || !out_f16) return FG_ERR_NULL;
  if (!aligned16(x_f16) || !aligned16(out_f16)) return FG_ERR_SHAPE;
  const size_t need = linear_workspace_bytes(w->dtype, w->rows, w->cols, m);
  if (need > kStaticScratchBytes) return FG_ERR_WORKSPACE;   // beyond what the library's own scratch array holds
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  // Nothing in the scratch has to start at zero: every partial-sum slot that the reduction pass reads
  // was written by the contraction kernel of the same call.
  return linear_launch(make_linear(*w, bias_f16, reinterpret_cast<const half_t*>(x_f16), w->cols, m,
                                   reinterpret_cast<const half_t*>(residual_f16), w->rows, relu,
                                   reinterpret_cast<half_t*>(out_f16), w->rows),
                       ws, kStaticScratchBytes, as_stream(stream));
}

extern "C" size_t fg_lm_head_workspace_bytes(const fg_model_cfg* cfg, int64_t rows) {
  if (!cfg || rows <= 0 || check_cfg(cfg)) return 0;
  return carve_head_ws(*cfg, rows, nullptr).total;
}

extern "C" int fg_lm_head_greedy(const fg_model_cfg* cfg, const void* x_f16, int64_t x_row_stride, int64_t rows,
                                 const void* lnf_g, const void* lnf_b, const void* embed_f16, int32_t* out_ids,
                                 int64_t out_stride, float* logits_f32, void* ws, size_t ws_bytes,
                                 void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (rows < 0 || rows > 0x7fffffff || x_row_stride < cfg->h1 || x_row_stride % 8 != 0 || out_stride < 1)
    return FG_ERR_SHAPE;
  if (cfg->vocab % 8 != 0) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!x_f16 || !lnf_g || !lnf_b || !embed_f16 || !out_ids || !logits_f32) return FG_ERR_NULL;
  if (!ws || ws_bytes < carve_head_ws(*cfg, rows, nullptr).total) return FG_ERR_WORKSPACE;
  return run_lm_head(*cfg, reinterpret_cast<const half_t*>(x_f16), x_row_stride, rows,
                     reinterpret_cast<const half_t*>(lnf_g), reinterpret_cast<const half_t*>(lnf_b),
                     reinterpret_cast<const half_t*>(embed_f16), out_ids, out_stride, logits_f32, ws, ws_bytes,
                     as_stream(stream));
}

extern "C" size_t fg_layer_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* wts, int64_t rows) {
  if (!cfg || !wts || rows <= 0 || check_cfg(cfg)) return 0;
  return carve_layer_ws(*cfg, *wts, rows, nullptr).total;
}

static int check_layer_call(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in,
                            const fg_kv_cache* kv, void* x_out) {
  if (!cfg || !wts || !kv) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if ((rc = check_layer(cfg, wts))) return rc;
  if ((rc = check_kv(cfg, kv))) return rc;
  (void)x_in;
  (void)x_out;
  return FG_OK;
}

extern "C" int fg_prefill_layer(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                                int32_t s, const fg_kv_cache* kv, int32_t batch_offset, void* x_out, void* ws,
                                size_t ws_bytes, void* stream) {
  int rc = check_layer_call(cfg, wts, x_in, kv, x_out);
  if (rc) return rc;
  if (b < 0 || s < 0 || batch_offset < 0 || b > 65535) return FG_ERR_SHAPE;
  if ((int64_t)batch_offset + b > kv->batch || s > kv->cap) return FG_ERR_SHAPE;
  if ((int64_t)b * s > 0x7fffffff) return FG_ERR_SHAPE;
  if (b == 0 || s == 0) return FG_OK;
  if (!x_in || !x_out) return FG_ERR_NULL;
  if (!aligned16(x_in) || !aligned16(x_out)) return FG_ERR_SHAPE;
  const size_t need = carve_layer_ws(*cfg, *wts, (int64_t)b * s, nullptr).total;
  if (!ws || ws_bytes < need) return FG_ERR_WORKSPACE;
  if (!aligned16(ws)) return FG_ERR_SHAPE;
  return run_layer(*cfg, *wts, reinterpret_cast<const half_t*>(x_in), b, s, true, 0, *kv, batch_offset,
                   reinterpret_cast<half_t*>(x_out), ws, ws_bytes, as_stream(stream));
}

extern "C" int fg_decode_layer(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                               int32_t t, int32_t topk, const fg_kv_cache* kv, int32_t batch_offset, void* x_out,
                               void* ws, size_t ws_bytes, void* stream) {
  int rc = check_layer_call(cfg, wts, x_in, kv, x_out);
  if (rc) return rc;
  if (b < 0 || t < 0 || batch_offset < 0 || b > 65535 || topk < 0) return FG_ERR_SHAPE;
  if (topk > 0 && kv->dtype != FG_Q4G64 && kv->dtype != FG_Q4G64_H16) return FG_ERR_UNSUPPORTED;
  if (topk > 0 && topk < t + 1 && (int64_t)(t + 1 + 127) / 128 * 128 + topk > 36864) return FG_ERR_UNSUPPORTED;
  if ((int64_t)batch_offset + b > kv->batch || t >= kv->cap) return FG_ERR_SHAPE;
  if (b == 0) return FG_OK;
  if (!x_in || !x_out) return FG_ERR_NULL;
  if (!aligned16(x_in) || !aligned16(x_out)) return FG_ERR_SHAPE;
  const size_t need = carve_layer_ws(*cfg, *wts, b, nullptr).total;
  if (!ws || ws_bytes < need) return FG_ERR_WORKSPACE;
  if (!aligned16(ws)) return FG_ERR_SHAPE;
  return run_layer(*cfg, *wts, reinterpret_cast<const half_t*>(x_in), b, 1, false, t, *kv, batch_offset,
                   reinterpret_cast<half_t*>(x_out), ws, ws_bytes, as_stream(stream), nullptr, topk);
}

static int paged_layer_entry(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                             int32_t s, bool prefill, const fg_kv_pages* pages, const fg_ragged* seqs, void* x_out,
                             void* ws, size_t ws_bytes, void* stream, int32_t topk = 0) {
  if (!cfg || !wts) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if ((rc = check_layer(cfg, wts))) return rc;
  if ((rc = check_pages(cfg, pages, seqs))) return rc;
  if (!prefill && !seqs->pos) return FG_ERR_NULL;
  if (b < 0 || s < 0 || b > 65535 || (int64_t)b * s > 0x7fffffff || topk < 0) return FG_ERR_SHAPE;
  if (topk > 0 && pages->dtype != FG_Q4G64 && pages->dtype != FG_Q4G64_H16) return FG_ERR_UNSUPPORTED;
  if (topk > 0 && ((int64_t)seqs->table_stride * FG_PAGE_ROWS + 127) / 128 * 128 + topk > 36864) return FG_ERR_UNSUPPORTED;
  if (prefill && s > (int64_t)seqs->table_stride * FG_PAGE_ROWS) return FG_ERR_SHAPE;
  if (b == 0 || s == 0) return FG_OK;
  if (!x_in || !x_out) return FG_ERR_NULL;
  if (!aligned16(x_in) || !aligned16(x_out)) return FG_ERR_SHAPE;
  const size_t need = carve_layer_ws(*cfg, *wts, (int64_t)b * s, nullptr).total;
  if (!ws || ws_bytes < need) return FG_ERR_WORKSPACE;
  if (!aligned16(ws)) return FG_ERR_SHAPE;
  const PagedKv pk = {pages, seqs};
  const fg_kv_cache none = {};
  return run_layer(*cfg, *wts, reinterpret_cast<const half_t*>(x_in), b, s, prefill, 0, none, 0,
                   reinterpret_cast<half_t*>(x_out), ws, ws_bytes, as_stream(stream), &pk, topk);
}

extern "C" int fg_decode_layer_paged(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in,
                                     int32_t b, int32_t topk, const fg_kv_pages* pages, const fg_ragged* seqs,
                                     void* x_out, void* ws, size_t ws_bytes, void* stream) {
  return paged_layer_entry(cfg, wts, x_in, b, 1, false, pages, seqs, x_out, ws, ws_bytes, stream, topk);
}

extern "C" int fg_prefill_layer_paged(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in,
                                      int32_t b, int32_t s, const fg_kv_pages* pages, const fg_ragged* seqs,
                                      void* x_out, void* ws, size_t ws_bytes, void* stream) {
  return paged_layer_entry(cfg, wts, x_in, b, s, true, pages, seqs, x_out, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------- block generation
namespace {
struct GenWs {
  half_t* x_all;    // [bls*s, h1] prefill activations of the whole block
  half_t* x_dec;    // [bls, h1]
  float* logits;    // [bls, vocab]
  void* layer;      // per-layer scratch (max of prefill GPU batch and decode block)
  size_t layer_bytes;
  void* head;
  size_t head_bytes;
  size_t total;
};
GenWs carve_gen_ws(const fg_model_cfg& c, const fg_layer_weights& w0, int32_t gbs, int32_t ngb, int32_t s,
                   void* base) {
  GenWs G;
  unsigned char* p = reinterpret_cast<unsigned char*>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    unsigned char* r = p ? p + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  };
  const int64_t bls = (int64_t)gbs * ngb;
  G.x_all = reinterpret_cast<half_t*>(take((size_t)bls * s * c.h1 * 2));
  G.x_dec = reinterpret_cast<half_t*>(take((size_t)bls * c.h1 * 2));
  G.logits = reinterpret_cast<float*>(take((size_t)bls * c.vocab * 4));
  const size_t lp = carve_layer_ws(c, w0, (int64_t)gbs * s, nullptr).total;
  const size_t ld = carve_layer_ws(c, w0, bls, nullptr).total;
  G.layer_bytes = lp > ld ? lp : ld;
  G.layer = take(G.layer_bytes);
  G.head_bytes = carve_head_ws(c, bls, nullptr).total;
  G.head = take(G.head_bytes);
  G.total = off;
  return G;
}
}  // namespace

extern "C" size_t fg_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* layer0, int32_t gpu_batch_size,
                                     int32_t num_gpu_batches, int32_t s) {
  if (!cfg || !layer0 || gpu_batch_size <= 0 || num_gpu_batches <= 0 || s <= 0 || check_cfg(cfg)) return 0;
  return carve_gen_ws(*cfg, *layer0, gpu_batch_size, num_gpu_batches, s, nullptr).total;
}

extern "C" int fg_generate(const fg_model_cfg* cfg, int32_t l, const fg_layer_weights* layers,
                           const void* embed_f16, const void* pos_f16, const void* lnf_g, const void* lnf_b,
                           const int32_t* prompt, int32_t s, int32_t n, int32_t num_gpu_batches,
                           int32_t gpu_batch_size, const fg_kv_cache* kv, int32_t* out_ids, void* ws,
                           size_t ws_bytes, void* stream, fg_stats* stats) {
  if (!cfg || !layers || !kv) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (l <= 0 || s <= 0 || n <= 0 || num_gpu_batches <= 0 || gpu_batch_size <= 0) return FG_ERR_SHAPE;
  const int64_t bls64 = (int64_t)num_gpu_batches * gpu_batch_size;
  if (bls64 > 65535 || (int64_t)gpu_batch_size * s > 0x7fffffff) return FG_ERR_SHAPE;
  if ((int64_t)s + n - 1 > cfg->max_pos || cfg->vocab % 8 != 0) return FG_ERR_SHAPE;
  const int32_t bls = (int32_t)bls64;
  for (int j = 0; j < l; ++j) {
    if ((rc = check_layer(cfg, &layers[j]))) return rc;
    if ((rc = check_kv(cfg, &kv[j]))) return rc;
    if (kv[j].batch < bls || kv[j].cap < s + n - 1) return FG_ERR_SHAPE;
    // one scratch size serves all layers: they must share the storage format of layer 0
    if (layers[j].wqkv.dtype != layers[0].wqkv.dtype || layers[j].wo.dtype != layers[0].wo.dtype ||
        layers[j].w1.dtype != layers[0].w1.dtype || layers[j].w2.dtype != layers[0].w2.dtype)
      return FG_ERR_UNSUPPORTED;
  }
  if (!embed_f16 || !pos_f16 || !lnf_g || !lnf_b || !prompt || !out_ids) return FG_ERR_NULL;
  const GenWs need = carve_gen_ws(*cfg, layers[0], gpu_batch_size, num_gpu_batches, s, nullptr);
  if (!ws || ws_bytes < need.total) return FG_ERR_WORKSPACE;
  if (!aligned16(ws)) return FG_ERR_SHAPE;
  const GenWs G = carve_gen_ws(*cfg, layers[0], gpu_batch_size, num_gpu_batches, s, ws);
  hipStream_t st = as_stream(stream);
  const half_t* emb = reinterpret_cast<const half_t*>(embed_f16);
  const half_t* pos = reinterpret_cast<const half_t*>(pos_f16);
  const half_t* fg_ = reinterpret_cast<const half_t*>(lnf_g);
  const half_t* fb_ = reinterpret_cast<const half_t*>(lnf_b);
  const int64_t h1 = cfg->h1;

  std::vector<hipEvent_t> ev;
  auto mark = [&]() -> int {
    if (!stats) return FG_OK;
    hipEvent_t e;
    FG_HIP(hipEventCreate(&e));
    FG_HIP(hipEventRecord(e, st));
    ev.push_back(e);
    return FG_OK;
  };
  auto cleanup = [&]() {
    for (auto e : ev) (void)hipEventDestroy(e);
  };
#define FG_TRY(expr)       \
  do {                     \
    int _rc = (expr);      \
    if (_rc) {             \
      cleanup();           \
      return _rc;          \
    }                      \
  } while (0)

  // ---- token step 1: prefill.  Layer outermost, GPU batch innermost (zig-zag block schedule):
  // all GPU batches pass through layer j before layer j+1 is touched.
  FG_TRY(mark());
  FG_TRY(embed_launch(emb, pos, prompt, 1, (int64_t)bls * s, s, 0, cfg->h1, cfg->vocab, G.x_all, st));
  for (int j = 0; j < l; ++j) {
    for (int k = 0; k < num_gpu_batches; ++k) {
      half_t* xk = G.x_all + (int64_t)k * gpu_batch_size * s * h1;
      FG_TRY(run_layer(*cfg, layers[j], xk, gpu_batch_size, s, true, 0, kv[j], k * gpu_batch_size, xk, G.layer,
                       G.layer_bytes, st));
    }
  }
  FG_TRY(run_lm_head(*cfg, G.x_all + (int64_t)(s - 1) * h1, (int64_t)s * h1, bls, fg_, fb_, emb, out_ids, n,
                     G.logits, G.head, G.head_bytes, st));
  FG_TRY(mark());
  // ---- token steps 2..n: decode.  Every layer takes all bls rows in one pass, so its weights are
  // streamed from HBM once per step for the whole block.
  for (int i = 1; i < n; ++i) {
    const int t = s + i - 1;   // rows already cached = absolute position of the token fed back
    FG_TRY(embed_launch(emb, pos, out_ids + (i - 1), n, bls, 1, t, cfg->h1, cfg->vocab, G.x_dec, st));
    for (int j = 0; j < l; ++j)
      FG_TRY(run_layer(*cfg, layers[j], G.x_dec, bls, 1, false, t, kv[j], 0, G.x_dec, G.layer, G.layer_bytes, st));
    FG_TRY(run_lm_head(*cfg, G.x_dec, h1, bls, fg_, fb_, emb, out_ids + i, n, G.logits, G.head, G.head_bytes, st));
    FG_TRY(mark());
  }
#undef FG_TRY

  if (stats) {
    if (hipEventSynchronize(ev.back()) != hipSuccess) {
      cleanup();
      return FG_ERR_DEVICE;
    }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, ev[0], ev[1]);
    stats->prefill_s = ms * 1e-3;
    double dec = 0.0;
    for (int i = 1; i < n; ++i) {
      (void)hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
      dec += ms * 1e-3;
      if (stats->decode_step_s) stats->decode_step_s[i - 1] = ms * 1e-3;
    }
    stats->decode_s = dec;
    stats->tokens = (int64_t)bls * n;
    auto mat_bytes = [](const fg_mat& m) -> int64_t {
      const int64_t e = m.rows * m.cols;
      if (m.dtype == FG_F16) return e * 2;
      return e / 2 + e / kGroup * (m.dtype == FG_Q4G64_H16_TILED ? 4 : 8);
    };
    int64_t wb = 0;
    for (int j = 0; j < l; ++j)
      wb += mat_bytes(layers[j].wqkv) + mat_bytes(layers[j].wo) + mat_bytes(layers[j].w1) + mat_bytes(layers[j].w2);
    stats->weight_bytes_per_step = wb;
    const int64_t rows_last = (int64_t)s + n - 1;
    const int64_t el = 2 * (int64_t)bls * l * h1 * (n > 1 ? rows_last : 0);
    stats->kv_bytes_last_step = kv[0].dtype == FG_Q4G64       ? el / 2 + el / kGroup * 8
                                : kv[0].dtype == FG_Q4G64_H16 ? el / 2 + el / kGroup * 4
                                                              : el * 2;
    cleanup();
  }
  return FG_OK;
}

// ---------------------------------------------------------------- diagonal block schedule
namespace {
// Host bookkeeping of the diagonal order (appendix, "Diagonal block schedule"): GPU batch g is admitted
// in iteration g, so in iteration `it` it is at token step it - g; it is retired after step n - 1.
// Pages are taken one at a time as a sequence grows and returned when its batch retires.
struct DiagPlan {
  int n_seqs, s, n, gbs, ng, max_pages;
  std::vector<int32_t> table;   // [n_seqs][max_pages], -1 = none
  std::vector<int32_t> free_list;
  int in_use = 0, peak = 0;
  DiagPlan(int n_seqs_, int s_, int n_, int gbs_, int pool_pages)
      : n_seqs(n_seqs_), s(s_), n(n_), gbs(gbs_), ng(n_seqs_ / gbs_),
        max_pages((s_ + n_ + FG_PAGE_ROWS - 1) / FG_PAGE_ROWS), table((size_t)n_seqs_ * max_pages, -1) {
    free_list.reserve(pool_pages);
    for (int p = pool_pages - 1; p >= 0; --p) free_list.push_back(p);
  }
  int iterations() const { return ng + n - 1; }
  bool ensure(int seq, int rows) {   // pages for positions 0 .. rows-1
    const int need = (rows + FG_PAGE_ROWS - 1) / FG_PAGE_ROWS;
    for (int slot = 0; slot < need; ++slot) {
      int32_t& e = table[(size_t)seq * max_pages + slot];
      if (e >= 0) continue;
      if (free_list.empty()) return false;
      e = free_list.back();
      free_list.pop_back();
      ++in_use;
    }
    peak = in_use > peak ? in_use : peak;
    return true;
  }
  void release(int seq) {
    for (int slot = 0; slot < max_pages; ++slot) {
      int32_t& e = table[(size_t)seq * max_pages + slot];
      if (e >= 0) {
        free_list.push_back(e);
        e = -1;
        --in_use;
      }
    }
  }
  // groups active in iteration it: [g_lo, g_hi]; the admitted one (if any) is `it` itself
  void active(int it, int& g_lo, int& g_hi) const {
    g_lo = it - (n - 1) > 0 ? it - (n - 1) : 0;
    g_hi = it < ng - 1 ? it : ng - 1;
  }
  // Takes the pages iteration `it` needs; false if the pool runs dry.
  bool begin_iteration(int it) {
    int g_lo, g_hi;
    active(it, g_lo, g_hi);
    for (int g = g_lo; g <= g_hi; ++g) {
      const int rows = g == it ? s : s + (it - g);   // after this iteration's append
      for (int q = g * gbs; q < (g + 1) * gbs; ++q)
        if (!ensure(q, rows)) return false;
    }
    return true;
  }
  void end_iteration(int it) {
    const int g = it - (n - 1);
    if (g >= 0 && g < ng)
      for (int q = g * gbs; q < (g + 1) * gbs; ++q) release(q);
  }
};

struct DiagWs {
  half_t* x_new;    // [gbs*s, h1]
  half_t* x_dec;    // [bmax, h1]
  float* logits;    // [max(gbs, bmax), vocab]
  int32_t* ints;    // page table and the per-iteration row arrays
  size_t n_ints;
  void* layer;
  size_t layer_bytes;
  void* head;
  size_t head_bytes;
  size_t total;
};
int diag_bmax(int n_seqs, int n, int gbs) {
  const int ng = n_seqs / gbs;
  const int groups = ng < n - 1 ? ng : n - 1;
  return groups * gbs;
}
DiagWs carve_diag_ws(const fg_model_cfg& c, const fg_layer_weights& w0, int n_seqs, int s, int n, int gbs,
                     void* base) {
  DiagWs D;
  unsigned char* p = reinterpret_cast<unsigned char*>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    unsigned char* r = p ? p + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  };
  const int bmax = diag_bmax(n_seqs, n, gbs);
  const int brow = bmax > 0 ? bmax : 1;
  const int max_pages = (s + n + FG_PAGE_ROWS - 1) / FG_PAGE_ROWS;
  D.x_new = reinterpret_cast<half_t*>(take((size_t)gbs * s * c.h1 * 2));
  D.x_dec = reinterpret_cast<half_t*>(take((size_t)brow * c.h1 * 2));
  D.logits = reinterpret_cast<float*>(take((size_t)(gbs > brow ? gbs : brow) * c.vocab * 4));
  D.n_ints = (size_t)n_seqs * max_pages + gbs + 4 * (size_t)brow;
  D.ints = reinterpret_cast<int32_t*>(take(D.n_ints * 4));
  // Per-layer scratch: the largest need over the prefill square and EVERY decode row count the schedule
  // runs (gbs, 2*gbs, ..., bmax).  Not just the largest row count: the partial-sum area of the GEMMs
  // depends on the tile shape picked for the row count and can shrink when the rows grow.
  D.layer_bytes = carve_layer_ws(c, w0, (int64_t)gbs * s, nullptr).total;
  size_t head_bytes = carve_head_ws(c, gbs, nullptr).total;
  for (int b = gbs; b <= bmax; b += gbs) {
    const size_t ld = carve_layer_ws(c, w0, b, nullptr).total;
    D.layer_bytes = ld > D.layer_bytes ? ld : D.layer_bytes;
    const size_t hd = carve_head_ws(c, b, nullptr).total;
    head_bytes = hd > head_bytes ? hd : head_bytes;
  }
  D.layer = take(D.layer_bytes);
  D.head_bytes = head_bytes;
  D.head = take(head_bytes);
  D.total = off;
  return D;
}
bool diag_args_ok(int32_t n_seqs, int32_t s, int32_t n, int32_t gbs) {
  return n_seqs > 0 && s > 0 && n > 0 && gbs > 0 && n_seqs % gbs == 0 && (int64_t)s + n <= 0x3fffffff &&
         (int64_t)n_seqs * n <= 0x7fffffff &&
         (int64_t)gbs * s <= 0x7fffffff && diag_bmax(n_seqs, n, gbs) <= 65535;
}
}  // namespace

extern "C" int64_t fg_diagonal_pages_needed(int32_t n_seqs, int32_t s, int32_t n, int32_t gpu_batch_size) {
  if (!diag_args_ok(n_seqs, s, n, gpu_batch_size)) return -1;
  const int64_t all = (int64_t)n_seqs * ((s + n + FG_PAGE_ROWS - 1) / FG_PAGE_ROWS);
  if (all > 0x7fffffff) return -1;
  DiagPlan plan(n_seqs, s, n, gpu_batch_size, (int)all);
  for (int it = 0; it < plan.iterations(); ++it) {
    plan.begin_iteration(it);
    plan.end_iteration(it);
  }
  return plan.peak;
}

extern "C" size_t fg_diagonal_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* layer0, int32_t n_seqs,
                                              int32_t s, int32_t n, int32_t gpu_batch_size) {
  if (!cfg || !layer0 || check_cfg(cfg) || !diag_args_ok(n_seqs, s, n, gpu_batch_size)) return 0;
  return carve_diag_ws(*cfg, *layer0, n_seqs, s, n, gpu_batch_size, nullptr).total;
}

extern "C" int fg_generate_diagonal(const fg_model_cfg* cfg, int32_t l, const fg_layer_weights* layers,
                                    const void* embed_f16, const void* pos_f16, const void* lnf_g, const void* lnf_b,
                                    const int32_t* prompt, int32_t n_seqs, int32_t s, int32_t n,
                                    int32_t gpu_batch_size, const fg_kv_pages* pages, int32_t* out_ids, void* ws,
                                    size_t ws_bytes, void* stream, fg_stats* stats, int32_t* peak_pages) {
  if (!cfg || !layers || !pages) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (l <= 0 || !diag_args_ok(n_seqs, s, n, gpu_batch_size)) return FG_ERR_SHAPE;
  if ((int64_t)s + n - 1 > cfg->max_pos || cfg->vocab % 8 != 0) return FG_ERR_SHAPE;
  const int gbs = gpu_batch_size;
  for (int j = 0; j < l; ++j) {
    if ((rc = check_layer(cfg, &layers[j]))) return rc;
    const bool q4 = pages[j].dtype == FG_Q4G64 || pages[j].dtype == FG_Q4G64_H16;
    if (!q4 && pages[j].dtype != FG_F16) return FG_ERR_UNSUPPORTED;
    if (pages[j].n_pages != pages[0].n_pages || pages[j].n_pages <= 0) return FG_ERR_SHAPE;
    if (!pages[j].k_codes || !pages[j].v_codes || (q4 && (!pages[j].k_meta || !pages[j].v_meta))) return FG_ERR_NULL;
    if (layers[j].wqkv.dtype != layers[0].wqkv.dtype || layers[j].wo.dtype != layers[0].wo.dtype ||
        layers[j].w1.dtype != layers[0].w1.dtype || layers[j].w2.dtype != layers[0].w2.dtype)
      return FG_ERR_UNSUPPORTED;
  }
  if (!embed_f16 || !pos_f16 || !lnf_g || !lnf_b || !prompt || !out_ids) return FG_ERR_NULL;
  const int64_t needed = fg_diagonal_pages_needed(n_seqs, s, n, gbs);
  if (needed < 0 || pages[0].n_pages < needed) return FG_ERR_WORKSPACE;   // the pool cannot hold the schedule
  const DiagWs need = carve_diag_ws(*cfg, layers[0], n_seqs, s, n, gbs, nullptr);
  if (!ws || ws_bytes < need.total) return FG_ERR_WORKSPACE;
  if (!aligned16(ws)) return FG_ERR_SHAPE;
  const DiagWs D = carve_diag_ws(*cfg, layers[0], n_seqs, s, n, gbs, ws);
  hipStream_t st = as_stream(stream);
  const half_t* emb = reinterpret_cast<const half_t*>(embed_f16);
  const half_t* pos = reinterpret_cast<const half_t*>(pos_f16);
  const half_t* fg_ = reinterpret_cast<const half_t*>(lnf_g);
  const half_t* fb_ = reinterpret_cast<const half_t*>(lnf_b);
  const int64_t h1 = cfg->h1;

  DiagPlan plan(n_seqs, s, n, gbs, pages[0].n_pages);
  const int bmax = diag_bmax(n_seqs, n, gbs) > 0 ? diag_bmax(n_seqs, n, gbs) : 1;
  // device int32 arrays, refreshed once per iteration in one copy: the page table, the admitted batch's
  // sequence ids, and per decode row: sequence, position, where its input token is, where its output goes
  const size_t tab_n = (size_t)n_seqs * plan.max_pages;
  int32_t* d_table = D.ints;
  int32_t* d_new = d_table + tab_n;
  int32_t* d_seq = d_new + gbs;
  int32_t* d_pos = d_seq + bmax;
  int32_t* d_in = d_pos + bmax;
  int32_t* d_out = d_in + bmax;
  std::vector<int32_t> h(D.n_ints, 0);

  hipEvent_t e0 = nullptr, e1 = nullptr, copied = nullptr;
  auto cleanup = [&]() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (copied) {
      (void)hipEventSynchronize(copied);   // the host buffer must outlive the last copy that reads it
      (void)hipEventDestroy(copied);
    }
  };
  FG_HIP(hipEventCreateWithFlags(&copied, hipEventDisableTiming));
#define FG_TRY(expr)       \
  do {                     \
    int _rc = (expr);      \
    if (_rc) {             \
      cleanup();           \
      return _rc;          \
    }                      \
  } while (0)
  if (stats && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess ||
                hipEventRecord(e0, st) != hipSuccess)) {
    cleanup();
    return FG_ERR_DEVICE;
  }
  for (int it = 0; it < plan.iterations(); ++it) {
    if (!plan.begin_iteration(it)) {
      cleanup();
      return FG_ERR_WORKSPACE;
    }
    int g_lo, g_hi;
    plan.active(it, g_lo, g_hi);
    const bool admit = it < plan.ng;
    if (it > 0 && hipEventSynchronize(copied) != hipSuccess) {   // the previous copy has read h
      cleanup();
      return FG_ERR_DEVICE;
    }
    int b = 0;   // decode rows of this iteration: every sequence of the batches at steps 1 .. n-1
    for (int g = g_lo; g <= g_hi; ++g) {
      const int step = it - g;
      if (step == 0) continue;
      for (int q = g * gbs; q < (g + 1) * gbs; ++q, ++b) {
        h[tab_n + gbs + b] = q;
        h[tab_n + gbs + bmax + b] = s + step - 1;             // rows already cached = position of the fed-back token
        h[tab_n + gbs + 2 * (size_t)bmax + b] = q * n + step - 1;   // its id in out_ids
        h[tab_n + gbs + 3 * (size_t)bmax + b] = q * n + step;       // where this step's id goes
      }
    }
    memcpy(h.data(), plan.table.data(), tab_n * 4);
    if (admit)
      for (int i = 0; i < gbs; ++i) h[tab_n + i] = it * gbs + i;
    // The copy is ordered behind the previous iteration's kernels on the stream.  The host buffer is
    // rewritten in the next iteration, so that iteration first waits until this copy has been done
    // (the wait above); the host therefore runs at most one iteration ahead of the GPU.
    if (hipMemcpyAsync(D.ints, h.data(), D.n_ints * 4, hipMemcpyHostToDevice, st) != hipSuccess ||
        hipEventRecord(copied, st) != hipSuccess) {
      cleanup();
      return FG_ERR_DEVICE;
    }
    fg_ragged rn = {d_table, d_new, nullptr, plan.max_pages, n_seqs};
    fg_ragged rd = {d_table, d_seq, d_pos, plan.max_pages, n_seqs};
    if (admit)
      FG_TRY(embed_launch(emb, pos, prompt + (int64_t)it * gbs * s, 1, (int64_t)gbs * s, s, 0, cfg->h1, cfg->vocab,
                          D.x_new, st));
    if (b > 0)
      FG_TRY(embed_ragged_launch(emb, pos, out_ids, d_in, d_pos, b, cfg->h1, cfg->vocab, cfg->max_pos, D.x_dec, st));
    // one diagonal: layer by layer, the admitted batch's prefill square and the decode squares of the rest
    const fg_kv_cache none = {};
    for (int j = 0; j < l; ++j) {
      if (admit) {
        const PagedKv pk = {&pages[j], &rn};
        FG_TRY(run_layer(*cfg, layers[j], D.x_new, gbs, s, true, 0, none, 0, D.x_new, D.layer, D.layer_bytes, st, &pk));
      }
      if (b > 0) {
        const PagedKv pk = {&pages[j], &rd};
        FG_TRY(run_layer(*cfg, layers[j], D.x_dec, b, 1, false, 0, none, 0, D.x_dec, D.layer, D.layer_bytes, st, &pk));
      }
    }
    if (admit)
      FG_TRY(run_lm_head(*cfg, D.x_new + (int64_t)(s - 1) * h1, (int64_t)s * h1, gbs, fg_, fb_, emb,
                         out_ids + (int64_t)it * gbs * n, n, D.logits, D.head, D.head_bytes, st));
    if (b > 0) FG_TRY(run_lm_head(*cfg, D.x_dec, h1, b, fg_, fb_, emb, out_ids, 0, D.logits, D.head, D.head_bytes, st, d_out));
    plan.end_iteration(it);
  }
#undef FG_TRY
  if (peak_pages) *peak_pages = plan.peak;
  if (stats) {
    float ms = 0.f;
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) {
      cleanup();
      return FG_ERR_DEVICE;
    }
    (void)hipEventElapsedTime(&ms, e0, e1);
    stats->prefill_s = 0.0;          // the phases interleave: the whole run is reported as one figure
    stats->decode_s = ms * 1e-3;
    stats->tokens = (int64_t)n_seqs * n;
    stats->weight_bytes_per_step = 0;
    stats->kv_bytes_last_step = 0;
  }
  cleanup();
  return FG_OK;
}
