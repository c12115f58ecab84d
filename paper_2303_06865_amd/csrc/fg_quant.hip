// Group-wise 4-bit asymmetric quantization (Section 5 of the paper): quantizer, inverse map,
// and the KV-cache append that stores new token rows in the compressed layout.
//
// This file is compiled with -ffp-contract=off: codes and {min, scale} must be bit-exact
// functions of the input (binary32, one rounding per operation, IEEE division).
#include "fg_common.h"

namespace fg {

// Eight lanes cooperate on one group of 64 FP16 values (16 bytes per lane), so a wavefront
// covers eight groups per pass: 1 KiB of coalesced input, 256 B of codes, 64 B of meta.
// H16: the 4.5-bit variant whose {min, scale} pair is stored as two FP16 numbers.  min is an FP16
// input value and needs no rounding; scale becomes the smallest FP16 number >= (max-min)/15, and it
// is that stored scale the codes are computed with (so they still lie in [0, 15] unclamped).
template <bool H16>
__device__ __forceinline__ void quantize_group_8lanes(const h8_t v, int sub, uint32_t& packed,
                                                      float& mn_out, float& scale_out) {
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (float)v[i];
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) {
    mn = fminf(mn, x[i]);
    mx = fmaxf(mx, x[i]);
  }
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, o, 64));
    mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  }
  const float range = mx - mn;
  float scale = range / 15.0f;  // IEEE-rounded division (see build flags)
  if (H16) {
    half_t hs = (half_t)scale;                         // round to nearest ...
    if ((float)hs < scale) {                           // ... then up, if that fell below
      const uint16_t b = __builtin_bit_cast(uint16_t, hs);
      hs = __builtin_bit_cast(half_t, (uint16_t)(b + 1));
    }
    scale = (float)hs;
  }
  uint32_t p = 0;
  if (scale > 0.0f) {
    // The code is rint(Q), Q = the correctly rounded quotient (x - min) / scale.  An IEEE division per
    // element makes this kernel VALU-bound, so the quotient is first taken as (x - min) * rcp(scale):
    // rcp is good to 1 ulp and the product adds half an ulp, so it is within 15 * 1.5 * 2^-23 < 3e-6
    // of the exact quotient, as is Q (half an ulp of 15 = 5e-7).  Both therefore round to the same
    // integer unless the fast quotient lies within 1e-4 of a half-integer; only then (2e-4 of all
    // elements, and every exact tie) the lane redoes its eight elements with the exact division.
    const float inv = __builtin_amdgcn_rcpf(scale);
    float t[8];
    bool near_half = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      t[i] = (x[i] - mn) * inv;
      const float frac = t[i] - floorf(t[i]);
      near_half |= fabsf(frac - 0.5f) < 1e-4f;
    }
    if (near_half) {
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = (x[i] - mn) / scale;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float r = rintf(t[i]);  // ties to even
      r = fminf(fmaxf(r, 0.0f), 15.0f);
      p |= ((uint32_t)(int)r) << (4 * i);
    }
  }
  packed = p;
  mn_out = mn;
  scale_out = scale;
  (void)sub;
}

// Plain layout: x [rows, cols] contiguous -> codes [rows, cols/2], meta [rows, cols/64].
template <bool H16>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const half_t* __restrict__ x,
                                                            int64_t n_groups,
                                                            uint32_t* __restrict__ codes,
                                                            void* __restrict__ meta) {
  const int sub = threadIdx.x & 7;
  int64_t g = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 3;
  const int64_t stride = ((int64_t)gridDim.x * blockDim.x) >> 3;
  for (; g < n_groups; g += stride) {  // uniform per 8-lane team, so shuffles stay converged
    const h8_t v = *reinterpret_cast<const h8_t*>(x + g * kGroup + sub * 8);
    uint32_t p;
    float mn, sc;
    quantize_group_8lanes<H16>(v, sub, p, mn, sc);
    codes[g * 8 + sub] = p;
    if (sub == 0) {
      if (H16)
        reinterpret_cast<h2_t*>(meta)[g] = (h2_t){(half_t)mn, (half_t)sc};
      else
        reinterpret_cast<float2*>(meta)[g] = make_float2(mn, sc);
    }
  }
}

template <bool H16>
__global__ __launch_bounds__(256) void dequantize_rows_kernel(const uint32_t* __restrict__ codes,
                                                              const void* __restrict__ meta,
                                                              int64_t n_words,
                                                              float* __restrict__ out) {
  int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; w < n_words; w += stride) {
    const uint32_t p = codes[w];
    float2 m;
    if (H16) {
      const h2_t hm = reinterpret_cast<const h2_t*>(meta)[w >> 3];
      m = make_float2((float)hm.x, (float)hm.y);
    } else {
      m = reinterpret_cast<const float2*>(meta)[w >> 3];
    }
    float4 lo, hi;
    float* o = reinterpret_cast<float*>(&lo);
    float* o2 = reinterpret_cast<float*>(&hi);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[i] = __builtin_fmaf((float)((p >> (4 * i)) & 15u), m.y, m.x);        // one rounding
      o2[i] = __builtin_fmaf((float)((p >> (4 * i + 16)) & 15u), m.y, m.x);
    }
    reinterpret_cast<float4*>(out)[w * 2] = lo;
    reinterpret_cast<float4*>(out)[w * 2 + 1] = hi;
  }
}

// Cache layout: token rows x [b*s, h1] (row stride `ld` elements) -> cache [batch, nh, cap, dh].
// z = 0 stores K, z = 1 stores V.
struct KvAppendArgs {
  const half_t* src[2];
  void* codes[2];
  void* meta[2];
  int64_t ld;
  int32_t b, s, nh, dh, cap, batch_offset, pos0;
  // paged destination (page_table != nullptr): row j of sequence i goes to position pos[i] + j of
  // sequence seq_ids[i]; cap, batch_offset and pos0 are unused
  const int32_t* page_table;
  const int32_t* seq_ids;
  const int32_t* pos;
  int32_t table_stride, n_seqs, n_pages;
};

// First cache row index (in rows of dh elements) of (sequence bi, head, row offset j), or -1 if the
// destination does not exist (paged: an id, position or page number out of range).
__device__ __forceinline__ int64_t kv_dest_row(const KvAppendArgs& a, int64_t bi, int head, int j) {
  if (!a.page_table) return ((int64_t)(a.batch_offset + bi) * a.nh + head) * a.cap + a.pos0 + j;
  const int sid = a.seq_ids ? a.seq_ids[bi] : (int)bi;
  const int p = (a.pos ? a.pos[bi] : 0) + j;
  const int slot = p >> 6;
  if (sid < 0 || sid >= a.n_seqs || p < 0 || slot >= a.table_stride) return -1;
  const int page = a.page_table[(int64_t)sid * a.table_stride + slot];
  if (page < 0 || page >= a.n_pages) return -1;
  return ((int64_t)page * a.nh + head) * FG_PAGE_ROWS + (p & (FG_PAGE_ROWS - 1));
}

// Grid (wave units / 4, 8-group chunks of a token row, {K, V}).  A wave unit is 8 consecutive
// positions of one sequence; the wave takes 8 consecutive groups of each of those token rows (512
// contiguous bytes per row), two rows per pass with both loads issued before either is used, and what
// it writes for a head (64 bytes of codes per position at head size 128) is contiguous over the unit.
// Which sequence and positions a wave covers is one scalar division per wave: the per-item index
// arithmetic has no division (64-bit divisions per item made the first version VALU-bound).
constexpr int kKvPosPerWave = 8;
template <bool H16>
__global__ __launch_bounds__(256) void kv_append_q4_kernel(KvAppendArgs a) {
  const int which = blockIdx.z;
  const half_t* __restrict__ x = a.src[which];
  uint32_t* __restrict__ codes = reinterpret_cast<uint32_t*>(a.codes[which]);
  void* __restrict__ meta = a.meta[which];
  const int gph = a.dh / kGroup;              // groups per head: 1 or 2
  const int gpr = a.nh * gph;                 // groups per token row
  const int sub = threadIdx.x & 7, lg = (threadIdx.x & 63) >> 3;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t units_per_seq = (uint32_t)(a.s + kKvPosPerWave - 1) / kKvPosPerWave;
  const uint32_t unit = blockIdx.x * 4u + (uint32_t)wave;
  const uint32_t bi = unit / units_per_seq;
  if (bi >= (uint32_t)a.b) return;
  const int pos_base = (int)(unit - bi * units_per_seq) * kKvPosPerWave;
  const int gi = blockIdx.y * 8 + lg;
  if (gi >= gpr) return;                      // whole groups of 8 lanes drop out together (partial last chunk)
  const int head = gph == 2 ? gi >> 1 : gi, gh = gph == 2 ? gi & 1 : 0;
  const half_t* src = x + (int64_t)bi * a.s * a.ld + (int64_t)gi * kGroup + sub * 8;
  auto finish = [&](int pos, const h8_t v) {
    uint32_t p;
    float mn, sc;
    quantize_group_8lanes<H16>(v, sub, p, mn, sc);   // all eight lanes of a group take part
    const int64_t crow = kv_dest_row(a, bi, head, pos);
    if (crow < 0) return;
    codes[(crow * gph + gh) * 8 + sub] = p;
    if (sub == 0) {
      if (H16)
        reinterpret_cast<h2_t*>(meta)[crow * gph + gh] = (h2_t){(half_t)mn, (half_t)sc};
      else
        reinterpret_cast<float2*>(meta)[crow * gph + gh] = make_float2(mn, sc);
    }
  };
#pragma unroll
  for (int k = 0; k < kKvPosPerWave; k += 2) {
    const int p0 = pos_base + k, p1 = p0 + 1;   // wave-uniform
    if (p0 >= a.s) break;
    const bool two = p1 < a.s;
    const h8_t v0 = *reinterpret_cast<const h8_t*>(src + (int64_t)p0 * a.ld);
    const h8_t v1 = *reinterpret_cast<const h8_t*>(src + (int64_t)(two ? p1 : p0) * a.ld);
    finish(p0, v0);
    if (two) finish(p1, v1);
  }
}

__global__ __launch_bounds__(256) void kv_append_f16_kernel(KvAppendArgs a) {
  const int which = blockIdx.y;
  const half_t* __restrict__ x = a.src[which];
  half_t* __restrict__ dst = reinterpret_cast<half_t*>(a.codes[which]);
  const int cpr = a.nh * a.dh / 8;            // 16-byte chunks per token row
  const int cph = a.dh / 8;
  const int64_t n_chunks = (int64_t)a.b * a.s * cpr;
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; c < n_chunks; c += stride) {
    const int64_t row = c / cpr;
    const int ci = (int)(c - row * cpr);
    const int head = ci / cph, ch = ci - head * cph;
    const int64_t bi = row / a.s;
    const u4_t v = *reinterpret_cast<const u4_t*>(x + row * a.ld + (int64_t)ci * 8);
    const int64_t crow = kv_dest_row(a, bi, head, (int)(row - bi * a.s));
    if (crow >= 0) *reinterpret_cast<u4_t*>(dst + crow * a.dh + ch * 8) = v;
  }
}

static int grid_for(int64_t work_items, int per_block) {
  int64_t blocks = ceil_div(work_items, per_block);
  const int64_t cap = 256 * 64;  // enough to fill the chip many times over; loops cover the rest
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

int kv_append_launch(const fg_model_cfg& cfg, const half_t* k, const half_t* v, int64_t row_stride,
                     int32_t b, int32_t s, const fg_kv_cache& kv, int32_t batch_offset, int32_t pos0,
                     hipStream_t stream) {
  if (b == 0 || s == 0) return FG_OK;
  KvAppendArgs a;
  a.src[0] = k;
  a.src[1] = v;
  a.codes[0] = kv.k_codes;
  a.codes[1] = kv.v_codes;
  a.meta[0] = kv.k_meta;
  a.meta[1] = kv.v_meta;
  a.ld = row_stride;
  a.b = b;
  a.s = s;
  a.nh = cfg.nh;
  a.dh = cfg.h1 / cfg.nh;
  a.cap = kv.cap;
  a.batch_offset = batch_offset;
  a.pos0 = pos0;
  a.page_table = nullptr;
  a.seq_ids = nullptr;
  a.pos = nullptr;
  a.table_stride = a.n_seqs = a.n_pages = 0;
  ProfScope prof(FG_K_KV_APPEND, stream);
  if (kv.dtype == FG_Q4G64 || kv.dtype == FG_Q4G64_H16) {
    const int gpr = cfg.h1 / kGroup;
    dim3 grid((unsigned)ceil_div(b * ceil_div(s, kKvPosPerWave), 4), (unsigned)ceil_div(gpr, 8), 2);
    if (kv.dtype == FG_Q4G64_H16)
      hipLaunchKernelGGL(kv_append_q4_kernel<true>, grid, dim3(256), 0, stream, a);
    else
      hipLaunchKernelGGL(kv_append_q4_kernel<false>, grid, dim3(256), 0, stream, a);
  } else {
    const int64_t chunks = (int64_t)b * s * cfg.h1 / 8;
    dim3 grid(grid_for(chunks, 256), 2);
    hipLaunchKernelGGL(kv_append_f16_kernel, grid, dim3(256), 0, stream, a);
  }
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int kv_append_paged_launch(const fg_model_cfg& cfg, const half_t* k, const half_t* v, int64_t row_stride,
                           int32_t b, int32_t s, const fg_kv_pages& pages, const fg_ragged& seqs, bool use_pos,
                           hipStream_t stream) {
  if (b == 0 || s == 0) return FG_OK;
  KvAppendArgs a;
  a.src[0] = k;
  a.src[1] = v;
  a.codes[0] = pages.k_codes;
  a.codes[1] = pages.v_codes;
  a.meta[0] = pages.k_meta;
  a.meta[1] = pages.v_meta;
  a.ld = row_stride;
  a.b = b;
  a.s = s;
  a.nh = cfg.nh;
  a.dh = cfg.h1 / cfg.nh;
  a.cap = 0;
  a.batch_offset = 0;
  a.pos0 = 0;
  a.page_table = seqs.page_table;
  a.seq_ids = seqs.seq_ids;
  a.pos = use_pos ? seqs.pos : nullptr;
  a.table_stride = seqs.table_stride;
  a.n_seqs = seqs.n_seqs;
  a.n_pages = pages.n_pages;
  ProfScope prof(FG_K_KV_APPEND, stream);
  if (pages.dtype == FG_F16) {
    const int64_t chunks = (int64_t)b * s * cfg.h1 / 8;
    dim3 grid(grid_for(chunks, 256), 2);
    hipLaunchKernelGGL(kv_append_f16_kernel, grid, dim3(256), 0, stream, a);
    FG_LAUNCH_CHECK();
    return FG_OK;
  }
  const int gpr = cfg.h1 / kGroup;
  dim3 grid((unsigned)ceil_div(b * ceil_div(s, kKvPosPerWave), 4), (unsigned)ceil_div(gpr, 8), 2);
  if (pages.dtype == FG_Q4G64_H16)
    hipLaunchKernelGGL(kv_append_q4_kernel<true>, grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL(kv_append_q4_kernel<false>, grid, dim3(256), 0, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg

using namespace fg;

static int quantize_entry(bool h16, const void* x_f16, int64_t rows, int64_t cols, int group, int bits,
                          void* codes_out, void* meta_out, void* stream) {
  if (group != kGroup || bits != 4) return FG_ERR_UNSUPPORTED;
  if (rows < 0 || cols <= 0 || cols % kGroup != 0) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!x_f16 || !codes_out || !meta_out) return FG_ERR_NULL;
  const int64_t groups = rows * (cols / kGroup);
  hipStream_t st = as_stream(stream);
  ProfScope prof(FG_K_QUANTIZE, st);
  if (h16)
    hipLaunchKernelGGL(quantize_rows_kernel<true>, dim3(grid_for(groups, 32)), dim3(256), 0, st,
                       reinterpret_cast<const half_t*>(x_f16), groups, reinterpret_cast<uint32_t*>(codes_out), meta_out);
  else
    hipLaunchKernelGGL(quantize_rows_kernel<false>, dim3(grid_for(groups, 32)), dim3(256), 0, st,
                       reinterpret_cast<const half_t*>(x_f16), groups, reinterpret_cast<uint32_t*>(codes_out), meta_out);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

extern "C" int fg_quantize_groupwise(const void* x_f16, int64_t rows, int64_t cols, int group, int bits,
                                     void* codes_out, void* meta_out, void* stream) {
  return quantize_entry(false, x_f16, rows, cols, group, bits, codes_out, meta_out, stream);
}

extern "C" int fg_quantize_groupwise_h16(const void* x_f16, int64_t rows, int64_t cols, int group, int bits,
                                         void* codes_out, void* meta_out_f16, void* stream) {
  return quantize_entry(true, x_f16, rows, cols, group, bits, codes_out, meta_out_f16, stream);
}

static int dequantize_entry(bool h16, const void* codes, const void* meta, int64_t rows, int64_t cols, void* out_f32,
                            void* stream) {
  if (rows < 0 || cols <= 0 || cols % kGroup != 0) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!codes || !meta || !out_f32) return FG_ERR_NULL;
  const int64_t words = rows * cols / 8;
  hipStream_t st = as_stream(stream);
  ProfScope prof(FG_K_DEQUANTIZE, st);
  if (h16)
    hipLaunchKernelGGL(dequantize_rows_kernel<true>, dim3(grid_for(words, 256)), dim3(256), 0, st,
                       reinterpret_cast<const uint32_t*>(codes), meta, words, reinterpret_cast<float*>(out_f32));
  else
    hipLaunchKernelGGL(dequantize_rows_kernel<false>, dim3(grid_for(words, 256)), dim3(256), 0, st,
                       reinterpret_cast<const uint32_t*>(codes), meta, words, reinterpret_cast<float*>(out_f32));
  FG_LAUNCH_CHECK();
  return FG_OK;
}

extern "C" int fg_dequantize_groupwise(const void* codes, const void* meta, int64_t rows, int64_t cols,
                                       void* out_f32, void* stream) {
  return dequantize_entry(false, codes, meta, rows, cols, out_f32, stream);
}

extern "C" int fg_dequantize_groupwise_h16(const void* codes, const void* meta_f16, int64_t rows, int64_t cols,
                                           void* out_f32, void* stream) {
  return dequantize_entry(true, codes, meta_f16, rows, cols, out_f32, stream);
}

extern "C" int fg_kv_append(const fg_model_cfg* cfg, const void* k_f16, const void* v_f16,
                            int64_t row_stride, int32_t b, int32_t s, const fg_kv_cache* kv,
                            int32_t batch_offset, int32_t pos0, void* stream) {
  if (!cfg || !kv) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_kv(cfg, kv);
  if (rc) return rc;
  if (b < 0 || s < 0 || batch_offset < 0 || pos0 < 0) return FG_ERR_SHAPE;
  if ((int64_t)batch_offset + b > kv->batch || (int64_t)pos0 + s > kv->cap) return FG_ERR_SHAPE;
  if (row_stride < cfg->h1 || row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0 || s == 0) return FG_OK;
  if (!k_f16 || !v_f16) return FG_ERR_NULL;
  if (((uintptr_t)k_f16 | (uintptr_t)v_f16) & 15u) return FG_ERR_SHAPE;   // the kernels load 16 bytes per lane
  return kv_append_launch(*cfg, reinterpret_cast<const half_t*>(k_f16), reinterpret_cast<const half_t*>(v_f16),
                          row_stride, b, s, *kv, batch_offset, pos0, as_stream(stream));
}

extern "C" int fg_kv_append_paged(const fg_model_cfg* cfg, const void* k_f16, const void* v_f16, int64_t row_stride,
                                  int32_t b, int32_t s, const fg_kv_pages* pages, const fg_ragged* seqs,
                                  void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_pages(cfg, pages, seqs);
  if (rc) return rc;
  if (b < 0 || s < 0) return FG_ERR_SHAPE;
  if (row_stride < cfg->h1 || row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0 || s == 0) return FG_OK;
  if (!k_f16 || !v_f16) return FG_ERR_NULL;
  if (((uintptr_t)k_f16 | (uintptr_t)v_f16) & 15u) return FG_ERR_SHAPE;
  return kv_append_paged_launch(*cfg, reinterpret_cast<const half_t*>(k_f16), reinterpret_cast<const half_t*>(v_f16),
                                row_stride, b, s, *pages, *seqs, true, as_stream(stream));
}
