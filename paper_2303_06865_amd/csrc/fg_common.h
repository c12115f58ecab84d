// Internal helpers shared by the HIP sources of libfg (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fg.h"

namespace fg {

typedef _Float16 half_t;
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));
typedef float f16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2_t __attribute__((ext_vector_type(2)));

constexpr int kGroup = 64;           // elements per quantization group (Section 5)
constexpr int kWave = 64;            // CDNA wavefront width

// ---- error plumbing ---------------------------------------------------------------------
void set_device_error(hipError_t e, const char* what);

#define FG_HIP(expr)                                   \
  do {                                                 \
    hipError_t _e = (expr);                            \
    if (_e != hipSuccess) {                            \
      ::fg::set_device_error(_e, #expr);               \
      return FG_ERR_DEVICE;                            \
    }                                                  \
  } while (0)

// Call after a kernel launch: picks up launch-configuration errors.
#define FG_LAUNCH_CHECK() FG_HIP(hipGetLastError())

// ---- per-kernel-class event timing --------------------------------------------------------
bool profile_enabled();
void profile_mark(int kclass, hipStream_t stream, bool begin);

struct ProfScope {
  int k;
  hipStream_t s;
  bool on;
  ProfScope(int kclass, hipStream_t stream) : k(kclass), s(stream), on(profile_enabled()) {
    if (on) profile_mark(k, s, true);
  }
  ~ProfScope() {
    if (on) profile_mark(k, s, false);
  }
};

static inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- entry points of the individual kernel files (host side, already validated) ----------
struct LinearArgs {
  const void* w_data;      // codes or FP16
  const void* w_meta;      // {min,scale} pairs or NULL
  int dtype;
  int64_t n, k;            // W is [n, k]
  const half_t* x;         // [m, k], row stride ldx
  int64_t ldx;
  int64_t m;
  const half_t* bias;      // [n] or NULL
  const half_t* residual;  // [m, n] row stride ldr, or NULL
  int64_t ldr;
  int relu;
  half_t* out_f16;         // [m, n] row stride ldo (NULL when out_f32 is used)
  float* out_f32;          // [m, n] row stride ldo, no FP16 rounding (LM head logits)
  int64_t ldo;
};
size_t linear_workspace_bytes(int dtype, int64_t n, int64_t k, int64_t m);
int linear_launch(const LinearArgs& a, void* ws, size_t ws_bytes, hipStream_t stream);

// small-M (decode) and large-M (prefill) kernels behind linear_launch
size_t gemm_small_m_workspace(int dtype, int64_t n, int64_t k, int64_t m);
int gemm_small_m_launch(const LinearArgs& a, void* ws, size_t ws_bytes, hipStream_t stream);
int gemm_large_m_launch(const LinearArgs& a, hipStream_t stream);
// tiled 4-bit weights: weight-streaming kernel for few rows, and the repacking kernel
// row-major FP16 weights, up to 128 rows (csrc/fg_gemm_f16w.hip); pick_cols returns 0 for shapes it does not take
int gemm_f16w_pick_cols(int64_t n, int64_t k, int64_t m);
size_t gemm_f16w_workspace(int64_t n, int64_t k, int64_t m);
int gemm_f16w_launch(const LinearArgs& a, void* ws, size_t ws_bytes, hipStream_t stream);
size_t gemm_stream_workspace(int64_t n, int64_t k, int64_t m);
int gemm_stream_launch(const LinearArgs& a, void* ws, size_t ws_bytes, hipStream_t stream);
int pack_weights_launch(const void* codes, const void* meta, bool meta_f16, int64_t n, int64_t k, void* codes_out, void* meta_out,
                        hipStream_t stream);

int layernorm_launch(const half_t* x, int64_t ldx, const half_t* g, const half_t* b, int64_t rows,
                     int64_t cols, float eps, half_t* out, int64_t ldo, hipStream_t stream);
int embed_launch(const half_t* emb, const half_t* pos, const int32_t* ids, int64_t ids_stride, int64_t rows,
                 int32_t s_len, int32_t pos0, int32_t h1, int32_t vocab, half_t* out, hipStream_t stream);
int embed_ragged_launch(const half_t* emb, const half_t* pos, const int32_t* ids, const int32_t* id_index,
                        const int32_t* positions, int64_t rows, int32_t h1, int32_t vocab, int32_t max_pos,
                        half_t* out, hipStream_t stream);
int argmax_launch(const float* logits, int64_t rows, int64_t cols, int32_t* out, int64_t out_stride,
                  hipStream_t stream, const int32_t* out_index = nullptr);

int kv_append_launch(const fg_model_cfg& cfg, const half_t* k, const half_t* v, int64_t row_stride,
                     int32_t b, int32_t s, const fg_kv_cache& kv, int32_t batch_offset, int32_t pos0,
                     hipStream_t stream);
int decode_attention_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                            int32_t rows, const fg_kv_cache& kv, int32_t batch_offset, half_t* out,
                            hipStream_t stream);
int prefill_attention_launch(const fg_model_cfg& cfg, const half_t* qkv, int32_t b, int32_t s,
                             half_t* out, hipStream_t stream);
// paged cache (sequences at different steps): s rows per sequence from position pos[i] (nullptr: 0);
// attention over pos[i] + rows_bias rows
int kv_append_paged_launch(const fg_model_cfg& cfg, const half_t* k, const half_t* v, int64_t row_stride,
                           int32_t b, int32_t s, const fg_kv_pages& pages, const fg_ragged& seqs, bool use_pos,
                           hipStream_t stream);
int decode_attention_paged_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                                  const fg_kv_pages& pages, const fg_ragged& seqs, int32_t rows_bias, half_t* out,
                                  hipStream_t stream);
int check_pages(const fg_model_cfg* cfg, const fg_kv_pages* pages, const fg_ragged* seqs);
// Top-K sparse decode attention (4-bit caches): contiguous cache, and paged cache with a length per row
int decode_attention_topk_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b, int32_t rows,
                                 int32_t topk, const fg_kv_cache& kv, int32_t batch_offset, half_t* out,
                                 int32_t* sel_out, hipStream_t stream);
int decode_attention_topk_paged_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                                       int32_t topk, const fg_kv_pages& pages, const fg_ragged& seqs,
                                       int32_t rows_bias, half_t* out, int32_t* sel_out, hipStream_t stream);

// validation helpers (host only)
int check_cfg(const fg_model_cfg* cfg);
int check_mat(const fg_mat* w, bool for_pack = false);
int check_kv(const fg_model_cfg* cfg, const fg_kv_cache* kv);

// ---- device helpers -------------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Unpack one 32-bit word of eight 4-bit codes c0..c7 (c0 in the lowest nibble) into four FP16
// pairs WITHOUT leaving the register file.  The pairs come out in the order
//   p[0] = (c0, c4) + 1024,  p[1] = (c1, c5) + 64,  p[2] = (c2, c6) + 1024,  p[3] = (c3, c7) + 64
// because OR-ing a nibble into the mantissa of 1024.0 (0x6400, ulp 1) or, four bits higher, of
// 64.0 (0x5400, ulp 1/16) yields those integers exactly.
__device__ __forceinline__ void unpack8_biased(uint32_t x, uint32_t p[4]) {
  const uint32_t y = x >> 8;
  p[0] = (x & 0x000F000Fu) | 0x64006400u;
  p[1] = (x & 0x00F000F0u) | 0x54005400u;
  p[2] = (y & 0x000F000Fu) | 0x64006400u;
  p[3] = (y & 0x00F000F0u) | 0x54005400u;
}

// Same word -> eight FP16 codes (exact small integers), pair order (c0,c4),(c1,c5),(c2,c6),(c3,c7).
__device__ __forceinline__ void unpack8_codes(uint32_t x, h2_t p[4]) {
  uint32_t r[4];
  unpack8_biased(x, r);
  const h2_t k1024 = {(half_t)1024.0f, (half_t)1024.0f};
  const h2_t k64 = {(half_t)64.0f, (half_t)64.0f};
  p[0] = __builtin_bit_cast(h2_t, r[0]) - k1024;
  p[1] = __builtin_bit_cast(h2_t, r[1]) - k64;
  p[2] = __builtin_bit_cast(h2_t, r[2]) - k1024;
  p[3] = __builtin_bit_cast(h2_t, r[3]) - k64;
}

// Exact dequantization of one word of eight codes to FP16: w_i = RN16(mn + c_i * scale), one rounding
// from the real number (Section 5: "converted back to FP16 before computation").
// A nibble masked in place is the FP16 subnormal c * 2^-24 (low nibble of a half) or c * 2^-20 (next
// nibble); gfx950 mixed-precision FMAs take FP16 subnormals at full rate, multiply by the pre-scaled
// s24 = scale * 2^24 / s20 = scale * 2^20 (exact scalings), add mn and round once into an FP16 half
// of the destination (v_fma_mixlo_f16 / v_fma_mixhi_f16).  Thirteen VALU instructions per eight
// weights.  Output in natural order: p[0] = (w0,w1), p[1] = (w2,w3), p[2] = (w4,w5), p[3] = (w6,w7).
__device__ __forceinline__ void dequant8_exact(uint32_t x, float s24, float s20, float mn, uint32_t p[4]) {
  const uint32_t y = x >> 8;
  const uint32_t a = x & 0x000F000Fu;   // halves: c0 * 2^-24 , c4 * 2^-24
  const uint32_t b = x & 0x00F000F0u;   //         c1 * 2^-20 , c5 * 2^-20
  const uint32_t c = y & 0x000F000Fu;   //         c2 * 2^-24 , c6 * 2^-24
  const uint32_t d = y & 0x00F000F0u;   //         c3 * 2^-20 , c7 * 2^-20
  const h2_t ha = __builtin_bit_cast(h2_t, a), hb = __builtin_bit_cast(h2_t, b);
  const h2_t hc = __builtin_bit_cast(h2_t, c), hd = __builtin_bit_cast(h2_t, d);
  const h2_t q0 = {(half_t)__builtin_fmaf((float)ha.x, s24, mn), (half_t)__builtin_fmaf((float)hb.x, s20, mn)};
  const h2_t q1 = {(half_t)__builtin_fmaf((float)hc.x, s24, mn), (half_t)__builtin_fmaf((float)hd.x, s20, mn)};
  const h2_t q2 = {(half_t)__builtin_fmaf((float)ha.y, s24, mn), (half_t)__builtin_fmaf((float)hb.y, s20, mn)};
  const h2_t q3 = {(half_t)__builtin_fmaf((float)hc.y, s24, mn), (half_t)__builtin_fmaf((float)hd.y, s20, mn)};
  const uint32_t r0 = __builtin_bit_cast(uint32_t, q0), r1 = __builtin_bit_cast(uint32_t, q1);
  const uint32_t r2 = __builtin_bit_cast(uint32_t, q2), r3 = __builtin_bit_cast(uint32_t, q3);
  p[0] = r0;
  p[1] = r1;
  p[2] = r2;
  p[3] = r3;
}

// Reorder eight consecutive FP16 values h0..h7 (four words) into the pair order produced by
// unpack8_*: (h0,h4),(h1,h5),(h2,h6),(h3,h7), so that a contraction against unpacked codes lines up.
__device__ __forceinline__ u4_t permute8_like_codes(u4_t d) {
  u4_t o;
  o.x = __builtin_amdgcn_perm(d.z, d.x, 0x05040100u);  // (h0, h4)
  o.y = __builtin_amdgcn_perm(d.z, d.x, 0x07060302u);  // (h1, h5)
  o.z = __builtin_amdgcn_perm(d.w, d.y, 0x05040100u);  // (h2, h6)
  o.w = __builtin_amdgcn_perm(d.w, d.y, 0x07060302u);  // (h3, h7)
  return o;
}

#endif  // __HIPCC__

}  // namespace fg
