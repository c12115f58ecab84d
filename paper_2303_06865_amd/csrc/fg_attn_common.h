// Pieces shared by the decode-attention kernels over the 4-bit cache (dense and Top-K): the query
// set-up and the scores of one 128-group chunk of the K stream on the matrix cores.
//
//   q.k_hat = sum_g scale_g * (q_g . c_g) + min_g * sum(q_g)     (Sections 3 and 5)
// The code dot products run on v_mfma_f32_16x16x32_f16: the K codes, expanded to FP16 in registers
// with a bias (nibble OR-ed into the mantissa of 1024 or 64), are the B operand (lane = row, 8
// consecutive codes per lane); the A operand holds the query, masked so that output rows 4j and 4j+1
// separate the two groups a lane pair covers.  Each of the four 32-group loads of a chunk is four MFMAs
// into a fresh accumulator; lane group j keeps load j's result, which leaves, in lane L, the two group
// sums of groups 2L and 2L+1 of the chunk; the bias is removed with a per-head constant.
#pragma once
#include "fg_common.h"

namespace fg {

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// a value that is the same in every lane, moved to a scalar register
__device__ __forceinline__ float uniform(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}

// {min, scale} of one group as stored: two binary32 (FG_Q4G64) or two FP16 (FG_Q4G64_H16).  Kept raw
// in the prefetch buffers and converted only when the chunk is processed, so that a conversion
// never waits for a load that has just been issued.
template <bool H16>
struct MetaRaw {
  using type = float2;
};
template <>
struct MetaRaw<true> {
  using type = h2_t;
};
__device__ __forceinline__ float2 meta_f32(float2 m) { return m; }
__device__ __forceinline__ float2 meta_f32(h2_t m) { return make_float2((float)m.x, (float)m.y); }

template <int DH>
struct QueryOps {
  float Qs[2], Os[2];   // per-group sums of q and of bias * q
  h8_t qop[4];          // masked A operands, one per 8-code step of a lane's 32 codes
};

// my_q: the head's query in LDS (DH halves, 16-byte aligned).  Lane roles: r = lane & 15,
// h = lane >> 5, half = (lane >> 4) & 1.
template <int DH>
__device__ __forceinline__ void query_setup(const half_t* my_q, int lane, QueryOps<DH>& Q) {
  const int q4 = lane >> 4, h = q4 >> 1, half = q4 & 1;
  // Qs = sum q_d, Os = sum off_d q_d with off = 1024 (even d) / 64 (odd d), the biases the register
  // unpacking leaves on the codes
  const float qa_ = (float)my_q[lane];
  const float qb_ = DH == 128 ? (float)my_q[(lane + 64) % DH] : qa_;
  const float off = (lane & 1) ? 64.f : 1024.f;
  // (the sums are the same in every lane: kept in scalar registers)
  Q.Qs[0] = uniform(wave_sum(qa_));
  Q.Os[0] = uniform(wave_sum(qa_ * off));
  Q.Qs[1] = uniform(wave_sum(qb_));
  Q.Os[1] = uniform(wave_sum(qb_ * off));
  // qop[u] is non-zero only in lanes whose output row (lane & 15) is 4 j + h for some j: rows 4 j take
  // the k positions that belong to the first group of a lane pair, rows 4 j + 1 those of the second
  const int m = lane & 15;
  const bool valid = (m & 3) == h;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int d0 = (DH == 128 ? 64 * h : 0) + 32 * half + 8 * u;
    const u4_t raw = *reinterpret_cast<const u4_t*>(my_q + d0);
    const u4_t pm = permute8_like_codes(raw);
    const u4_t z = {0u, 0u, 0u, 0u};
    Q.qop[u] = __builtin_bit_cast(h8_t, valid ? pm : z);
  }
}

// Scores of the chunk starting at group gbase: kq[i] = the lane's 16 bytes of load i (group
// gbase + 32 i + 2 (lane&15) + h, half (lane>>4)&1), km0/km1 = {min, scale} of groups gbase + 2 lane
// and + 1.  G = groups in the stream.  Head size 128: sc[0] = score of row (gbase/2 + lane);
// head size 64: sc[0], sc[1] = scores of rows gbase + 2 lane and + 1.  Rows past the end get -inf.
template <int DH>
__device__ __forceinline__ void chunk_scores(const u4_t kq[4], float2 km0, float2 km1, const QueryOps<DH>& Q,
                                             float scale, int G, int gbase, int lane, float* sc) {
  constexpr int NS = 2 / (DH / 64);
  const int g0 = gbase + 2 * lane, g1 = g0 + 1;
  // load i of a chunk covers 32 groups; the last chunk of a stream may need only the first few
  // (wave-uniform count, so the skipped work costs nothing)
  const int ni = (G - gbase + 31) >> 5;
  // Rows 4 j and 4 j + 1 of a load's accumulator hold, for every j, the two group sums of the load's
  // column; lane group j = lane >> 4 keeps load j's, so lane L ends up owning groups 2 L and 2 L + 1 of
  // the chunk.  One accumulator is live at a time.
  const int j = lane >> 4;
  float a0 = 0.f, a1 = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i >= ni) break;
    f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      uint32_t pk[4];
      unpack8_biased(kq[i][u], pk);
      const u4_t bw = {pk[0], pk[1], pk[2], pk[3]};
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(Q.qop[u], __builtin_bit_cast(h8_t, bw), acc, 0, 0, 0);
    }
    a0 = j == i ? acc[0] : a0;
    a1 = j == i ? acc[1] : a1;
  }
  const float s0 = km0.y * (a0 - Q.Os[0]) + km0.x * Q.Qs[0];
  const float s1 = km1.y * (a1 - Q.Os[1]) + km1.x * Q.Qs[1];
  if (DH == 128) {
    sc[0] = g0 < G ? (s0 + s1) * scale : -INFINITY;
  } else {
    sc[0] = g0 < G ? s0 * scale : -INFINITY;
    sc[NS - 1] = g1 < G ? s1 * scale : -INFINITY;
  }
}

}  // namespace fg
