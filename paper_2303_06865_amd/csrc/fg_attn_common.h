// Pieces shared by the decode-attention kernels over the 4-bit cache (dense and Top-K): the query
// set-up and the scores of one 128-group chunk of the K stream on the matrix cores.
//
//   q.k_hat = sum_g scale_g * (q_g . c_g) + min_g * sum(q_g)     (Sections 3 and 5)
// The code dot products run on v_mfma_f32_16x16x32_f16: the K codes, expanded to FP16 in registers
// with a bias (nibble OR-ed into the mantissa of 1024 or 64), are the B operand (lane = row, 8
// consecutive codes per lane); the A operand holds the query, masked so that output row 0/1 of
// each lane group separates the two groups a lane pair covers.  Sixteen MFMAs leave, in lane L, the
// two group sums of groups 2L and 2L+1 of the chunk; the bias is removed with a per-head constant.
#pragma once
#include "fg_common.h"

namespace fg {

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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
  h8_t qop[4][4];       // masked A operands
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
  Q.Qs[0] = wave_sum(qa_);
  Q.Os[0] = wave_sum(qa_ * off);
  Q.Qs[1] = wave_sum(qb_);
  Q.Os[1] = wave_sum(qb_ * off);
  // qop[i][u] is non-zero only in lanes whose output row (lane&15) equals 4*i + h, so that load i's
  // sixteen rows land in lane group i of the accumulator
  const int m = lane & 15;
  const bool valid_h = (m & 3) == h;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int d0 = (DH == 128 ? 64 * h : 0) + 32 * half + 8 * u;
    const u4_t raw = *reinterpret_cast<const u4_t*>(my_q + d0);
    const u4_t pm = permute8_like_codes(raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool valid = valid_h && ((m >> 2) == i);
      const u4_t z = {0u, 0u, 0u, 0u};
      Q.qop[i][u] = __builtin_bit_cast(h8_t, valid ? pm : z);
    }
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
  f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i >= ni) break;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      uint32_t pk[4];
      unpack8_biased(kq[i][u], pk);
      const u4_t bw = {pk[0], pk[1], pk[2], pk[3]};
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(Q.qop[i][u], __builtin_bit_cast(h8_t, bw), acc, 0, 0, 0);
    }
  }
  const float s0 = km0.y * (acc[0] - Q.Os[0]) + km0.x * Q.Qs[0];
  const float s1 = km1.y * (acc[1] - Q.Os[1]) + km1.x * Q.Qs[1];
  if (DH == 128) {
    sc[0] = g0 < G ? (s0 + s1) * scale : -INFINITY;
  } else {
    sc[0] = g0 < G ? s0 * scale : -INFINITY;
    sc[NS - 1] = g1 < G ? s1 * scale : -INFINITY;
  }
}

}  // namespace fg
