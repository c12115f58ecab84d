// Prefill-phase attention (Section 3, prefill: softmax(xQ.xK^T/sqrt(h)).xV, causal) over the fresh
// FP16 q, k, v of one GPU batch, before k and v are stored into the compressed cache.
//
// One workgroup per (sequence, head, 64 queries); each of its four waves owns 16 queries.  Keys are
// walked in tiles of 64 staged in LDS (K as is, V transposed); the next tile's rows are fetched into
// registers while the current tile is in use.  Both contractions run on
// v_mfma_f32_16x16x32_f16 in the transposed form
//     S^T[key][query] = K . Q^T          O^T[d][query] = V^T . P^T
// so that every per-query quantity (running max, sum, rescale factor) lives in the lane that owns
// the query column, and the S^T accumulator registers are, after exponentiation and packing to
// FP16, already the B operand of the second product: P never leaves the register file.
#include "fg_common.h"

namespace fg {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kKT = 64;   // keys per tile

struct PrefillAttnArgs {
  const half_t* qkv;   // [b*s, 3*h1]
  half_t* out;         // [b*s, h1]
  int s, nh, h1;
  int n_pairs;         // b * nh
  float scale;
};

template <int DH>
__global__ __launch_bounds__(256) void attn_prefill_kernel(PrefillAttnArgs a) {
  constexpr int NU = DH / 32;     // K-dimension steps of the first product
  constexpr int ND = DH / 16;     // output tiles of the second product
  constexpr int NB = kKT / 16;    // 16-key blocks per tile
  constexpr int LDK = DH + 8;     // LDS pitch of K rows (halves)
  constexpr int LDV = kKT + 8;    // LDS pitch of V^T rows (halves)
  constexpr int NP = kKT * (DH / 8) / 256;   // 16-byte pieces of K (and of V) per thread per tile
  __shared__ __attribute__((aligned(16))) half_t Ks[kKT * LDK];
  __shared__ __attribute__((aligned(16))) half_t Vt[DH * LDV];

  // Workgroups go to the 8 XCDs round-robin by their index.  All query tiles of one (sequence, head)
  // read the same K and V rows, so they are numbered to land on the same XCD (and its L2), one after
  // the other, the longest (last) tile first.
  const int nq = (a.s + 63) >> 6;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int hs = (slot / nq) * 8 + xcd;          // (sequence, head) pair
  if (hs >= a.n_pairs) return;
  const int qt = nq - 1 - slot % nq;
  const int seq = hs / a.nh, head = hs - seq * a.nh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, ib = lane >> 4;
  const int64_t ld = 3 * (int64_t)a.h1;
  const half_t* base = a.qkv + (int64_t)seq * a.s * ld + head * DH;
  const int q0 = qt * 64;
  const int my_q = q0 + wave * 16 + n;                 // the query this lane's column belongs to
  const int my_qc = my_q < a.s ? my_q : a.s - 1;

  // B operand of the first product: this query's row, 8 head dims per K block
  h8_t qreg[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u)
    qreg[u] = *reinterpret_cast<const h8_t*>(base + (int64_t)my_qc * ld + 32 * u + 8 * ib);

  f4_t o[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d) o[d] = (f4_t){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  const int last_q = (q0 + 63) < (a.s - 1) ? (q0 + 63) : (a.s - 1);
  const int n_tiles = last_q / kKT + 1;

  // the next tile's K and V rows travel through registers while the current tile is being used
  u4_t kreg[NP];
  h8_t vreg[NP];
  // consecutive lanes take consecutive 16-byte pieces of one row: DH/8 lanes cover a K (or V) row;
  // piece i of this thread is key (tid + 256 i) / (DH/8) of the tile
  constexpr int kKeysPerPass = 256 / (DH / 8);
  const int key0 = tid / (DH / 8), dc0 = tid % (DH / 8);
  const half_t* kv_col = base + a.h1 + dc0 * 8;
  auto fetch = [&](int kt) {
    const int k0 = kt * kKT + key0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      int kg = k0 + kKeysPerPass * i;
      kg = kg < a.s ? kg : a.s - 1;
      const half_t* row = kv_col + (int64_t)kg * ld;
      kreg[i] = *reinterpret_cast<const u4_t*>(row);
      vreg[i] = *reinterpret_cast<const h8_t*>(row + a.h1);
    }
  };
  // K [kKT][DH] as is; V transposed to [DH][kKT] with the keys of row d rotated by 4 * (d / 8)
  // positions, so that the DH/8 lanes that hold one key write to different banks
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int key = key0 + kKeysPerPass * i, dc = dc0;
      *reinterpret_cast<u4_t*>(Ks + key * LDK + dc * 8) = kreg[i];
      const int col = (key + 4 * dc) & (kKT - 1);
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(dc * 8 + e) * LDV + col] = vreg[i][e];
    }
  };

  fetch(0);
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * kKT;
    __syncthreads();   // previous tile fully consumed
    stage();
    __syncthreads();
    if (kt + 1 < n_tiles) fetch(kt + 1);   // in flight during this tile's MFMAs

    // ---- S^T blocks: block j = keys k0 + 16 j .. + 15
    f4_t t[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) t[j] = (f4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < NU; ++u) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const h8_t ka = *reinterpret_cast<const h8_t*>(Ks + (16 * j + n) * LDK + 32 * u + 8 * ib);
        t[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qreg[u], t[j], 0, 0, 0);
      }
    }
    // lane holds, for query my_q, keys k0 + 16 j + 4 ib + r
    float sc[4 * NB];
    float cmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int key = k0 + 16 * j + 4 * ib + r;
        sc[4 * j + r] = key <= my_q ? t[j][r] * a.scale : -INFINITY;
        cmax = fmaxf(cmax, sc[4 * j + r]);
      }
    cmax = fmaxf(cmax, __shfl_xor(cmax, 16, 64));
    cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
    const float m_new = fmaxf(m_run, cmax);
    // a query can see no key of this tile only in tiles past its own position; then m_new may
    // still be -inf for rows beyond s (clamped duplicates) - guard the exponent
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * kLog2e);
    m_run = m_new;
    float psum = 0.f;
    h8_t pop[NB / 2];   // B operands of the second product: 32 keys each = blocks 2h, 2h+1
#pragma unroll
    for (int e = 0; e < 4 * NB; ++e) {
      const float p = __builtin_amdgcn_exp2f((sc[e] - m_use) * kLog2e);
      psum += p;
      pop[e / 8][e % 8] = (half_t)p;
    }
    l_run = l_run * alpha + psum;
    // the running maximum rarely moves after the first tiles: skip the rescale when no lane needs it
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int d = 0; d < ND; ++d) {
#pragma unroll
        for (int r = 0; r < 4; ++r) o[d][r] *= alpha;
      }
    }
    // ---- O^T += V^T . P^T ; A operand: V^T rows d, K slots of half h = keys 32 h + {4 ib .. +3, 16 + 4 ib .. +3}
#pragma unroll
    for (int h = 0; h < NB / 2; ++h) {
#pragma unroll
      for (int d = 0; d < ND; ++d) {
        const int row = d * 16 + n, rot = 4 * (row >> 3);
        const half_t* vr = Vt + row * LDV;
        const h4_t lo = *reinterpret_cast<const h4_t*>(vr + ((32 * h + 4 * ib + rot) & (kKT - 1)));
        const h4_t hi = *reinterpret_cast<const h4_t*>(vr + ((32 * h + 16 + 4 * ib + rot) & (kKT - 1)));
        const h8_t va = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        o[d] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pop[h], o[d], 0, 0, 0);
      }
    }
  }

  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (my_q < a.s) {
    const float inv = 1.0f / l_run;
    half_t* orow = a.out + ((int64_t)seq * a.s + my_q) * a.h1 + head * DH;
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      h4_t v;
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = (half_t)(o[d][r] * inv);
      *reinterpret_cast<h4_t*>(orow + d * 16 + 4 * ib) = v;
    }
  }
}

}  // namespace

int prefill_attention_launch(const fg_model_cfg& cfg, const half_t* qkv, int32_t b, int32_t s, half_t* out,
                             hipStream_t stream) {
  if (b == 0 || s == 0) return FG_OK;
  const int dh = cfg.h1 / cfg.nh;
  PrefillAttnArgs a;
  a.qkv = qkv;
  a.out = out;
  a.s = s;
  a.nh = cfg.nh;
  a.h1 = cfg.h1;
  a.scale = 1.0f / sqrtf((float)dh);
  a.n_pairs = b * cfg.nh;
  const dim3 grid((unsigned)(ceil_div(a.n_pairs, 8) * 8 * ceil_div(s, 64)));
  ProfScope prof(FG_K_ATTN_PREFILL, stream);
  if (dh == 128)
    hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, dim3(256), 0, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg

using namespace fg;

extern "C" int fg_prefill_attention(const fg_model_cfg* cfg, const void* qkv_f16, int32_t b, int32_t s,
                                    void* out_f16, void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (b < 0 || s < 0 || b > 65535) return FG_ERR_SHAPE;
  if (b == 0 || s == 0) return FG_OK;
  if (!qkv_f16 || !out_f16) return FG_ERR_NULL;
  return prefill_attention_launch(*cfg, reinterpret_cast<const half_t*>(qkv_f16), b, s,
                                  reinterpret_cast<half_t*>(out_f16), as_stream(stream));
}
