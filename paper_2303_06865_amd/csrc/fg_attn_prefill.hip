// Prefill-phase attention (Section 3, prefill: softmax(xQ.xK^T/sqrt(h)).xV, causal) over the fresh
// FP16 q, k, v of one GPU batch, before k and v are stored into the compressed cache.
//
// One workgroup per (sequence, head, 128 queries); each of its four waves owns 32 queries.  Keys are
// walked in tiles of 64 staged in LDS (K as is, V transposed); the next tile's rows are fetched into
// registers while the current tile is in use.  Both contractions run on
// v_mfma_f32_32x32x16_f16 in the transposed form
//     S^T[key][query] = K . Q^T          O^T[d][query] = V^T . P^T
// so that every per-query quantity (running max, sum, rescale factor) lives in the lanes that own
// the query column, and the S^T accumulator registers are, after exponentiation and packing to
// FP16, already the B operand of the second product: P never leaves the register file.  (The
// accumulator gives lane (query, h) the keys {4h..4h+3, 8+4h..8+4h+3} of every 16; the A operand of
// the second product reads V^T in that same order, so no shuffle is needed.)  32 queries per wave
// halve the LDS bytes read per MFMA cycle against a 16-query tiling; a wave skips the tiles that lie
// wholly above its queries' diagonal.
#include "fg_common.h"

namespace fg {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kKT = 64;    // keys per tile
constexpr int kQT = 128;   // queries per workgroup

struct PrefillAttnArgs {
  const half_t* qkv;   // [b*s, 3*h1]
  half_t* out;         // [b*s, h1]
  int s, nh, h1;
  int n_pairs;         // b * nh
  float scale;
};

template <int DH>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillAttnArgs a) {
  constexpr int NU = DH / 16;     // K-dimension steps of the first product
  constexpr int NDB = DH / 32;    // 32-row output blocks of the second product
  constexpr int NKB = kKT / 32;   // 32-key blocks per tile
  constexpr int LDK = DH + 8;     // LDS pitch of K rows (halves)
  constexpr int LDV = kKT + 8;    // LDS pitch of V^T rows (halves)
  constexpr int NP = kKT * (DH / 8) / 256;   // 16-byte pieces of K (and of V) per thread per tile
  __shared__ __attribute__((aligned(16))) half_t Ks[kKT * LDK];
  __shared__ __attribute__((aligned(16))) half_t Vt[DH * LDV];

  // Work items = (sequence, head, 128-query tile).  The workgroups are persistent: workgroup g takes
  // items g, g + gridDim.x, ... and fetches the next item's query rows and first key tile while it
  // finishes the current one, so that no load latency is exposed between items.  Workgroups go to the
  // 8 XCDs round-robin by their index (gridDim.x is a multiple of 8); all query tiles of one
  // (sequence, head) read the same K and V rows, so items are numbered to land on the same XCD (and
  // its L2), next to each other.
  const int nq = (a.s + kQT - 1) / kQT;
  const int n_items = ((a.n_pairs + 7) >> 3) * 8 * nq;
  const int pairs_per_round = (int)(gridDim.x >> 3) / nq > 0 ? (int)(gridDim.x >> 3) / nq : 1;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int64_t ld = 3 * (int64_t)a.h1;
  const float c2 = a.scale * kLog2e;
  constexpr int kKeysPerPass = 256 / (DH / 8);
  // consecutive lanes take consecutive 16-byte pieces of one row: DH/8 lanes cover a K (or V) row;
  // piece i of this thread is key (tid + 256 i) / (DH/8) of the tile
  const int key0 = tid / (DH / 8), dc0 = tid % (DH / 8);

  struct Item {
    const half_t* base;   // q row 0 of the (sequence, head)
    int q0, seq, head;
    bool valid;
  };
  auto decode = [&](int item) -> Item {
    Item it;
    const int xcd = item & 7, slot = item >> 3;
    const int pair = slot / nq;
    const int hs = pair * 8 + xcd;          // (sequence, head) pair
    it.valid = item < n_items && hs < a.n_pairs;
    const int hsc = hs < a.n_pairs ? hs : a.n_pairs - 1;
    it.seq = hsc / a.nh;
    it.head = hsc - it.seq * a.nh;
    // Query tiles differ in length (causal), and a workgroup's successive items are a fixed stride
    // apart: rotate the tile index by the round the pair falls in, so that every workgroup sees all
    // lengths in turn (all nq slots of a pair share the rotation, so each tile is still taken once).
    const int round = pair / pairs_per_round;
    it.q0 = ((slot - pair * nq + round) % nq) * kQT;
    it.base = a.qkv + (int64_t)it.seq * a.s * ld + it.head * DH;
    return it;
  };
  // first item at or after `item` (in this workgroup's stride) that exists; items past the last pair
  // of a partly filled group of 8 are skipped
  auto next_valid = [&](int item) -> int {
    while (item < n_items && !decode(item).valid) item += gridDim.x;
    return item;
  };

  h8_t qreg[NU];   // B operand of the first product: the lane's query row, 8 head dims per K step
  auto load_q = [&](const Item& it) {
    int q = it.q0 + wave * 32 + l32;
    q = q < a.s ? q : a.s - 1;
#pragma unroll
    for (int u = 0; u < NU; ++u)
      qreg[u] = *reinterpret_cast<const h8_t*>(it.base + (int64_t)q * ld + 16 * u + 8 * hi);
  };
  // the next tile's K and V rows travel through registers while the current tile is being used
  u4_t kreg[NP];
  h8_t vreg[NP];
  auto fetch = [&](const Item& it, int kt) {
    const half_t* kv_col = it.base + a.h1 + dc0 * 8;
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

  int item = next_valid(blockIdx.x);
  if (item >= n_items) return;
  Item cur = decode(item);
  load_q(cur);
  fetch(cur, 0);

  while (true) {
    const int nxt_item = next_valid(item + gridDim.x);
    const bool has_next = nxt_item < n_items;
    const Item nxt = decode(has_next ? nxt_item : item);
    const int wq0 = cur.q0 + wave * 32;                  // this wave's first query
    const int my_q = wq0 + l32;                          // the query this lane's column belongs to
    const int last_q = (cur.q0 + kQT - 1) < (a.s - 1) ? (cur.q0 + kQT - 1) : (a.s - 1);
    const int n_tiles = last_q / kKT + 1;

    f16_t o[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;   // running maximum (log2 units) and sum over this lane's keys

    for (int kt = 0; kt < n_tiles; ++kt) {
      const int k0 = kt * kKT;
      const bool last = kt + 1 == n_tiles;
      __syncthreads();   // previous tile fully consumed
      stage();
      __syncthreads();
      // in flight during this tile's MFMAs: the next tile, or the next item's first tile
      if (!last)
        fetch(cur, kt + 1);
      else if (has_next)
        fetch(nxt, 0);
      // a wave has nothing to do in tiles that lie wholly above its diagonal (wave-uniform)
      const bool active = k0 <= wq0 + 31;

      f16_t t[NKB];
      if (active) {
        // ---- S^T blocks: block j = keys k0 + 32 j .. + 31
#pragma unroll
        for (int j = 0; j < NKB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) t[j][r] = 0.f;
#pragma unroll
        for (int u = 0; u < NU; ++u) {
#pragma unroll
          for (int j = 0; j < NKB; ++j) {
            const h8_t ka = *reinterpret_cast<const h8_t*>(Ks + (32 * j + l32) * LDK + 16 * u + 8 * hi);
            t[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ka, qreg[u], t[j], 0, 0, 0);
          }
        }
      }
      // the query rows are dead after the item's last S^T: bring in the next item's
      if (last && has_next) load_q(nxt);
      if (!active) continue;

      // lane holds, for query my_q, keys k0 + 32 j + 8 (r / 4) + 4 hi + r % 4 (raw dot products).
      // Only tiles that reach past the wave's first query need the causal mask.
      if (__builtin_amdgcn_readfirstlane(k0 + kKT - 1 > wq0)) {
#pragma unroll
        for (int j = 0; j < NKB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + 32 * j + 8 * (r >> 2) + 4 * hi + (r & 3);
            t[j][r] = key <= my_q ? t[j][r] : -INFINITY;
          }
        __builtin_amdgcn_sched_barrier(0);   // keep the masking out of the common path below
      }
      float cmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < NKB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) cmax = fmaxf(cmax, t[j][r]);
      cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64)) * c2;   // scale > 0: the maximum commutes with it
      const float m_new = fmaxf(m_run, cmax);
      // every key of a processed tile may still be masked for the clamped duplicate rows beyond s:
      // guard the exponent
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      m_run = m_new;
      float psum = 0.f;
      h8_t pop[NKB][2];   // B operands of the second product: 16 keys each
#pragma unroll
      for (int j = 0; j < NKB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(t[j][r], c2, -m_use));
          psum += p;
          pop[j][r >> 3][r & 7] = (half_t)p;
        }
      l_run = l_run * alpha + psum;
      // the running maximum rarely moves after the first tiles: skip the rescale when no lane needs it
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
      }
      // ---- O^T += V^T . P^T ; A operand: V^T rows d, K slots of lane half hi of the 16 keys starting
      // at kb = keys kb + {4 hi .. +3, 8 + 4 hi .. +3} (the order the accumulator left them in)
#pragma unroll
      for (int j = 0; j < NKB; ++j)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const int kb = 32 * j + 16 * c;
#pragma unroll
          for (int d = 0; d < NDB; ++d) {
            const int row = d * 32 + l32, rot = 4 * (row >> 3);
            const half_t* vr = Vt + row * LDV;
            const h4_t lo = *reinterpret_cast<const h4_t*>(vr + ((kb + 4 * hi + rot) & (kKT - 1)));
            const h4_t up = *reinterpret_cast<const h4_t*>(vr + ((kb + 8 + 4 * hi + rot) & (kKT - 1)));
            const h8_t va = {lo[0], lo[1], lo[2], lo[3], up[0], up[1], up[2], up[3]};
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pop[j][c], o[d], 0, 0, 0);
          }
        }
    }

    l_run += __shfl_xor(l_run, 32, 64);
    if (my_q < a.s) {
      const float inv = 1.0f / l_run;
      half_t* orow = a.out + ((int64_t)cur.seq * a.s + my_q) * a.h1 + cur.head * DH;
      // lane (query, hi) holds head dims 32 d + 8 g + 4 hi + 0..3 in registers 4 g .. 4 g + 3 of block d
#pragma unroll
      for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          h4_t v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = (half_t)(o[d][4 * g + r] * inv);
          *reinterpret_cast<h4_t*>(orow + d * 32 + 8 * g + 4 * hi) = v;
        }
    }
    if (!has_next) break;
    item = nxt_item;
    cur = nxt;
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
  // persistent workgroups: two per CU (what the kernel's registers allow), a multiple of 8 for the XCDs
  const int64_t items = ceil_div(a.n_pairs, 8) * 8 * ceil_div(s, kQT);
  const dim3 grid((unsigned)(items < 512 ? items : 512));
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
