// Decode-phase attention over the stored KV cache (Section 3, decode: softmax(tQ.K^T/sqrt(h)).V),
// with the cache read in its storage format of Section 5 and dequantized in registers.
//
// WPH = 1, 2 or 4 waves per (sequence, head), four waves per workgroup.  The rows of that head's K
// and V are one contiguous byte stream in the cache, read 16 bytes per lane (1 KiB per wave load).
// The waves of a head take 4 KiB chunks of the stream round-robin, keep a running (max, sum, output)
// triple each, and the triples are merged through LDS at the end (log-sum-exp merge); with one wave
// per head there is nothing to merge.  The host picks the smallest WPH that still fills the chip:
// a stream of c chunks costs ceil(c / WPH) chunk times, so at 528 rows (8.25 chunks) four waves
// per head would idle a quarter of the time.  The next chunk's loads are issued before the current
// one is processed.
//
// 4-bit path, per chunk of 128 quantization groups (64 rows at head size 128, 128 rows at 64):
//   scores  : q.k_hat = sum_g scale_g * (q_g . c_g) + min_g * sum(q_g).  The code dot products run on
//             the matrix cores: the K codes, expanded to FP16 in registers, are the B operand of
//             v_mfma_f32_16x16x32_f16 (lane = row, 8 consecutive codes per lane); the A operand
//             holds the query, masked so that output row 0/1 of each lane group separates the two
//             groups a lane pair covers.  Sixteen MFMAs leave, in lane L, the two group sums of
//             groups 2L and 2L+1 of the chunk, which is also the lane that loaded their {min,scale}.
//   softmax : one or two scores per lane, wavefront shuffles for the running max.
//   output  : sum_j p_j v_hat_j = sum_j (p_j scale_j) c_j + sum_j p_j min_j; the first term is
//             accumulated per lane over its 32 head dimensions with FP16->FP32 mixed FMAs on the
//             nibbles taken in place as FP16 subnormals, the second is one scalar per group.
#include "fg_attn_common.h"

namespace fg {

namespace {

struct AttnArgs {
  const half_t* q;
  int64_t q_stride;
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const void* k_meta;   // float2 or (H16) FP16 pairs
  const void* v_meta;
  half_t* out;       // [b, nh*dh]
  int nh, cap, rows, batch_offset;
  int n_heads;       // b * nh
  float scale;       // 1/sqrt(dh)
  // paged cache (PAGED kernels): k/v pointers are the page pools; cap, rows, batch_offset are unused
  const int32_t* page_table;   // [n_seqs][table_stride]
  const int32_t* seq_ids;      // [b] or nullptr
  const int32_t* seq_rows;     // [b]: rows attended = seq_rows[i] + rows_bias
  int table_stride, n_seqs, n_pages, rows_bias;
};

// Merge the WPH per-wave triples of each head of the block and write the outputs.  o_w already
// includes the per-group constant term.  out0 = output row of the block's first head.
template <int DH, int WPH>
__device__ __forceinline__ void merge_and_store(const float* sm_m, const float* sm_l, const float* sm_o, half_t* out0,
                                                int heads_valid) {
  __syncthreads();
  constexpr int HPB = 4 / WPH;
  for (int idx = threadIdx.x; idx < HPB * DH; idx += 256) {
    const int hl = idx / DH, t = idx - hl * DH;
    if (hl >= heads_valid) break;
    const float* mm = sm_m + hl * WPH;
    float M = mm[0];
#pragma unroll
    for (int w = 1; w < WPH; ++w) M = fmaxf(M, mm[w]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < WPH; ++w) {
      const float f = mm[w] == -INFINITY ? 0.f : fast_exp2((mm[w] - M) * kLog2e);
      num += f * sm_o[(hl * WPH + w) * DH + t];
      den += f * sm_l[hl * WPH + w];
    }
    out0[(int64_t)hl * DH + t] = (half_t)(den > 0.f ? num / den : 0.f);   // no rows attended: zeros
  }
}

// PAGED: the head's stream is cut into pages of 64 rows (FG_PAGE_ROWS) found through the sequence's
// row of the page table, and every sequence has its own length.  A wave keeps 64 consecutive table
// entries in one register (one per lane) and picks the page of a chunk with a lane read.
template <int DH, int WPH, bool H16, bool PAGED = false>
__global__ __launch_bounds__(256, 3) void attn_decode_q4_kernel(AttnArgs a) {
  using meta_t = typename MetaRaw<H16>::type;
  constexpr int GPR = DH / 64;       // quantization groups per row of this head
  constexpr int NS = 2 / GPR;        // scores per lane per chunk (lane owns groups 2L, 2L+1)
  constexpr int HPB = 4 / WPH;       // heads per workgroup
  __shared__ __attribute__((aligned(16))) half_t sm_q[HPB * DH];
  __shared__ float sm_m[4], sm_l[4];
  __shared__ float sm_o[WPH > 1 ? 4 * DH : 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = wave / WPH, part = wave - hl * WPH;
  const int hid0 = blockIdx.x * HPB;
  const int heads_valid = a.n_heads - hid0 < HPB ? a.n_heads - hid0 : HPB;
  const int hid = hl < heads_valid ? hid0 + hl : hid0;   // surplus waves of the last block redo its first head
  const int seq = hid / a.nh, head = hid - seq * a.nh;
  const int r = lane & 15, q4 = lane >> 4, h = q4 >> 1, half = q4 & 1;

  // contiguous: the stream starts at cache row hrow; paged: group indices are formed per page
  const int64_t hrow = PAGED ? 0 : ((int64_t)(a.batch_offset + seq) * a.nh + head) * a.cap;
  const uint8_t* kc = a.k_codes;
  const uint8_t* vc = a.v_codes;
  const meta_t* km = reinterpret_cast<const meta_t*>(a.k_meta);
  const meta_t* vm = reinterpret_cast<const meta_t*>(a.v_meta);
  int rows = a.rows;
  const int32_t* tbl = nullptr;
  int n_slots = 0;
  if constexpr (PAGED) {
    int sid = a.seq_ids ? a.seq_ids[seq] : seq;
    sid = sid < 0 ? 0 : (sid >= a.n_seqs ? a.n_seqs - 1 : sid);
    tbl = a.page_table + (int64_t)sid * a.table_stride;
    rows = a.seq_rows[seq] + a.rows_bias;
    rows = rows < 0 ? 0 : rows;
    rows = rows > a.table_stride * FG_PAGE_ROWS ? a.table_stride * FG_PAGE_ROWS : rows;   // never read past the table
    n_slots = (rows + FG_PAGE_ROWS - 1) / FG_PAGE_ROWS;
  }
  const int G = rows * GPR;                    // groups in the stream
  const int n_chunks = (G + 127) >> 7;
  // paged: the table entries of slots 64*win .. 64*win + 63, one per lane
  int win = -1, tbl_reg = 0;
  auto page_of = [&](int slot) -> int {   // slot is wave-uniform and < n_slots
    if ((slot >> 6) != win) {
      win = slot >> 6;
      const int sl = win * 64 + lane;
      tbl_reg = tbl[sl < n_slots ? sl : n_slots - 1];
    }
    int pg = __builtin_amdgcn_readlane(tbl_reg, slot & 63);
    return pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);   // a bad entry reads page 0 / the last page
  };
  // index (in quantization groups) into the code / meta arrays of group g (< G) of this head's stream;
  // pgA, pgB: pages of the first and (head size 64 only) second slot of the chunk being loaded
  constexpr int kGPP = FG_PAGE_ROWS * GPR;     // groups per (page, head)
  auto gidx = [&](int g, int slot0, int pgA, int pgB) -> int64_t {
    if constexpr (!PAGED) {
      return hrow * GPR + g;
    } else {
      const int slot = g / kGPP;
      const int pg = slot == slot0 ? pgA : pgB;
      return ((int64_t)pg * a.nh + head) * kGPP + (g - slot * kGPP);
    }
  };

  // one chunk's worth of registers: 4 + 4 code loads of 16 bytes and the meta of the lane's two groups
  struct Buf {
    u4_t kq[4], vq[4];
    meta_t km0, km1, vm0, vm1;
  };
  // all addresses clamped into the stream; rows past the end are masked when the chunk is processed
  auto load = [&](Buf& b, int chunk) {
    const int gbase = chunk << 7;
    int slot0 = 0, pgA = 0, pgB = 0;
    if constexpr (PAGED) {   // a chunk of 128 groups is one page at head size 128, two at 64
      slot0 = gbase / kGPP;
      pgA = page_of(slot0);
      pgB = (GPR == 1 && slot0 + 1 < n_slots) ? page_of(slot0 + 1) : pgA;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int g = gbase + 32 * i + 2 * r + h;
      g = g < G ? g : G - 1;
      const int64_t gi = gidx(g, slot0, pgA, pgB);
      b.kq[i] = *reinterpret_cast<const u4_t*>(kc + gi * 32 + half * 16);
      b.vq[i] = *reinterpret_cast<const u4_t*>(vc + gi * 32 + half * 16);
    }
    const int g0 = gbase + 2 * lane, g1 = g0 + 1;
    const int c0 = g0 < G ? g0 : G - 1, c1 = g1 < G ? g1 : G - 1;
    const int64_t i0 = gidx(c0, slot0, pgA, pgB), i1 = gidx(c1, slot0, pgA, pgB);
    b.km0 = km[i0];
    b.km1 = km[i1];
    b.vm0 = vm[i0];
    b.vm1 = vm[i1];
  };
  // the first chunk's loads go out before anything else: they overlap the query set-up below
  Buf b0, b1;
  if (part < n_chunks) load(b0, part);

  half_t* my_q = sm_q + hl * DH;
  if (part == 0 && lane < DH / 8)
    *reinterpret_cast<u4_t*>(my_q + lane * 8) =
        *reinterpret_cast<const u4_t*>(a.q + (int64_t)seq * a.q_stride + head * DH + lane * 8);
  __syncthreads();

  QueryOps<DH> Q;
  query_setup<DH>(my_q, lane, Q);

  float m_run = -INFINITY, l_run = 0.f;
  float mterm[2] = {0.f, 0.f};   // sum_j p_j min_j for the groups this lane owns
  float o[32];
#pragma unroll
  for (int e = 0; e < 32; ++e) o[e] = 0.f;

  auto process = [&](const Buf& b, int chunk) {
    const int gbase = chunk << 7;
    const int ni = (G - gbase + 31) >> 5;   // 32-group loads of this chunk that hold valid rows
    // ---- scores on the matrix cores
    float sc[NS];
    chunk_scores<DH>(b.kq, meta_f32(b.km0), meta_f32(b.km1), Q, a.scale, G, gbase, lane, sc);
    // ---- online softmax (every processed chunk has at least one valid row)
    float cmax = sc[0];
    if (NS == 2) cmax = fmaxf(cmax, sc[NS - 1]);
    cmax = uniform(wave_max(cmax));
    const float m_new = fmaxf(m_run, cmax);
    if (m_new > m_run) {   // wave-uniform
      const float alpha = fast_exp2((m_run - m_new) * kLog2e);
      l_run *= alpha;
      mterm[0] *= alpha;
      mterm[1] *= alpha;
#pragma unroll
      for (int e = 0; e < 32; ++e) o[e] *= alpha;
      m_run = m_new;
    }
    float p[2];
    p[0] = fast_exp2((sc[0] - m_run) * kLog2e);
    p[1] = NS == 2 ? fast_exp2((sc[NS - 1] - m_run) * kLog2e) : p[0];
    l_run += NS == 2 ? p[0] + p[1] : p[0];
    // weights of the V codes of the two groups this lane owns, and their constant terms
    const float2 vm0 = meta_f32(b.vm0), vm1 = meta_f32(b.vm1);
    const float wv0 = p[0] * vm0.y, wv1 = p[1] * vm1.y;
    mterm[0] += p[0] * vm0.x;
    mterm[1] += p[1] * vm1.x;

    // ---- output accumulation: lane (r, q4) handles group 32 i + 2 r + h of each load, half `half`.
    // A nibble masked in place is the FP16 subnormal c * 2^-24 (low nibble of a half) or c * 2^-20;
    // the mixed-precision FMA takes it as it is, the weight carries the inverse power of two.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i >= ni) break;
      const int src = 16 * i + r;
      const float w0 = __shfl(wv0, src, 64), w1 = __shfl(wv1, src, 64);
      const float w = h ? w1 : w0;
      const float w24 = w * 16777216.0f, w20 = w * 1048576.0f;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t x = b.vq[i][u], y = x >> 8;
        const h2_t c04 = __builtin_bit_cast(h2_t, x & 0x000F000Fu);
        const h2_t c15 = __builtin_bit_cast(h2_t, x & 0x00F000F0u);
        const h2_t c26 = __builtin_bit_cast(h2_t, y & 0x000F000Fu);
        const h2_t c37 = __builtin_bit_cast(h2_t, y & 0x00F000F0u);
        o[8 * u + 0] = __builtin_fmaf((float)c04.x, w24, o[8 * u + 0]);
        o[8 * u + 4] = __builtin_fmaf((float)c04.y, w24, o[8 * u + 4]);
        o[8 * u + 1] = __builtin_fmaf((float)c15.x, w20, o[8 * u + 1]);
        o[8 * u + 5] = __builtin_fmaf((float)c15.y, w20, o[8 * u + 5]);
        o[8 * u + 2] = __builtin_fmaf((float)c26.x, w24, o[8 * u + 2]);
        o[8 * u + 6] = __builtin_fmaf((float)c26.y, w24, o[8 * u + 6]);
        o[8 * u + 3] = __builtin_fmaf((float)c37.x, w20, o[8 * u + 3]);
        o[8 * u + 7] = __builtin_fmaf((float)c37.y, w20, o[8 * u + 7]);
      }
    }
  };

  // (the first chunk is already on its way; the loop is unrolled by two so that neither buffer is ever
  // moved while loads fly)
  for (int chunk = part; chunk < n_chunks; chunk += 2 * WPH) {
    const bool more1 = chunk + WPH < n_chunks;
    if (more1) load(b1, chunk + WPH);
    __builtin_amdgcn_sched_barrier(0);
    process(b0, chunk);
    if (more1) {
      if (chunk + 2 * WPH < n_chunks) load(b0, chunk + 2 * WPH);
      __builtin_amdgcn_sched_barrier(0);
      process(b1, chunk + WPH);
    }
  }

  // ---- reduce inside the wave: lanes with the same head-dimension range add up
#pragma unroll
  for (int e = 0; e < 32; ++e) {
    float v = o[e];
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    if (DH == 64) v += __shfl_xor(v, 32, 64);
    o[e] = v;
  }
  const float lw = wave_sum(l_run);
  const float mt0 = wave_sum(mterm[0]), mt1 = wave_sum(mterm[1]);
  // this lane's range: head dims [dbase, dbase + 32), all in one quantization group
  const int dbase = DH == 128 ? 32 * q4 : 32 * half;
  const float c = DH == 128 ? (h ? mt1 : mt0) : (mt0 + mt1);
  const bool writer = r == 0 && (DH == 128 || h == 0);
  half_t* out0 = a.out + (int64_t)hid0 * DH;
  if (WPH == 1) {
    if (writer && hl < heads_valid) {
      const float inv = lw > 0.f ? 1.0f / lw : 0.f;   // no rows attended (paged, empty sequence): zeros
      half_t* dst = out0 + (int64_t)hl * DH + dbase;
#pragma unroll
      for (int v8 = 0; v8 < 4; ++v8) {
        h8_t pk;
#pragma unroll
        for (int e = 0; e < 8; ++e) pk[e] = (half_t)((o[8 * v8 + e] + c) * inv);
        *reinterpret_cast<h8_t*>(dst + 8 * v8) = pk;
      }
    }
  } else {
    if (lane == 0) {
      sm_m[wave] = m_run;
      sm_l[wave] = lw;
    }
    if (writer) {
#pragma unroll
      for (int e = 0; e < 32; ++e) sm_o[wave * DH + dbase + e] = o[e] + c;
    }
    merge_and_store<DH, WPH>(sm_m, sm_l, sm_o, out0, heads_valid);
  }
}

// FP16 cache: the same streaming structure without the unpacking.  K rows are the B operand
// directly (lane = row, 8 consecutive head dimensions per lane).
// PAGED: a chunk of 64 rows is exactly one page of the sequence (FG_PAGE_ROWS = 64), found through the
// page table; every sequence has its own length.
template <int DH, int WPH, bool PAGED = false>
__global__ __launch_bounds__(256) void attn_decode_f16_kernel(AttnArgs a) {
  constexpr int NU = DH / 32;        // 32-wide head-dimension blocks
  constexpr int HPB = 4 / WPH;       // heads per workgroup
  __shared__ __attribute__((aligned(16))) half_t sm_q[HPB * DH];
  __shared__ float sm_m[4], sm_l[4];
  __shared__ float sm_o[WPH > 1 ? 4 * DH : 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = wave / WPH, part = wave - hl * WPH;
  const int hid0 = blockIdx.x * HPB;
  const int heads_valid = a.n_heads - hid0 < HPB ? a.n_heads - hid0 : HPB;
  const int hid = hl < heads_valid ? hid0 + hl : hid0;
  const int seq = hid / a.nh, head = hid - seq * a.nh;
  const int r = lane & 15, q4 = lane >> 4;
  const int64_t hrow = PAGED ? 0 : ((int64_t)(a.batch_offset + seq) * a.nh + head) * a.cap;
  const half_t* kp = reinterpret_cast<const half_t*>(a.k_codes) + hrow * DH;
  const half_t* vp = reinterpret_cast<const half_t*>(a.v_codes) + hrow * DH;
  int n_rows = a.rows;
  const int32_t* tbl = nullptr;
  if constexpr (PAGED) {
    int sid = a.seq_ids ? a.seq_ids[seq] : seq;
    sid = sid < 0 ? 0 : (sid >= a.n_seqs ? a.n_seqs - 1 : sid);
    tbl = a.page_table + (int64_t)sid * a.table_stride;
    n_rows = a.seq_rows[seq] + a.rows_bias;
    n_rows = n_rows < 0 ? 0 : n_rows;
    n_rows = n_rows > a.table_stride * FG_PAGE_ROWS ? a.table_stride * FG_PAGE_ROWS : n_rows;
  }
  const int n_chunks = (n_rows + 63) >> 6;
  // first cache row (in rows of DH elements) of chunk c of this head's stream
  auto chunk_row0 = [&](int c) -> int64_t {
    if constexpr (!PAGED) {
      return (int64_t)c << 6;
    } else {
      int pg = tbl[c];                                             // c < n_chunks <= table_stride
      pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);   // a bad entry reads some page of the pool
      return ((int64_t)pg * a.nh + head) * FG_PAGE_ROWS;
    }
  };

  half_t* my_q = sm_q + hl * DH;
  if (part == 0 && lane < DH / 8)
    *reinterpret_cast<u4_t*>(my_q + lane * 8) =
        *reinterpret_cast<const u4_t*>(a.q + (int64_t)seq * a.q_stride + head * DH + lane * 8);
  __syncthreads();

  // A operand: the query in rows 0, 4, 8, 12 of the 16 x 32 tile, zeros elsewhere.  Lane (n = l % 16,
  // g = l / 16) of the result holds D[4g][n] in its first register, so with the query in all four of
  // those rows every lane group g gets q . k_n of the 16 keys at hand; group g keeps the product of
  // keys 16 g .. 16 g + 15, which leaves lane l the score of row l of the chunk.
  h8_t qop[NU];
  {
    const int m = lane & 15;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const u4_t raw = *reinterpret_cast<const u4_t*>(my_q + 32 * u + 8 * q4);
      const u4_t z = {0u, 0u, 0u, 0u};
      qop[u] = __builtin_bit_cast(h8_t, (m & 3) == 0 ? raw : z);
    }
  }

  float m_run = -INFINITY, l_run = 0.f;
  float o[8 * NU];
#pragma unroll
  for (int e = 0; e < 8 * NU; ++e) o[e] = 0.f;

  // Two register sets, one for a chunk's K rows and one for its V rows (16 KiB each at DH = 128).  The V
  // rows of a chunk are requested before its scores are computed and the K rows of the wave's next
  // chunk right after them, so a wave has 16 to 32 KiB on their way all the time instead of waiting
  // out one load latency for K and another for V in every chunk.
  h8_t kreg[4][NU], vreg[4][NU];
  auto load_rows = [&](const half_t* base, int chunk, h8_t (&dst)[4][NU]) {
    const int64_t crow0 = chunk_row0(chunk);
    const int last = n_rows - 1 - (chunk << 6);   // rows of the chunk past the end re-read its last valid row
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int row = 16 * i + r;
      row = row < last ? row : last;
#pragma unroll
      for (int u = 0; u < NU; ++u)
        dst[i][u] = *reinterpret_cast<const h8_t*>(base + (crow0 + row) * DH + 32 * u + 8 * q4);
    }
  };
  if (part < n_chunks) load_rows(kp, part, kreg);
  for (int chunk = part; chunk < n_chunks; chunk += WPH) {
    const int rbase = chunk << 6;
    load_rows(vp, chunk, vreg);
    __builtin_amdgcn_sched_barrier(0);
    float sc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < NU; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qop[u], kreg[i][u], acc, 0, 0, 0);
      sc = q4 == i ? acc[0] : sc;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (chunk + WPH < n_chunks) load_rows(kp, chunk + WPH, kreg);
    __builtin_amdgcn_sched_barrier(0);
    sc = (rbase + lane) < n_rows ? sc * a.scale : -INFINITY;
    const float cmax = wave_max(sc);
    const float m_new = fmaxf(m_run, cmax);
    if (m_new > m_run) {
      const float alpha = fast_exp2((m_run - m_new) * kLog2e);
      l_run *= alpha;
#pragma unroll
      for (int e = 0; e < 8 * NU; ++e) o[e] *= alpha;
      m_run = m_new;
    }
    const float p = fast_exp2((sc - m_run) * kLog2e);
    l_run += p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float w = __shfl(p, 16 * i + r, 64);
#pragma unroll
      for (int u = 0; u < NU; ++u) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[8 * u + e] += w * (float)vreg[i][u][e];
      }
    }
  }

#pragma unroll
  for (int e = 0; e < 8 * NU; ++e) {
    float v = o[e];
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    o[e] = v;
  }
  const float lw = wave_sum(l_run);
  half_t* out0 = a.out + (int64_t)hid0 * DH;
  if (WPH == 1) {
    if (r == 0 && hl < heads_valid) {
      const float inv = lw > 0.f ? 1.0f / lw : 0.f;   // no rows attended (paged, empty sequence): zeros
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        h8_t pk;
#pragma unroll
        for (int e = 0; e < 8; ++e) pk[e] = (half_t)(o[8 * u + e] * inv);
        *reinterpret_cast<h8_t*>(out0 + (int64_t)hl * DH + 32 * u + 8 * q4) = pk;
      }
    }
  } else {
    if (lane == 0) {
      sm_m[wave] = m_run;
      sm_l[wave] = lw;
    }
    if (r == 0) {
#pragma unroll
      for (int u = 0; u < NU; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) sm_o[wave * DH + 32 * u + 8 * q4 + e] = o[8 * u + e];
    }
    merge_and_store<DH, WPH>(sm_m, sm_l, sm_o, out0, heads_valid);
  }
}

}  // namespace

// Waves per (sequence, head): 1, 2 or 4.  A stream of c chunks costs a wave ceil(c / WPH) chunk times
// plus the merge, so one wave per head wastes the least, and measured it is the fastest from a few
// thousand heads up even where the launch is only one or two rounds of workgroups (4096 heads x 528
// rows: 4.6 / 4.4 / 4.2 TB/s with 1 / 2 / 4 waves per head; 13824 heads: 5.4 / 4.9 / 4.3).  Fewer
// heads than that get more waves each, so that the chip is not left empty, but never more waves than
// the stream has chunks.
static int pick_waves_per_head(int64_t heads, int rows, int rows_per_chunk) {
  const int chunks = (rows + rows_per_chunk - 1) / rows_per_chunk;
  int wph = heads >= 2048 ? 1 : (heads >= 1024 ? 2 : 4);
  while (wph > 1 && chunks < wph) wph >>= 1;
  return wph;
}

int decode_attention_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                            int32_t rows, const fg_kv_cache& kv, int32_t batch_offset, half_t* out,
                            hipStream_t stream) {
  if (b == 0) return FG_OK;
  const int dh = cfg.h1 / cfg.nh;
  AttnArgs a;
  a.q = q;
  a.q_stride = q_stride;
  a.k_codes = reinterpret_cast<const uint8_t*>(kv.k_codes);
  a.v_codes = reinterpret_cast<const uint8_t*>(kv.v_codes);
  a.k_meta = kv.k_meta;
  a.v_meta = kv.v_meta;
  a.out = out;
  a.nh = cfg.nh;
  a.cap = kv.cap;
  a.rows = rows;
  a.batch_offset = batch_offset;
  a.scale = 1.0f / sqrtf((float)dh);
  a.n_heads = b * cfg.nh;
  a.page_table = a.seq_ids = a.seq_rows = nullptr;
  a.table_stride = a.n_seqs = a.n_pages = a.rows_bias = 0;
  const int64_t heads = (int64_t)b * cfg.nh;
  const bool q4 = kv.dtype == FG_Q4G64 || kv.dtype == FG_Q4G64_H16;
  const bool h16 = kv.dtype == FG_Q4G64_H16;
  const int wph = pick_waves_per_head(heads, rows, q4 ? 8192 / dh : 64);
  const dim3 grid((unsigned)ceil_div(heads * wph, 4));
  ProfScope prof(FG_K_ATTN_DECODE, stream);
#define FG_ATTN_LAUNCH(DH_, ...)                                                                      \
  do {                                                                                                \
    if (wph == 1)                                                                                     \
      hipLaunchKernelGGL((__VA_ARGS__<DH_, 1 FG_ATTN_EXTRA>), grid, dim3(256), 0, stream, a);         \
    else if (wph == 2)                                                                                \
      hipLaunchKernelGGL((__VA_ARGS__<DH_, 2 FG_ATTN_EXTRA>), grid, dim3(256), 0, stream, a);         \
    else                                                                                              \
      hipLaunchKernelGGL((__VA_ARGS__<DH_, 4 FG_ATTN_EXTRA>), grid, dim3(256), 0, stream, a);         \
  } while (0)
  if (q4 && h16) {
#define FG_ATTN_EXTRA , true
    if (dh == 128)
      FG_ATTN_LAUNCH(128, attn_decode_q4_kernel);
    else
      FG_ATTN_LAUNCH(64, attn_decode_q4_kernel);
#undef FG_ATTN_EXTRA
  } else if (q4) {
#define FG_ATTN_EXTRA , false
    if (dh == 128)
      FG_ATTN_LAUNCH(128, attn_decode_q4_kernel);
    else
      FG_ATTN_LAUNCH(64, attn_decode_q4_kernel);
#undef FG_ATTN_EXTRA
  } else {
#define FG_ATTN_EXTRA
    if (dh == 128)
      FG_ATTN_LAUNCH(128, attn_decode_f16_kernel);
    else
      FG_ATTN_LAUNCH(64, attn_decode_f16_kernel);
#undef FG_ATTN_EXTRA
  }
#undef FG_ATTN_LAUNCH
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int decode_attention_paged_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                                  const fg_kv_pages& pages, const fg_ragged& seqs, int32_t rows_bias, half_t* out,
                                  hipStream_t stream) {
  if (b == 0) return FG_OK;
  const int dh = cfg.h1 / cfg.nh;
  AttnArgs a;
  a.q = q;
  a.q_stride = q_stride;
  a.k_codes = reinterpret_cast<const uint8_t*>(pages.k_codes);
  a.v_codes = reinterpret_cast<const uint8_t*>(pages.v_codes);
  a.k_meta = pages.k_meta;
  a.v_meta = pages.v_meta;
  a.out = out;
  a.nh = cfg.nh;
  a.cap = 0;
  a.rows = 0;
  a.batch_offset = 0;
  a.scale = 1.0f / sqrtf((float)dh);
  a.n_heads = b * cfg.nh;
  a.page_table = seqs.page_table;
  a.seq_ids = seqs.seq_ids;
  a.seq_rows = seqs.pos;
  a.table_stride = seqs.table_stride;
  a.n_seqs = seqs.n_seqs;
  a.n_pages = pages.n_pages;
  a.rows_bias = rows_bias;
  const int64_t heads = (int64_t)b * cfg.nh;
  // as in the contiguous launch, with the longest sequence the page table can address standing in for the
  // lengths, which only the device knows
  const int wph = pick_waves_per_head(heads, seqs.table_stride * FG_PAGE_ROWS, pages.dtype == FG_F16 ? 64 : 8192 / dh);
  const dim3 grid((unsigned)ceil_div(heads * wph, 4));
  const bool h16 = pages.dtype == FG_Q4G64_H16;
  ProfScope prof(FG_K_ATTN_DECODE, stream);
  if (pages.dtype == FG_F16) {
#define FG_PAGED_F16(DH_)                                                                                     \
  do {                                                                                                        \
    if (wph == 1)                                                                                             \
      hipLaunchKernelGGL((attn_decode_f16_kernel<DH_, 1, true>), grid, dim3(256), 0, stream, a);              \
    else if (wph == 2)                                                                                        \
      hipLaunchKernelGGL((attn_decode_f16_kernel<DH_, 2, true>), grid, dim3(256), 0, stream, a);              \
    else                                                                                                      \
      hipLaunchKernelGGL((attn_decode_f16_kernel<DH_, 4, true>), grid, dim3(256), 0, stream, a);              \
  } while (0)
    if (dh == 128) FG_PAGED_F16(128); else FG_PAGED_F16(64);
#undef FG_PAGED_F16
    FG_LAUNCH_CHECK();
    return FG_OK;
  }
#define FG_PAGED_LAUNCH(DH_, WPH_)                                                                          \
  do {                                                                                                      \
    if (h16)                                                                                                \
      hipLaunchKernelGGL((attn_decode_q4_kernel<DH_, WPH_, true, true>), grid, dim3(256), 0, stream, a);    \
    else                                                                                                    \
      hipLaunchKernelGGL((attn_decode_q4_kernel<DH_, WPH_, false, true>), grid, dim3(256), 0, stream, a);   \
  } while (0)
  if (dh == 128) {
    if (wph == 1) FG_PAGED_LAUNCH(128, 1); else if (wph == 2) FG_PAGED_LAUNCH(128, 2); else FG_PAGED_LAUNCH(128, 4);
  } else {
    if (wph == 1) FG_PAGED_LAUNCH(64, 1); else if (wph == 2) FG_PAGED_LAUNCH(64, 2); else FG_PAGED_LAUNCH(64, 4);
  }
#undef FG_PAGED_LAUNCH
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg

using namespace fg;

extern "C" int fg_decode_attention_paged(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                                         const fg_kv_pages* pages, const fg_ragged* seqs, int32_t rows_bias,
                                         void* out_f16, void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_pages(cfg, pages, seqs);
  if (rc) return rc;
  if (!seqs->pos) return FG_ERR_NULL;
  if (b < 0 || rows_bias < 0) return FG_ERR_SHAPE;
  if (q_row_stride < cfg->h1 || q_row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0) return FG_OK;
  if (!q_f16 || !out_f16) return FG_ERR_NULL;
  return decode_attention_paged_launch(*cfg, reinterpret_cast<const half_t*>(q_f16), q_row_stride, b, *pages, *seqs,
                                       rows_bias, reinterpret_cast<half_t*>(out_f16), as_stream(stream));
}

extern "C" int fg_decode_attention(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                                   int32_t rows, const fg_kv_cache* kv, int32_t batch_offset, void* out_f16,
                                   void* stream) {
  if (!cfg || !kv) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_kv(cfg, kv);
  if (rc) return rc;
  if (b < 0 || rows < 1 || rows > kv->cap || batch_offset < 0 || (int64_t)batch_offset + b > kv->batch)
    return FG_ERR_SHAPE;
  if (q_row_stride < cfg->h1 || q_row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0) return FG_OK;
  if (!q_f16 || !out_f16) return FG_ERR_NULL;
  return decode_attention_launch(*cfg, reinterpret_cast<const half_t*>(q_f16), q_row_stride, b, rows, *kv,
                                 batch_offset, reinterpret_cast<half_t*>(out_f16), as_stream(stream));
}
