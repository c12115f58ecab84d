// Top-K sparse decode attention over the 4-bit KV cache (Section 5, sparse attention; decode phase of
// Section 3): the attention weights of the query are those of the full softmax over all cached rows;
// only the `topk` highest-weighted rows of V are then read, the rest is dropped without
// renormalisation.  Among equal scores the lowest row index is kept.
//
// One workgroup of four waves per (sequence, head), three phases:
//   1. scores   the K stream is read once, exactly as in the dense kernel (MFMA on the codes); the
//               scaled scores of all rows go to LDS;
//   2. select   exact k-th largest score by a four-pass radix select over the order-preserving
//               integer image of the scores (256-bin LDS histograms), then a compaction in row order:
//               rows above the threshold, plus the first rows equal to it until k rows are kept;
//   3. gather   the kept rows of V (DH/2 bytes of codes + their {min,scale} each) are fetched by
//               DH/16 lanes per row and accumulated with the full-softmax weights.
// K is half of the dense kernel's bytes and V shrinks to k/rows of it.
#include "fg_attn_common.h"

namespace fg {

namespace {

struct TopkArgs {
  const half_t* q;
  int64_t q_stride;
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const void* k_meta;   // float2 or (H16) FP16 pairs
  const void* v_meta;
  half_t* out;       // [b, nh*dh]
  int32_t* sel_out;  // [b, nh, topk] kept row indices, ascending, or NULL
  int nh, cap, rows, topk, batch_offset;
  int rows_pad;      // rows rounded up to whole chunks: size of the score array in LDS
  float scale;       // 1/sqrt(dh)
  // paged cache (PAGED kernels): k/v pointers are the page pools; cap, rows, batch_offset are unused.
  // Row i attends seq_rows[i] + rows_bias rows and keeps min(topk, that many) of them.
  const int32_t* page_table;   // [n_seqs][table_stride]
  const int32_t* seq_ids;      // [b] or nullptr
  const int32_t* seq_rows;     // [b]
  int table_stride, n_seqs, n_pages, rows_bias;
};

__device__ __forceinline__ uint32_t order_key(float s) {
  const uint32_t u = __builtin_bit_cast(uint32_t, s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // larger score <=> larger key
}

// exclusive prefix sum of one value per thread over the 256 threads; *total gets the sum
__device__ __forceinline__ int block_excl_scan(int v, int* s_wave, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(incl, d, 64);
    if (lane >= d) incl += t;
  }
  __syncthreads();   // s_wave may still be read from a previous call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w < wave) base += s_wave[w];
  *total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
  return base + incl - v;
}

template <int DH, bool H16, bool PAGED = false>
__global__ __launch_bounds__(256) void attn_decode_topk_q4_kernel(TopkArgs a) {
  using meta_t = typename MetaRaw<H16>::type;
  constexpr int GPR = DH / 64;       // quantization groups per row
  constexpr int NS = 2 / GPR;        // scores per lane per chunk
  constexpr int RPC = 128 / GPR;     // rows per chunk
  constexpr int LPR = DH / 16;       // gather: lanes per V row (8 bytes = 16 codes each)
  constexpr int RPI = 64 / LPR;      // gather: rows per wave iteration
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
  float* s_sc = reinterpret_cast<float*>(dyn);                    // [rows_pad]
  int* s_sel = reinterpret_cast<int*>(dyn) + a.rows_pad;          // [topk]
  __shared__ __attribute__((aligned(16))) half_t sm_q[DH];
  __shared__ int s_hist[256];
  __shared__ int s_wave[4];
  __shared__ float s_red[8];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  __shared__ float s_o[4 * DH];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hid = blockIdx.x;
  const int seq = hid / a.nh, head = hid - seq * a.nh;
  const int r = lane & 15, q4 = lane >> 4, h = q4 >> 1, half = q4 & 1;
  int n = a.rows, topk = a.topk;
  const int32_t* tbl = nullptr;
  if constexpr (PAGED) {
    int sid = a.seq_ids ? a.seq_ids[seq] : seq;
    sid = sid < 0 ? 0 : (sid >= a.n_seqs ? a.n_seqs - 1 : sid);
    tbl = a.page_table + (int64_t)sid * a.table_stride;
    n = a.seq_rows[seq] + a.rows_bias;
    n = n < 0 ? 0 : n;
    n = n > a.table_stride * FG_PAGE_ROWS ? a.table_stride * FG_PAGE_ROWS : n;   // never read past the table
    topk = topk < n ? topk : n;
    if (n == 0) {   // nothing to attend (uniform over the workgroup): zeros, no kept rows
      if (tid < DH) a.out[(int64_t)hid * DH + tid] = (half_t)0.f;
      if (a.sel_out)
        for (int e = tid; e < a.topk; e += 256) a.sel_out[(int64_t)hid * a.topk + e] = -1;
      return;
    }
  }

  // cache row (in rows of DH elements) that holds position `row` of this head's stream
  const int64_t hrow = PAGED ? 0 : ((int64_t)(a.batch_offset + seq) * a.nh + head) * a.cap;
  auto rowidx = [&](int row) -> int64_t {
    if constexpr (!PAGED) {
      return hrow + row;
    } else {
      int pg = tbl[row >> 6];
      pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);   // a bad entry reads some page, never outside the pool
      return ((int64_t)pg * a.nh + head) * FG_PAGE_ROWS + (row & (FG_PAGE_ROWS - 1));
    }
  };
  const uint8_t* kc = a.k_codes;
  const uint8_t* vc = a.v_codes;
  const meta_t* km = reinterpret_cast<const meta_t*>(a.k_meta);
  const meta_t* vm = reinterpret_cast<const meta_t*>(a.v_meta);
  const int G = n * GPR;
  const int n_chunks = (G + 127) >> 7;
  // index, in quantization groups, of group g (< G) of the stream
  auto gidx = [&](int g) -> int64_t { return rowidx(g / GPR) * GPR + (g & (GPR - 1)); };

  struct Buf {
    u4_t kq[4];
    meta_t km0, km1;
  };
  auto load = [&](Buf& b, int chunk) {
    const int gbase = chunk << 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int g = gbase + 32 * i + 2 * r + h;
      g = g < G ? g : G - 1;
      b.kq[i] = *reinterpret_cast<const u4_t*>(kc + gidx(g) * 32 + half * 16);
    }
    const int g0 = gbase + 2 * lane, g1 = g0 + 1;
    b.km0 = km[gidx(g0 < G ? g0 : G - 1)];
    b.km1 = km[gidx(g1 < G ? g1 : G - 1)];
  };
  Buf b0, b1;
  if (wave < n_chunks) load(b0, wave);

  if (tid < DH / 8)
    *reinterpret_cast<u4_t*>(sm_q + tid * 8) =
        *reinterpret_cast<const u4_t*>(a.q + (int64_t)seq * a.q_stride + head * DH + tid * 8);
  __syncthreads();
  QueryOps<DH> Q;
  query_setup<DH>(sm_q, lane, Q);

  // ---- phase 1: scores of all rows -> LDS (rows past the end hold -inf), with each wave's running
  // maximum and sum of exponentials (merged below into the softmax denominator)
  float m_run = -INFINITY, l_run = 0.f;
  auto scores = [&](const Buf& b, int chunk) {
    float sc[NS];
    chunk_scores<DH>(b.kq, meta_f32(b.km0), meta_f32(b.km1), Q, a.scale, G, chunk << 7, lane, sc);
    float cmax = sc[0];
    if (NS == 2) cmax = fmaxf(cmax, sc[NS - 1]);
    cmax = wave_max(cmax);              // a processed chunk has at least one valid row
    if (cmax > m_run) {                 // wave-uniform
      l_run *= fast_exp2((m_run - cmax) * kLog2e);
      m_run = cmax;
    }
    l_run += fast_exp2((sc[0] - m_run) * kLog2e);
    if (NS == 2) l_run += fast_exp2((sc[NS - 1] - m_run) * kLog2e);
    if (DH == 128) {
      s_sc[chunk * RPC + lane] = sc[0];
    } else {
      s_sc[chunk * RPC + 2 * lane] = sc[0];
      s_sc[chunk * RPC + 2 * lane + 1] = sc[NS - 1];
    }
  };
  for (int chunk = wave; chunk < n_chunks; chunk += 8) {
    const bool more1 = chunk + 4 < n_chunks;
    if (more1) load(b1, chunk + 4);
    __builtin_amdgcn_sched_barrier(0);
    scores(b0, chunk);
    if (more1) {
      if (chunk + 8 < n_chunks) load(b0, chunk + 8);
      __builtin_amdgcn_sched_barrier(0);
      scores(b1, chunk + 4);
    }
  }
  // ---- maximum and softmax denominator over all rows: log-sum-exp merge of the four waves
  l_run = wave_sum(l_run);
  if (lane == 0) {
    s_red[wave] = m_run;
    s_red[4 + wave] = l_run;
  }
  __syncthreads();
  const float M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  float den = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (s_red[w] != -INFINITY) den += s_red[4 + w] * fast_exp2((s_red[w] - M) * kLog2e);
  const float inv_den = 1.0f / den;

  // ---- phase 2: radix select of the topk-th largest key, most significant byte first
  if (tid == 0) {
    s_prefix = 0u;
    s_need = topk;
  }
  uint32_t mask = 0u;
#pragma unroll 1
  for (int shift = 24; shift >= 0; shift -= 8) {
    s_hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    for (int i = tid; i < n; i += 256) {
      const uint32_t key = order_key(s_sc[i]);
      if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (wave == 0) {
      // bins in descending order: lane l owns bins 255-4l .. 252-4l
      const int need = s_need;
      int c[4], sum = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c[j] = s_hist[255 - (4 * lane + j)];
        sum += c[j];
      }
      int incl = sum;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
      }
      const uint64_t reach = __builtin_amdgcn_ballot_w64(incl >= need);
      const int first = __builtin_ctzll(reach);   // reach != 0: the candidates number at least `need`
      if (lane == first) {
        int above = incl - sum;                   // keys in higher bins
        int j = 0;
        while (j < 3 && above + c[j] < need) {
          above += c[j];
          ++j;
        }
        s_prefix = prefix | ((uint32_t)(255 - (4 * lane + j)) << shift);
        s_need = need - above;
      }
    }
    mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t T = s_prefix;     // key of the topk-th largest score
  const int need_eq = s_need;      // rows equal to it that are kept (the lowest indices)

  // ---- compaction in row order: thread t owns rows [t*per, (t+1)*per)
  const int per = (n + 255) >> 8;
  const int r0 = tid * per, r1 = (r0 + per) < n ? (r0 + per) : n;
  int n_gt = 0, n_eq = 0;
  for (int i = r0; i < r1; ++i) {
    const uint32_t key = order_key(s_sc[i]);
    n_gt += key > T;
    n_eq += key == T;
  }
  int tot;
  const int eq_before = block_excl_scan(n_eq, s_wave, &tot);
  int eq_take = need_eq - eq_before;
  eq_take = eq_take < 0 ? 0 : (eq_take > n_eq ? n_eq : eq_take);
  int pos = block_excl_scan(n_gt + eq_take, s_wave, &tot);
  for (int i = r0; i < r1; ++i) {
    const uint32_t key = order_key(s_sc[i]);
    bool keep = key > T;
    if (key == T && eq_take > 0) {
      keep = true;
      --eq_take;
    }
    if (keep) s_sel[pos++] = i;
  }
  __syncthreads();
  if (a.sel_out)
    for (int e = tid; e < a.topk; e += 256) a.sel_out[(int64_t)hid * a.topk + e] = e < topk ? s_sel[e] : -1;

  // ---- phase 3: gather the kept V rows.  Lane = (row slot rs, 8-byte piece pc of the row).
  const int rs = lane / LPR, pc = lane - rs * LPR;
  float o[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) o[e] = 0.f;
  float mterm = 0.f;
  for (int e0 = wave * RPI; e0 < topk; e0 += 4 * RPI) {
    const int e = e0 + rs;
    const bool valid = e < topk;
    const int row = s_sel[valid ? e : topk - 1];
    const float p = valid ? fast_exp2((s_sc[row] - M) * kLog2e) * inv_den : 0.f;
    const int64_t ri = rowidx(row);
    const uint2 cw = *reinterpret_cast<const uint2*>(vc + ri * (DH / 2) + pc * 8);
    const float2 mt = meta_f32(vm[ri * GPR + (pc >> 2)]);
    const float w = p * mt.y;
    const float w24 = w * 16777216.0f, w20 = w * 1048576.0f;   // nibbles are read as FP16 subnormals
    mterm += p * mt.x;
    const uint32_t xs[2] = {cw.x, cw.y};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const uint32_t x = xs[u], y = x >> 8;
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
  // lanes with the same piece add up over the row slots, then the four waves through LDS
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    float v = o[e] + mterm;
#pragma unroll
    for (int d = LPR; d < 64; d <<= 1) v += __shfl_xor(v, d, 64);
    o[e] = v;
  }
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < 16; ++e) s_o[wave * DH + 16 * pc + e] = o[e];
  }
  __syncthreads();
  if (tid < DH)
    a.out[(int64_t)hid * DH + tid] = (half_t)(s_o[tid] + s_o[DH + tid] + s_o[2 * DH + tid] + s_o[3 * DH + tid]);
}

constexpr int kMaxLdsWords = 36 * 1024;   // score array + index list, 4 bytes each (144 KiB)

}  // namespace

static int topk_launch(TopkArgs& a, int dh, bool h16, bool paged, int64_t heads, hipStream_t stream) {
  if ((int64_t)a.rows_pad + a.topk > kMaxLdsWords) return FG_ERR_UNSUPPORTED;
  const size_t smem = ((size_t)a.rows_pad + a.topk) * 4;
  const dim3 grid((unsigned)heads);
  const int variant = (paged ? 4 : 0) + (dh == 128 ? 2 : 0) + (h16 ? 1 : 0);
  typedef void (*kernel_t)(TopkArgs);
  static const kernel_t kernels[8] = {
      attn_decode_topk_q4_kernel<64, false>,        attn_decode_topk_q4_kernel<64, true>,
      attn_decode_topk_q4_kernel<128, false>,       attn_decode_topk_q4_kernel<128, true>,
      attn_decode_topk_q4_kernel<64, false, true>,  attn_decode_topk_q4_kernel<64, true, true>,
      attn_decode_topk_q4_kernel<128, false, true>, attn_decode_topk_q4_kernel<128, true, true>};
  static bool attr_done[8] = {false, false, false, false, false, false, false, false};
  if (!attr_done[variant]) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[variant]),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsWords * 4));
    attr_done[variant] = true;
  }
  ProfScope prof(FG_K_ATTN_DECODE, stream);
  hipLaunchKernelGGL(kernels[variant], grid, dim3(256), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int decode_attention_topk_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b, int32_t rows,
                                 int32_t topk, const fg_kv_cache& kv, int32_t batch_offset, half_t* out,
                                 int32_t* sel_out, hipStream_t stream) {
  if (b == 0) return FG_OK;
  const int dh = cfg.h1 / cfg.nh;
  const int rpc = dh == 128 ? 64 : 128;
  TopkArgs a;
  a.q = q;
  a.q_stride = q_stride;
  a.k_codes = reinterpret_cast<const uint8_t*>(kv.k_codes);
  a.v_codes = reinterpret_cast<const uint8_t*>(kv.v_codes);
  a.k_meta = kv.k_meta;
  a.v_meta = kv.v_meta;
  a.out = out;
  a.sel_out = sel_out;
  a.nh = cfg.nh;
  a.cap = kv.cap;
  a.rows = rows;
  a.topk = topk;
  a.batch_offset = batch_offset;
  a.rows_pad = (int)(ceil_div(rows, rpc) * rpc);
  a.scale = 1.0f / sqrtf((float)dh);
  a.page_table = a.seq_ids = a.seq_rows = nullptr;
  a.table_stride = a.n_seqs = a.n_pages = a.rows_bias = 0;
  return topk_launch(a, dh, kv.dtype == FG_Q4G64_H16, false, (int64_t)b * cfg.nh, stream);
}

// Paged cache, a length per sequence: the score array in LDS is sized for the longest sequence the page
// table can address.
int decode_attention_topk_paged_launch(const fg_model_cfg& cfg, const half_t* q, int64_t q_stride, int32_t b,
                                       int32_t topk, const fg_kv_pages& pages, const fg_ragged& seqs,
                                       int32_t rows_bias, half_t* out, int32_t* sel_out, hipStream_t stream) {
  if (b == 0) return FG_OK;
  const int dh = cfg.h1 / cfg.nh;
  const int rpc = dh == 128 ? 64 : 128;
  TopkArgs a;
  a.q = q;
  a.q_stride = q_stride;
  a.k_codes = reinterpret_cast<const uint8_t*>(pages.k_codes);
  a.v_codes = reinterpret_cast<const uint8_t*>(pages.v_codes);
  a.k_meta = pages.k_meta;
  a.v_meta = pages.v_meta;
  a.out = out;
  a.sel_out = sel_out;
  a.nh = cfg.nh;
  a.cap = 0;
  a.rows = 0;
  a.topk = topk;
  a.batch_offset = 0;
  a.rows_pad = (int)(ceil_div((int64_t)seqs.table_stride * FG_PAGE_ROWS, rpc) * rpc);
  a.scale = 1.0f / sqrtf((float)dh);
  a.page_table = seqs.page_table;
  a.seq_ids = seqs.seq_ids;
  a.seq_rows = seqs.pos;
  a.table_stride = seqs.table_stride;
  a.n_seqs = seqs.n_seqs;
  a.n_pages = pages.n_pages;
  a.rows_bias = rows_bias;
  return topk_launch(a, dh, pages.dtype == FG_Q4G64_H16, true, (int64_t)b * cfg.nh, stream);
}

}  // namespace fg

using namespace fg;

extern "C" int fg_decode_attention_topk(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                                        int32_t rows, int32_t topk, const fg_kv_cache* kv, int32_t batch_offset,
                                        void* out_f16, int32_t* kept_rows, void* stream) {
  if (!cfg || !kv) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_kv(cfg, kv);
  if (rc) return rc;
  if (kv->dtype != FG_Q4G64 && kv->dtype != FG_Q4G64_H16) return FG_ERR_UNSUPPORTED;
  if (b < 0 || rows < 1 || rows > kv->cap || batch_offset < 0 || (int64_t)batch_offset + b > kv->batch)
    return FG_ERR_SHAPE;
  if (topk < 1 || topk > rows) return FG_ERR_SHAPE;
  if (q_row_stride < cfg->h1 || q_row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0) return FG_OK;
  if (!q_f16 || !out_f16) return FG_ERR_NULL;
  return decode_attention_topk_launch(*cfg, reinterpret_cast<const half_t*>(q_f16), q_row_stride, b, rows, topk, *kv,
                                      batch_offset, reinterpret_cast<half_t*>(out_f16), kept_rows, as_stream(stream));
}

extern "C" int fg_decode_attention_topk_paged(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride,
                                              int32_t b, int32_t topk, const fg_kv_pages* pages,
                                              const fg_ragged* seqs, int32_t rows_bias, void* out_f16,
                                              int32_t* kept_rows, void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rc = check_pages(cfg, pages, seqs);
  if (rc) return rc;
  if (pages->dtype != FG_Q4G64 && pages->dtype != FG_Q4G64_H16) return FG_ERR_UNSUPPORTED;
  if (!seqs->pos) return FG_ERR_NULL;
  if (b < 0 || rows_bias < 0 || topk < 1) return FG_ERR_SHAPE;
  if (q_row_stride < cfg->h1 || q_row_stride % 8 != 0) return FG_ERR_SHAPE;
  if (b == 0) return FG_OK;
  if (!q_f16 || !out_f16) return FG_ERR_NULL;
  return decode_attention_topk_paged_launch(*cfg, reinterpret_cast<const half_t*>(q_f16), q_row_stride, b, topk, *pages,
                                            *seqs, rows_bias, reinterpret_cast<half_t*>(out_f16), kept_rows,
                                            as_stream(stream));
}
