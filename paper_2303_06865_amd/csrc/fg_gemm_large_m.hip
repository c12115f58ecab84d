// Fused dequant + MFMA GEMM for the prefill-phase projections (Section 3, prefill: x.wQ, x.wK,
// x.wV, .wO, .w1, .w2 over b*s rows, weights stored as in Section 5), for FP16 weights and for 4-bit
// weights in the canonical row-major format.  Tiled 4-bit weights take fg_gemm_stream.hip instead.
//
// out[M, N] = act(x[M, K] . W[N, K]^T + bias) + residual,  M large (thousands of rows)
//
// Design (gfx950): 256x256 output tile per workgroup, four waves in a 2x2 arrangement, each wave
// owning 128x128 = 4x4 v_mfma_f32_32x32x16_f16 tiles (256 accumulator registers).  A K step is 64
// elements = one quantization group.  The activation tile (and an FP16 weight tile) is copied
// global -> LDS asynchronously, 16 bytes per lane, without passing through registers; a 4-bit
// weight tile goes global (codes + one {min,scale} per row) -> registers -> exact FP16 -> LDS, so
// compressed weights never exist as FP16 in HBM.  Two LDS stages, XOR-swizzled instead of padded;
// the copies of step k+1 are issued before the MFMAs of step k, the MFMA operands of K slice
// kk+1 are read from LDS under the MFMAs of slice kk, and the next weight tile is dequantized
// under them too.  Tiles are walked in an order that keeps the 32
// workgroups resident on one XCD inside an 8x4 patch of tiles, so its L2 sees 12 panel streams
// instead of 64.
#include "fg_common.h"

namespace fg {

namespace {

constexpr int BM = 256, BN = 256, KS = 64;
constexpr int STAGE = BM * KS;                // halves per operand per stage (no padding: swizzled)
constexpr int GROUP_M = 8;

struct LargeArgs {
  const uint8_t* w;
  const float2* meta;
  const half_t* x;
  int64_t ldx;
  int M, N, K;
  int tm, tn;
  const half_t* bias;
  const half_t* residual;
  int64_t ldr;
  int relu;
  half_t* out16;
  float* out32;
  int64_t ldo;
};

// LDS tiles are [256 rows][8 chunks of 8 halves] = 128 bytes per row.  Logical chunk kc of a row
// sits at physical chunk kc ^ ((row >> 1) & 7): sixteen consecutive rows reading the same logical
// chunk then touch sixteen different 16-byte columns of the 64 banks (measured: fewer bank-conflict
// cycles than the row & 7 map, and 1.6x the read rate of the unswizzled tile), without padding.
__device__ __forceinline__ int swz(int row, int kc) { return kc ^ ((row >> 1) & 7); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Asynchronous 16-byte-per-lane copy global -> LDS (no registers): lane l lands at lds_base + 16*l.
__device__ __forceinline__ void async_copy16(const void* g, half_t* lds_base) {
  __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)lds_base, 16, 0, 0);
}

// WF: weight format, 0 = FP16, 1 = 4-bit canonical (row-major codes); tiled 4-bit weights have their
// own kernel family (fg_gemm_stream.hip)
template <int WF>
__global__ __launch_bounds__(256) void gemm_large_m_kernel(LargeArgs a) {
  constexpr bool Q4 = WF != 0;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  half_t* As = reinterpret_cast<half_t*>(smem_raw);   // [2][BM][KS]
  half_t* Bs = As + 2 * STAGE;                        // [2][BN][KS]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, kb = lane >> 5;

  // tile walk: XCD-major, then groups of GROUP_M row tiles walked column by column
  const int per_xcd = gridDim.x >> 3;
  const int w = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (w >= a.tm * a.tn) return;
  const int per_group = GROUP_M * a.tn;
  const int grp = w / per_group;
  const int first_m = grp * GROUP_M;
  const int gsize = (a.tm - first_m) < GROUP_M ? (a.tm - first_m) : GROUP_M;
  const int in_g = w - grp * per_group;
  const int m_tile = first_m + in_g % gsize;
  const int n_tile = in_g / gsize;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  f16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- loader roles
  // Async copies: a wave instruction fills 8 consecutive LDS rows (64 lanes x 16 B); lane l holds
  // physical chunk l%8 of row l/8, i.e. logical chunk (l%8) ^ swizzle(row).  Wave w issues copies
  // c = 0..7 for rows (8w + c)*8 .. +8 of the tile.
  const int a_lrow = lane >> 3;
  const half_t* a_src[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int prow = (wave * 8 + c) * 8 + a_lrow;
    int row = m0 + prow;
    row = row < a.M ? row : a.M - 1;
    a_src[c] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
  }
  const half_t* bf_src[Q4 ? 1 : 8];
  if (!Q4) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int prow = (wave * 8 + c) * 8 + a_lrow;
      int col = n0 + prow;
      col = col < a.N ? col : a.N - 1;
      bf_src[c] = reinterpret_cast<const half_t*>(a.w) + (int64_t)col * a.K + swz(prow, lane & 7) * 8;
    }
  }
  // Q4 weights: 512 pieces of 32 codes per step, 2 per thread.  Piece id -> (tile row, half of the
  // 64-element K step): canonical layout (id/2, id%2); tiled layout: 32-column tile id/64, and
  // inside it the wavefront order of the tile (column id%32, half (id/32)%2), 1 KiB contiguous.
  u4_t gb[2];
  float2 gm[2];
  const uint8_t* bq_src[2];
  const float2* bm_src[2];
  int bq_row[2], bq_hb[2];
  constexpr int kBqStep = KS / 2;   // bytes between K steps
  constexpr int kBmStep = 1;        // pairs between K steps
  if (Q4) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int id = tid + 256 * c;
      bq_row[c] = id >> 1;
      bq_hb[c] = id & 1;
      int col = n0 + (id >> 1);
      col = col < a.N ? col : a.N - 1;
      bq_src[c] = a.w + (int64_t)col * (a.K >> 1) + (id & 1) * 16;
      bm_src[c] = a.meta + (int64_t)col * (a.K >> 6);
    }
  }

  auto issue_async = [&](int ks, int buf) {
    const int kk = ks * KS;
#pragma unroll
    for (int c = 0; c < 8; ++c) async_copy16(a_src[c] + kk, As + buf * STAGE + (wave * 8 + c) * 8 * KS);
    if (!Q4) {
#pragma unroll
      for (int c = 0; c < 8; ++c) async_copy16(bf_src[c] + kk, Bs + buf * STAGE + (wave * 8 + c) * 8 * KS);
    }
  };
  auto load_bq = [&](int ks) {
    if (Q4) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        gb[c] = *reinterpret_cast<const u4_t*>(bq_src[c] + (int64_t)ks * kBqStep);
        gm[c] = bm_src[c][(int64_t)ks * kBmStep];
      }
    }
  };
  // One eighth of the next weight tile (one word of 8 codes -> 8 FP16 weights -> LDS), cut into four
  // sub-steps of a few VALU instructions each so that every sub-step fits in the shadow of one MFMA.
  uint32_t dq_m[4], dq_r[4];
  float dq_s24 = 0.f, dq_s20 = 0.f, dq_mn = 0.f;
  auto dq_sub = [&](int buf, int piece, int sub) {
    if (!Q4) return;
    const int c = piece >> 2, u = piece & 3;
    const int row = bq_row[c], hb = bq_hb[c];
    if (sub == 0) {
      const uint32_t x = gb[c][u], y = x >> 8;
      dq_m[0] = x & 0x000F000Fu;
      dq_m[1] = x & 0x00F000F0u;
      dq_m[2] = y & 0x000F000Fu;
      dq_m[3] = y & 0x00F000F0u;
      dq_s24 = gm[c].y * 16777216.0f;
      dq_s20 = gm[c].y * 1048576.0f;
      dq_mn = gm[c].x;
    } else if (sub == 1 || sub == 2) {
      const h2_t ha = __builtin_bit_cast(h2_t, dq_m[0]), hb2 = __builtin_bit_cast(h2_t, dq_m[1]);
      const h2_t hc = __builtin_bit_cast(h2_t, dq_m[2]), hd = __builtin_bit_cast(h2_t, dq_m[3]);
      if (sub == 1) {
        const h2_t q0 = {(half_t)__builtin_fmaf((float)ha.x, dq_s24, dq_mn), (half_t)__builtin_fmaf((float)hb2.x, dq_s20, dq_mn)};
        const h2_t q1 = {(half_t)__builtin_fmaf((float)hc.x, dq_s24, dq_mn), (half_t)__builtin_fmaf((float)hd.x, dq_s20, dq_mn)};
        dq_r[0] = __builtin_bit_cast(uint32_t, q0);
        dq_r[1] = __builtin_bit_cast(uint32_t, q1);
      } else {
        const h2_t q2 = {(half_t)__builtin_fmaf((float)ha.y, dq_s24, dq_mn), (half_t)__builtin_fmaf((float)hb2.y, dq_s20, dq_mn)};
        const h2_t q3 = {(half_t)__builtin_fmaf((float)hc.y, dq_s24, dq_mn), (half_t)__builtin_fmaf((float)hd.y, dq_s20, dq_mn)};
        dq_r[2] = __builtin_bit_cast(uint32_t, q2);
        dq_r[3] = __builtin_bit_cast(uint32_t, q3);
      }
    } else {
      const u4_t o = {dq_r[0], dq_r[1], dq_r[2], dq_r[3]};
      *reinterpret_cast<u4_t*>(Bs + buf * STAGE + row * KS + swz(row, hb * 4 + u) * 8) = o;
    }
  };
  auto store_bq_piece = [&](int buf, int piece) {
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) dq_sub(buf, piece, sub);
  };

  // MFMA operand addresses: lane (l32, kb) reads chunk 2*kk + kb of rows wm*128 + i*32 + l32
  const int arow = wm * 128 + l32, brow = wn * 128 + l32;
  int a_off[4], b_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    a_off[kk] = arow * KS + swz(arow, 2 * kk + kb) * 8;   // (row + 32 i) has the same swizzle
    b_off[kk] = brow * KS + swz(brow, 2 * kk + kb) * 8;
  }

  const int nk = a.K / KS;
  load_bq(0);
  issue_async(0, 0);
#pragma unroll
  for (int pc = 0; pc < 8; ++pc) store_bq_piece(0, pc);
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int buf = 0;
  for (int ks = 0; ks < nk; ++ks) {
    // The last iteration re-fetches its own tile into the idle stage: no branch in the loop body.
    const int kn = ks + 1 < nk ? ks + 1 : ks;
    load_bq(kn);
    __builtin_amdgcn_sched_barrier(0);   // register loads first: they can then be awaited with the copies in flight
    issue_async(kn, buf ^ 1);
    const half_t* At = As + buf * STAGE;
    const half_t* Bt = Bs + buf * STAGE;
    h8_t aop[2][4], bop[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) aop[0][i] = *reinterpret_cast<const h8_t*>(At + a_off[0] + i * 32 * KS);
#pragma unroll
    for (int j = 0; j < 4; ++j) bop[0][j] = *reinterpret_cast<const h8_t*>(Bt + b_off[0] + j * 32 * KS);
    __builtin_amdgcn_sched_barrier(0);
    // The issue order below is pinned with scheduling fences: a wave issues in order, so whatever
    // is to overlap with an MFMA has to sit right behind it in the instruction stream.
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk < 3) {   // operands of the next K slice are fetched under this slice's MFMAs
#pragma unroll
        for (int i = 0; i < 4; ++i)
          aop[nxt][i] = *reinterpret_cast<const h8_t*>(At + a_off[kk + 1] + i * 32 * KS);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          bop[nxt][j] = *reinterpret_cast<const h8_t*>(Bt + b_off[kk + 1] + j * 32 * KS);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop[cur][i], bop[cur][j], acc[i][j], 0, 0, 0);
          // the next weight tile is dequantized under the MFMAs of slices 2 and 3: 32 sub-steps
          if (kk >= 2) {
            __builtin_amdgcn_sched_barrier(0);
            dq_sub(buf ^ 1, (kk - 2) * 4 + i, j);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // async copies of the next stage landed
    __syncthreads();
    buf ^= 1;
  }

  // epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*kb + r%4
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int col = n0 + wn * 128 + j * 32 + l32;
    if (col >= a.N) continue;
    const float bv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 128 + i * 32 + (r >> 2) * 8 + kb * 4 + (r & 3);
        if (row < a.M) {
          float v = acc[i][j][r] + bv;
          if (a.relu) v = fmaxf(v, 0.f);
          if (a.residual) v += (float)a.residual[(int64_t)row * a.ldr + col];
          if (a.out32)
            a.out32[(int64_t)row * a.ldo + col] = v;
          else
            a.out16[(int64_t)row * a.ldo + col] = (half_t)v;
        }
      }
    }
  }
}

}  // namespace

int gemm_large_m_launch(const LinearArgs& la, hipStream_t stream) {
  if (la.m == 0 || la.n == 0) return FG_OK;
  LargeArgs a;
  a.w = reinterpret_cast<const uint8_t*>(la.w_data);
  a.meta = reinterpret_cast<const float2*>(la.w_meta);
  a.x = la.x;
  a.ldx = la.ldx;
  a.M = (int)la.m;
  a.N = (int)la.n;
  a.K = (int)la.k;
  a.tm = (int)ceil_div(la.m, BM);
  a.tn = (int)ceil_div(la.n, BN);
  a.bias = la.bias;
  a.residual = la.residual;
  a.ldr = la.ldr;
  a.relu = la.relu;
  a.out16 = la.out_f16;
  a.out32 = la.out_f32;
  a.ldo = la.ldo;
  const int64_t tiles = (int64_t)a.tm * a.tn;
  const unsigned grid = (unsigned)(ceil_div(tiles, 8) * 8);
  const size_t smem = (size_t)4 * STAGE * sizeof(half_t);   // 128 KiB
  if (la.dtype != FG_F16 && la.dtype != FG_Q4G64) return FG_ERR_UNSUPPORTED;
  const int wf = la.dtype == FG_F16 ? 0 : 1;
  static bool attr_done[2] = {false, false};
  const void* fn = wf == 0 ? (const void*)&gemm_large_m_kernel<0> : (const void*)&gemm_large_m_kernel<1>;
  if (!attr_done[wf]) {
    FG_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_done[wf] = true;
  }
  ProfScope prof(FG_K_GEMM_LARGE_M, stream);
  if (wf == 0)
    hipLaunchKernelGGL(gemm_large_m_kernel<0>, dim3(grid), dim3(256), smem, stream, a);
  else
    hipLaunchKernelGGL(gemm_large_m_kernel<1>, dim3(grid), dim3(256), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg
