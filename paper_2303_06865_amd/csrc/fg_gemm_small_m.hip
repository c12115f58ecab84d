// Fused dequant + GEMM for the decode-phase projections (Section 3: t.wQ, t.wK, t.wV, .wO, .w1, .w2
// with the weights stored as in Section 5), for a small number of activation rows M (the block
// of sequences in a decode step), on weights in the CANONICAL row-major 4-bit format, and on FP16
// weights whose shape the streaming kernels do not take (N % 32 != 0, or 320 < M <= 512).  Tiled
// 4-bit weights and the common FP16 cases go through fg_gemm_stream.hip, which is faster: in the
// canonical format the 32 bytes a lane pair needs per K step lie K/2 bytes apart from row to row.
//
// out[M, N] = act(x[M, K] . W[N, K]^T + bias) + residual
//
// Design (gfx950):
//   * The weight matrix is streamed from HBM exactly once, straight into registers, 16 bytes per
//     lane; 4-bit codes are dequantized to FP16 in registers (exactly: one rounding of
//     min + code * scale; never through LDS or HBM) and fed to
//     v_mfma_f32_16x16x32_f16 as the B operand.  The activation tile (all M rows x 128 K) is
//     staged in LDS once per workgroup and shared by its four waves as the A operand.
//   * A workgroup covers 256 output columns (4 waves x 4 column tiles of 16), so each A-operand
//     read from LDS feeds four MFMAs.
//   * Work is the flattened list of (output tile, K step) pairs, cut into equal contiguous ranges,
//     one per workgroup of a fixed-size grid ("stream-K"): every CU streams the same number of
//     weight bytes whatever N is.  A tile whose K range is shared by several workgroups is
//     reduced in a fixed order by a second small kernel, so results are deterministic.
#include "fg_common.h"

namespace fg {

namespace {

constexpr int kBN = 256;        // output columns per workgroup
constexpr int kNTW = 4;         // 16-column tiles per wave
constexpr int kLdA = 136;       // LDS row pitch in halves (128 + 8: conflict-free 16-byte reads)
constexpr int kMaxMT = 10;      // at most 160 rows per tile

struct SmallArgs {
  const uint8_t* w;       // codes or FP16 values
  const float2* meta;     // Q4 only
  const half_t* x;
  int64_t ldx;
  int M, N, K;
  int m_blocks;           // tiles along M
  int n_tiles;            // tiles along N
  int ksteps;             // K steps per tile
  int64_t total_work;     // m_blocks * n_tiles * ksteps
  int grid;               // number of workgroups sharing total_work
  // epilogue
  const half_t* bias;
  const half_t* residual;
  int64_t ldr;
  int relu;
  half_t* out16;
  float* out32;
  int64_t ldo;
  float* partial;         // [grid][2][MT*16][256]
};

__device__ __forceinline__ int64_t work_begin(int64_t total, int grid, int p) {
  return (total * p) / grid;
}

template <bool Q4>
struct Cfg {
  static constexpr int KS = Q4 ? 128 : 64;   // K elements per step
  static constexpr int NSUB = KS / 32;       // MFMA K-substeps per step
};

template <int MT, bool Q4>
__global__ __launch_bounds__(256) void gemm_small_m_kernel(SmallArgs a) {
  constexpr int KS = Cfg<Q4>::KS;
  constexpr int NSUB = Cfg<Q4>::NSUB;
  constexpr int CPR = KS / 8;                 // 16-byte chunks per A row per step
  constexpr int NCH = MT * 16 * CPR;          // A chunks per step
  constexpr int ACH = (NCH + 255) / 256;      // A chunks per thread per step (last one may be idle)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  half_t* As = reinterpret_cast<half_t*>(smem_raw);          // [2][MT*16][kLdA]
  constexpr int kStage = MT * 16 * kLdA;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ln = lane & 15;    // row of A / column of B inside a 16x16 tile
  const int kb4 = lane >> 4;   // which 8-wide K block of the MFMA this lane feeds

  // XCD-aware placement: consecutive work ranges go to workgroups that share an XCD (and its L2).
  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  int64_t pos = work_begin(a.total_work, a.grid, p);
  const int64_t pos_end = work_begin(a.total_work, a.grid, p + 1);
  int seg = 0;

  while (pos < pos_end) {
    const int64_t tile = pos / a.ksteps;
    const int ks0 = (int)(pos - tile * a.ksteps);
    const int64_t left = pos_end - pos;
    const int ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    const int n_tile = (int)(tile / a.m_blocks);
    const int mblk = (int)(tile - (int64_t)n_tile * a.m_blocks);
    const int m0 = mblk * (MT * 16);
    const int n0 = n_tile * kBN + wave * (kNTW * 16);

    f4_t acc[MT][kNTW];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int j = 0; j < kNTW; ++j) acc[m][j] = (f4_t){0.f, 0.f, 0.f, 0.f};

    // per-lane weight row pointers (columns clamped so that loads stay inside the matrix)
    const uint8_t* wrow[kNTW];
    const float2* mrow[kNTW];
#pragma unroll
    for (int j = 0; j < kNTW; ++j) {
      int col = n0 + j * 16 + ln;
      col = col < a.N ? col : a.N - 1;
      if (Q4) {
        wrow[j] = a.w + (int64_t)col * (a.K >> 1);
        mrow[j] = a.meta + (int64_t)col * (a.K >> 6);
      } else {
        wrow[j] = a.w + (int64_t)col * a.K * 2;
        mrow[j] = nullptr;
      }
    }

    u4_t bq[kNTW][Q4 ? 1 : NSUB];   // weight words of the current step
    float2 bm[kNTW];
    u4_t aq[ACH];                   // activation chunks in flight to LDS

    auto load_b = [&](int ks) {
      const int kk = ks * KS;
#pragma unroll
      for (int j = 0; j < kNTW; ++j) {
        if (Q4) {
          int k = kk + 32 * kb4;
          k = k < a.K ? k : a.K - 32;           // tail step of a K that is 64 mod 128: A is zero there
          bq[j][0] = *reinterpret_cast<const u4_t*>(wrow[j] + (k >> 1));
          bm[j] = mrow[j][k >> 6];
        } else {
#pragma unroll
          for (int i = 0; i < NSUB; ++i) {
            const int k = kk + 32 * i + 8 * kb4;   // K % 64 == 0 and KS == 64: always in range
            bq[j][i] = *reinterpret_cast<const u4_t*>(wrow[j] + (int64_t)k * 2);
          }
        }
      }
    };
    auto load_a = [&](int ks) {
      const int kk = ks * KS;
#pragma unroll
      for (int c = 0; c < ACH; ++c) {
        const int id = tid + 256 * c;
        const int row = id / CPR, kc = id % CPR;
        int gr = m0 + row;
        gr = gr < a.M ? gr : a.M - 1;
        const int k = kk + kc * 8;
        if (k < a.K && id < NCH) {
          aq[c] = *reinterpret_cast<const u4_t*>(a.x + (int64_t)gr * a.ldx + k);
        } else {
          aq[c] = (u4_t){0u, 0u, 0u, 0u};
        }
      }
    };
    auto store_a = [&](int buf) {
#pragma unroll
      for (int c = 0; c < ACH; ++c) {
        const int id = tid + 256 * c;
        const int row = id / CPR, kc = id % CPR;
        const u4_t v = aq[c];
        if (id < NCH) *reinterpret_cast<u4_t*>(As + buf * kStage + row * kLdA + kc * 8) = v;
      }
    };

    // prologue
    load_a(ks0);
    load_b(ks0);
    __syncthreads();   // previous segment's readers are done with both LDS stages
    store_a(0);
    __syncthreads();

    int buf = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      // operands of this step, moved out of the prefetch registers
      u4_t bcur[kNTW][Q4 ? 1 : NSUB];
      float s24[kNTW], s20[kNTW], mnf[kNTW];
#pragma unroll
      for (int j = 0; j < kNTW; ++j) {
#pragma unroll
        for (int i = 0; i < (Q4 ? 1 : NSUB); ++i) bcur[j][i] = bq[j][i];
        if (Q4) {
          s24[j] = bm[j].y * 16777216.0f;
          s20[j] = bm[j].y * 1048576.0f;
          mnf[j] = bm[j].x;
        }
      }
      const bool more = ks + 1 < ks1;
      if (more) {
        load_a(ks + 1);
        load_b(ks + 1);
      }
      const half_t* At = As + buf * kStage;
#pragma unroll
      for (int i = 0; i < NSUB; ++i) {
        h8_t aop[MT];
        const int koff = Q4 ? (32 * kb4 + 8 * i) : (32 * i + 8 * kb4);
#pragma unroll
        for (int m = 0; m < MT; ++m)
          aop[m] = *reinterpret_cast<const h8_t*>(At + (m * 16 + ln) * kLdA + koff);
#pragma unroll
        for (int j = 0; j < kNTW; ++j) {
          h8_t bop;
          if (Q4) {
            uint32_t c[4];
            dequant8_exact(bcur[j][0][i], s24[j], s20[j], mnf[j], c);
            const u4_t cw = {c[0], c[1], c[2], c[3]};
            bop = __builtin_bit_cast(h8_t, cw);
          } else {
            bop = __builtin_bit_cast(h8_t, bcur[j][i]);
          }
#pragma unroll
          for (int m = 0; m < MT; ++m)
            acc[m][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aop[m], bop, acc[m][j], 0, 0, 0);
        }
      }
      if (more) store_a(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }

    // ---- epilogue of this segment
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    if (full) {
#pragma unroll
      for (int j = 0; j < kNTW; ++j) {
        const int col = n0 + j * 16 + ln;
        if (col < a.N) {
          const float bv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int row = m0 + m * 16 + kb4 * 4 + r;
              if (row < a.M) {
                float v = acc[m][j][r] + bv;
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
    } else {
      float* dst = a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * (MT * 16 * kBN);
#pragma unroll
      for (int j = 0; j < kNTW; ++j) {
        const int cl = wave * (kNTW * 16) + j * 16 + ln;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int r = 0; r < 4; ++r) dst[(m * 16 + kb4 * 4 + r) * kBN + cl] = acc[m][j][r];
      }
    }
    pos += ks1 - ks0;
    ++seg;
  }
}

// Second pass of the stream-K schedule: every tile whose K range was shared by several workgroups
// gets its partial sums added in ascending K order, then the epilogue.
__global__ __launch_bounds__(256) void gemm_small_m_finish_kernel(SmallArgs a, int mt) {
  const int64_t tile = blockIdx.x;
  const int64_t w0 = tile * a.ksteps, w1 = w0 + a.ksteps;
  // workgroups whose range intersects [w0, w1): p_lo = last p with begin(p) <= w0
  int p_lo = (int)((w0 * a.grid) / a.total_work);
  while (p_lo + 1 < a.grid && work_begin(a.total_work, a.grid, p_lo + 1) <= w0) ++p_lo;
  while (p_lo > 0 && work_begin(a.total_work, a.grid, p_lo) > w0) --p_lo;
  if (work_begin(a.total_work, a.grid, p_lo + 1) >= w1) return;   // one workgroup owned the whole tile
  int p_hi = p_lo;
  while (p_hi + 1 < a.grid && work_begin(a.total_work, a.grid, p_hi + 1) < w1) ++p_hi;

  const int n_tile = (int)(tile / a.m_blocks);
  const int mblk = (int)(tile - (int64_t)n_tile * a.m_blocks);
  const int rows_t = mt * 16;
  const int m0 = mblk * rows_t;
  const int64_t slot = (int64_t)rows_t * kBN;
  for (int e = threadIdx.x + blockIdx.y * 256; e < rows_t * kBN; e += 256 * gridDim.y) {
    const int r = e / kBN, c = e - r * kBN;
    const int row = m0 + r, col = n_tile * kBN + c;
    if (row >= a.M || col >= a.N) continue;
    float v = 0.f;
    for (int p = p_lo; p <= p_hi; ++p) {
      const int64_t pb = work_begin(a.total_work, a.grid, p);
      if (work_begin(a.total_work, a.grid, p + 1) == pb) continue;   // a workgroup with no work
      const int s = pb >= w0 ? 0 : 1;
      v += a.partial[((int64_t)p * 2 + s) * slot + e];
    }
    if (a.bias) v += (float)a.bias[col];
    if (a.relu) v = fmaxf(v, 0.f);
    if (a.residual) v += (float)a.residual[(int64_t)row * a.ldr + col];
    if (a.out32)
      a.out32[(int64_t)row * a.ldo + col] = v;
    else
      a.out16[(int64_t)row * a.ldo + col] = (half_t)v;
  }
}

int pick_mt(int64_t m) {
  // number of 16-row tiles per workgroup tile; instantiated sizes only
  static const int sizes[] = {1, 2, 3, 4, 6, 8, 9, 10};
  if (m > kMaxMT * 16) {
    // several row blocks: balance them
    const int64_t blocks = ceil_div(m, kMaxMT * 16);
    m = ceil_div(m, blocks);
  }
  const int need = (int)ceil_div(m, 16);
  for (int s : sizes)
    if (s >= need) return s;
  return kMaxMT;
}

int pick_grid(int mt) { return mt >= 5 ? 256 : 512; }

template <int MT, bool Q4>
int launch_t(const SmallArgs& a, hipStream_t stream) {
  const size_t smem = (size_t)2 * MT * 16 * kLdA * sizeof(half_t);
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_small_m_kernel<MT, Q4>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_small_m_kernel<MT, Q4>), dim3(a.grid), dim3(256), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

template <bool Q4>
int launch_q(int mt, const SmallArgs& a, hipStream_t stream) {
  switch (mt) {
    case 1: return launch_t<1, Q4>(a, stream);
    case 2: return launch_t<2, Q4>(a, stream);
    case 3: return launch_t<3, Q4>(a, stream);
    case 4: return launch_t<4, Q4>(a, stream);
    case 6: return launch_t<6, Q4>(a, stream);
    case 8: return launch_t<8, Q4>(a, stream);
    case 9: return launch_t<9, Q4>(a, stream);
    case 10: return launch_t<10, Q4>(a, stream);
  }
  return FG_ERR_UNSUPPORTED;
}

}  // namespace

size_t gemm_small_m_workspace(int dtype, int64_t n, int64_t k, int64_t m) {
  (void)dtype;
  (void)n;
  (void)k;
  if (m <= 0) return 0;
  const int mt = pick_mt(m);
  return (size_t)pick_grid(mt) * 2 * mt * 16 * kBN * sizeof(float);
}

int gemm_small_m_launch(const LinearArgs& la, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (la.m == 0 || la.n == 0) return FG_OK;
  const bool q4 = la.dtype == FG_Q4G64;
  const int mt = pick_mt(la.m);
  SmallArgs a;
  a.w = reinterpret_cast<const uint8_t*>(la.w_data);
  a.meta = reinterpret_cast<const float2*>(la.w_meta);
  a.x = la.x;
  a.ldx = la.ldx;
  a.M = (int)la.m;
  a.N = (int)la.n;
  a.K = (int)la.k;
  a.m_blocks = (int)ceil_div(la.m, mt * 16);
  a.n_tiles = (int)ceil_div(la.n, kBN);
  const int ks = q4 ? 128 : 64;
  a.ksteps = (int)ceil_div(la.k, ks);
  a.total_work = (int64_t)a.m_blocks * a.n_tiles * a.ksteps;
  a.grid = pick_grid(mt);
  a.bias = la.bias;
  a.residual = la.residual;
  a.ldr = la.ldr;
  a.relu = la.relu;
  a.out16 = la.out_f16;
  a.out32 = la.out_f32;
  a.ldo = la.ldo;
  a.partial = reinterpret_cast<float*>(ws);
  const size_t need = gemm_small_m_workspace(la.dtype, la.n, la.k, la.m);
  if (need > 0 && (!ws || ws_bytes < need)) return FG_ERR_WORKSPACE;
  {
    ProfScope prof(FG_K_GEMM_SMALL_M, stream);
    const int rc = q4 ? launch_q<true>(mt, a, stream) : launch_q<false>(mt, a, stream);
    if (rc) return rc;
  }
  {
    ProfScope prof(FG_K_GEMM_SMALL_M_FINISH, stream);
    const int ysplit = mt >= 5 ? 4 : 1;
    hipLaunchKernelGGL(gemm_small_m_finish_kernel, dim3(a.m_blocks * a.n_tiles, ysplit), dim3(256), 0, stream, a,
                       mt);
    FG_LAUNCH_CHECK();
  }
  return FG_OK;
}

}  // namespace fg
