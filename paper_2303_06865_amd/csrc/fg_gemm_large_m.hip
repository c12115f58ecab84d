// Fused dequant + MFMA GEMM for the prefill-phase projections (Section 3, prefill: x.wQ, x.wK,
// x.wV, .wO, .w1, .w2 over b*s rows, weights stored as in Section 5).
//
// out[M, N] = act(x[M, K] . W[N, K]^T + bias) + residual,  M large (thousands of rows)
//
// Design (gfx950): 256x256 output tile per workgroup, four waves in a 2x2 arrangement, each wave
// owning 128x128 = 4x4 v_mfma_f32_32x32x16_f16 tiles (256 accumulator registers).  A K step is 64
// elements = one quantization group: the activation tile goes global -> registers -> LDS; the
// weight tile goes global (4-bit codes + one {min,scale} per row) -> registers -> dequantized FP16
// -> LDS, so compressed weights never exist as FP16 in HBM.  Two LDS stages; global loads of step
// k+1 are issued before the MFMAs of step k.  Tiles are walked in an order that keeps the 32
// workgroups resident on one XCD inside an 8x4 patch of tiles, so its L2 sees 12 panel streams
// instead of 64.
#include "fg_common.h"

namespace fg {

namespace {

constexpr int BM = 256, BN = 256, KS = 64;
constexpr int LDT = 72;                       // LDS row pitch in halves (64 + 8)
constexpr int STAGE = BM * LDT;               // halves per operand per stage
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

template <bool Q4>
__global__ __launch_bounds__(256) void gemm_large_m_kernel(LargeArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  half_t* As = reinterpret_cast<half_t*>(smem_raw);   // [2][BM][LDT]
  half_t* Bs = As + 2 * STAGE;                        // [2][BN][LDT]

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

  // loader roles
  //   A (and FP16 B): 2048 16-byte chunks per step, 8 per thread: chunk id -> (row = id/8, kc = id%8)
  //   Q4 B: 512 chunks of 32 codes, 2 per thread: id -> (row = id/2, half = id%2)
  u4_t ga[8];
  u4_t gb[Q4 ? 2 : 8];
  float2 gm[2];

  auto gload = [&](int ks) {
    const int kk = ks * KS;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int id = tid + 256 * c;
      int row = m0 + (id >> 3);
      row = row < a.M ? row : a.M - 1;
      ga[c] = *reinterpret_cast<const u4_t*>(a.x + (int64_t)row * a.ldx + kk + (id & 7) * 8);
    }
    if (Q4) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int id = tid + 256 * c;
        int col = n0 + (id >> 1);
        col = col < a.N ? col : a.N - 1;
        gb[c] = *reinterpret_cast<const u4_t*>(a.w + (int64_t)col * (a.K >> 1) + (kk >> 1) + (id & 1) * 16);
        gm[c] = a.meta[(int64_t)col * (a.K >> 6) + ks];
      }
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int id = tid + 256 * c;
        int col = n0 + (id >> 3);
        col = col < a.N ? col : a.N - 1;
        gb[c] = *reinterpret_cast<const u4_t*>(a.w + ((int64_t)col * a.K + kk + (id & 7) * 8) * 2);
      }
    }
  };
  auto lstore = [&](int buf) {
    half_t* Ad = As + buf * STAGE;
    half_t* Bd = Bs + buf * STAGE;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int id = tid + 256 * c;
      const u4_t v = Q4 ? permute8_like_codes(ga[c]) : ga[c];
      *reinterpret_cast<u4_t*>(Ad + (id >> 3) * LDT + (id & 7) * 8) = v;
    }
    if (Q4) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int id = tid + 256 * c;
        const float s24 = gm[c].y * 16777216.0f, s20 = gm[c].y * 1048576.0f, mnf = gm[c].x;
        half_t* dst = Bd + (id >> 1) * LDT + (id & 1) * 32;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          h2_t cc[4];
          dequant8_exact(gb[c][u], s24, s20, mnf, cc);
          h8_t o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[2 * e] = cc[e].x;
            o[2 * e + 1] = cc[e].y;
          }
          *reinterpret_cast<h8_t*>(dst + u * 8) = o;
        }
      }
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int id = tid + 256 * c;
        *reinterpret_cast<u4_t*>(Bd + (id >> 3) * LDT + (id & 7) * 8) = gb[c];
      }
    }
  };

  const int nk = a.K / KS;
  gload(0);
  lstore(0);
  __syncthreads();
  int buf = 0;
  for (int ks = 0; ks < nk; ++ks) {
    const bool more = ks + 1 < nk;
    if (more) gload(ks + 1);
    const half_t* At = As + buf * STAGE + (wm * 128 + l32) * LDT + kb * 8;
    const half_t* Bt = Bs + buf * STAGE + (wn * 128 + l32) * LDT + kb * 8;
#pragma unroll
    for (int kk = 0; kk < KS / 16; ++kk) {
      h8_t aop[4], bop[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) aop[i] = *reinterpret_cast<const h8_t*>(At + i * 32 * LDT + kk * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) bop[j] = *reinterpret_cast<const h8_t*>(Bt + j * 32 * LDT + kk * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop[i], bop[j], acc[i][j], 0, 0, 0);
    }
    if (more) lstore(buf ^ 1);
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
  const size_t smem = (size_t)4 * STAGE * sizeof(half_t);
  const bool q4 = la.dtype == FG_Q4G64;
  static bool attr_done[2] = {false, false};
  if (!attr_done[q4]) {
    if (q4)
      FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_large_m_kernel<true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    else
      FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_large_m_kernel<false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_done[q4] = true;
  }
  ProfScope prof(FG_K_GEMM_LARGE_M, stream);
  if (q4)
    hipLaunchKernelGGL(gemm_large_m_kernel<true>, dim3(grid), dim3(256), smem, stream, a);
  else
    hipLaunchKernelGGL(gemm_large_m_kernel<false>, dim3(grid), dim3(256), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg
