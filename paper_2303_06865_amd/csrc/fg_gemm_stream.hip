// Decode-phase projections on TILED 4-bit weights (Section 3 decode: t.wQ, t.wK, t.wV, .wO, .w1, .w2;
// weights stored as in Section 5), and the one-time repacking that produces the tiled layout.
//
// Why a second layout: in the canonical row-major format the 64 codes one lane pair needs per K step
// are 32 bytes of a row, and neighbouring rows are K/2 bytes apart, so a weight-streaming kernel
// touches thousands of DRAM pages with 32..64-byte pieces.  FG_Q4G64_TILED stores, for every
// (32 output columns, 64 input elements) tile, the 1 KiB of codes in exactly the order the 64 lanes
// of a wavefront consume them as the B operand of v_mfma_f32_32x32x16_f16 (lane l: column l%32,
// codes k = 32*(l/32) .. +32), tiles of one column block consecutive along K.  A wave then streams
// contiguous kilobytes, like the decode attention does.  Same bytes, same 0.625 B/element.
//
// Kernel: out[M, N] = act(x[M, K] . W^T + bias) + residual for M <= 160 per row block.
//   * 4 waves, each owning 64 output columns (two 32-column tiles) and all rows: the activation tile
//     is copied global -> LDS asynchronously (4 stages, XOR-swizzled) and shared as the A operand;
//     weights go HBM -> registers -> exact FP16 (in registers) -> MFMA B operand, prefetched three K
//     steps ahead, so ~6 KiB per wave are in flight at any time.
//   * stream-K over a fixed grid with a deterministic second-pass reduction, as in the canonical
//     small-M kernel.
#include "fg_common.h"

namespace fg {

namespace {

constexpr int kBN = 256;      // output columns per workgroup (4 waves x 2 tiles x 32)
constexpr int kKS = 64;       // K elements per step = one quantization group
constexpr int kPD = 3;        // prefetch distance in K steps
constexpr int kNST = kPD + 1; // LDS stages of the activation tile
constexpr int kMaxMT = 5;     // 32-row tiles per workgroup tile (160 rows)

struct StreamArgs {
  const uint8_t* w;     // tiled codes
  const float2* meta;   // tiled {min, scale}
  const half_t* x;
  int64_t ldx;
  int M, N, K;
  int m_blocks, n_tiles, ksteps, n32;   // n32 = N / 32
  int64_t total_work;
  int grid;
  const half_t* bias;
  const half_t* residual;
  int64_t ldr;
  int relu;
  half_t* out16;
  float* out32;
  int64_t ldo;
  float* partial;       // [grid][2][MT*32][256]
};

__device__ __forceinline__ int64_t work_begin(int64_t total, int grid, int p) { return (total * p) / grid; }
__device__ __forceinline__ int swz(int row, int kc) { return kc ^ ((row >> 1) & 7); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int MT>
__global__ __launch_bounds__(256) void gemm_stream_kernel(StreamArgs a) {
  constexpr int kStage = MT * 32 * kKS;          // halves per LDS stage
  constexpr int kWait = (kPD - 1) * (MT + 4);    // VMEM ops a wave issues after the copies of a step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  half_t* As = reinterpret_cast<half_t*>(smem_raw);   // [kNST][MT*32][64]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kb = lane >> 5;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  int64_t pos = work_begin(a.total_work, a.grid, p);
  const int64_t pos_end = work_begin(a.total_work, a.grid, p + 1);
  int seg = 0;

  // operand read offsets inside a stage: lane (l32, kb) reads logical chunk 4*kb + kk of row 32*m + l32
  int a_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) a_off[kk] = l32 * kKS + swz(l32, 4 * kb + kk) * 8;

  while (pos < pos_end) {
    const int64_t tile = pos / a.ksteps;
    const int ks0 = (int)(pos - tile * a.ksteps);
    const int64_t left = pos_end - pos;
    const int ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    const int n_tile = (int)(tile / a.m_blocks);
    const int mblk = (int)(tile - (int64_t)n_tile * a.m_blocks);
    const int m0 = mblk * (MT * 32);
    const int nt0 = n_tile * 8 + wave * 2;   // first 32-column tile of this wave

    f16_t acc[MT][2];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][j][r] = 0.f;

    // this wave's MT async activation copies per step: copy c covers rows 8c .. 8c+7 of the tile
    const half_t* a_src[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int c = wave + 4 * i;
      const int prow = 8 * c + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    const uint8_t* w_src[2];
    const float2* m_src[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int nt = nt0 + j;
      nt = nt < a.n32 ? nt : a.n32 - 1;   // ragged last column block: load valid data, never store it
      w_src[j] = a.w + (int64_t)nt * a.ksteps * 1024 + lane * 16;
      m_src[j] = a.meta + (int64_t)nt * a.ksteps * 32 + l32;
    }

    u4_t bq[kPD][2];
    float2 bm[kPD][2];
    auto issue = [&](int ks, int stage, u4_t* q, float2* mm) {
      const int kc = ks < ks1 ? ks : ks1 - 1;   // past the end: harmless re-fetch, keeps VMEM counts uniform
#pragma unroll
      for (int i = 0; i < MT; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + kc * kKS),
                                         (lptr_t)(As + stage * kStage + (wave + 4 * i) * 8 * kKS), 16, 0, 0);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        q[j] = *reinterpret_cast<const u4_t*>(w_src[j] + (int64_t)kc * 1024);
        mm[j] = m_src[j][(int64_t)kc * 32];
      }
    };

    __syncthreads();   // the previous segment no longer reads any stage
#pragma unroll
    for (int t = 0; t < kPD; ++t) issue(ks0 + t, t, bq[t], bm[t]);

    int stage = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      // copies and weights of this step were issued kPD steps ago; everything issued since may still fly
      __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(kWait) : "memory");
      __syncthreads();
      u4_t cq[2] = {bq[0][0], bq[0][1]};
      float s24[2], s20[2], mn[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        s24[j] = bm[0][j].y * 16777216.0f;
        s20[j] = bm[0][j].y * 1048576.0f;
        mn[j] = bm[0][j].x;
      }
#pragma unroll
      for (int t = 0; t + 1 < kPD; ++t) {
        bq[t][0] = bq[t + 1][0];
        bq[t][1] = bq[t + 1][1];
        bm[t][0] = bm[t + 1][0];
        bm[t][1] = bm[t + 1][1];
      }
      int nstage = stage + kPD;
      nstage = nstage >= kNST ? nstage - kNST : nstage;
      issue(ks + kPD, nstage, bq[kPD - 1], bm[kPD - 1]);
      __builtin_amdgcn_sched_barrier(0);

      const half_t* At = As + stage * kStage;
      h8_t aop[2][MT];
      uint32_t bop[2][2][4];
#pragma unroll
      for (int m = 0; m < MT; ++m) aop[0][m] = *reinterpret_cast<const h8_t*>(At + m * 32 * kKS + a_off[0]);
#pragma unroll
      for (int j = 0; j < 2; ++j) dequant8_exact(cq[j][0], s24[j], s20[j], mn[j], bop[0][j]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int cur = kk & 1, nxt = cur ^ 1;
        if (kk < 3) {
#pragma unroll
          for (int m = 0; m < MT; ++m)
            aop[nxt][m] = *reinterpret_cast<const h8_t*>(At + m * 32 * kKS + a_off[kk + 1]);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const u4_t bw = {bop[cur][j][0], bop[cur][j][1], bop[cur][j][2], bop[cur][j][3]};
          const h8_t bv = __builtin_bit_cast(h8_t, bw);
#pragma unroll
          for (int m = 0; m < MT; ++m)
            acc[m][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop[cur][m], bv, acc[m][j], 0, 0, 0);
          if (kk < 3) {   // next slice's weights are dequantized in the shadow of these MFMAs
            __builtin_amdgcn_sched_barrier(0);
            dequant8_exact(cq[j][kk + 1], s24[j], s20[j], mn[j], bop[nxt][j]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      stage = stage + 1 == kNST ? 0 : stage + 1;
    }

    // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*kb + r%4
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    if (full) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = (nt0 + j) * 32 + l32;
        if (nt0 + j < a.n32) {
          const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int row = m0 + m * 32 + (r >> 2) * 8 + kb * 4 + (r & 3);
              if (row < a.M) {
                float v = acc[m][j][r] + bvv;
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
      float* dst = a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * (MT * 32 * kBN);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int cl = (wave * 2 + j) * 32 + l32;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[(m * 32 + (r >> 2) * 8 + kb * 4 + (r & 3)) * kBN + cl] = acc[m][j][r];
      }
    }
    pos += ks1 - ks0;
    ++seg;
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may still target LDS when the wave ends
}

// Second pass of the stream-K schedule: tiles whose K range was shared get their partial sums added
// in ascending K order, then the epilogue.  One thread per four columns.
__global__ __launch_bounds__(256) void gemm_stream_finish_kernel(StreamArgs a, int mt) {
  const int64_t tile = blockIdx.x;
  const int64_t w0 = tile * a.ksteps, w1 = w0 + a.ksteps;
  int p_lo = (int)((w0 * a.grid) / a.total_work);
  while (p_lo + 1 < a.grid && work_begin(a.total_work, a.grid, p_lo + 1) <= w0) ++p_lo;
  while (p_lo > 0 && work_begin(a.total_work, a.grid, p_lo) > w0) --p_lo;
  if (work_begin(a.total_work, a.grid, p_lo + 1) >= w1) return;   // one workgroup owned the whole tile
  int p_hi = p_lo;
  while (p_hi + 1 < a.grid && work_begin(a.total_work, a.grid, p_hi + 1) < w1) ++p_hi;

  const int n_tile = (int)(tile / a.m_blocks);
  const int mblk = (int)(tile - (int64_t)n_tile * a.m_blocks);
  const int rows_t = mt * 32;
  const int m0 = mblk * rows_t;
  const int64_t slot = (int64_t)rows_t * kBN;
  const int n_quads = rows_t * (kBN / 4);
  for (int e = threadIdx.x + blockIdx.y * 256; e < n_quads; e += 256 * gridDim.y) {
    const int r = e / (kBN / 4), c = (e - r * (kBN / 4)) * 4;
    const int row = m0 + r, col = n_tile * kBN + c;
    if (row >= a.M || col >= a.N) continue;   // N % 32 == 0, so a quad is inside or outside as a whole
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = p_lo; p <= p_hi; ++p) {
      const int64_t pb = work_begin(a.total_work, a.grid, p);
      if (work_begin(a.total_work, a.grid, p + 1) == pb) continue;
      const int s = pb >= w0 ? 0 : 1;
      const float4 t = *reinterpret_cast<const float4*>(a.partial + ((int64_t)p * 2 + s) * slot + (int64_t)r * kBN + c);
      v.x += t.x;
      v.y += t.y;
      v.z += t.z;
      v.w += t.w;
    }
    float o[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (a.bias) o[i] += (float)a.bias[col + i];
      if (a.relu) o[i] = fmaxf(o[i], 0.f);
      if (a.residual) o[i] += (float)a.residual[(int64_t)row * a.ldr + col + i];
    }
    if (a.out32) {
      *reinterpret_cast<float4*>(a.out32 + (int64_t)row * a.ldo + col) = make_float4(o[0], o[1], o[2], o[3]);
    } else {
      h4_t h = {(half_t)o[0], (half_t)o[1], (half_t)o[2], (half_t)o[3]};
      *reinterpret_cast<h4_t*>(a.out16 + (int64_t)row * a.ldo + col) = h;
    }
  }
}

// canonical [N][K/2] codes + [N][K/64] meta  ->  tiled: one thread per 16-byte piece
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint8_t* __restrict__ codes,
                                                           const float2* __restrict__ meta, int N, int K,
                                                           uint8_t* __restrict__ codes_out,
                                                           float2* __restrict__ meta_out) {
  const int ksteps = K >> 6;
  const int64_t pieces = (int64_t)N * ksteps * 2;   // 16-byte pieces
  int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; id < pieces; id += stride) {
    const int lane = (int)(id & 63);
    const int64_t t = id >> 6;               // tile index = nt * ksteps + ks
    const int ks = (int)(t % ksteps);
    const int64_t nt = t / ksteps;
    const int col = (int)(nt * 32) + (lane & 31), kbb = lane >> 5;
    const u4_t v = *reinterpret_cast<const u4_t*>(codes + (int64_t)col * (K >> 1) + ks * 32 + kbb * 16);
    *reinterpret_cast<u4_t*>(codes_out + id * 16) = v;
    if (kbb == 0) meta_out[t * 32 + (lane & 31)] = meta[(int64_t)col * ksteps + ks];
  }
}

int pick_mt(int64_t m) {
  if (m > kMaxMT * 32) {
    const int64_t blocks = ceil_div(m, kMaxMT * 32);
    m = ceil_div(m, blocks);
  }
  const int need = (int)ceil_div(m, 32);
  return need < 1 ? 1 : (need > kMaxMT ? kMaxMT : need);
}

template <int MT>
int launch_t(const StreamArgs& a, hipStream_t stream) {
  const size_t smem = (size_t)kNST * MT * 32 * kKS * sizeof(half_t);
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_stream_kernel<MT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_stream_kernel<MT>), dim3(a.grid), dim3(256), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace

size_t gemm_stream_workspace(int64_t n, int64_t k, int64_t m) {
  (void)n;
  (void)k;
  if (m <= 0) return 0;
  return (size_t)256 * 2 * pick_mt(m) * 32 * kBN * sizeof(float);
}

int gemm_stream_launch(const LinearArgs& la, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (la.m == 0 || la.n == 0) return FG_OK;
  const int mt = pick_mt(la.m);
  StreamArgs a;
  a.w = reinterpret_cast<const uint8_t*>(la.w_data);
  a.meta = reinterpret_cast<const float2*>(la.w_meta);
  a.x = la.x;
  a.ldx = la.ldx;
  a.M = (int)la.m;
  a.N = (int)la.n;
  a.K = (int)la.k;
  a.m_blocks = (int)ceil_div(la.m, mt * 32);
  a.n_tiles = (int)ceil_div(la.n, kBN);
  a.ksteps = (int)(la.k / kKS);
  a.n32 = (int)(la.n / 32);
  a.total_work = (int64_t)a.m_blocks * a.n_tiles * a.ksteps;
  a.grid = 256;
  a.bias = la.bias;
  a.residual = la.residual;
  a.ldr = la.ldr;
  a.relu = la.relu;
  a.out16 = la.out_f16;
  a.out32 = la.out_f32;
  a.ldo = la.ldo;
  a.partial = reinterpret_cast<float*>(ws);
  const size_t need = gemm_stream_workspace(la.n, la.k, la.m);
  if (!ws || ws_bytes < need) return FG_ERR_WORKSPACE;
  {
    ProfScope prof(FG_K_GEMM_SMALL_M, stream);
    int rc = FG_ERR_UNSUPPORTED;
    switch (mt) {
      case 1: rc = launch_t<1>(a, stream); break;
      case 2: rc = launch_t<2>(a, stream); break;
      case 3: rc = launch_t<3>(a, stream); break;
      case 4: rc = launch_t<4>(a, stream); break;
      case 5: rc = launch_t<5>(a, stream); break;
    }
    if (rc) return rc;
  }
  {
    ProfScope prof(FG_K_GEMM_SMALL_M_FINISH, stream);
    hipLaunchKernelGGL(gemm_stream_finish_kernel, dim3(a.m_blocks * a.n_tiles, mt >= 3 ? 4 : 2), dim3(256), 0, stream,
                       a, mt);
    FG_LAUNCH_CHECK();
  }
  return FG_OK;
}

int pack_weights_launch(const void* codes, const void* meta, int64_t n, int64_t k, void* codes_out, void* meta_out,
                        hipStream_t stream) {
  const int64_t pieces = n * (k / 64) * 2;
  int64_t blocks = ceil_div(pieces, 256);
  if (blocks > 256 * 64) blocks = 256 * 64;
  ProfScope prof(FG_K_QUANTIZE, stream);
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     reinterpret_cast<const uint8_t*>(codes), reinterpret_cast<const float2*>(meta), (int)n, (int)k,
                     reinterpret_cast<uint8_t*>(codes_out), reinterpret_cast<float2*>(meta_out));
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg
