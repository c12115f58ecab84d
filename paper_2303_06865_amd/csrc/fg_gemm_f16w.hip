// Decode-phase projections on uncompressed (row-major FP16) weights with up to 128 rows of
// activations (Section 3: the decode-phase products with wQ, wK, wV, wO, w1, w2; Section 6's smaller
// models run without compression).  At this row count the product is bound by reading the weights once
// from HBM (128 flop per weight byte, under the machine's 312 flop/B), and at the sizes of a 6.7B-scale
// layer a projection is 30..130 MB, i.e. 4..17 us of HBM time: what decides the time is how the matrix
// is cut over the 256 CUs, not the matrix cores.
//
//   * Output tile = all rows x BN columns, BN = 16, 32, 48 or 64, chosen per launch (pick_cols) so that
//     the tiles are a multiple of 256 wherever the matrix allows it (N = 12288: 256 tiles of 48; 16384:
//     256 of 64; 4096 x 4096: 256 of 16): every CU then owns one tile over the whole contraction, nothing
//     is split along K, no partial sums are written and no reduction pass runs.  Narrow tiles have a
//     price: every workgroup pulls the whole activation block through its L1 (rows / BN times the bytes
//     of its weights), and a CU takes in only 45..55 GB/s of asynchronous copies; so for a long
//     contraction (4096 x 16384) wider tiles cut stream-K fashion into 256 equal ranges, with a small
//     deterministic reduction pass, are cheaper, and long ragged matrices (an LM head) stay on the
//     256-column kernel.  The choice is made with a cost model fitted to measurements (pick_cols).
//   * Both operands are [rows][64 k] tiles of 128-byte rows, copied global -> LDS asynchronously and
//     read back as MFMA operands with one ds_read_b128 each (XOR swizzle, conflict-free).  The weight
//     tiles, which come from HBM, sit in a ring of up to 10 K steps; the activation tiles, which come
//     from L2, in a ring of 5: one vmcnt wait per step covers both, because a step's weight copy is
//     always older than its activation copy.
//   * v_mfma_f32_16x16x32_f16; eight waves, wave w owns the 16-row tile w and all BN columns (the async
//     copies of a CU run faster issued from eight waves than from four).
#include <cstdlib>

#include "fg_common.h"
#include "fg_async_lds.h"

namespace fg {

namespace {

constexpr int kKS = 64;            // K elements per step: 128-byte rows in LDS
constexpr int kLds = 160 * 1024;
constexpr int kDA = 5;             // activation stages
constexpr int kGrid = 256;

struct F16wArgs {
  const half_t* w;      // [N, K] row-major
  const half_t* x;      // [M, K], row stride ldx
  int64_t ldx;
  int M, N, K;
  int n_tiles, ksteps;
  int rounds;           // whole rounds: tiles [0, rounds * 256) go one per workgroup per round
  int64_t rem_work;     // (remaining tiles) * ksteps, cut into 256 equal ranges
  const half_t* bias;
  const half_t* residual;
  int64_t ldr;
  int relu;
  half_t* out16;
  float* out32;
  int64_t ldo;
  float* partial;       // [256][2][128 rows x BN columns] in register order
};

constexpr int kNW = 8;             // waves per workgroup (two per SIMD): wave w owns the 16-row tile w

template <int MT32, int CT>
struct F16wCfg {
  static constexpr int kBN = CT * 16;
  static constexpr int kAC = (MT32 * 4 + kNW - 1) / kNW;   // activation copies (8 rows each) per wave per step
  static constexpr int kAStage = kNW * kAC * 8 * kKS * 2;  // room for every wave's pieces (>= MT32 * 32 rows)
  static constexpr int kWStage = kNW * 8 * kKS * 2;        // one weight piece per wave: 64 rows, BN of them used
  static constexpr int kDWmax = (kLds - kDA * kAStage) / kWStage;
  static constexpr int kDW = kDWmax > 10 ? 10 : kDWmax;    // weight stages
  static constexpr int kLdsBytes = kDA * kAStage + kDW * kWStage;
  static constexpr int kSlotRows = kNW * 16;               // rows of a partial-sum slot
  static_assert(kDW >= kDA, "the weight ring is at least as deep as the activation ring");
  static_assert((kDW - 1) + (kDA - 1) * kAC < 60, "more copies in flight than the counter holds");
};

template <int MT32, int CT>
__global__ __launch_bounds__(kNW * 64) void gemm_f16w_kernel(F16wArgs a) {
  using C = F16wCfg<MT32, CT>;
  constexpr int kAStage = C::kAStage, kWStage = C::kWStage, kDW = C::kDW, kAC = C::kAC, kBN = C::kBN;
  constexpr int kWBase = kDA * kAStage;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [kDA] A tiles | [kDW] W tiles

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;
  const int p = (blockIdx.x & 7) * (kGrid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, kGrid, p), rem_end = work_begin(a.rem_work, kGrid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  const bool has_w = wave < 2 * CT;   // this wave's 8-row weight piece lies inside the tile

  // operand offsets inside a tile of 128-byte rows: lane (l16, g4) reads logical chunk 4 sl + g4 of row l16
  int op_off[2];
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) op_off[sl] = (l16 * kKS + swz(l16, 4 * sl + g4) * 8) * 2;

  while (round < a.rounds || pos < rem_end) {
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * kGrid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * kGrid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    const int n0 = (int)tile * kBN;

    f4_t acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = (f4_t){0.f, 0.f, 0.f, 0.f};

    // this wave's copies per step: piece c covers rows 8c .. 8c + 7 of a tile, 16 bytes per lane
    const half_t* a_src[kAC];
#pragma unroll
    for (int i = 0; i < kAC; ++i) {
      const int prow = 8 * (wave + kNW * i) + (lane >> 3);
      const int row = prow < a.M ? prow : a.M - 1;   // rows past the block fetch its last row again (never stored)
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    const half_t* w_src;
    {
      const int prow = 8 * wave + (lane >> 3);
      w_src = a.w + (int64_t)(n0 + (has_w ? prow : 0)) * a.K + swz(prow, lane & 7) * 8;
    }
    // Past the end of the segment the last step is fetched again: harmless, and the counts stay uniform.
    auto copy_w = [&](int ks, int stage) {
      const int kc = ks < ks1 ? ks : ks1 - 1;
      if (has_w)
        __builtin_amdgcn_global_load_lds((gptr_t)(w_src + kc * kKS), (lptr_t)(smem + kWBase + stage * kWStage + wave * 1024), 16,
                                         0, 0);
    };
    auto copy_a = [&](int ks, int stage) {
      const int kc = ks < ks1 ? ks : ks1 - 1;
#pragma unroll
      for (int i = 0; i < kAC; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + kc * kKS),
                                         (lptr_t)(smem + stage * kAStage + (wave + kNW * i) * 1024), 16, 0, 0);
    };
    // all but the newest n steps' worth of this wave's copies have landed
    auto wait_steps = [&](auto N_) {
      constexpr int n = decltype(N_)::value;
      if (has_w)
        __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(n * (kAC + 1)) : "memory");
      else
        __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(n * kAC) : "memory");
    };

    // nobody reads the stages of the previous segment any more, and none of its copies is in flight
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // Steps ks0 .. ks0 + depth - 1 of each ring, issued in the order the loop below issues its refills
    // (one weight step, then one activation step, per turn): a step's weight copy is then always older
    // than its activation copy, and after any activation step come exactly the copies of the turns
    // since, so one count serves every wait.
#pragma unroll
    for (int t = 0; t < kDW; ++t) {
      copy_w(ks0 + t, t);
      if (t >= kDW - kDA) copy_a(ks0 + t - (kDW - kDA), t - (kDW - kDA));
    }
    // operands of one K step: two K slices of 32, this wave's row tile and the CT column tiles
    h8_t aop[2][2], bop[2][2][CT];
    auto read_ops = [&](int sa, int sw, auto SET_) __attribute__((always_inline)) {
      constexpr int set = decltype(SET_)::value;
      const uint32_t At = lds0 + sa * kAStage + wave * 16 * kKS * 2, Wt = lds0 + kWBase + sw * kWStage;
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        aop[set][sl] = __builtin_bit_cast(h8_t, lds_read128<0>(At + op_off[sl]));
        static_for<0, CT>([&](auto T_) __attribute__((always_inline)) {
          constexpr int ct = decltype(T_)::value;
          bop[set][sl][ct] = __builtin_bit_cast(h8_t, lds_read128<ct * 16 * kKS * 2>(Wt + op_off[sl]));
        });
      }
    };
    wait_steps(IdxC<kDA - 1>{});   // step ks0 has landed
    __builtin_amdgcn_s_barrier();
    read_ops(0, 0, IdxC<0>{});

    int sa = 0, sw = 0;   // stages holding step ks
    // One K step: the operands of step ks are in register set SET (on their way from LDS); once they
    // are there and step ks + 1 has landed for every wave, its operands are requested into the other
    // set and the stages of step ks are refilled, both behind the MFMAs of step ks.
    auto step = [&](int ks, auto SET_) __attribute__((always_inline)) {
      constexpr int set = decltype(SET_)::value;
      lds_wait();
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        lds_landed(aop[set][sl]);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) lds_landed(bop[set][sl][ct]);
      }
      // step ks + 1: its activation copy was issued kDA - 2 turns ago, followed only by those turns' copies
      wait_steps(IdxC<kDA - 2>{});
      __builtin_amdgcn_s_barrier();   // bare barrier: the copies in flight stay in flight
      const int sa1 = sa + 1 == kDA ? 0 : sa + 1, sw1 = sw + 1 == kDW ? 0 : sw + 1;
      read_ops(sa1, sw1, IdxC<1 - set>{});
      copy_w(ks + kDW, sw);   // every wave has the operands of step ks in registers: its stages are free
      copy_a(ks + kDA, sa);
      __builtin_amdgcn_sched_barrier(0);   // reads and copies go out first, the MFMAs run behind them
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aop[set][sl], bop[set][sl][ct], acc[ct], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      sa = sa1;
      sw = sw1;
    };
    for (int ks = ks0; ks < ks1; ks += 2) {
      step(ks, IdxC<0>{});
      if (ks + 1 < ks1) step(ks + 1, IdxC<1>{});
    }
    lds_wait();   // the operand reads of the step after the last one (never used) are not left in flight

    // ---- epilogue: lane holds column l16 of each 16 x 16 tile, rows 16 wave + 4 g4 + 0..3
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    if (full) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const int col = n0 + 16 * ct + l16;
        const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = 16 * wave + 4 * g4 + r;
          if (row < a.M) {
            float v = acc[ct][r] + bvv;
            if (a.relu) v = fmaxf(v, 0.f);
            if (a.residual) v += (float)a.residual[(int64_t)row * a.ldr + col];
            if (a.out32)
              a.out32[(int64_t)row * a.ldo + col] = v;
            else
              a.out16[(int64_t)row * a.ldo + col] = (half_t)v;
          }
        }
      }
    } else if (16 * wave < a.M) {
      // partial sums in register order: float4 number ct of thread tid
      float4* dst = reinterpret_cast<float4*>(a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * ((int64_t)C::kSlotRows * kBN)) + tid;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) dst[ct * (kNW * 64)] = make_float4(acc[ct][0], acc[ct][1], acc[ct][2], acc[ct][3]);
    }
    if (whole_round) {
      ++round;
    } else {
      pos += ks1 - ks0;
      ++seg;
    }
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Reduction pass: thread tid of a block adds, in ascending K order, the float4s that thread tid of the
// contributing workgroups wrote for one tile, then applies the epilogue.  One block per tile.
template <int CT>
__global__ __launch_bounds__(kNW * 64) void gemm_f16w_finish_kernel(F16wArgs a) {
  constexpr int kBN = CT * 16;
  const int64_t t = blockIdx.x;
  const int64_t w0 = t * a.ksteps, w1 = w0 + a.ksteps;
  int p_lo = (int)((w0 * kGrid) / a.rem_work);
  while (p_lo + 1 < kGrid && work_begin(a.rem_work, kGrid, p_lo + 1) <= w0) ++p_lo;
  while (p_lo > 0 && work_begin(a.rem_work, kGrid, p_lo) > w0) --p_lo;
  if (work_begin(a.rem_work, kGrid, p_lo + 1) >= w1) return;   // one workgroup owned the whole tile and stored it
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
  if (16 * wave >= a.M) return;
  const int64_t slot = (int64_t)kNW * 16 * kBN;
  float4 v[CT];
#pragma unroll
  for (int e = 0; e < CT; ++e) v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = p_lo; p < kGrid; ++p) {
    const int64_t pb = work_begin(a.rem_work, kGrid, p), pe = work_begin(a.rem_work, kGrid, p + 1);
    if (pb >= w1) break;
    if (pe == pb) continue;
    const int s = pb >= w0 ? 0 : 1;   // the tile is the workgroup's first segment, or its second
    const float4* src = reinterpret_cast<const float4*>(a.partial + ((int64_t)p * 2 + s) * slot) + tid;
#pragma unroll
    for (int e = 0; e < CT; ++e) {
      const float4 x = src[e * (kNW * 64)];
      v[e].x += x.x;
      v[e].y += x.y;
      v[e].z += x.z;
      v[e].w += x.w;
    }
  }
  const int n0 = (int)((int64_t)a.rounds * kGrid + t) * kBN;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int col = n0 + 16 * ct + l16;
    const float o[4] = {v[ct].x, v[ct].y, v[ct].z, v[ct].w};
    const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 16 * wave + 4 * g4 + r;
      if (row >= a.M) continue;
      float x = o[r] + bvv;
      if (a.relu) x = fmaxf(x, 0.f);
      if (a.residual) x += (float)a.residual[(int64_t)row * a.ldr + col];
      if (a.out32)
        a.out32[(int64_t)row * a.ldo + col] = x;
      else
        a.out16[(int64_t)row * a.ldo + col] = (half_t)x;
    }
  }
}

template <int MT32, int CT>
int launch_f16w(const F16wArgs& a, int64_t rem_tiles, hipStream_t stream) {
  using C = F16wCfg<MT32, CT>;
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_f16w_kernel<MT32, CT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes));
    attr_done = true;
  }
  {
    ProfScope prof(FG_K_GEMM_SMALL_M, stream);
    hipLaunchKernelGGL((gemm_f16w_kernel<MT32, CT>), dim3(kGrid), dim3(kNW * 64), C::kLdsBytes, stream, a);
    FG_LAUNCH_CHECK();
  }
  if (rem_tiles > 0) {
    ProfScope prof(FG_K_GEMM_SMALL_M_FINISH, stream);
    hipLaunchKernelGGL((gemm_f16w_finish_kernel<CT>), dim3((unsigned)rem_tiles), dim3(kNW * 64), 0, stream, a);
    FG_LAUNCH_CHECK();
  }
  return FG_OK;
}

template <int MT32>
int launch_f16w_ct(int ct, const F16wArgs& a, int64_t rem_tiles, hipStream_t stream) {
  switch (ct) {
    case 1: return launch_f16w<MT32, 1>(a, rem_tiles, stream);
    case 2: return launch_f16w<MT32, 2>(a, rem_tiles, stream);
    case 3: return launch_f16w<MT32, 3>(a, rem_tiles, stream);
    default: return launch_f16w<MT32, 4>(a, rem_tiles, stream);
  }
}

}  // namespace

// Column tiles of 16 per workgroup tile (0: this kernel does not take the shape, the caller falls back
// on the 256-column stream kernel).  Cost of a choice in microseconds, fitted to measurements at 128 rows
// (12288 x 4096, 4096 x 4096, 16384 x 4096, 4096 x 16384 and 50272 x 4096, every width): the HBM time of
// the weights, plus 0.15 us per K step of a CU (measured the same at 32, 64 and 128 rows and at every
// width: a cost of the step itself - copies issued, waits, barrier - that does not overlap the weight
// stream), plus, where tiles are split along K, the reduction pass (4 us + 0.6 us per MB of partial sums).  The 256-column kernel is priced the same way
// (0.3 us per of its fatter K steps, its 34 MB of partial sums) and wins for long, ragged matrices such
// as the LM head.
int gemm_f16w_pick_cols(int64_t n, int64_t k, int64_t m) {
  if (m < 1 || m > 128 || k % kKS != 0 || k < kKS || n < 16) return 0;
  // FG_F16W_COLS = 1..4 in the environment fixes the choice where the width divides N (tests cover every
  // instantiation with it; sweeps calibrate the model)
  if (const char* env = getenv("FG_F16W_COLS")) {
    const int ct = atoi(env);
    if (ct >= 1 && ct <= 4 && n % (16 * ct) == 0) return ct;
  }
  const double rows = (double)(((m + 31) / 32) * 32), ksteps = (double)(k / kKS);
  const double hbm_us = (double)n * k * 2 / 6.0e6;
  int best = 0;
  double best_us = 0;
  for (int ct = 4; ct >= 1; --ct) {
    const int bn = 16 * ct;
    if (n % bn) continue;
    const int64_t tiles = n / bn;
    const int64_t rounds = tiles / kGrid, rem = tiles - rounds * kGrid;
    double us = hbm_us + ((double)rounds + (double)rem / kGrid) * ksteps * 0.15;
    if (rem) {
      // a CU's range starts inside one tile and may end inside the next: between rem and 2 x 256 pieces
      const double pieces = (double)(rem < kGrid / 2 ? 2 * rem : kGrid) * 1.5;
      us += 4.0 + 0.6e-6 * pieces * (kNW * 16) * bn * 4;
    }
    if (!best || us < best_us) {
      best = ct;
      best_us = us;
    }
  }
  const int64_t tiles256 = (n + 255) / 256;
  double old_us = hbm_us + (double)tiles256 * ksteps / kGrid * 0.3;
  if (tiles256 % kGrid) old_us += 4.0 + 0.6e-6 * (2.0 * kGrid * rows * 256 * 4) * 0.5;
  return best_us < old_us ? best : 0;
}

size_t gemm_f16w_workspace(int64_t n, int64_t k, int64_t m) {
  const int ct = gemm_f16w_pick_cols(n, k, m);
  if (!ct) return 0;
  (void)m;
  return (size_t)kGrid * 2 * (kNW * 16) * (16 * ct) * sizeof(float);
}

int gemm_f16w_launch(const LinearArgs& la, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (la.m == 0 || la.n == 0) return FG_OK;
  const int ct = gemm_f16w_pick_cols(la.n, la.k, la.m);
  if (!ct || la.dtype != FG_F16) return FG_ERR_UNSUPPORTED;
  F16wArgs a;
  a.w = reinterpret_cast<const half_t*>(la.w_data);
  a.x = la.x;
  a.ldx = la.ldx;
  a.M = (int)la.m;
  a.N = (int)la.n;
  a.K = (int)la.k;
  a.n_tiles = (int)(la.n / (16 * ct));
  a.ksteps = (int)(la.k / kKS);
  a.rounds = a.n_tiles / kGrid;
  const int64_t rem_tiles = a.n_tiles - (int64_t)a.rounds * kGrid;
  a.rem_work = rem_tiles * a.ksteps;
  a.bias = la.bias;
  a.residual = la.residual;
  a.ldr = la.ldr;
  a.relu = la.relu;
  a.out16 = la.out_f16;
  a.out32 = la.out_f32;
  a.ldo = la.ldo;
  a.partial = reinterpret_cast<float*>(ws);
  if (rem_tiles > 0 && (!ws || ws_bytes < gemm_f16w_workspace(la.n, la.k, la.m))) return FG_ERR_WORKSPACE;
  switch ((la.m + 31) / 32) {
    case 1: return launch_f16w_ct<1>(ct, a, rem_tiles, stream);
    case 2: return launch_f16w_ct<2>(ct, a, rem_tiles, stream);
    case 3: return launch_f16w_ct<3>(ct, a, rem_tiles, stream);
    default: return launch_f16w_ct<4>(ct, a, rem_tiles, stream);
  }
}

}  // namespace fg
