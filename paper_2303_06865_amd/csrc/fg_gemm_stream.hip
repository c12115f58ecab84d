// Projections on TILED 4-bit weights (Section 3: t.wQ, t.wK, t.wV, .wO, .w1, .w2 in the prefill and
// the decode phase; weights stored as in Section 5), and the one-time repacking that produces the
// tiled layout.
//
// Why a second layout: in the canonical row-major format the 64 codes one lane pair needs per K step
// are 32 bytes of a row, and neighbouring rows are K/2 bytes apart, so a weight-streaming kernel
// touches thousands of DRAM pages with 32..64-byte pieces.  FG_Q4G64_TILED stores, for every
// (32 output columns, 64 input elements) tile, the 1 KiB of codes in exactly the order the 64 lanes
// of a wavefront consume them as the B operand of v_mfma_f32_32x32x16_f16 (lane l: column l%32,
// codes k = 32*(l/32) .. +32), tiles of one column block consecutive along K.  A wave then streams
// contiguous kilobytes, like the decode attention does.  Same bytes, same 0.625 B/element.
//
// Kernel: out[M, N] = act(x[M, K] . W^T + bias) + residual.  One kernel template, two shapes:
//   decode   M <= 160 per row block: 4 waves side by side, each all rows x 64 columns
//            (MT = 1..5 row tiles of 32, NT = 2 column tiles, WM = 1);
//   prefill  row blocks of 256: 8 waves side by side, each all 256 rows x 32 columns (MT = 8, NT = 1,
//            WM = 1; two waves per SIMD, so that one wave's MFMAs overlap the other's LDS reads and
//            dequantization, and no weight is dequantized twice in a workgroup: measured 2 % faster
//            than 2 x 4 waves of 128 x 64, which halve the LDS reads but dequantize everything twice).
//            This shape now runs in gemm_prefill16_kernel / gemm_prefill16_f16_kernel further down (the
//            same tile, wave layout, tile walk and partial sums on v_mfma_f32_16x16x32_f16, which is
//            worth 7-10 % under the chip's power limit); the template keeps the parameters, the
//            launcher no longer instantiates them.
//   * Nothing but MFMA operands passes through registers.  The activation tile (XOR-swizzled, the A
//     operand) and the weight tiles (1 KiB of codes + 256 B of {min,scale} each) are copied
//     global -> LDS asynchronously, several K steps ahead.  A wave reads its codes back, dequantizes
//     them exactly in registers (no LDS round trip for FP16 weights) and feeds them to the MFMA as
//     the B operand.
//   * Work = (output tile, K step) pairs.  Whole rounds of tiles go one tile per workgroup, walked in
//     groups of 4 row blocks so that concurrently running workgroups share activations and weights
//     in L2; the remaining tiles are cut stream-K fashion into equal contiguous ranges with a
//     deterministic second-pass reduction.  The grid is always 256 workgroups, one per CU.
#include "fg_common.h"
#include "fg_async_lds.h"

namespace fg {

namespace {

constexpr int kBN = 256;      // output columns per workgroup
constexpr int kKS = 64;       // K elements per step = one quantization group
constexpr int kBStageQ4 = 8 * (1024 + 256);   // bytes of weight codes + meta per stage (8 column tiles)
constexpr int kBStageF16 = kBN * kKS * 2;     // FP16 weights: 256 rows of 128 bytes, laid out like the activations
constexpr int kMaxMT = 5;     // decode shape: up to 5 row tiles of 32 (160 rows)
constexpr int kGroupM = 4;    // row blocks per group in the tile walk
constexpr int kLdsBytes = 160 * 1024;
constexpr int kFinishItems = 4;   // float4 items per thread of the reduction pass
constexpr int kFinishParts = 4;   // contributors whose loads are in flight together

struct StreamArgs {
  const uint8_t* w;     // tiled codes
  const float2* meta;   // tiled {min, scale}
  const half_t* x;
  int64_t ldx;
  int M, N, K;
  int m_blocks, n_tiles, ksteps, n32;   // n32 = N / 32
  int rounds;           // whole rounds: tiles [0, rounds*grid) go one per workgroup per round
  int64_t rem_work;     // (remaining tiles) * ksteps, cut into grid equal ranges
  int grid;
  const half_t* bias;
  const half_t* residual;
  int64_t ldr;
  int relu;
  half_t* out16;
  float* out32;
  int64_t ldo;
  float* partial;       // [grid][2][block rows][256]
};

// linear tile number -> (row block, column block): groups of kGroupM row blocks, inside a group the
// row block runs fastest, so 32 consecutive tiles (one XCD's share of a round) form a patch of 4 row blocks x 8 column
// blocks: per K step the 32 workgroups then fetch 4 activation tiles (32 KiB each) and 8 weight tiles
// (10 KiB each) into that XCD's L2, the least of all patch shapes
__device__ __forceinline__ void tile_coords(int64_t t, int m_blocks, int n_tiles, int& mblk, int& n_tile) {
  const int64_t per_group = (int64_t)kGroupM * n_tiles;
  const int g = (int)(t / per_group);
  const int first = g * kGroupM;
  const int gm = m_blocks - first < kGroupM ? m_blocks - first : kGroupM;
  const int r = (int)(t - (int64_t)g * per_group);
  mblk = first + r % gm;
  n_tile = r / gm;
}

// F16W: the weights are plain row-major FP16 (no repacking needed: a [256 columns][64 k] block of W is
// copied and read exactly like the activation tile) instead of tiled 4-bit codes.
template <int MT, int NT, int WM, int NW, bool F16W>
struct StreamCfg {
  static constexpr int kWN = NW / WM;                      // waves along N
  static constexpr int kRows = WM * MT * 32;               // rows per workgroup tile
  static constexpr int kAStage = kRows * kKS * 2;          // bytes of the activation tile per stage
  static constexpr int kBStage = F16W ? kBStageF16 : kBStageQ4;
  static constexpr int kStageBytes = kAStage + kBStage;
  static constexpr int kNST = kLdsBytes / kStageBytes > 5 ? 5 : kLdsBytes / kStageBytes;   // LDS stages
  static constexpr int kACopies = kRows / 8 / NW;          // wave-wide copies per wave per K step: activations
  static constexpr int kBCopies = (F16W ? kBN / 8 : 16) / NW;   // ... weights (8 tiles x {codes, meta}, or 32 x 8 rows)
  static constexpr int kCopies = kACopies + kBCopies;
  static_assert(kWN * NT == 8, "a workgroup covers 8 column tiles of 32");
  static_assert(kACopies * 8 * NW == kRows, "activation rows must split evenly over the waves");
  // (two stages: the 256 x 256 tile pair of FP16 weights, 64 KiB per stage; its operands come from L2,
  // one K step of look-ahead covers that)
  static_assert(kNST >= 2, "needs two stages");
};

// H16M: the {min, scale} pairs of the tiled 4-bit weights are two FP16 numbers (4 bytes) instead of two
// binary32 numbers; a tile's 32 pairs then fill half of its 256-byte slot of the stage (the copy stays
// wave-wide: lanes 32..63 fetch the same pairs again into the other half).
template <int MT, int NT, int WM, int NW, bool F16W, bool H16M = false>
__global__ __launch_bounds__(NW * 64) void gemm_stream_kernel(StreamArgs a) {
  using C = StreamCfg<MT, NT, WM, NW, F16W>;
  constexpr int kWN = C::kWN, kAStage = C::kAStage, kStageBytes = C::kStageBytes, kNST = C::kNST;
  constexpr int kACopies = C::kACopies, kBCopies = C::kBCopies, kCopies = C::kCopies;
  constexpr int kBT = F16W ? kBCopies : (kBCopies + 1) / 2;   // weight tiles (FP16: 8-row pieces) this wave copies
  // Outstanding copies allowed when step ks+1 must have landed (end of slice 2 of step ks): those of
  // the steps after it that are already issued.
  constexpr int kWait = (kNST - 2) * kCopies;
  constexpr int kNM = MT * NT;                          // MFMAs per K slice
  constexpr int kDq = 3 * NT;                           // dequantization pieces per K slice
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [kNST][A tile | B tiles]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / kWN, wn = wave - wm * kWN;
  const int l32 = lane & 31, kb = lane >> 5;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, a.grid, p), rem_end = work_begin(a.rem_work, a.grid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;

  // operand read offsets inside a stage: lane (l32, kb) reads logical chunk 4*kb + kk of its row
  int a_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) a_off[kk] = ((wm * MT * 32 + l32) * kKS + swz(l32, 4 * kb + kk) * 8) * 2;
  // this wave's weight tiles inside a stage
  const int bq_off = kAStage + wn * NT * 1024 + lane * 16;           // + j * 1024
  const int bm_off = kAStage + 8 * 1024 + wn * NT * 256 + l32 * (H16M ? 4 : 8);   // + j * 256
  // FP16 weights: operand offsets like a_off, for this wave's first column tile
  int b_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) b_off[kk] = kAStage + ((wn * NT * 32 + l32) * kKS + swz(l32, 4 * kb + kk) * 8) * 2;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

  while (round < a.rounds || pos < rem_end) {
    // ---- next segment: a whole tile of a round, or a piece of this workgroup's stream-K range
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * a.grid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * a.grid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    int mblk, n_tile;
    tile_coords(tile, a.m_blocks, a.n_tiles, mblk, n_tile);
    const int m0 = mblk * C::kRows;
    const int nt0 = n_tile * 8 + wn * NT;   // first 32-column tile of this wave

    f16_t acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][j][r] = 0.f;

    // this wave's async activation copies per step: copy c covers rows 8c .. 8c+7 of the tile
    const half_t* a_src[kACopies];
#pragma unroll
    for (int i = 0; i < kACopies; ++i) {
      const int c = wave + NW * i;
      const int prow = 8 * c + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    // ... and its share of the weight copies: kBT of the workgroup's 8 column tiles
    const uint8_t* w_src[kBT];
    const float* m_src[F16W ? 1 : kBT];
#pragma unroll
    for (int j = 0; j < kBT; ++j) {
      if constexpr (F16W) {   // piece c = wave + NW*j covers weight rows (output columns) 8c .. 8c+7 of the block
        const int c = wave + NW * j;
        const int prow = 8 * c + (lane >> 3);
        int col = n_tile * kBN + prow;
        col = col < a.N ? col : a.N - 1;
        w_src[j] = a.w + ((int64_t)col * a.K + swz(prow, lane & 7) * 8) * 2;
      } else {
        int nt = n_tile * 8 + wave * kBT + j;
        nt = nt < a.n32 ? nt : a.n32 - 1;   // ragged last column block: load valid data, never store it
        w_src[j] = a.w + (int64_t)nt * a.ksteps * 1024 + lane * 16;
        m_src[j] = reinterpret_cast<const float*>(a.meta) + (H16M ? (int64_t)nt * a.ksteps * 32 + l32
                                                                  : (int64_t)nt * a.ksteps * 64 + lane);
      }
    }

    // The kCopies wave-wide asynchronous global -> LDS transfers of one K step.  Past the end of the
    // segment the last step is fetched again: harmless, and it keeps the VMEM counts uniform.
    auto copy_one = [&](int c, int ks, int stage) {
      const int kc = ks < ks1 ? ks : ks1 - 1;
      unsigned char* st = smem + stage * kStageBytes;
      if (c < kACopies) {
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[c] + kc * kKS), (lptr_t)(st + (wave + NW * c) * 8 * kKS * 2), 16,
                                         0, 0);
      } else if constexpr (F16W) {
        const int j = c - kACopies;
        __builtin_amdgcn_global_load_lds((gptr_t)(w_src[j] + (int64_t)kc * (kKS * 2)),
                                         (lptr_t)(st + kAStage + (wave + NW * j) * 8 * kKS * 2), 16, 0, 0);
      } else {
        const int b = c - kACopies, j = b >> 1;   // b = 2 * j + (0: codes, 1: {min, scale})
        if ((b & 1) == 0)
          __builtin_amdgcn_global_load_lds((gptr_t)(w_src[j] + (int64_t)kc * 1024),
                                           (lptr_t)(st + kAStage + (wave * kBT + j) * 1024), 16, 0, 0);
        else
          __builtin_amdgcn_global_load_lds((gptr_t)(m_src[j] + (int64_t)kc * (H16M ? 32 : 64)),
                                           (lptr_t)(st + kAStage + 8 * 1024 + (wave * kBT + j) * 256), 4, 0, 0);
      }
    };
    u4_t cq[NT];
    float2 cm[NT];
    uint32_t cmh[NT];   // H16M: the pair as stored
    auto read_b = [&](int stage) {
      const uint32_t st = lds0 + stage * kStageBytes;
      static_for<0, NT>([&](auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        cq[j] = lds_read128<j * 1024>(st + bq_off);
        if constexpr (H16M) cmh[j] = lds_read32<j * 256>(st + bm_off); else cm[j] = lds_read64<j * 256>(st + bm_off);
      });
    };
    // operand slice kk of this wave's MT row tiles of a stage
    auto read_a = [&](uint32_t st, int kk, h8_t* dst) {
      const uint32_t ad = st + a_off[kk];
      static_for<0, MT>([&](auto m) __attribute__((always_inline)) {
        constexpr int off = decltype(m)::value * 32 * kKS * 2;
        dst[decltype(m)::value] = __builtin_bit_cast(h8_t, lds_read128<off>(ad));
      });
    };
    // FP16 weights: operand slice kk of this wave's NT column tiles, straight from the stage
    auto read_w16 = [&](uint32_t st, int kk, u4_t* dst) {
      const uint32_t ad = st + b_off[kk];
      static_for<0, NT>([&](auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        dst[j] = lds_read128<j * 32 * kKS * 2>(ad);
      });
    };
    h8_t aop[2][MT];
    u4_t bop[2][NT];
    float s24[NT], s20[NT], mn[NT];
    uint32_t msk[4];
    // Exact dequantization (fg_common.h: dequant8_exact) of word kk of tile j, cut into three pieces so
    // that it can be spread between MFMAs: 0 = masks, 1 = weights 0..3, 2 = weights 4..7.
    auto dq = [&](int kk, int j, int sub, int buf) {
      if (sub == 0) {
        const uint32_t x = cq[j][kk], y = x >> 8;
        msk[0] = x & 0x000F000Fu;
        msk[1] = x & 0x00F000F0u;
        msk[2] = y & 0x000F000Fu;
        msk[3] = y & 0x00F000F0u;
      } else {
        const h2_t ha = __builtin_bit_cast(h2_t, msk[0]), hb = __builtin_bit_cast(h2_t, msk[1]);
        const h2_t hc = __builtin_bit_cast(h2_t, msk[2]), hd = __builtin_bit_cast(h2_t, msk[3]);
        if (sub == 1) {
          const h2_t q0 = {(half_t)__builtin_fmaf((float)ha.x, s24[j], mn[j]), (half_t)__builtin_fmaf((float)hb.x, s20[j], mn[j])};
          const h2_t q1 = {(half_t)__builtin_fmaf((float)hc.x, s24[j], mn[j]), (half_t)__builtin_fmaf((float)hd.x, s20[j], mn[j])};
          bop[buf][j][0] = __builtin_bit_cast(uint32_t, q0);
          bop[buf][j][1] = __builtin_bit_cast(uint32_t, q1);
        } else {
          const h2_t q2 = {(half_t)__builtin_fmaf((float)ha.y, s24[j], mn[j]), (half_t)__builtin_fmaf((float)hb.y, s20[j], mn[j])};
          const h2_t q3 = {(half_t)__builtin_fmaf((float)hc.y, s24[j], mn[j]), (half_t)__builtin_fmaf((float)hd.y, s20[j], mn[j])};
          bop[buf][j][2] = __builtin_bit_cast(uint32_t, q2);
          bop[buf][j][3] = __builtin_bit_cast(uint32_t, q3);
        }
      }
    };
    // the freshly read {min, scale} pairs -> FMA constants
    auto set_meta = [&]() {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if constexpr (H16M) {
          const h2_t pr = __builtin_bit_cast(h2_t, cmh[j]);
          cm[j].x = (float)pr.x;
          cm[j].y = (float)pr.y;
        }
        s24[j] = cm[j].y * 16777216.0f;
        s20[j] = cm[j].y * 1048576.0f;
        mn[j] = cm[j].x;
      }
    };
    auto landed_b = [&]() {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        lds_landed(cq[j]);
        if constexpr (H16M) lds_landed(cmh[j]); else lds_landed(cm[j]);
      }
    };

    // no copy of the previous segment may still be in flight towards a stage, and no wave still reads one
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kNST; ++t)
#pragma unroll
      for (int c = 0; c < kCopies; ++c) copy_one(c, ks0 + t, t);
    __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"((kNST - 1) * kCopies) : "memory");
    __builtin_amdgcn_s_barrier();
    read_a(lds0, 0, aop[0]);
    if constexpr (F16W) read_w16(lds0, 0, bop[0]); else read_b(0);
    lds_wait();
#pragma unroll
    for (int m = 0; m < MT; ++m) lds_landed(aop[0][m]);
    if constexpr (F16W) {
#pragma unroll
      for (int j = 0; j < NT; ++j) lds_landed(bop[0][j]);
    } else {
      landed_b();
      set_meta();
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int sub = 0; sub < 3; ++sub) dq(0, j, sub, 0);
    }

    // Steady state.  At the top of a step the operands of its first K slice are already in registers.
    // Every slice issues its MFMAs with the preparation of the NEXT slice spread between them (a wave
    // issues in order, and an MFMA occupies the matrix pipe for 32 cycles: a few independent
    // instructions after each one are free, a block of them is not):
    //   slices 0..2: LDS reads of the next A slice and dequantization of the next code word;
    //   end of 2   : this wave's copies of step ks+1 have landed (vmcnt), barrier: now every wave's
    //                have, and nobody reads this stage any more (its weights were read one step ago);
    //   slice 3    : copies of step ks+kNST into this stage, LDS reads of step ks+1 (first A slice,
    //                codes, meta), then dequantization of its first code word.
    int stage = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage1 = stage + 1 == kNST ? 0 : stage + 1;
      const uint32_t At = lds0 + stage * kStageBytes;
      static_for<0, 4>([&](auto KK) __attribute__((always_inline)) {
        constexpr int kk = decltype(KK)::value;
        constexpr int cur = kk & 1, nxt = cur ^ 1;
        if constexpr (kk < 3) {
          read_a(At, kk + 1, aop[nxt]);
          if constexpr (F16W) read_w16(At, kk + 1, bop[nxt]);
        } else {
          read_a(lds0 + stage1 * kStageBytes, 0, aop[nxt]);
          if constexpr (F16W) read_w16(lds0 + stage1 * kStageBytes, 0, bop[nxt]); else read_b(stage1);
        }
        __builtin_amdgcn_sched_barrier(0);
        // slice 3: the copies go between the MFMAs of the first kH, the dequantization between the rest
        constexpr int kH = kNM / 2 > 0 ? kNM / 2 : 1;
        static_for<0, kNM>([&](auto I) __attribute__((always_inline)) {
          constexpr int i = decltype(I)::value;
          constexpr int j = i / MT, m = i - j * MT;
          acc[m][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop[cur][m], __builtin_bit_cast(h8_t, bop[cur][j]), acc[m][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (kk < 3) {
            if constexpr (!F16W)
              static_for<i * kDq / kNM, (i + 1) * kDq / kNM>([&](auto IT) __attribute__((always_inline)) {
                constexpr int it = decltype(IT)::value;
                dq(kk + 1, it / 3, it % 3, nxt);
              });
          } else if constexpr (i < kH) {
            static_for<i * kCopies / kH, (i + 1) * kCopies / kH>([&](auto CC) __attribute__((always_inline)) {
              copy_one(decltype(CC)::value, ks + kNST, stage);
            });
            if constexpr (i == kH - 1) {
              lds_wait();
#pragma unroll
              for (int mm = 0; mm < MT; ++mm) lds_landed(aop[nxt][mm]);
              if constexpr (F16W) {
#pragma unroll
                for (int jj = 0; jj < NT; ++jj) lds_landed(bop[nxt][jj]);
              } else {
                landed_b();
                set_meta();
              }
            }
          } else if constexpr (!F16W) {
            static_for<(i - kH) * kDq / (kNM - kH), (i - kH + 1) * kDq / (kNM - kH)>([&](auto IT) __attribute__((always_inline)) {
              constexpr int it = decltype(IT)::value;
              dq(0, it / 3, it % 3, nxt);
            });
          }
          __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (kk < 3) {
          lds_wait();
#pragma unroll
          for (int m = 0; m < MT; ++m) lds_landed(aop[nxt][m]);
          if constexpr (F16W) {
#pragma unroll
            for (int j = 0; j < NT; ++j) lds_landed(bop[nxt][j]);
          }
          if constexpr (kk == 2) {
            __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(kWait) : "memory");
            __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the copies in flight stay in flight
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      });
      stage = stage1;
    }

    // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*kb + r%4
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    if (full) {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int col = (nt0 + j) * 32 + l32;
        if (nt0 + j < a.n32) {
          const float bvv = a.bias ? (float)a.bias[col] : 0.f;
          // running offsets instead of 16 * MT independent ones (which would all be kept in registers)
          int row = m0 + wm * MT * 32 + kb * 4;
          int64_t o_off = (int64_t)row * a.ldo + col, r_off = (int64_t)row * a.ldr + col;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              if (row < a.M) {
                float v = acc[m][j][r] + bvv;
                if (a.relu) v = fmaxf(v, 0.f);
                if (a.residual) v += (float)a.residual[r_off];
                if (a.out32)
                  a.out32[o_off] = v;
                else
                  a.out16[o_off] = (half_t)v;
              }
              const int step = (r & 3) == 3 ? 5 : 1;   // rows 8*(r/4) + 4*kb + r%4
              row += step;
              o_off += step * a.ldo;
              r_off += step * a.ldr;
            }
          }
        }
      }
    } else {
      // partial sums in register order: float4 number ((m*NT + j)*4 + q) of thread tid holds rows
      // 32m + 8q + 4kb + 0..3 of one column -> every store is 1 KiB contiguous per wave
      float4* dst = reinterpret_cast<float4*>(a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * ((int64_t)C::kRows * kBN)) + tid;
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (m0 + (wm * MT + m) * 32 + q * 8 < a.M)   // rows beyond M: padding, never read back
              *dst = make_float4(acc[m][j][4 * q], acc[m][j][4 * q + 1], acc[m][j][4 * q + 2], acc[m][j][4 * q + 3]);
            dst += NW * 64;
          }
    }
    if (whole_round) {
      ++round;
    } else {
      pos += ks1 - ks0;
      ++seg;
    }
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may still target LDS when the wave ends
}

// Second pass of the stream-K schedule: tiles whose K range was shared get their partial sums added
// in ascending K order, then the epilogue.  Thread tid of a block takes the float4s that thread tid of
// the GEMM kernel wrote (four rows of one column each).  blockIdx.x counts the tiles after the whole
// rounds.
__global__ __launch_bounds__(512) void gemm_stream_finish_kernel(StreamArgs a, int mt, int nt, int wm_n) {
  const int64_t t = blockIdx.x;
  const int64_t w0 = t * a.ksteps, w1 = w0 + a.ksteps;
  int p_lo = (int)((w0 * a.grid) / a.rem_work);
  while (p_lo + 1 < a.grid && work_begin(a.rem_work, a.grid, p_lo + 1) <= w0) ++p_lo;
  while (p_lo > 0 && work_begin(a.rem_work, a.grid, p_lo) > w0) --p_lo;
  if (work_begin(a.rem_work, a.grid, p_lo + 1) >= w1) return;   // one workgroup owned the whole tile
  int p_hi = p_lo;
  while (p_hi + 1 < a.grid && work_begin(a.rem_work, a.grid, p_hi + 1) < w1) ++p_hi;

  int mblk, n_tile;
  tile_coords((int64_t)a.rounds * a.grid + t, a.m_blocks, a.n_tiles, mblk, n_tile);
  const int nthr = blockDim.x;   // = threads of the GEMM workgroup
  const int rows_t = wm_n * mt * 32, wn_n = (nthr >> 6) / wm_n;
  const int m0 = mblk * rows_t;
  const int64_t slot = (int64_t)rows_t * kBN;
  const int tid = threadIdx.x, wave = tid >> 6, l32 = tid & 31, kb = (tid >> 5) & 1;
  const int wm = wave / wn_n, wn = wave - wm * wn_n;
  // this thread's float4 items e = blockIdx.y + i * gridDim.y, e = (m*nt + j)*4 + q; the launch keeps
  // their number within kFinishItems.  The loads of up to kFinishParts contributors for all items are
  // in flight together (a tile of the decode shapes has 2 to 7 contributors: one or two dependent
  // round trips instead of one per contributor); the sum still runs in ascending K order per item.
  const int n_items = mt * nt * 4;
  float4 v[kFinishItems];
#pragma unroll
  for (int i = 0; i < kFinishItems; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  int p = p_lo;
  while (p <= p_hi) {
    const float4* src[kFinishParts];
    int n = 0;
    for (; p <= p_hi && n < kFinishParts; ++p) {
      const int64_t pb = work_begin(a.rem_work, a.grid, p);
      if (work_begin(a.rem_work, a.grid, p + 1) == pb) continue;
      const int s = pb >= w0 ? 0 : 1;
      src[n++] = reinterpret_cast<const float4*>(a.partial + ((int64_t)p * 2 + s) * slot) + tid;
    }
    float4 x[kFinishParts][kFinishItems];
#pragma unroll
    for (int c = 0; c < kFinishParts; ++c)
#pragma unroll
      for (int i = 0; i < kFinishItems; ++i) {
        const int e = blockIdx.y + i * gridDim.y;
        // items whose eight rows (8q .. 8q+7 of row tile m) all lie beyond M were never written
        const bool live = e < n_items && m0 + (wm * mt + (e >> 2) / nt) * 32 + (e & 3) * 8 < a.M;
        x[c][i] = (c < n && live) ? src[c < n ? c : 0][(int64_t)e * nthr] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
    for (int c = 0; c < kFinishParts; ++c)
      if (c < n) {
#pragma unroll
        for (int i = 0; i < kFinishItems; ++i) {
          v[i].x += x[c][i].x;
          v[i].y += x[c][i].y;
          v[i].z += x[c][i].z;
          v[i].w += x[c][i].w;
        }
      }
  }
#pragma unroll
  for (int i = 0; i < kFinishItems; ++i) {
    const int e = blockIdx.y + i * gridDim.y;
    if (e >= n_items) break;
    const int q = e & 3, mj = e >> 2, m = mj / nt, j = mj - m * nt;
    const int row0 = m0 + (wm * mt + m) * 32 + q * 8 + kb * 4;
    const int col = n_tile * kBN + (wn * nt + j) * 32 + l32;
    if (row0 >= a.M || col >= a.N) continue;
    const float o[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + r;
      if (row >= a.M) break;
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

// ---------------------------------------------------------------------------------------------
// Decode shape on 16-row tiles.  The 32 x 32 tiles above round a block of rows up to a multiple of 32:
// the 144 rows of a 4 x 36 block are computed as 160, a tenth of the matrix-core time for nothing.
// This kernel is the same pipeline (same stages, copies, tile walk, stream-K ranges and partial-sum
// scheme) on v_mfma_f32_16x16x32_f16: MT16 = ceil(rows / 16) row tiles, each wave all rows x 64 columns
// as four column tiles of 16.  It is used where the row count fills an odd number of 16-row tiles.
//   A operand  lane (i = l % 16, g = l / 16): row 16 m + i, the 8 halves of logical chunk 4 s + g of the
//              64-wide K step (s = 0, 1: the two K slices of 32); one ds_read_b128, conflict-free under
//              the stage's XOR swizzle.
//   B operand  lane (j = l % 16, g): column 16 c + j of a 32-column weight tile, codes 32 s + 8 g .. + 8:
//              word g of the 16-byte piece (column, half s) of the tiled layout, i.e. one ds_read_b32 at
//              16 (32 s + 16 c + j) + 4 g (64 distinct banks), dequantized exactly as above.
//   K step     slice 0: its 9 x 4 MFMAs with the reads of slice 1's A operands and the dequantization of
//              slice 1's weights between them; then this wave's copies of the next step have landed
//              (vmcnt) and a barrier: every wave's have, and nobody reads this stage any more;
//              slice 1: copies for step ks + kNST into this stage, the next stage's A operands, code
//              words and {min, scale}, and the dequantization of its first slice, between the MFMAs.
// acc += A . B on v_mfma_f32_16x16x32_f16 with the accumulator updated IN PLACE in accumulation
// registers.  Written as an instruction because the register allocator, given 36 four-register
// accumulators per wave through the builtin, keeps rotating them through other registers (three
// register moves and wait states per MFMA); an in-place operand leaves it nothing to rotate.
__device__ __forceinline__ void mfma16_inplace(f4_t& acc, const h8_t& a, const h8_t& b) {
  __asm__ volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// The same with the accumulator in an ordinary vector register: a kernel with two waves per SIMD has 256
// registers per lane in all, of either kind, and keeping the accumulators among the ordinary ones spares
// it every move between the two files where the sums are finished.
__device__ __forceinline__ void mfma16_inplace_v(f4_t& acc, const h8_t& a, const h8_t& b) {
  __asm__ volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

template <int MT16, bool H16M>
struct Dec16Cfg {
  static constexpr int kMT32 = (MT16 + 1) / 2;
  static constexpr int kRowsLds = kMT32 * 32;             // rows of the activation tile in a stage (copied in 8-row pieces)
  static constexpr int kRows = MT16 * 16;                 // rows computed
  static constexpr int kAStage = kRowsLds * kKS * 2;
  static constexpr int kStageBytes = kAStage + kBStageQ4;
  static constexpr int kNST = kLdsBytes / kStageBytes > 5 ? 5 : kLdsBytes / kStageBytes;
  static constexpr int kACopies = kRowsLds / 8 / 4;
  static constexpr int kCopies = kACopies + 4;
};

template <int MT16, bool H16M>
__global__ __launch_bounds__(256) void gemm_decode16_kernel(StreamArgs a) {
  using C = Dec16Cfg<MT16, H16M>;
  constexpr int kAStage = C::kAStage, kStageBytes = C::kStageBytes, kNST = C::kNST;
  constexpr int kACopies = C::kACopies, kCopies = C::kCopies;
  constexpr int kWait = (kNST - 2) * kCopies;
  constexpr int kNM = MT16 * 4;                 // MFMAs per K slice
  constexpr int NW = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, a.grid, p), rem_end = work_begin(a.rem_work, a.grid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;

  // operand read offsets inside a stage
  int a_off[2];
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) a_off[sl] = (l16 * kKS + swz(l16, 4 * sl + g4) * 8) * 2;
  // code word of (column tile ct, slice sl): + (ct >> 1) * 1024 + (ct & 1) * 256 + sl * 512
  const int bq_off = kAStage + wave * 2 * 1024 + l16 * 16 + g4 * 4;
  // {min, scale} of column tile ct: + (ct >> 1) * 256 + (ct & 1) * 16 * (H16M ? 4 : 8)
  const int bm_off = kAStage + 8 * 1024 + wave * 2 * 256 + l16 * (H16M ? 4 : 8);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

  while (round < a.rounds || pos < rem_end) {
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * a.grid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * a.grid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    int mblk, n_tile;
    tile_coords(tile, a.m_blocks, a.n_tiles, mblk, n_tile);
    const int m0 = mblk * C::kRows;
    const int nt0 = n_tile * 8 + wave * 2;   // first 32-column tile of this wave

    f4_t acc[MT16][4];
#pragma unroll
    for (int m = 0; m < MT16; ++m)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) acc[m][ct] = (f4_t){0.f, 0.f, 0.f, 0.f};

    const half_t* a_src[kACopies];
#pragma unroll
    for (int i = 0; i < kACopies; ++i) {
      const int c = wave + NW * i;
      const int prow = 8 * c + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    const uint8_t* w_src[2];
    const float* m_src[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int nt = nt0 + j;
      nt = nt < a.n32 ? nt : a.n32 - 1;   // ragged last column block: load valid data, never store it
      w_src[j] = a.w + (int64_t)nt * a.ksteps * 1024 + lane * 16;
      m_src[j] = reinterpret_cast<const float*>(a.meta) +
                 (H16M ? (int64_t)nt * a.ksteps * 32 + (lane & 31) : (int64_t)nt * a.ksteps * 64 + lane);
    }
    auto copy_one = [&](int c, int ks, int stage) {
      const int kc = ks < ks1 ? ks : ks1 - 1;
      unsigned char* st = smem + stage * kStageBytes;
      if (c < kACopies) {
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[c] + kc * kKS), (lptr_t)(st + (wave + NW * c) * 8 * kKS * 2), 16,
                                         0, 0);
      } else {
        const int b = c - kACopies, j = b >> 1;
        if ((b & 1) == 0)
          __builtin_amdgcn_global_load_lds((gptr_t)(w_src[j] + (int64_t)kc * 1024),
                                           (lptr_t)(st + kAStage + (wave * 2 + j) * 1024), 16, 0, 0);
        else
          __builtin_amdgcn_global_load_lds((gptr_t)(m_src[j] + (int64_t)kc * (H16M ? 32 : 64)),
                                           (lptr_t)(st + kAStage + 8 * 1024 + (wave * 2 + j) * 256), 4, 0, 0);
      }
    };

    h8_t aop[2][MT16];
    u4_t bop[2][4];
    uint32_t cw[2][4];     // raw code words [slice][column tile] of the current stage
    float2 cm[4];
    uint32_t cmh[4];
    float s24[4], s20[4], mn[4];
    auto read_a = [&](uint32_t st, int sl, h8_t* dst) {
      const uint32_t ad = st + a_off[sl];
      static_for<0, MT16>([&](auto m) __attribute__((always_inline)) {
        constexpr int off = decltype(m)::value * 16 * kKS * 2;
        dst[decltype(m)::value] = __builtin_bit_cast(h8_t, lds_read128<off>(ad));
      });
    };
    auto read_b = [&](int stage) {
      const uint32_t st = lds0 + stage * kStageBytes;
      static_for<0, 4>([&](auto CT) __attribute__((always_inline)) {
        constexpr int ct = decltype(CT)::value;
        constexpr int qoff = (ct >> 1) * 1024 + (ct & 1) * 256;
        cw[0][ct] = lds_read32<qoff>(st + bq_off);
        cw[1][ct] = lds_read32<qoff + 512>(st + bq_off);
        constexpr int moff = (ct >> 1) * 256 + (ct & 1) * 16 * (H16M ? 4 : 8);
        if constexpr (H16M) cmh[ct] = lds_read32<moff>(st + bm_off); else cm[ct] = lds_read64<moff>(st + bm_off);
      });
    };
    auto landed_b = [&]() {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        lds_landed(cw[0][ct]);
        lds_landed(cw[1][ct]);
        if constexpr (H16M) lds_landed(cmh[ct]); else lds_landed(cm[ct]);
      }
    };
    auto set_meta = [&]() {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        if constexpr (H16M) {
          const h2_t pr = __builtin_bit_cast(h2_t, cmh[ct]);
          cm[ct].x = (float)pr.x;
          cm[ct].y = (float)pr.y;
        }
        s24[ct] = cm[ct].y * 16777216.0f;
        s20[ct] = cm[ct].y * 1048576.0f;
        mn[ct] = cm[ct].x;
      }
    };
    // Exact dequantization of one code word (fg_common.h: dequant8_exact) into the B operand of
    // (slice, ct), cut into four pieces of two to four VALU instructions so that it can be spread
    // between MFMAs of 16 cycles: 0, 1 = nibble masks, 2 = operand registers 0 and 1 (weights 0..3),
    // 3 = registers 2 and 3 (weights 4..7); the two halves of one register are never written back to back.
    // Every piece ends in an empty volatile statement on its result: the MFMAs here are volatile
    // instructions too, so a piece stays where it is written, between the same two MFMAs, instead of
    // being sunk next to its consumer.  That matters for correctness, not only for speed: the compiler
    // does not know that the consumer is an MFMA and puts no wait state between a VALU write of an
    // operand register and the MFMA that reads it in the next cycle (seen: wrong sums in one column tile).
    uint32_t msk[4];
    auto dq_piece = [&](int sl, int ct, int buf, int piece) {
      if (piece == 0) {
        const uint32_t x = cw[sl][ct];
        msk[0] = x & 0x000F000Fu;
        msk[1] = x & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[0]), "+v"(msk[1]));
      } else if (piece == 1) {
        const uint32_t y = cw[sl][ct] >> 8;
        msk[2] = y & 0x000F000Fu;
        msk[3] = y & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[2]), "+v"(msk[3]));
      } else {
        const h2_t ha = __builtin_bit_cast(h2_t, msk[0]), hb = __builtin_bit_cast(h2_t, msk[1]);
        const h2_t hc = __builtin_bit_cast(h2_t, msk[2]), hd = __builtin_bit_cast(h2_t, msk[3]);
        h2_t q0, q1;
        if (piece == 2) {
          q0 = (h2_t){(half_t)__builtin_fmaf((float)ha.x, s24[ct], mn[ct]), (half_t)__builtin_fmaf((float)hb.x, s20[ct], mn[ct])};
          q1 = (h2_t){(half_t)__builtin_fmaf((float)hc.x, s24[ct], mn[ct]), (half_t)__builtin_fmaf((float)hd.x, s20[ct], mn[ct])};
        } else {
          q0 = (h2_t){(half_t)__builtin_fmaf((float)ha.y, s24[ct], mn[ct]), (half_t)__builtin_fmaf((float)hb.y, s20[ct], mn[ct])};
          q1 = (h2_t){(half_t)__builtin_fmaf((float)hc.y, s24[ct], mn[ct]), (half_t)__builtin_fmaf((float)hd.y, s20[ct], mn[ct])};
        }
        uint32_t r0 = __builtin_bit_cast(uint32_t, q0), r1 = __builtin_bit_cast(uint32_t, q1);
        __asm__ volatile("" : "+v"(r0), "+v"(r1));
        bop[buf][ct][2 * (piece - 2)] = r0;
        bop[buf][ct][2 * (piece - 2) + 1] = r1;
      }
    };
    constexpr int kPieces = 16;   // 4 column tiles x 4 pieces per K slice

    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kNST; ++t)
#pragma unroll
      for (int c = 0; c < kCopies; ++c) copy_one(c, ks0 + t, t);
    __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"((kNST - 1) * kCopies) : "memory");
    __builtin_amdgcn_s_barrier();
    read_a(lds0, 0, aop[0]);
    read_b(0);
    lds_wait();
#pragma unroll
    for (int m = 0; m < MT16; ++m) lds_landed(aop[0][m]);
    landed_b();
    set_meta();
#pragma unroll
    for (int q = 0; q < kPieces; ++q) dq_piece(0, q / 4, 0, q % 4);

    int stage = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage1 = stage + 1 == kNST ? 0 : stage + 1;
      const uint32_t At = lds0 + stage * kStageBytes;
      // ---- slice 0
      read_a(At, 1, aop[1]);
      __builtin_amdgcn_sched_barrier(0);
      static_for<0, kNM>([&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        constexpr int ct = i / MT16, m = i - ct * MT16;
        mfma16_inplace(acc[m][ct], aop[0][m], __builtin_bit_cast(h8_t, bop[0][ct]));
        __builtin_amdgcn_sched_barrier(0);
        // the dequantization of slice 1, spread evenly over the MFMAs
        static_for<i * kPieces / kNM, (i + 1) * kPieces / kNM>([&](auto Q) __attribute__((always_inline)) {
          constexpr int q = decltype(Q)::value;
          dq_piece(1, q / 4, 1, q % 4);
        });
        __builtin_amdgcn_sched_barrier(0);
      });
      lds_wait();
#pragma unroll
      for (int m = 0; m < MT16; ++m) lds_landed(aop[1][m]);
      __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(kWait) : "memory");
      __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the copies in flight stay in flight
      __builtin_amdgcn_sched_barrier(0);
      // ---- slice 1
      read_a(lds0 + stage1 * kStageBytes, 0, aop[0]);
      read_b(stage1);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int kH = kNM / 2;
      static_for<0, kNM>([&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        constexpr int ct = i / MT16, m = i - ct * MT16;
        mfma16_inplace(acc[m][ct], aop[1][m], __builtin_bit_cast(h8_t, bop[1][ct]));
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (i < kH) {
          static_for<i * kCopies / kH, (i + 1) * kCopies / kH>([&](auto CC) __attribute__((always_inline)) {
            copy_one(decltype(CC)::value, ks + kNST, stage);
          });
          if constexpr (i == kH - 1) {
            lds_wait();
#pragma unroll
            for (int mm = 0; mm < MT16; ++mm) lds_landed(aop[0][mm]);
            landed_b();
            set_meta();
          }
        } else {
          // the dequantization of the next step's slice 0, spread over the second half
          constexpr int r = i - kH, n2 = kNM - kH;
          static_for<r * kPieces / n2, (r + 1) * kPieces / n2>([&](auto Q) __attribute__((always_inline)) {
            constexpr int q = decltype(Q)::value;
            dq_piece(0, q / 4, 0, q % 4);
          });
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      stage = stage1;
    }

    // The MFMAs above are opaque instructions to the compiler, so it does not know that the last of them
    // are still in the matrix pipe (16 cycles each) when the accumulators are read below: wait them out.
    __asm__ volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int m = 0; m < MT16; ++m)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) __asm__ volatile("" : "+a"(acc[m][ct]));
    // ---- epilogue: lane holds column l16 of each 16 x 16 tile, rows 4 * g4 + 0..3
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    if (full) {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        const int col = (nt0 + (ct >> 1)) * 32 + (ct & 1) * 16 + l16;
        if (nt0 + (ct >> 1) < a.n32) {
          const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
          for (int m = 0; m < MT16; ++m) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int row = m0 + 16 * m + 4 * g4 + r;
              if (row < a.M && row < m0 + C::kRows) {
                float v = acc[m][ct][r] + bvv;
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
      // partial sums in register order: float4 number (m * 4 + ct) of thread tid holds rows
      // 16 m + 4 g4 + 0..3 of one column -> every store is 1 KiB contiguous per wave
      float4* dst = reinterpret_cast<float4*>(a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * ((int64_t)C::kRows * kBN)) + tid;
#pragma unroll
      for (int m = 0; m < MT16; ++m)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          *dst = make_float4(acc[m][ct][0], acc[m][ct][1], acc[m][ct][2], acc[m][ct][3]);
          dst += NW * 64;
        }
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

// One half of d = nearest FP16 of (FP16 half SEL of x) * s + b, computed in FP32 with a single rounding; the
// other half of d is kept.  Written as instructions so that the two halves of an operand register can be
// produced in different gaps between MFMAs (the compiler would merge separately computed halves with
// extra moves), and, being volatile, they stay where they are written.
template <int SEL>
__device__ __forceinline__ void fma_mixlo(uint32_t& d, uint32_t x, float s, float b) {
  // (output only: the high half of d is whatever it was, and the caller overwrites it next)
  if constexpr (SEL == 0)
    __asm__ volatile("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(x), "v"(s), "v"(b));
  else
    __asm__ volatile("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(x), "v"(s), "v"(b));
}
template <int SEL>
__device__ __forceinline__ void fma_mixhi(uint32_t& d, uint32_t x, float s, float b) {
  if constexpr (SEL == 0)
    __asm__ volatile("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "+v"(d) : "v"(x), "v"(s), "v"(b));
  else
    __asm__ volatile("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(d) : "v"(x), "v"(s), "v"(b));
}

// pieces [spread7(i, n), spread7(i + 1, n)) of seven go behind item i of n (none behind items >= n)
constexpr int spread7(int i, int n) { return i * 7 / n > 7 ? 7 : i * 7 / n; }

// The same tiles on eight waves, two per SIMD.  Measured on the four-wave kernel above, everything that is
// not an MFMA adds to the time instead of hiding behind the matrix pipe (per 144 x 36864 launch: MFMAs
// alone 79 us of 177; the exact dequantization +41, the operand reads +24, the copies +34, the barrier
// +12): a wave issues in order, and a 16-cycle MFMA covers only four to eight cycles of the same wave's
// other work.  Here wave w = (column group w & 3, K slice w >> 2): the two waves of a SIMD work on the two
// 32-wide K slices of the same 64 columns, so nothing is read or dequantized twice, each wave's 36 MFMAs
// per step fall into four groups of nine (one column tile each) with the next column tile's
// dequantization spread one or two instructions per MFMA between them, and one wave's waits (LDS,
// copies, barrier) are the other wave's matrix time.  The activation operands are single-buffered: a
// row tile's register is reloaded for the next step right after its last MFMA of this step.  The two
// K-slice sums of a column group are added through LDS once per tile segment (each wave finishes two of
// the four column tiles), so the partial-sum layout and the reduction pass are those of the kernel above.
template <int MT16, bool H16M>
__global__ __launch_bounds__(512) void gemm_decode16x2_kernel(StreamArgs a) {
  using C = Dec16Cfg<MT16, H16M>;
  constexpr int kAStage = C::kAStage, kStageBytes = C::kStageBytes, kNST = C::kNST;
  constexpr int kPieces = C::kRowsLds / 8;                          // 8-row activation pieces per stage
  constexpr int kAC0 = (kPieces + 7) / 8, kAC1 = kPieces / 8;       // activation copies per step: waves 0..3, waves 4..7
  constexpr int kDqSpan = MT16 > 2 ? MT16 - 2 : 1;
  static_assert(MT16 * 16 * 1024 <= kNST * kStageBytes, "the exchange of the K-slice sums needs 16 KiB per row tile");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cg = wave & 3, sl = wave >> 2;
  const int l16 = lane & 15, g4 = lane >> 4;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, a.grid, p), rem_end = work_begin(a.rem_work, a.grid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;

  // operand read offsets inside a stage (see the kernel above), for this wave's K slice
  const int a_off = (l16 * kKS + swz(l16, 4 * sl + g4) * 8) * 2;
  const int bq_off = kAStage + cg * 2 * 1024 + l16 * 16 + g4 * 4 + sl * 512;
  const int bm_off = kAStage + 8 * 1024 + cg * 2 * 256 + l16 * (H16M ? 4 : 8);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

  while (round < a.rounds || pos < rem_end) {
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * a.grid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * a.grid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    int mblk, n_tile;
    tile_coords(tile, a.m_blocks, a.n_tiles, mblk, n_tile);
    const int m0 = mblk * C::kRows;
    const int nt0 = n_tile * 8 + cg * 2;   // first 32-column tile of this wave's column group

    f4_t acc[MT16][4];
#pragma unroll
    for (int m = 0; m < MT16; ++m)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) acc[m][ct] = (f4_t){0.f, 0.f, 0.f, 0.f};

    // this wave's copies per step: activation pieces wave, wave + 8, (wave + 16), and weight tile `wave`
    // of the block's eight (codes + {min, scale})
    const half_t* a_src[kAC0];
#pragma unroll
    for (int i = 0; i < kAC0; ++i) {
      const int prow = 8 * (wave + 8 * i) + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    const uint8_t* w_src;
    const float* m_src;
    {
      int nt = n_tile * 8 + wave;
      nt = nt < a.n32 ? nt : a.n32 - 1;   // ragged last column block: load valid data, never store it
      w_src = a.w + (int64_t)nt * a.ksteps * 1024 + lane * 16;
      m_src = reinterpret_cast<const float*>(a.meta) +
              (H16M ? (int64_t)nt * a.ksteps * 32 + (lane & 31) : (int64_t)nt * a.ksteps * 64 + lane);
    }
    // copy number c (0 .. kAC0 + 1) of a step; waves 4..7 have no activation piece number kAC1 where
    // the pieces do not divide by eight
    auto copy_one = [&](int c, int ks, int stage) {
      const int kc = ks < ks1 ? ks : ks1 - 1;   // past the end the last step is fetched again
      unsigned char* st = smem + stage * kStageBytes;
      if (c < kAC0) {
        if (c < kAC1 || wave < 4)
          __builtin_amdgcn_global_load_lds((gptr_t)(a_src[c] + kc * kKS), (lptr_t)(st + (wave + 8 * c) * 8 * kKS * 2), 16, 0, 0);
      } else if (c == kAC0) {
        __builtin_amdgcn_global_load_lds((gptr_t)(w_src + (int64_t)kc * 1024), (lptr_t)(st + kAStage + wave * 1024), 16, 0, 0);
      } else {
        __builtin_amdgcn_global_load_lds((gptr_t)(m_src + (int64_t)kc * (H16M ? 32 : 64)),
                                         (lptr_t)(st + kAStage + 8 * 1024 + wave * 256), 4, 0, 0);
      }
    };
    constexpr int kCopies = kAC0 + 2;
    // this wave's copies have landed, all but those of the newest N steps
    auto wait_steps = [&](auto N_) {
      constexpr int n = decltype(N_)::value;
      if (kAC0 == kAC1 || wave < 4)
        __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(n * (kAC0 + 2)) : "memory");
      else
        __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(n * (kAC1 + 2)) : "memory");
    };

    h8_t aop[MT16];
    u4_t bop[2];           // B operands of two column tiles in turn
    uint32_t cw[4];        // this wave's code words of the step, one per column tile
    float2 cm[4];
    uint32_t cmh[4];
    auto read_a_tile = [&](uint32_t st, auto M_) __attribute__((always_inline)) {
      constexpr int m = decltype(M_)::value;
      aop[m] = __builtin_bit_cast(h8_t, lds_read128<m * 16 * kKS * 2>(st + a_off));
    };
    auto read_b = [&](uint32_t st) {
      static_for<0, 4>([&](auto CT) __attribute__((always_inline)) {
        constexpr int ct = decltype(CT)::value;
        constexpr int qoff = (ct >> 1) * 1024 + (ct & 1) * 256;
        cw[ct] = lds_read32<qoff>(st + bq_off);
        constexpr int moff = (ct >> 1) * 256 + (ct & 1) * 16 * (H16M ? 4 : 8);
        if constexpr (H16M) cmh[ct] = lds_read32<moff>(st + bm_off); else cm[ct] = lds_read64<moff>(st + bm_off);
      });
    };
    auto landed_b = [&]() {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        lds_landed(cw[ct]);
        if constexpr (H16M) lds_landed(cmh[ct]); else lds_landed(cm[ct]);
      }
    };
    // Exact dequantization of column tile ct's code word into bop[ct & 1] in seven pieces of two or
    // three VALU instructions (0: FMA constants, 1 and 2: nibble masks, 3..6: two weights each into two
    // different registers), every piece pinned where it is written (see dq_piece above).
    float s24, s20, mn;
    uint32_t msk[4], r01[2];
    auto dq7 = [&](int ct, int piece) {
      if (piece == 0) {
        float2 m2 = cm[ct];
        if constexpr (H16M) {
          const h2_t pr = __builtin_bit_cast(h2_t, cmh[ct]);
          m2.x = (float)pr.x;
          m2.y = (float)pr.y;
        }
        s24 = m2.y * 16777216.0f;
        s20 = m2.y * 1048576.0f;
        mn = m2.x;
        __asm__ volatile("" : "+v"(s24), "+v"(s20), "+v"(mn));
      } else if (piece == 1) {
        msk[0] = cw[ct] & 0x000F000Fu;
        msk[1] = cw[ct] & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[0]), "+v"(msk[1]));
      } else if (piece == 2) {
        const uint32_t y = cw[ct] >> 8;
        msk[2] = y & 0x000F000Fu;
        msk[3] = y & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[2]), "+v"(msk[3]));
      } else if (piece == 3) {   // weights 0 and 2: low halves of operand registers 0 and 1
        fma_mixlo<0>(r01[0], msk[0], s24, mn);
        fma_mixlo<0>(r01[1], msk[2], s24, mn);
      } else if (piece == 4) {   // weights 1 and 3: high halves; registers 0 and 1 are complete
        fma_mixhi<0>(r01[0], msk[1], s20, mn);
        fma_mixhi<0>(r01[1], msk[3], s20, mn);
        bop[ct & 1][0] = r01[0];
        bop[ct & 1][1] = r01[1];
      } else if (piece == 5) {   // weights 4 and 6
        fma_mixlo<1>(r01[0], msk[0], s24, mn);
        fma_mixlo<1>(r01[1], msk[2], s24, mn);
      } else {                   // weights 5 and 7; registers 2 and 3 are complete
        fma_mixhi<1>(r01[0], msk[1], s20, mn);
        fma_mixhi<1>(r01[1], msk[3], s20, mn);
        bop[ct & 1][2] = r01[0];
        bop[ct & 1][3] = r01[1];
      }
    };

    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kNST; ++t)
#pragma unroll
      for (int c = 0; c < kCopies; ++c) copy_one(c, ks0 + t, t);
    wait_steps(IdxC<kNST - 1>{});   // step ks0 has landed
    __builtin_amdgcn_s_barrier();
    static_for<0, MT16>([&](auto M_) __attribute__((always_inline)) { read_a_tile(lds0, M_); });
    read_b(lds0);
    lds_wait();
    landed_b();
#pragma unroll
    for (int q = 0; q < 7; ++q) dq7(0, q);

    int stage = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage1 = stage + 1 == kNST ? 0 : stage + 1;
      const uint32_t Nt = lds0 + stage1 * kStageBytes;
      lds_wait();   // the activation operands of this step, requested during the last step
#pragma unroll
      for (int m = 0; m < MT16; ++m) lds_landed(aop[m]);
      __builtin_amdgcn_sched_barrier(0);
      // ---- column tiles 0, 1, 2: MFMAs with the dequantization of the next column tile between them
      static_for<0, 3 * MT16>([&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        constexpr int ct = i / MT16, m = i - ct * MT16;
        mfma16_inplace_v(acc[m][ct], aop[m], __builtin_bit_cast(h8_t, bop[ct & 1]));
        __builtin_amdgcn_sched_barrier(0);
        // seven pieces over the first MT16 - 2 MFMAs of the group: the last two MFMAs separate the
        // last register write from the first MFMA that reads it
        static_for<spread7(m, kDqSpan), spread7(m + 1, kDqSpan)>(
            [&](auto Q) __attribute__((always_inline)) { dq7(ct + 1, decltype(Q)::value); });
        if constexpr (MT16 < 3 && m == MT16 - 1) __asm__ volatile("s_nop 3");
        __builtin_amdgcn_sched_barrier(0);
      });
      // every wave's copies of step ks + 1 have landed, and nobody reads the stage of step ks any more
      wait_steps(IdxC<kNST - 2>{});
      __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the copies in flight stay in flight
      __builtin_amdgcn_sched_barrier(0);
      // ---- column tile 3: the next step's code words and {min, scale} first, its copies between the
      // first MFMAs, then the reloads of the activation operands and the dequantization of the next
      // step's column tile 0
      read_b(Nt);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int kH = MT16 / 2;   // MFMAs before the wait for the code words
      static_for<0, MT16>([&](auto M_) __attribute__((always_inline)) {
        constexpr int m = decltype(M_)::value;
        mfma16_inplace_v(acc[m][3], aop[m], __builtin_bit_cast(h8_t, bop[1]));
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (m < kH || MT16 == 1) {
          static_for<m * kCopies / (kH > 0 ? kH : 1), (MT16 == 1 ? kCopies : (m + 1) * kCopies / kH)>(
              [&](auto CC) __attribute__((always_inline)) { copy_one(decltype(CC)::value, ks + kNST, stage); });
        }
        if constexpr (m == kH || MT16 == 1) {
          lds_wait();
          landed_b();
          static_for<0, (MT16 == 1 ? 1 : kH + 1)>([&](auto R_) __attribute__((always_inline)) { read_a_tile(Nt, R_); });
        }
        if constexpr (m > kH) read_a_tile(Nt, M_);
        if constexpr (MT16 == 1) {
          static_for<0, 7>([&](auto Q) __attribute__((always_inline)) { dq7(0, decltype(Q)::value); });
          __asm__ volatile("s_nop 3");
        } else if constexpr (m >= kH && m < MT16 - 1) {
          constexpr int r = m - kH, n2 = MT16 - 1 - kH;
          static_for<r * 7 / n2, (r + 1) * 7 / n2>([&](auto Q) __attribute__((always_inline)) { dq7(0, decltype(Q)::value); });
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      stage = stage1;
    }

    // The MFMAs are opaque instructions to the compiler: wait out the last of them (16 cycles each)
    // before the accumulators are read.
    __asm__ volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int m = 0; m < MT16; ++m)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) __asm__ volatile("" : "+v"(acc[m][ct]));
    // ---- the two K-slice sums of a column group meet in LDS: the wave of slice 1 hands over column
    // tiles 0 and 1, the wave of slice 0 column tiles 2 and 3, and each finishes the two it keeps
    lds_wait();
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    float4* xb = reinterpret_cast<float4*>(smem);
    // (the accumulator array is only ever indexed with constants: each K slice has its own copy of the code)
    auto hand_over = [&](auto SL_) __attribute__((always_inline)) {
      constexpr int give = decltype(SL_)::value == 0 ? 2 : 0;
#pragma unroll
      for (int m = 0; m < MT16; ++m)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const f4_t v = acc[m][give + c];
          xb[(wave * (MT16 * 2) + m * 2 + c) * 64 + lane] = make_float4(v[0], v[1], v[2], v[3]);
          __builtin_amdgcn_sched_barrier(0);   // one tile at a time: this code must not raise the kernel's register count
        }
    };
    const bool full = (ks0 == 0) && (ks1 == a.ksteps);
    // adds the partner's sums to the two column tiles this wave keeps and stores them: lane holds
    // column l16, rows 4 g4 + 0..3 of each 16 x 16 tile
    auto finish_kept = [&](auto SL_) __attribute__((always_inline)) {
      constexpr int keep = decltype(SL_)::value == 0 ? 0 : 2;
      const int partner = wave ^ 4;
      float4* pdst = reinterpret_cast<float4*>(a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * ((int64_t)C::kRows * kBN)) +
                     (cg * 64 + lane);
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        constexpr int dummy = 0;
        (void)dummy;
        const int ct = keep + c;
        const int col = (nt0 + (ct >> 1)) * 32 + (ct & 1) * 16 + l16;
        const bool col_ok = nt0 + (ct >> 1) < a.n32;
        const float bvv = (full && col_ok && a.bias) ? (float)a.bias[col] : 0.f;
#pragma unroll
        for (int m = 0; m < MT16; ++m) {
          const float4 o = xb[(partner * (MT16 * 2) + m * 2 + c) * 64 + lane];
          const f4_t mine = acc[m][keep + c];
          const float v4[4] = {mine[0] + o.x, mine[1] + o.y, mine[2] + o.z, mine[3] + o.w};
          if (!full) {
            // partial sums in the order of the four-wave kernel: float4 number (m * 4 + ct) of thread cg * 64 + lane
            pdst[(m * 4 + ct) * 256] = make_float4(v4[0], v4[1], v4[2], v4[3]);
          } else if (col_ok) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int row = m0 + 16 * m + 4 * g4 + r;
              if (row < a.M && row < m0 + C::kRows) {
                float v = v4[r] + bvv;
                if (a.relu) v = fmaxf(v, 0.f);
                if (a.residual) v += (float)a.residual[(int64_t)row * a.ldr + col];
                if (a.out32)
                  a.out32[(int64_t)row * a.ldo + col] = v;
                else
                  a.out16[(int64_t)row * a.ldo + col] = (half_t)v;
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    if (sl == 0) hand_over(IdxC<0>{}); else hand_over(IdxC<1>{});
    __syncthreads();
    if (sl == 0) finish_kept(IdxC<0>{}); else finish_kept(IdxC<1>{});
    if (whole_round) {
      ++round;
    } else {
      pos += ks1 - ks0;
      ++seg;
    }
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// ---------------------------------------------------------------------------------------------
// Prefill shape on v_mfma_f32_16x16x32_f16.  With random operands the chip is limited by power, not by
// issue slots, and the 16 x 16 x 32 instruction delivers more flops per joule than the 32 x 32 x 16 one
// (MFMAs alone, random FP16 operands, every CU busy: 1.88 against 1.62 PFLOP/s), so the 256 x 256 tile of
// the prefill projections is computed on the small shape.
//   Wave w of eight: all 256 rows (16 row tiles) x the 32 columns of weight tile w (two column tiles of 16):
//   32 accumulators of four registers, kept in ordinary vector registers and updated in place.
//   Activations: three stages of 32 KiB, copied by all waves, one barrier per K step (as in the kernel
//   above).  Weights: a wave copies, reads and dequantizes only its own tile, so its codes and {min, scale}
//   pairs sit in a ring of five slots private to the wave in effect: its own vmcnt wait is all the
//   synchronisation they need, and the code words of step ks + 1 are read in the middle of step ks, which
//   leaves half a K step to dequantize them between MFMAs.
//   A K step is eight phases (K slice s = 0, 1) x (four groups of four row tiles); a phase issues the LDS
//   reads of the next phase's four A operands, then its 8 MFMAs (column tile 0: four row tiles, column
//   tile 1: the same four) with dequantization pieces and, in the last phase, the copies between them.
//     phases 0..3: dequantize slice 1 of this step;  phase 4: read the code words of step ks + 1;
//     phases 5..7: dequantize slice 0 of step ks + 1;  end of phase 6: vmcnt + barrier (stage ks + 1 has
//     landed for everyone, nobody reads stage ks any more);  phase 7: copies for ks + 3 (activations) and
//     ks + 5 (weights), A operands of the next step's first phase.
//   Copies are issued weights first, then activations, so that the one vmcnt count that guarantees the
//   activations of step ks + 1 also covers the weights of step ks + 2.
constexpr int kP16AStages = 3, kP16WSlots = 5, kP16Rows = 256;
constexpr int kP16AStage = kP16Rows * kKS * 2;
constexpr int kP16WBase = kP16AStages * kP16AStage;
constexpr int kP16Lds = kP16WBase + kP16WSlots * kBStageQ4;
constexpr int kP16Copies = 6;   // per wave per K step: codes, {min, scale}, four 8-row activation pieces
static_assert(kP16Lds <= kLdsBytes, "stages must fit in LDS");

// position (MFMA number within the K step, 0..63) behind which dequantization piece p of 14 goes: slice 1 of
// this step over MFMAs 0..29, slice 0 of the next step over MFMAs 41..61
constexpr int p16_pos_cur(int p) { return p * 30 / 14; }
constexpr int p16_pos_nxt(int p) { return 41 + p * 21 / 14; }
// slice 1's operands are first used by MFMA 32, the next step's slice 0 operands by MFMA 64 (= 0 of the next
// step), and the code words they are made from land with the wait that ends phase 4 (behind MFMA 39): a
// piece writes an operand register at least three MFMAs before the first MFMA that reads it
static_assert(p16_pos_cur(13) <= 32 - 4 && p16_pos_nxt(0) > 39 && p16_pos_nxt(13) <= 64 - 4, "dequantization windows");

// What both prefill kernels on 16 x 16 x 32 MFMAs do with a finished segment of a 256 x 256 tile: acc[m][ct]
// of wave w holds rows 16 m + 4 g4 + 0..3 of column 32 w + 16 ct + l16.
__device__ __forceinline__ void prefill16_finish_tile(const StreamArgs& a, f4_t (&acc)[16][2], bool full, int m0, int nt0, int p,
                                                      int seg, int wave, int l16, int g4) {
  // The MFMAs are opaque instructions to the compiler: wait out the last of them (16 cycles each)
  // before the accumulators are read.
  __asm__ volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int m = 0; m < 16; ++m)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) __asm__ volatile("" : "+v"(acc[m][ct]));
  // ---- epilogue: lane holds column l16 of each 16 x 16 tile, rows 4 * g4 + 0..3.  Neighbouring lanes
  // swap one value each (even lanes give away their column of column tile 1, odd lanes theirs of column
  // tile 0), after which every lane owns two adjacent columns and a store instruction covers 64
  // contiguous bytes of each of its four rows instead of 32.
  if (full) {
    if (nt0 < a.n32) {
      const bool odd = (l16 & 1) != 0;
      const int c0 = nt0 * 32 + l16, c1 = c0 + 16;
      const float b0 = a.bias ? (float)a.bias[c0] : 0.f, b1 = a.bias ? (float)a.bias[c1] : 0.f;
      const int cs = odd ? c1 - 1 : c0;   // first of the two adjacent columns this lane stores
      int row = m0 + 4 * g4;
      int64_t o_off = (int64_t)row * a.ldo + cs, r_off = (int64_t)row * a.ldr + cs;
#pragma unroll
      for (int m = 0; m < 16; ++m) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float x0 = acc[m][0][r] + b0, x1 = acc[m][1][r] + b1;
          if (a.relu) {
            x0 = fmaxf(x0, 0.f);
            x1 = fmaxf(x1, 0.f);
          }
          const float keep = odd ? x1 : x0, send = odd ? x0 : x1;
          // lane l <-> lane l ^ 1 (quad_perm [1, 0, 3, 2])
          const float recv = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
          float lo = odd ? recv : keep, hi = odd ? keep : recv;
          if (row < a.M) {
            if (a.residual) {
              const h2_t rr = *reinterpret_cast<const h2_t*>(a.residual + r_off);
              lo += (float)rr.x;
              hi += (float)rr.y;
            }
            if (a.out32)
              *reinterpret_cast<float2*>(a.out32 + o_off) = make_float2(lo, hi);
            else
              *reinterpret_cast<h2_t*>(a.out16 + o_off) = (h2_t){(half_t)lo, (half_t)hi};
          }
          const int step = r == 3 ? 13 : 1;   // rows 16 m + 4 g4 + r
          row += step;
          o_off += step * a.ldo;
          r_off += step * a.ldr;
        }
      }
    }
  } else {
    // Partial sums in the layout of gemm_stream_kernel<8, 1, 1, 8> (its reduction pass finishes these
    // tiles too): float4 number (2 m + g4 / 2) of "thread" 64 wave + 32 (g4 % 2) + 16 ct + l16 holds
    // rows 16 m + 4 g4 + 0..3 of column 32 wave + 16 ct + l16.
    float4* base = reinterpret_cast<float4*>(a.partial + ((int64_t)p * 2 + (seg == 0 ? 0 : 1)) * ((int64_t)kP16Rows * kBN));
#pragma unroll
    for (int m = 0; m < 16; ++m)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        if (m0 + 16 * m + 8 * (g4 >> 1) < a.M)   // rows beyond M: padding, never read back
          base[(2 * m + (g4 >> 1)) * 512 + wave * 64 + (g4 & 1) * 32 + ct * 16 + l16] =
              make_float4(acc[m][ct][0], acc[m][ct][1], acc[m][ct][2], acc[m][ct][3]);
      }
  }
}

template <bool H16M>
__global__ __launch_bounds__(512) void gemm_prefill16_kernel(StreamArgs a) {
  constexpr int NW = 8, RH = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, a.grid, p), rem_end = work_begin(a.rem_work, a.grid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;

  // A operand of (row tile m, slice sl): + m * 16 * kKS * 2
  int a_off[2];
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) a_off[sl] = (l16 * kKS + swz(l16, 4 * sl + g4) * 8) * 2;
  // code word of (column tile ct, slice sl) in a weight slot: + ct * 256 + sl * 512
  const int bq_off = kP16WBase + wave * 1024 + l16 * 16 + g4 * 4;
  // {min, scale} of column tile ct: + ct * 16 * (H16M ? 4 : 8)
  const int bm_off = kP16WBase + 8 * 1024 + wave * 256 + l16 * (H16M ? 4 : 8);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

  while (round < a.rounds || pos < rem_end) {
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * a.grid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * a.grid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    int mblk, n_tile;
    tile_coords(tile, a.m_blocks, a.n_tiles, mblk, n_tile);
    const int m0 = mblk * kP16Rows;
    const int nt0 = n_tile * 8 + wave;   // this wave's 32-column weight tile

    f4_t acc[16][2];
#pragma unroll
    for (int m = 0; m < 16; ++m)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) acc[m][ct] = (f4_t){0.f, 0.f, 0.f, 0.f};

    // this wave's four activation pieces per step: piece c = wave + 8 i covers rows 8 c .. 8 c + 7
    const half_t* a_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = wave + NW * i;
      const int prow = 8 * c + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
    }
    const uint8_t* w_src;
    const float* m_src;
    {
      int nt = nt0 < a.n32 ? nt0 : a.n32 - 1;   // ragged last column block: load valid data, never store it
      w_src = a.w + (int64_t)nt * a.ksteps * 1024 + lane * 16;
      m_src = reinterpret_cast<const float*>(a.meta) +
              (H16M ? (int64_t)nt * a.ksteps * 32 + (lane & 31) : (int64_t)nt * a.ksteps * 64 + lane);
    }
    // copy c of step ks: 0 = codes, 1 = {min, scale} (into weight slot wslot), 2..5 = activation pieces
    // (into stage).  Past the end of the segment the last step is fetched again: harmless, and it keeps
    // the VMEM counts uniform.
    auto copy_one = [&](int c, int ks_w, int wslot, int ks_a, int stage) {
      if (c == 0) {
        const int kc = ks_w < ks1 ? ks_w : ks1 - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(w_src + (int64_t)kc * 1024),
                                         (lptr_t)(smem + kP16WBase + wslot * kBStageQ4 + wave * 1024), 16, 0, 0);
      } else if (c == 1) {
        const int kc = ks_w < ks1 ? ks_w : ks1 - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(m_src + (int64_t)kc * (H16M ? 32 : 64)),
                                         (lptr_t)(smem + kP16WBase + wslot * kBStageQ4 + 8 * 1024 + wave * 256), 4, 0, 0);
      } else {
        const int kc = ks_a < ks1 ? ks_a : ks1 - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[c - 2] + kc * kKS),
                                         (lptr_t)(smem + stage * kP16AStage + (wave + NW * (c - 2)) * 8 * kKS * 2), 16, 0, 0);
      }
    };

    h8_t aop[2][RH];
    u4_t bop[2][2];        // [slice][column tile]
    uint32_t cw[2][2];     // raw code words [slice][column tile]
    float2 cm[2];
    uint32_t cmh[2];
    float s24, s20, mn;
    uint32_t msk[4], r01[2];
    // A operands of phase q (slice q / 4, row tiles 4 (q % 4) .. + 3) of the stage at st
    auto read_a = [&](uint32_t st, auto Q_, h8_t* dst) {
      constexpr int q = decltype(Q_)::value;
      const uint32_t ad = st + a_off[q >> 2];
      static_for<0, RH>([&](auto M_) __attribute__((always_inline)) {
        constexpr int off = ((q & 3) * RH + decltype(M_)::value) * 16 * kKS * 2;
        dst[decltype(M_)::value] = __builtin_bit_cast(h8_t, lds_read128<off>(ad));
      });
    };
    auto read_b = [&](int wslot) {
      const uint32_t st = lds0 + wslot * kBStageQ4;
      static_for<0, 2>([&](auto CT) __attribute__((always_inline)) {
        constexpr int ct = decltype(CT)::value;
        cw[0][ct] = lds_read32<ct * 256>(st + bq_off);
        cw[1][ct] = lds_read32<ct * 256 + 512>(st + bq_off);
        constexpr int moff = ct * 16 * (H16M ? 4 : 8);
        if constexpr (H16M) cmh[ct] = lds_read32<moff>(st + bm_off); else cm[ct] = lds_read64<moff>(st + bm_off);
      });
    };
    auto landed_b = [&]() {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        lds_landed(cw[0][ct]);
        lds_landed(cw[1][ct]);
        if constexpr (H16M) lds_landed(cmh[ct]); else lds_landed(cm[ct]);
      }
    };
    // Exact dequantization (fg_common.h: dequant8_exact) of code word (sl, ct) into bop[sl][ct], in seven
    // pieces of one to three instructions that stay where they are written (see gemm_decode16_kernel).
    auto dq7 = [&](int sl, int ct, int piece) {
      if (piece == 0) {
        float2 m2 = cm[ct];
        if constexpr (H16M) {
          const h2_t pr = __builtin_bit_cast(h2_t, cmh[ct]);
          m2.x = (float)pr.x;
          m2.y = (float)pr.y;
        }
        s24 = m2.y * 16777216.0f;
        s20 = m2.y * 1048576.0f;
        mn = m2.x;
        __asm__ volatile("" : "+v"(s24), "+v"(s20), "+v"(mn));
      } else if (piece == 1) {
        msk[0] = cw[sl][ct] & 0x000F000Fu;
        msk[1] = cw[sl][ct] & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[0]), "+v"(msk[1]));
      } else if (piece == 2) {
        const uint32_t y = cw[sl][ct] >> 8;
        msk[2] = y & 0x000F000Fu;
        msk[3] = y & 0x00F000F0u;
        __asm__ volatile("" : "+v"(msk[2]), "+v"(msk[3]));
      } else if (piece == 3) {   // weights 0 and 2: low halves of operand registers 0 and 1
        fma_mixlo<0>(r01[0], msk[0], s24, mn);
        fma_mixlo<0>(r01[1], msk[2], s24, mn);
      } else if (piece == 4) {   // weights 1 and 3: high halves; registers 0 and 1 are complete
        fma_mixhi<0>(r01[0], msk[1], s20, mn);
        fma_mixhi<0>(r01[1], msk[3], s20, mn);
        bop[sl][ct][0] = r01[0];
        bop[sl][ct][1] = r01[1];
      } else if (piece == 5) {   // weights 4 and 6
        fma_mixlo<1>(r01[0], msk[0], s24, mn);
        fma_mixlo<1>(r01[1], msk[2], s24, mn);
      } else {                   // weights 5 and 7; registers 2 and 3 are complete
        fma_mixhi<1>(r01[0], msk[1], s20, mn);
        fma_mixhi<1>(r01[1], msk[3], s20, mn);
        bop[sl][ct][2] = r01[0];
        bop[sl][ct][3] = r01[1];
      }
    };

    // no copy of the previous segment may still be in flight towards a stage, and no wave still reads one
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // the copy groups of steps ks0 - 5 .. ks0 - 1, as the steady state would have issued them
    copy_one(0, ks0, 0, 0, 0);
    copy_one(1, ks0, 0, 0, 0);
    copy_one(0, ks0 + 1, 1, 0, 0);
    copy_one(1, ks0 + 1, 1, 0, 0);
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int c = 0; c < kP16Copies; ++c) copy_one(c, ks0 + 2 + t, 2 + t, ks0 + t, t);
    __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kP16Copies) : "memory");   // weights ks0 .. ks0 + 2, activations ks0
    __builtin_amdgcn_s_barrier();
    read_a(lds0, IdxC<0>{}, aop[0]);
    read_b(0);
    lds_wait();
#pragma unroll
    for (int m = 0; m < RH; ++m) lds_landed(aop[0][m]);
    landed_b();
#pragma unroll
    for (int q = 0; q < 14; ++q) dq7(0, q / 7, q % 7);

    int stage = 0, wslot = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage1 = stage + 1 == kP16AStages ? 0 : stage + 1;
      const int wslot1 = wslot + 1 == kP16WSlots ? 0 : wslot + 1;
      const uint32_t At = lds0 + stage * kP16AStage;
      static_for<0, 8>([&](auto Q_) __attribute__((always_inline)) {
        constexpr int q = decltype(Q_)::value;
        constexpr int sl = q >> 2, cur = q & 1, nxt = cur ^ 1;
        if constexpr (q < 7)
          read_a(At, IdxC<q + 1>{}, aop[nxt]);
        else
          read_a(lds0 + stage1 * kP16AStage, IdxC<0>{}, aop[nxt]);
        if constexpr (q == 4) read_b(wslot1);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, 2 * RH>([&](auto I) __attribute__((always_inline)) {
          constexpr int i = decltype(I)::value;
          constexpr int ct = i / RH, m = i - ct * RH, g = q * 8 + i;
          mfma16_inplace_v(acc[(q & 3) * RH + m][ct], aop[cur][m], __builtin_bit_cast(h8_t, bop[sl][ct]));
          __builtin_amdgcn_sched_barrier(0);
          static_for<0, 14>([&](auto P_) __attribute__((always_inline)) {
            constexpr int pc = decltype(P_)::value;
            if constexpr (p16_pos_cur(pc) == g) dq7(1, pc / 7, pc % 7);
            if constexpr (p16_pos_nxt(pc) == g) dq7(0, pc / 7, pc % 7);
          });
          if constexpr (q == 7 && i < kP16Copies) copy_one(i, ks + kP16WSlots, wslot, ks + kP16AStages, stage);
          __builtin_amdgcn_sched_barrier(0);
        });
        lds_wait();
#pragma unroll
        for (int m = 0; m < RH; ++m) lds_landed(aop[nxt][m]);
        if constexpr (q == 4) landed_b();
        if constexpr (q == 6) {
          __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(kP16Copies) : "memory");
          __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the copies in flight stay in flight
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      stage = stage1;
      wslot = wslot1;
    }

    prefill16_finish_tile(a, acc, (ks0 == 0) && (ks1 == a.ksteps), m0, nt0, p, seg, wave, l16, g4);
    if (whole_round) {
      ++round;
    } else {
      pos += ks1 - ks0;
      ++seg;
    }
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may still target LDS when the wave ends
}

// The same tile on row-major FP16 weights (the uncompressed workload's prefill projections).  Nothing to
// dequantize: a wave's B operands are read from LDS like its A operands.  Activations: three stages of
// 32 KiB behind the per-step barrier, as above.  Weights: wave w copies and reads only rows 32 w .. + 31 of
// the [256 columns][64 k] block (4 KiB per step), so they sit in two 32 KiB slots that the wave's own vmcnt
// wait synchronises; the copies of a step are issued weights (for step ks + 2) first, then activations (for
// step ks + 3), and one count covers "activations of ks + 1 and weights of ks + 1 have landed".
// Phases as above; slice 1's B operands are read at the start of phase 2, the next step's slice 0 operands at
// the start of the last phase, after the barrier.
constexpr int kP16FWSlots = 2;
constexpr int kP16FLds = kP16WBase + kP16FWSlots * kBStageF16;
constexpr int kP16FCopies = 8;   // per wave per K step: four 8-row weight pieces, four 8-row activation pieces
static_assert(kP16FLds <= kLdsBytes, "stages must fit in LDS");

__global__ __launch_bounds__(512) void gemm_prefill16_f16_kernel(StreamArgs a) {
  constexpr int NW = 8, RH = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;

  const int p = (blockIdx.x & 7) * (a.grid >> 3) + (blockIdx.x >> 3);
  const int64_t rem_begin = work_begin(a.rem_work, a.grid, p), rem_end = work_begin(a.rem_work, a.grid, p + 1);
  int64_t pos = rem_begin;
  int round = 0, seg = 0;

  // A operand of (row tile m, slice sl): + m * 16 * kKS * 2
  int a_off[2];
  // B operand of (column tile ct, slice sl) in a weight slot: row 32 wave + 16 ct + l16 of the block
  int b_off[2][2];
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) {
    a_off[sl] = (l16 * kKS + swz(l16, 4 * sl + g4) * 8) * 2;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int r = wave * 32 + ct * 16 + l16;
      b_off[sl][ct] = kP16WBase + (r * kKS + swz(r, 4 * sl + g4) * 8) * 2;
    }
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

  while (round < a.rounds || pos < rem_end) {
    int64_t tile;
    int ks0, ks1;
    const bool whole_round = round < a.rounds;
    if (whole_round) {
      tile = (int64_t)round * a.grid + p;
      ks0 = 0;
      ks1 = a.ksteps;
    } else {
      const int64_t t = pos / a.ksteps;
      tile = (int64_t)a.rounds * a.grid + t;
      ks0 = (int)(pos - t * a.ksteps);
      const int64_t left = rem_end - pos;
      ks1 = (int)((int64_t)(a.ksteps - ks0) < left ? a.ksteps : ks0 + left);
    }
    int mblk, n_tile;
    tile_coords(tile, a.m_blocks, a.n_tiles, mblk, n_tile);
    const int m0 = mblk * kP16Rows;
    const int nt0 = n_tile * 8 + wave;   // this wave's 32 columns, as a 32-column tile number

    f4_t acc[16][2];
#pragma unroll
    for (int m = 0; m < 16; ++m)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) acc[m][ct] = (f4_t){0.f, 0.f, 0.f, 0.f};

    // this wave's four activation pieces per step: piece c = wave + 8 i covers rows 8 c .. 8 c + 7 of the tile;
    // its four weight pieces: rows (output columns) 32 wave + 8 i .. + 7 of the block
    const half_t* a_src[4];
    const uint8_t* w_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = wave + NW * i;
      const int prow = 8 * c + (lane >> 3);
      int row = m0 + prow;
      row = row < a.M ? row : a.M - 1;
      a_src[i] = a.x + (int64_t)row * a.ldx + swz(prow, lane & 7) * 8;
      const int wrow = wave * 32 + 8 * i + (lane >> 3);
      int col = n_tile * kBN + wrow;
      col = col < a.N ? col : a.N - 1;   // ragged last column block: load valid data, never store it
      w_src[i] = a.w + ((int64_t)col * a.K + swz(wrow, lane & 7) * 8) * 2;
    }
    // copy c of a step: 0..3 = weight pieces of step ks_w (into weight slot wslot), 4..7 = activation pieces
    // of step ks_a (into stage).  Past the end of the segment the last step is fetched again: harmless, and it
    // keeps the VMEM counts uniform.
    auto copy_one = [&](int c, int ks_w, int wslot, int ks_a, int stage) {
      if (c < 4) {
        const int kc = ks_w < ks1 ? ks_w : ks1 - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(w_src[c] + (int64_t)kc * (kKS * 2)),
                                         (lptr_t)(smem + kP16WBase + wslot * kBStageF16 + (wave * 4 + c) * 8 * kKS * 2), 16, 0, 0);
      } else {
        const int kc = ks_a < ks1 ? ks_a : ks1 - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[c - 4] + kc * kKS),
                                         (lptr_t)(smem + stage * kP16AStage + (wave + NW * (c - 4)) * 8 * kKS * 2), 16, 0, 0);
      }
    };

    h8_t aop[2][RH];
    u4_t bop[2][2];   // [slice][column tile]
    auto read_a = [&](uint32_t st, auto Q_, h8_t* dst) {
      constexpr int q = decltype(Q_)::value;
      const uint32_t ad = st + a_off[q >> 2];
      static_for<0, RH>([&](auto M_) __attribute__((always_inline)) {
        constexpr int off = ((q & 3) * RH + decltype(M_)::value) * 16 * kKS * 2;
        dst[decltype(M_)::value] = __builtin_bit_cast(h8_t, lds_read128<off>(ad));
      });
    };
    auto read_b = [&](int wslot, auto SL_) {
      constexpr int sl = decltype(SL_)::value;
      const uint32_t st = lds0 + wslot * kBStageF16;
      bop[sl][0] = lds_read128<0>(st + b_off[sl][0]);
      bop[sl][1] = lds_read128<0>(st + b_off[sl][1]);
    };

    // no copy of the previous segment may still be in flight towards a stage, and no wave still reads one
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // the copy groups of steps ks0 - 3 .. ks0 - 1, as the steady state would have issued them
#pragma unroll
    for (int c = 4; c < kP16FCopies; ++c) copy_one(c, 0, 0, ks0, 0);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < kP16FCopies; ++c) copy_one(c, ks0 + t, t, ks0 + 1 + t, 1 + t);
    __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(12) : "memory");   // activations and weights of step ks0
    __builtin_amdgcn_s_barrier();
    read_a(lds0, IdxC<0>{}, aop[0]);
    read_b(0, IdxC<0>{});
    lds_wait();
#pragma unroll
    for (int m = 0; m < RH; ++m) lds_landed(aop[0][m]);
    lds_landed(bop[0][0]);
    lds_landed(bop[0][1]);

    int stage = 0, wslot = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage1 = stage + 1 == kP16AStages ? 0 : stage + 1;
      const int wslot1 = wslot ^ 1;
      const uint32_t At = lds0 + stage * kP16AStage;
      static_for<0, 8>([&](auto Q_) __attribute__((always_inline)) {
        constexpr int q = decltype(Q_)::value;
        constexpr int sl = q >> 2, cur = q & 1, nxt = cur ^ 1;
        if constexpr (q < 7)
          read_a(At, IdxC<q + 1>{}, aop[nxt]);
        else
          read_a(lds0 + stage1 * kP16AStage, IdxC<0>{}, aop[nxt]);
        if constexpr (q == 2) read_b(wslot, IdxC<1>{});
        if constexpr (q == 7) read_b(wslot1, IdxC<0>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, 2 * RH>([&](auto I) __attribute__((always_inline)) {
          constexpr int i = decltype(I)::value;
          constexpr int ct = i / RH, m = i - ct * RH;
          mfma16_inplace_v(acc[(q & 3) * RH + m][ct], aop[cur][m], __builtin_bit_cast(h8_t, bop[sl][ct]));
          __builtin_amdgcn_sched_barrier(0);
          // (weights into the slot whose last operands were read at phase 2 of this step)
          if constexpr (q == 7) copy_one(i, ks + kP16FWSlots, wslot, ks + kP16AStages, stage);
          __builtin_amdgcn_sched_barrier(0);
        });
        lds_wait();
#pragma unroll
        for (int m = 0; m < RH; ++m) lds_landed(aop[nxt][m]);
        if constexpr (q == 2) {
          lds_landed(bop[1][0]);
          lds_landed(bop[1][1]);
        }
        if constexpr (q == 7) {
          lds_landed(bop[0][0]);
          lds_landed(bop[0][1]);
        }
        if constexpr (q == 6) {
          // outstanding may stay: the four activation pieces of step ks + 2 (issued last in step ks - 1)
          __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(4) : "memory");
          __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the copies in flight stay in flight
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      stage = stage1;
      wslot = wslot1;
    }

    prefill16_finish_tile(a, acc, (ks0 == 0) && (ks1 == a.ksteps), m0, nt0, p, seg, wave, l16, g4);
    if (whole_round) {
      ++round;
    } else {
      pos += ks1 - ks0;
      ++seg;
    }
  }
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may still target LDS when the wave ends
}

// Reduction pass for gemm_decode16_kernel: thread tid of a block adds, in ascending K order, the float4s
// that thread tid of the contributing workgroups wrote, then applies the epilogue.  blockIdx.x counts the
// tiles after the whole rounds, blockIdx.y spreads a thread's MT16 * 4 items.
__global__ __launch_bounds__(256) void gemm_decode16_finish_kernel(StreamArgs a, int mt16) {
  const int64_t t = blockIdx.x;
  const int64_t w0 = t * a.ksteps, w1 = w0 + a.ksteps;
  int p_lo = (int)((w0 * a.grid) / a.rem_work);
  while (p_lo + 1 < a.grid && work_begin(a.rem_work, a.grid, p_lo + 1) <= w0) ++p_lo;
  while (p_lo > 0 && work_begin(a.rem_work, a.grid, p_lo) > w0) --p_lo;
  if (work_begin(a.rem_work, a.grid, p_lo + 1) >= w1) return;   // one workgroup owned the whole tile
  int p_hi = p_lo;
  while (p_hi + 1 < a.grid && work_begin(a.rem_work, a.grid, p_hi + 1) < w1) ++p_hi;

  int mblk, n_tile;
  tile_coords((int64_t)a.rounds * a.grid + t, a.m_blocks, a.n_tiles, mblk, n_tile);
  const int rows_t = mt16 * 16;
  const int m0 = mblk * rows_t;
  const int64_t slot = (int64_t)rows_t * kBN;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
  const int n_items = mt16 * 4;
  float4 v[kFinishItems];
#pragma unroll
  for (int i = 0; i < kFinishItems; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  int p = p_lo;
  while (p <= p_hi) {
    const float4* src[kFinishParts];
    int n = 0;
    for (; p <= p_hi && n < kFinishParts; ++p) {
      const int64_t pb = work_begin(a.rem_work, a.grid, p);
      if (work_begin(a.rem_work, a.grid, p + 1) == pb) continue;
      const int s = pb >= w0 ? 0 : 1;
      src[n++] = reinterpret_cast<const float4*>(a.partial + ((int64_t)p * 2 + s) * slot) + tid;
    }
    float4 x[kFinishParts][kFinishItems];
#pragma unroll
    for (int c = 0; c < kFinishParts; ++c)
#pragma unroll
      for (int i = 0; i < kFinishItems; ++i) {
        const int e = blockIdx.y + i * gridDim.y;
        x[c][i] = (c < n && e < n_items) ? src[c < n ? c : 0][(int64_t)e * 256] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
    for (int c = 0; c < kFinishParts; ++c)
      if (c < n) {
#pragma unroll
        for (int i = 0; i < kFinishItems; ++i) {
          v[i].x += x[c][i].x;
          v[i].y += x[c][i].y;
          v[i].z += x[c][i].z;
          v[i].w += x[c][i].w;
        }
      }
  }
#pragma unroll
  for (int i = 0; i < kFinishItems; ++i) {
    const int e = blockIdx.y + i * gridDim.y;
    if (e >= n_items) break;
    const int m = e >> 2, ct = e & 3;
    const int row0 = m0 + 16 * m + 4 * g4;
    const int col = n_tile * kBN + wave * 64 + ct * 16 + l16;
    if (col >= a.N) continue;
    const float o[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    const float bvv = a.bias ? (float)a.bias[col] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + r;
      if (row >= a.M || row >= m0 + rows_t) break;
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

// canonical [N][K/2] codes + [N][K/64] meta  ->  tiled: one thread per 16-byte piece
template <class PairT>   // float2, or uint32_t for a pair of FP16 numbers
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint8_t* __restrict__ codes,
                                                           const PairT* __restrict__ meta, int N, int K,
                                                           uint8_t* __restrict__ codes_out,
                                                           PairT* __restrict__ meta_out) {
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

// rows per workgroup tile and the kernel shape for m rows
struct Shape {
  int mt, nt, wm, nw;
  int rows() const { return wm * mt * 32; }
  // One workgroup per CU, except for the 32-row shape: its stages are small enough for two workgroups
  // per CU, which doubles the bytes in flight of what is then a pure weight streamer.
  int grid() const { return (wm == 1 && mt == 1) ? 512 : 256; }
};
Shape pick_shape(int64_t m) {
  // Up to two row blocks the side-by-side shape wins (few tiles: the 256-row shape would leave most of
  // its stream-K pieces short); beyond that the weights would be re-read too often.
  if (m > 2 * kMaxMT * 32) return {8, 1, 1, 8};
  if (m > kMaxMT * 32) m = ceil_div(m, 2);
  const int need = (int)ceil_div(m, 32);
  return {need < 1 ? 1 : need, 2, 1, 4};
}

// blocks along y of the reduction pass: every thread takes at most kFinishItems of the mt*nt*4 items
static inline unsigned finish_y(const Shape& sh) { return (unsigned)ceil_div(sh.mt * sh.nt * 4, kFinishItems); }

template <int MT, int NT, int WM, int NW, bool F16W, bool H16M = false>
int launch_t(const StreamArgs& a, hipStream_t stream) {
  using C = StreamCfg<MT, NT, WM, NW, F16W>;
  const size_t smem = (size_t)C::kNST * C::kStageBytes;
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_stream_kernel<MT, NT, WM, NW, F16W, H16M>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_stream_kernel<MT, NT, WM, NW, F16W, H16M>), dim3(a.grid), dim3(NW * 64), smem, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

// Eight waves from five row tiles up (measured against four waves in one run, 144 rows: QKV 162-167 vs
// 176-178 us, FFN1 210-218 vs 225-229, FFN2 219-221 vs 227-230; 112 rows 135-144 vs 151; level at 48 rows,
// 3-7 % slower at 4 and 16 rows, where a wave has too few MFMAs per step to spread anything between).
template <bool H16M>
int launch_prefill16(const StreamArgs& a, hipStream_t stream) {
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_prefill16_kernel<H16M>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kP16Lds));
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_prefill16_kernel<H16M>), dim3(a.grid), dim3(512), kP16Lds, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int launch_prefill16_f16(const StreamArgs& a, hipStream_t stream) {
  static bool attr_done = false;
  if (!attr_done) {
    FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_prefill16_f16_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kP16FLds));
    attr_done = true;
  }
  hipLaunchKernelGGL(gemm_prefill16_f16_kernel, dim3(a.grid), dim3(512), kP16FLds, stream, a);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

template <int MT16, bool H16M>
int launch_dec16(const StreamArgs& a, hipStream_t stream) {
  using C = Dec16Cfg<MT16, H16M>;
  const size_t smem = (size_t)C::kNST * C::kStageBytes;
  constexpr bool kEight = MT16 >= 5;
  static bool attr_done = false;
  if constexpr (kEight) {
    if (!attr_done) {
      FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_decode16x2_kernel<MT16, H16M>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      attr_done = true;
    }
    hipLaunchKernelGGL((gemm_decode16x2_kernel<MT16, H16M>), dim3(a.grid), dim3(512), smem, stream, a);
  } else {
    if (!attr_done) {
      FG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_decode16_kernel<MT16, H16M>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      attr_done = true;
    }
    hipLaunchKernelGGL((gemm_decode16_kernel<MT16, H16M>), dim3(a.grid), dim3(256), smem, stream, a);
  }
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace

size_t gemm_stream_workspace(int64_t n, int64_t k, int64_t m) {
  (void)n;
  (void)k;
  const Shape sh = pick_shape(m);
  return (size_t)sh.grid() * 2 * sh.rows() * kBN * sizeof(float);
}

int gemm_stream_launch(const LinearArgs& la, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (la.m == 0 || la.n == 0) return FG_OK;
  const Shape sh = pick_shape(la.m);
  StreamArgs a;
  a.w = reinterpret_cast<const uint8_t*>(la.w_data);
  a.meta = reinterpret_cast<const float2*>(la.w_meta);
  a.x = la.x;
  a.ldx = la.ldx;
  a.M = (int)la.m;
  a.N = (int)la.n;
  a.K = (int)la.k;
  a.m_blocks = (int)ceil_div(la.m, sh.rows());
  a.n_tiles = (int)ceil_div(la.n, kBN);
  a.ksteps = (int)(la.k / kKS);
  a.n32 = (int)(la.n / 32);
  a.grid = sh.grid();
  const int64_t tiles = (int64_t)a.m_blocks * a.n_tiles;
  a.rounds = (int)(tiles / a.grid);
  const int64_t rem_tiles = tiles - (int64_t)a.rounds * a.grid;
  a.rem_work = rem_tiles * a.ksteps;
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
  if (sh.nw == 8) {   // prefill shape: GEMM and reduction of the last partial round are one profile record
    ProfScope prof(FG_K_GEMM_LARGE_M, stream);
    if (la.dtype != FG_Q4G64_TILED && la.dtype != FG_Q4G64_H16_TILED && la.dtype != FG_F16) return FG_ERR_UNSUPPORTED;
    const int rc = la.dtype == FG_F16               ? launch_prefill16_f16(a, stream)
                   : la.dtype == FG_Q4G64_H16_TILED ? launch_prefill16<true>(a, stream)
                                                    : launch_prefill16<false>(a, stream);
    if (rc) return rc;
    if (rem_tiles > 0) {
      hipLaunchKernelGGL(gemm_stream_finish_kernel, dim3((unsigned)rem_tiles, finish_y(sh)), dim3(sh.nw * 64), 0, stream, a, sh.mt,
                         sh.nt, sh.wm);
      FG_LAUNCH_CHECK();
    }
    return FG_OK;
  }
  // 4-bit weights on 16-row tiles: where the rows fill an odd number of them (e.g. 144 = 9 x 16) the
  // 32-row tiles would compute 16 padding rows, and from six tiles up the eight-wave kernel is the faster
  // one at even counts too (measured in one run, 128 rows: 55-71 vs 56-73 us on the OPT-30B shapes, 150
  // vs 160 us at 36864 x 12288; two blocks of 128: 97-101 vs 106-109 us)
  const int rows_blk = sh.rows() < (int)la.m ? (int)ceil_div(la.m, a.m_blocks) : (int)la.m;
  const int mt16 = (int)ceil_div(rows_blk, 16);
  if (la.dtype != FG_F16 && ((mt16 & 1) || mt16 >= 6) && mt16 <= 9 && ceil_div(la.m, mt16 * 16) == a.m_blocks) {
    const bool h16m = la.dtype == FG_Q4G64_H16_TILED;
    {
      ProfScope prof(FG_K_GEMM_SMALL_M, stream);
      int rc = FG_ERR_UNSUPPORTED;
#define FG_DEC16_CASE(MT)                                                                          \
  case MT:                                                                                         \
    rc = h16m ? launch_dec16<MT, true>(a, stream) : launch_dec16<MT, false>(a, stream);            \
    break;
      switch (mt16) {
        FG_DEC16_CASE(1)
        FG_DEC16_CASE(3)
        FG_DEC16_CASE(5)
        FG_DEC16_CASE(6)
        FG_DEC16_CASE(7)
        FG_DEC16_CASE(8)
        FG_DEC16_CASE(9)
      }
#undef FG_DEC16_CASE
      if (rc) return rc;
    }
    if (rem_tiles > 0) {
      ProfScope prof(FG_K_GEMM_SMALL_M_FINISH, stream);
      hipLaunchKernelGGL(gemm_decode16_finish_kernel, dim3((unsigned)rem_tiles, (unsigned)ceil_div(mt16 * 4, kFinishItems)),
                         dim3(256), 0, stream, a, mt16);
      FG_LAUNCH_CHECK();
    }
    return FG_OK;
  }
  {
    ProfScope prof(FG_K_GEMM_SMALL_M, stream);
    int rc = FG_ERR_UNSUPPORTED;
    const bool f16w = la.dtype == FG_F16, h16m = la.dtype == FG_Q4G64_H16_TILED;
#define FG_STREAM_CASE(MT)                                                     \
  case MT:                                                                     \
    rc = f16w   ? launch_t<MT, 2, 1, 4, true>(a, stream)                       \
         : h16m ? launch_t<MT, 2, 1, 4, false, true>(a, stream)                \
                : launch_t<MT, 2, 1, 4, false>(a, stream);                     \
    break;
    switch (sh.mt) {
      FG_STREAM_CASE(1)
      FG_STREAM_CASE(2)
      FG_STREAM_CASE(3)
      FG_STREAM_CASE(4)
      FG_STREAM_CASE(5)
    }
#undef FG_STREAM_CASE
    if (rc) return rc;
  }
  if (rem_tiles > 0) {
    ProfScope prof(FG_K_GEMM_SMALL_M_FINISH, stream);
    hipLaunchKernelGGL(gemm_stream_finish_kernel, dim3((unsigned)rem_tiles, finish_y(sh)),
                       dim3(sh.nw * 64), 0, stream, a, sh.mt, sh.nt, sh.wm);
    FG_LAUNCH_CHECK();
  }
  return FG_OK;
}

int pack_weights_launch(const void* codes, const void* meta, bool meta_f16, int64_t n, int64_t k, void* codes_out,
                        void* meta_out, hipStream_t stream) {
  const int64_t pieces = n * (k / 64) * 2;
  int64_t blocks = ceil_div(pieces, 256);
  if (blocks > 256 * 64) blocks = 256 * 64;
  ProfScope prof(FG_K_QUANTIZE, stream);
  if (meta_f16)
    hipLaunchKernelGGL(pack_weights_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       reinterpret_cast<const uint8_t*>(codes), reinterpret_cast<const uint32_t*>(meta), (int)n, (int)k,
                       reinterpret_cast<uint8_t*>(codes_out), reinterpret_cast<uint32_t*>(meta_out));
  else
    hipLaunchKernelGGL(pack_weights_kernel<float2>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       reinterpret_cast<const uint8_t*>(codes), reinterpret_cast<const float2*>(meta), (int)n, (int)k,
                       reinterpret_cast<uint8_t*>(codes_out), reinterpret_cast<float2*>(meta_out));
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg
