// Row-wise kernels around the projections: LayerNorm (OPT pre-LN placement), token + position
// embedding, and the greedy argmax over logits.  All are HBM/L2-bound streaming kernels.
#include "fg_common.h"

namespace fg {

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  const float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

// One 256-thread block per row.  Mean first, then the centred second moment (both in binary32
// over FP16 inputs), then the normalised row; the re-reads hit L2.
__global__ __launch_bounds__(256) void layernorm_kernel(const half_t* __restrict__ x, int64_t ldx,
                                                        const half_t* __restrict__ gamma,
                                                        const half_t* __restrict__ beta, int cols,
                                                        float eps, half_t* __restrict__ out, int64_t ldo) {
  __shared__ float red[4];
  const half_t* xr = x + (int64_t)blockIdx.x * ldx;
  half_t* orow = out + (int64_t)blockIdx.x * ldo;
  const int nchunk = cols >> 3;
  float s = 0.f;
  for (int c = threadIdx.x; c < nchunk; c += 256) {
    const h8_t v = *reinterpret_cast<const h8_t*>(xr + c * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (float)v[i];
  }
  const float mean = block_sum_256(s, red) / (float)cols;
  float q = 0.f;
  for (int c = threadIdx.x; c < nchunk; c += 256) {
    const h8_t v = *reinterpret_cast<const h8_t*>(xr + c * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float d = (float)v[i] - mean;
      q += d * d;
    }
  }
  const float var = block_sum_256(q, red) / (float)cols;
  const float rstd = 1.0f / sqrtf(var + eps);
  for (int c = threadIdx.x; c < nchunk; c += 256) {
    const h8_t v = *reinterpret_cast<const h8_t*>(xr + c * 8);
    const h8_t g = *reinterpret_cast<const h8_t*>(gamma + c * 8);
    const h8_t b = *reinterpret_cast<const h8_t*>(beta + c * 8);
    h8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (half_t)(((float)v[i] - mean) * rstd * (float)g[i] + (float)b[i]);
    *reinterpret_cast<h8_t*>(orow + c * 8) = o;
  }
}

// The same arithmetic in the same order for rows of up to 256 * 8 * NC elements, with the row held in
// registers between the three phases (one read of x instead of three).
template <int NC>
__global__ __launch_bounds__(256) void layernorm_reg_kernel(const half_t* __restrict__ x, int64_t ldx,
                                                            const half_t* __restrict__ gamma,
                                                            const half_t* __restrict__ beta, int cols,
                                                            float eps, half_t* __restrict__ out, int64_t ldo) {
  __shared__ float red[4];
  const half_t* xr = x + (int64_t)blockIdx.x * ldx;
  half_t* orow = out + (int64_t)blockIdx.x * ldo;
  const int nchunk = cols >> 3;
  h8_t v[NC];
#pragma unroll
  for (int j = 0; j < NC; ++j) {
    const int c = threadIdx.x + 256 * j;
    if (c < nchunk) v[j] = *reinterpret_cast<const h8_t*>(xr + c * 8);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NC; ++j)
    if (threadIdx.x + 256 * j < nchunk) {
#pragma unroll
      for (int i = 0; i < 8; ++i) s += (float)v[j][i];
    }
  const float mean = block_sum_256(s, red) / (float)cols;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < NC; ++j)
    if (threadIdx.x + 256 * j < nchunk) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = (float)v[j][i] - mean;
        q += d * d;
      }
    }
  const float var = block_sum_256(q, red) / (float)cols;
  const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int j = 0; j < NC; ++j) {
    const int c = threadIdx.x + 256 * j;
    if (c < nchunk) {
      const h8_t g = *reinterpret_cast<const h8_t*>(gamma + c * 8);
      const h8_t b = *reinterpret_cast<const h8_t*>(beta + c * 8);
      h8_t o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = (half_t)(((float)v[j][i] - mean) * rstd * (float)g[i] + (float)b[i]);
      *reinterpret_cast<h8_t*>(orow + c * 8) = o;
    }
  }
}

int layernorm_launch(const half_t* x, int64_t ldx, const half_t* g, const half_t* b, int64_t rows,
                     int64_t cols, float eps, half_t* out, int64_t ldo, hipStream_t stream) {
  if (rows == 0) return FG_OK;
  ProfScope prof(FG_K_LAYERNORM, stream);
  const dim3 grid((unsigned)rows), block(256);
  if (cols <= 256 * 8 * 2)
    hipLaunchKernelGGL(layernorm_reg_kernel<2>, grid, block, 0, stream, x, ldx, g, b, (int)cols, eps, out, ldo);
  else if (cols <= 256 * 8 * 4)
    hipLaunchKernelGGL(layernorm_reg_kernel<4>, grid, block, 0, stream, x, ldx, g, b, (int)cols, eps, out, ldo);
  else if (cols <= 256 * 8 * 8)
    hipLaunchKernelGGL(layernorm_reg_kernel<8>, grid, block, 0, stream, x, ldx, g, b, (int)cols, eps, out, ldo);
  else
    hipLaunchKernelGGL(layernorm_kernel, grid, block, 0, stream, x, ldx, g, b, (int)cols, eps, out, ldo);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

// x0[row] = E[ids[row]] + P[pos0 + row % s_len]; one 16-byte chunk per thread.
__global__ __launch_bounds__(256) void embed_kernel(const half_t* __restrict__ emb,
                                                    const half_t* __restrict__ pos,
                                                    const int32_t* __restrict__ ids, int64_t ids_stride,
                                                    int64_t rows, int s_len, int pos0, int h1, int vocab,
                                                    half_t* __restrict__ out) {
  const int cpr = h1 >> 3;
  const int64_t n = rows * cpr;
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; c < n; c += stride) {
    const int64_t row = c / cpr;
    const int ci = (int)(c - row * cpr);
    int id = ids[row * ids_stride];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);  // never read outside the table
    const int p = pos0 + (int)(row % s_len);
    const h8_t e = *reinterpret_cast<const h8_t*>(emb + (int64_t)id * h1 + ci * 8);
    const h8_t q = *reinterpret_cast<const h8_t*>(pos + (int64_t)p * h1 + ci * 8);
    h8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (half_t)((float)e[i] + (float)q[i]);
    *reinterpret_cast<h8_t*>(out + row * h1 + ci * 8) = o;
  }
}

// The same with a position per row (rows of sequences that are at different steps); row r takes
// its token from ids[id_index[r]] (id_index == nullptr: ids[r]).
__global__ __launch_bounds__(256) void embed_ragged_kernel(const half_t* __restrict__ emb,
                                                           const half_t* __restrict__ pos,
                                                           const int32_t* __restrict__ ids,
                                                           const int32_t* __restrict__ id_index,
                                                           const int32_t* __restrict__ positions, int64_t rows,
                                                           int h1, int vocab, int max_pos,
                                                           half_t* __restrict__ out) {
  const int cpr = h1 >> 3;
  const int64_t n = rows * cpr;
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; c < n; c += stride) {
    const int64_t row = c / cpr;
    const int ci = (int)(c - row * cpr);
    int id = ids[id_index ? (int64_t)id_index[row] : row];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // never read outside the tables
    int p = positions[row];
    p = p < 0 ? 0 : (p >= max_pos ? max_pos - 1 : p);
    const h8_t e = *reinterpret_cast<const h8_t*>(emb + (int64_t)id * h1 + ci * 8);
    const h8_t q = *reinterpret_cast<const h8_t*>(pos + (int64_t)p * h1 + ci * 8);
    h8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (half_t)((float)e[i] + (float)q[i]);
    *reinterpret_cast<h8_t*>(out + row * h1 + ci * 8) = o;
  }
}

// Greedy token: argmax over a row of binary32 logits, lowest index on ties.
// Row r's result goes to out[r * out_stride], or to out[out_index[r]] when out_index is given.
__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int64_t cols,
                                                     int32_t* __restrict__ out, int64_t out_stride,
                                                     const int32_t* __restrict__ out_index) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const float* r = logits + (int64_t)blockIdx.x * cols;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  for (int64_t c = threadIdx.x; c < cols; c += 256) {
    const float v = r[c];
    if (v > best || (v == best && (int)c < idx)) {
      best = v;
      idx = (int)c;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(idx, o, 64);
    if (ov > best || (ov == best && oi < idx)) {
      best = ov;
      idx = oi;
    }
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    bv[w] = best;
    bi[w] = idx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; ++k)
      if (bv[k] > best || (bv[k] == best && bi[k] < idx)) {
        best = bv[k];
        idx = bi[k];
      }
    const int64_t dst = out_index ? (int64_t)out_index[blockIdx.x] : (int64_t)blockIdx.x * out_stride;
    out[dst] = idx == 0x7fffffff ? 0 : idx;
  }
}

int argmax_launch(const float* logits, int64_t rows, int64_t cols, int32_t* out, int64_t out_stride,
                  hipStream_t stream, const int32_t* out_index) {
  if (rows == 0) return FG_OK;
  ProfScope prof(FG_K_ARGMAX, stream);
  hipLaunchKernelGGL(argmax_kernel, dim3((unsigned)rows), dim3(256), 0, stream, logits, cols, out, out_stride,
                     out_index);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int embed_launch(const half_t* emb, const half_t* pos, const int32_t* ids, int64_t ids_stride, int64_t rows,
                 int32_t s_len, int32_t pos0, int32_t h1, int32_t vocab, half_t* out, hipStream_t stream) {
  if (rows == 0) return FG_OK;
  const int64_t chunks = rows * (h1 / 8);
  int64_t blocks = ceil_div(chunks, 256);
  if (blocks > 256 * 32) blocks = 256 * 32;
  ProfScope prof(FG_K_EMBED, stream);
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, emb, pos, ids, ids_stride, rows,
                     (int)s_len, (int)pos0, (int)h1, (int)vocab, out);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

int embed_ragged_launch(const half_t* emb, const half_t* pos, const int32_t* ids, const int32_t* id_index,
                        const int32_t* positions, int64_t rows, int32_t h1, int32_t vocab, int32_t max_pos,
                        half_t* out, hipStream_t stream) {
  if (rows == 0) return FG_OK;
  const int64_t chunks = rows * (h1 / 8);
  int64_t blocks = ceil_div(chunks, 256);
  if (blocks > 256 * 32) blocks = 256 * 32;
  ProfScope prof(FG_K_EMBED, stream);
  hipLaunchKernelGGL(embed_ragged_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, emb, pos, ids, id_index,
                     positions, rows, (int)h1, (int)vocab, (int)max_pos, out);
  FG_LAUNCH_CHECK();
  return FG_OK;
}

}  // namespace fg

using namespace fg;

extern "C" int fg_embed_ragged(const fg_model_cfg* cfg, const void* embed_f16, const void* pos_f16,
                               const int32_t* ids, const int32_t* positions, int64_t rows, void* out_f16,
                               void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (rows < 0) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!embed_f16 || !pos_f16 || !ids || !positions || !out_f16) return FG_ERR_NULL;
  return embed_ragged_launch(reinterpret_cast<const half_t*>(embed_f16), reinterpret_cast<const half_t*>(pos_f16), ids,
                             nullptr, positions, rows, cfg->h1, cfg->vocab, cfg->max_pos,
                             reinterpret_cast<half_t*>(out_f16), as_stream(stream));
}

extern "C" int fg_layernorm(const void* x_f16, const void* gamma_f16, const void* beta_f16, int64_t rows,
                            int64_t cols, float eps, void* out_f16, void* stream) {
  if (rows < 0 || cols <= 0 || cols % 8 != 0 || rows > 0x7fffffff) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!x_f16 || !gamma_f16 || !beta_f16 || !out_f16) return FG_ERR_NULL;
  return layernorm_launch(reinterpret_cast<const half_t*>(x_f16), cols, reinterpret_cast<const half_t*>(gamma_f16),
                          reinterpret_cast<const half_t*>(beta_f16), rows, cols, eps,
                          reinterpret_cast<half_t*>(out_f16), cols, as_stream(stream));
}

extern "C" int fg_embed(const fg_model_cfg* cfg, const void* embed_f16, const void* pos_f16, const int32_t* ids,
                        int64_t rows, int32_t s_len, int32_t pos0, void* out_f16, void* stream) {
  if (!cfg) return FG_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (rows < 0 || s_len <= 0 || pos0 < 0 || (int64_t)pos0 + s_len > cfg->max_pos) return FG_ERR_SHAPE;
  if (rows == 0) return FG_OK;
  if (!embed_f16 || !pos_f16 || !ids || !out_f16) return FG_ERR_NULL;
  return embed_launch(reinterpret_cast<const half_t*>(embed_f16), reinterpret_cast<const half_t*>(pos_f16), ids, 1,
                        rows, s_len, pos0, cfg->h1, cfg->vocab, reinterpret_cast<half_t*>(out_f16),
                        as_stream(stream));
}
