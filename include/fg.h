/*
 * fg.h — C ABI of the MI355X (gfx950) generation path for OPT-style decoders whose
 * weights and attention (KV) cache are compressed with group-wise 4-bit asymmetric
 * quantization (FlexGen, arXiv 2303.06865).
 *
 * Conventions shared by every call
 *   - Returns 0 (FG_OK) or a negative fg_status.  Never throws, never aborts.
 *   - Every buffer is a caller-owned DEVICE pointer unless the comment says "host".
 *     The library allocates no device memory: scratch space is the caller's `ws`
 *     argument, sized by the matching *_workspace_bytes call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously on it; the call returns before the GPU finishes, except
 *     fg_generate with a non-NULL `stats`, which synchronises the stream to read timers.
 *   - Arguments are validated on the host before anything is launched, so every error
 *     path can be exercised without a GPU (a NULL/shape/unsupported error is returned
 *     before the first HIP call).
 *   - FP16 means IEEE binary16.  Matrices are row-major.
 *
 * Storage formats
 *   FG_F16    plain FP16.
 *   FG_Q4G64  Section 5 of the paper: groups of 64 consecutive elements of the last
 *             (contiguous) dimension share one pair {float min, float scale}, with
 *             scale = (max-min)/15, and each element is stored as the 4-bit code
 *             round((x-min)/scale) (ties to even; a constant group has scale 0 and codes 0).
 *             codes: cols/2 bytes per row, element 2j in the low nibble of byte j;
 *             meta : cols/64 pairs per row, 8 bytes each {min, scale} (binary32).
 *             An element is recovered as min + code*scale: weights as the FP16 number nearest to
 *             that value (the projections multiply FP16 by FP16 into binary32), KV rows in
 *             binary32 inside the attention kernel.  0.625 bytes per element.
 *   FG_Q4G64_TILED  the same codes and pairs as FG_Q4G64, reordered for streaming (weights only;
 *             made by fg_pack_weights, rows % 32 == 0): for every tile of 32 rows (output columns)
 *             x 64 columns (one group per row) the 1 KiB of codes is stored contiguously, 16 bytes
 *             per (row r, half h of the group) at offset 16*(32*h + r); tiles of one row block
 *             follow each other along the input dimension, row blocks follow each other; meta has
 *             32 pairs per tile in the same tile order.  Same size as FG_Q4G64.
 *   FG_Q4G64_H16  the 4.5-bit variant (KV caches; weights only as the input of fg_pack_weights): as
 *             FG_Q4G64, but the pair is stored as two
 *             FP16 numbers {min, scale}, 4 bytes per group.  min is stored exactly (the inputs are
 *             FP16); scale is the smallest FP16 number >= (max-min)/15, and the codes are computed
 *             with that stored scale, so they lie in [0, 15] without clamping and every element is
 *             within scale/2 of min + code*scale; the maximum no longer round-trips exactly.
 *             0.5625 bytes per element.
 *   FG_Q4G64_H16_TILED  FG_Q4G64_H16 weights in the tile order of FG_Q4G64_TILED (32 pairs of 4 bytes
 *             per tile); made by fg_pack_weights.  Dequantized like FG_Q4G64 weights: the FP16 number
 *             nearest to min + code*scale with the stored FP16 min and scale.
 */
#ifndef FG_H
#define FG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FG_OK = 0,
  FG_ERR_NULL = -1,        /* a required pointer is NULL */
  FG_ERR_SHAPE = -2,       /* a dimension is <= 0, not a multiple of 64 where required, t >= cap, ... */
  FG_ERR_UNSUPPORTED = -3, /* bits != 4, group != 64, unknown dtype, head size not 64 or 128 */
  FG_ERR_WORKSPACE = -4,   /* ws is NULL or smaller than the matching *_workspace_bytes */
  FG_ERR_DEVICE = -5       /* a HIP runtime call failed (see fg_last_device_error) */
} fg_status;

typedef enum { FG_F16 = 0, FG_Q4G64 = 1, FG_Q4G64_TILED = 2, FG_Q4G64_H16 = 3, FG_Q4G64_H16_TILED = 4 } fg_dtype;

/* A weight matrix [rows = output features, cols = input features], row-major.
 * FG_F16:   data = FP16 values, meta = NULL.
 * FG_Q4G64: data = packed codes (rows*cols/2 bytes), meta = rows*cols/64 {min,scale} pairs;
 *           groups run along cols (the contraction dimension); cols % 64 == 0.
 * FG_Q4G64_TILED: the same bytes in the streaming order described above.
 * FG_Q4G64_H16_TILED: likewise with rows*cols/64 FP16 pairs (4 bytes each).  A canonical FG_Q4G64_H16
 *           matrix (codes as FG_Q4G64, FP16 pairs) is accepted by fg_pack_weights only. */
typedef struct {
  const void* data;
  const void* meta;
  int32_t dtype; /* fg_dtype */
  int32_t reserved;
  int64_t rows, cols;
} fg_mat;

/* Model shape in the paper's notation (Section 3): h1 hidden size, h2 hidden size of the
 * MLP, nh attention heads (head size dh = h1/nh must be 64 or 128), vocabulary size,
 * number of learned position rows, LayerNorm epsilon. */
typedef struct {
  int32_t h1, nh, h2, vocab, max_pos;
  float ln_eps;
} fg_model_cfg;

/* One decoder layer (Section 3: wQ, wK, wV, wO, w1, w2; OPT's pre-LayerNorm placement).
 * wqkv stacks Wq, Wk, Wv along rows: [3*h1, h1].  wo [h1,h1], w1 [h2,h1], w2 [h1,h2].
 * Biases are FP16 vectors and may be NULL (= 0).  LayerNorm gamma/beta are FP16 [h1]. */
typedef struct {
  fg_mat wqkv, wo, w1, w2;
  const void *bqkv, *bo, *b1, *b2;
  const void *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} fg_layer_weights;

/* The KV cache of one layer for `batch` sequences, logical layout [batch, nh, cap, dh].
 * FG_Q4G64: k_codes/v_codes hold dh/2 bytes per (sequence, head, row); k_meta/v_meta hold
 *           dh/64 {min,scale} pairs per (sequence, head, row).  Groups run along the hidden
 *           dimension of a token row (Section 5), so no group straddles a head.
 * FG_Q4G64_H16: the same with 4-byte FP16 pairs in k_meta/v_meta.
 * FG_F16:   k_codes/v_codes hold dh FP16 values per (sequence, head, row); metas are NULL. */
typedef struct {
  void *k_codes, *k_meta, *v_codes, *v_meta;
  int32_t dtype; /* fg_dtype */
  int32_t batch;
  int32_t cap; /* rows allocated per (sequence, head); >= s + n - 1 */
  int32_t reserved;
} fg_kv_cache;

/* One layer's compressed cache in NON-CONTIGUOUS memory (appendix, "Diagonal block schedule": the
 * schedule saves memory only with attention over a cache that is not one pre-allocated buffer per
 * sequence).  A pool of n_pages pages; a page holds FG_PAGE_ROWS = 64 consecutive positions of ONE
 * sequence for all heads:
 *   k_codes/v_codes [n_pages][nh][64][dh/2] bytes, k_meta/v_meta [n_pages][nh][64][dh/64] pairs
 * (8-byte pairs for FG_Q4G64, 4-byte FP16 pairs for FG_Q4G64_H16).  FG_F16 pages hold plain FP16 rows,
 * k_codes/v_codes [n_pages][nh][64][dh] halves, metas NULL.
 * Rows are stored exactly as in fg_kv_cache; only their place differs. */
#define FG_PAGE_ROWS 64
typedef struct {
  void *k_codes, *k_meta, *v_codes, *v_meta; /* device */
  int32_t dtype;                             /* FG_Q4G64, FG_Q4G64_H16 or FG_F16 */
  int32_t n_pages;
} fg_kv_pages;

/* Who the rows of a ragged step are and where their sequences live.  All arrays are DEVICE int32.
 * page_table [n_seqs][table_stride]: entry [q][j] is the page holding positions 64j .. 64j+63 of
 *   sequence q (only entries below the sequence's length are read; the table is shared by all layers
 *   when every layer's pool assigns the same page numbers).
 * seq_ids [b]: sequence of row i, or NULL for the identity (row i is sequence i).
 * pos [b]: number of rows of row i's sequence already cached BEFORE this call (its new row goes to
 *   position pos[i]); NULL means 0 for every row.
 * The kernels cannot report errors: an entry that is out of range (sequence id, position beyond
 * 64*table_stride, page number) makes them skip the store, and read page 0 or stop at the table's
 * end in the attention, so a wrong table yields wrong values, never an access outside the pool. */
typedef struct {
  const int32_t* page_table;
  const int32_t* seq_ids;
  const int32_t* pos;
  int32_t table_stride;
  int32_t n_seqs;
} fg_ragged;

/* Timers and byte counts written by fg_generate (host memory). */
typedef struct {
  double prefill_s;             /* token step 1: all layers, all GPU batches, first token */
  double decode_s;              /* token steps 2..n */
  int64_t tokens;               /* bls * n */
  int64_t weight_bytes_per_step;/* stored bytes of all layer matrices (read once per block and step) */
  int64_t kv_bytes_last_step;   /* stored K+V bytes attended to in the last decode step */
  double* decode_step_s;        /* host array of n-1 doubles or NULL: seconds of each decode step */
} fg_stats;

const char* fg_error_string(int status);
/* Text of the HIP error behind the last FG_ERR_DEVICE of the calling thread ("" if none). */
const char* fg_last_device_error(void);
/* 10000*major + 100*minor + patch */
int fg_version(void);

/* ---- Section 5: group-wise quantization ------------------------------------------------
 * Quantize x [rows, cols] FP16 (device, row-major, contiguous) into FG_Q4G64:
 * codes_out rows*cols/2 bytes, meta_out rows*cols/64 pairs.  group must be 64 and bits 4
 * (FG_ERR_UNSUPPORTED otherwise); cols % 64 == 0 and rows >= 0 (rows == 0 is a no-op).
 * The same routine serves weight matrices (groups along the input dimension) and KV token
 * rows (groups along the hidden dimension).  Results are bit-exact functions of the input:
 * binary32 arithmetic, IEEE division, no fused multiply-add. */
int fg_quantize_groupwise(const void* x_f16, int64_t rows, int64_t cols, int group, int bits,
                          void* codes_out, void* meta_out, void* stream);
/* The same quantizer for the FG_Q4G64_H16 variant (see "Storage formats"): meta_out_f16 receives
 * rows*cols/64 pairs of FP16 {min, scale}. */
int fg_quantize_groupwise_h16(const void* x_f16, int64_t rows, int64_t cols, int group, int bits,
                              void* codes_out, void* meta_out_f16, void* stream);

/* Reorder a canonical FG_Q4G64 matrix into FG_Q4G64_TILED, or a canonical FG_Q4G64_H16 one into
 * FG_Q4G64_H16_TILED (same byte counts as the source: rows*cols/2 codes and rows*cols/64 pairs of 8
 * or 4 bytes).  src->rows % 32 == 0.  Done once per weight matrix, e.g. at load time. */
int fg_pack_weights(const fg_mat* src, void* data_out, void* meta_out, void* stream);

/* Inverse map of Section 5 (stored 4-bit -> values before computation): out_f32[r][c] =
 * min + code*scale rounded once to binary32 (a fused multiply-add). */
int fg_dequantize_groupwise(const void* codes, const void* meta, int64_t rows, int64_t cols,
                            void* out_f32, void* stream);
int fg_dequantize_groupwise_h16(const void* codes, const void* meta_f16, int64_t rows, int64_t cols,
                                void* out_f32, void* stream);

/* ---- Section 3 pieces, exported so each can be checked on its own ---------------------- */

/* Row-wise LayerNorm of x [rows, cols] FP16 with FP16 gamma/beta, statistics in binary32,
 * FP16 result.  cols % 8 == 0. */
int fg_layernorm(const void* x_f16, const void* gamma_f16, const void* beta_f16, int64_t rows,
                 int64_t cols, float eps, void* out_f16, void* stream);

/* out[m, w.rows] = act(x[m, w.cols] . W^T + bias) + residual   (Section 3: x . w)
 * x, residual (nullable), out are FP16 row-major; bias FP16 (nullable); relu != 0 applies
 * max(.,0) before the residual is added.  4-bit weights (FG_Q4G64, FG_Q4G64_TILED) are dequantized
 * inside the kernel (never materialised in HBM); the tiled form is the fast one.
 * w.cols % 64 == 0; w.rows % 8 == 0 (% 32 for the tiled form); m >= 0.
 * ws must hold fg_linear_workspace_bytes(&w, m) bytes (may be 0 => ws may be NULL): the kernels
 * that split the contraction over workgroups keep their partial sums there and add them in a
 * fixed order, so results do not depend on scheduling.  One ws serves one call at a time. */
int fg_linear(const fg_mat* w, const void* bias_f16, const void* x_f16, int64_t m,
              const void* residual_f16, int relu, void* out_f16, void* ws, size_t ws_bytes,
              void* stream);
size_t fg_linear_workspace_bytes(const fg_mat* w, int64_t m);

/* fg_linear for callers that cannot allocate device memory or pass a workspace along: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels
 * and bit-identical results as fg_linear, but the partial sums live in an array of
 * fg_linear_static_scratch_bytes() = 80 MiB of device memory that the library itself owns (one copy
 * per GPU, held from the loading of the library until the process ends).  The call allocates and frees
 * nothing.  A call whose fg_linear_workspace_bytes(w, m) exceeds that size returns FG_ERR_WORKSPACE and
 * launches nothing: every projection of up to 320 rows fits (the decode phase), the 256-row-tile
 * prefill shape does not.  All calls on one GPU share the one array: calls that may overlap in time
 * on one GPU (different streams, different threads) race on it and must be serialised by the caller;
 * calls in one stream are ordered and safe. */
int fg_linear_static(const fg_mat* w, const void* bias_f16, const void* x_f16, int64_t m,
                     const void* residual_f16, int relu, void* out_f16, void* stream);
size_t fg_linear_static_scratch_bytes(void);

/* Store K and V token rows into a layer's cache (Section 3 "Concat", Section 5 storage):
 * k, v are FP16 [b, s, h1] views whose consecutive rows are row_stride elements apart
 * (so they may be column slices of a [b*s, 3*h1] QKV buffer).  Rows land at cache rows
 * pos0 .. pos0+s-1 of sequences batch_offset .. batch_offset+b-1; with FG_Q4G64 (FG_Q4G64_H16) every
 * 64-element group of a row is quantized exactly as fg_quantize_groupwise (_h16) does. */
int fg_kv_append(const fg_model_cfg* cfg, const void* k_f16, const void* v_f16, int64_t row_stride,
                 int32_t b, int32_t s, const fg_kv_cache* kv, int32_t batch_offset, int32_t pos0,
                 void* stream);

/* Decode-phase attention (Section 3): for each of b sequences and nh heads,
 * out = softmax(q . K^T / sqrt(dh)) . V over cache rows 0 .. rows-1 of sequence
 * batch_offset+i, K and V read in their stored format and dequantized in registers.
 * q is an FP16 [b, h1] view with row stride q_row_stride elements; out FP16 [b, h1]. */
int fg_decode_attention(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                        int32_t rows, const fg_kv_cache* kv, int32_t batch_offset, void* out_f16,
                        void* stream);

/* Top-K sparse variant of fg_decode_attention (Section 5, sparse attention), 4-bit caches only
 * (FG_ERR_UNSUPPORTED otherwise): the attention weights are those of the full softmax over rows
 * 0 .. rows-1; only the topk highest-weighted rows of V are read and summed with those weights (no
 * renormalisation); among equal scores the lowest row index is kept.  1 <= topk <= rows
 * (FG_ERR_SHAPE otherwise); rows (rounded up to a multiple of 128) + topk may not exceed 36864
 * (FG_ERR_UNSUPPORTED: the scores of one head are kept on chip).  kept_rows, if not NULL, is a device
 * int32 [b, nh, topk] array that receives the kept row indices in ascending order. */
int fg_decode_attention_topk(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                             int32_t rows, int32_t topk, const fg_kv_cache* kv, int32_t batch_offset,
                             void* out_f16, int32_t* kept_rows, void* stream);

/* Prefill-phase attention (Section 3): causal softmax(q . k^T / sqrt(dh)) . v per sequence and
 * head over the fresh FP16 q, k, v held in qkv [b*s, 3*h1] (columns q | k | v); out [b*s, h1]. */
int fg_prefill_attention(const fg_model_cfg* cfg, const void* qkv_f16, int32_t b, int32_t s,
                         void* out_f16, void* stream);

/* x0 = E[id] + P[pos] (FP16).  ids int32 [rows]; position of row r is pos0 + (r % s_len). */
int fg_embed(const fg_model_cfg* cfg, const void* embed_f16, const void* pos_f16, const int32_t* ids,
             int64_t rows, int32_t s_len, int32_t pos0, void* out_f16, void* stream);

/* Final LayerNorm, logits against the tied FP16 embedding [vocab, h1], greedy argmax with the
 * lowest index winning ties.  x FP16 [rows, h1] with row stride x_row_stride elements.
 * out_ids int32, written with stride out_stride elements; logits_f32 [rows, vocab] is scratch
 * the caller may inspect.  ws >= fg_lm_head_workspace_bytes. */
int fg_lm_head_greedy(const fg_model_cfg* cfg, const void* x_f16, int64_t x_row_stride, int64_t rows,
                      const void* lnf_g, const void* lnf_b, const void* embed_f16, int32_t* out_ids,
                      int64_t out_stride, float* logits_f32, void* ws, size_t ws_bytes, void* stream);
size_t fg_lm_head_workspace_bytes(const fg_model_cfg* cfg, int64_t rows);

/* ---- Section 3: one transformer layer --------------------------------------------------
 * Prefill: x_in [b, s, h1] FP16 -> x_out [b, s, h1].  Attention is causal over the fresh FP16
 * K/V; then the s K/V rows are stored at cache rows 0..s-1 of sequences batch_offset.. .
 * ws >= fg_layer_workspace_bytes(cfg, wts, b*s).  x_out may alias x_in. */
int fg_prefill_layer(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                     int32_t s, const fg_kv_cache* kv, int32_t batch_offset, void* x_out, void* ws,
                     size_t ws_bytes, void* stream);

/* Decode: x_in [b, h1] FP16 is the current token; t rows are already cached (0 <= t < cap).
 * Appends the new K/V row at row t in the storage format, attends to rows 0..t read back from
 * the cache, then output projection, residual, MLP, residual.  x_out [b, h1] may alias x_in.
 * topk = 0: dense attention.  topk > 0: the sparse attention of Section 5 as in
 * fg_decode_attention_topk, keeping min(topk, t + 1) rows of V per head (4-bit caches only:
 * FG_ERR_UNSUPPORTED otherwise, and where the scores of one head no longer fit on chip).
 * ws >= fg_layer_workspace_bytes(cfg, wts, b). */
int fg_decode_layer(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                    int32_t t, int32_t topk, const fg_kv_cache* kv, int32_t batch_offset, void* x_out,
                    void* ws, size_t ws_bytes, void* stream);
size_t fg_layer_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* wts, int64_t rows);

/* ---- Sections 3-4: generation of a block -----------------------------------------------
 * A model of l layers, prompts of s tokens, n generated tokens, a block of
 * num_gpu_batches x gpu_batch_size sequences (bls).  Token step 1 prefills the prompts and
 * emits token 1; steps 2..n decode.  Loop nest of the block schedule (Algorithm 1): token
 * step -> layer -> GPU batch, so a layer's weights are streamed once per block and step; in
 * decode steps all bls rows go through a layer's projections in one pass.
 * layers: host array of l structs (device pointers inside).  kv: host array of l caches with
 * batch == bls and cap >= s+n-1.  prompt int32 [bls, s] device; out_ids int32 [bls, n] device.
 * ws >= fg_workspace_bytes(...).  stats (host) may be NULL. */
int fg_generate(const fg_model_cfg* cfg, int32_t l, const fg_layer_weights* layers, const void* embed_f16,
                const void* pos_f16, const void* lnf_g, const void* lnf_b, const int32_t* prompt,
                int32_t s, int32_t n, int32_t num_gpu_batches, int32_t gpu_batch_size,
                const fg_kv_cache* kv, int32_t* out_ids, void* ws, size_t ws_bytes, void* stream,
                fg_stats* stats);
size_t fg_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* layer0, int32_t gpu_batch_size,
                          int32_t num_gpu_batches, int32_t s);

/* ---- Appendix, "Diagonal block schedule": paged cache, sequences at different steps --------
 * fg_kv_append_paged: like fg_kv_append, rows [b, s, h1]; row j of sequence i goes to position
 * pos[i] + j of sequence seq_ids[i], through the page table. */
int fg_kv_append_paged(const fg_model_cfg* cfg, const void* k_f16, const void* v_f16, int64_t row_stride,
                       int32_t b, int32_t s, const fg_kv_pages* pages, const fg_ragged* seqs, void* stream);

/* Decode attention over a paged cache with a length per sequence: row i attends positions
 * 0 .. pos[i] + rows_bias - 1 of sequence seq_ids[i] (rows_bias = 1 right after its new row was
 * appended at pos[i]; 0 if pos already counts every row to attend).  A row with no position to
 * attend gets zeros.  seqs->pos may not be NULL.  Same arithmetic as fg_decode_attention. */
int fg_decode_attention_paged(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                              const fg_kv_pages* pages, const fg_ragged* seqs, int32_t rows_bias,
                              void* out_f16, void* stream);

/* Top-K sparse attention (Section 5) over a paged cache with a length per sequence: as
 * fg_decode_attention_paged, but row i keeps only its min(topk, rows of row i) highest-weighted rows of
 * V.  kept_rows (device int32 [b, nh, topk] or NULL) receives the kept positions in ascending order,
 * padded with -1.  4-bit pages only; 64 * table_stride (rounded up to 128) + topk may not exceed 36864. */
int fg_decode_attention_topk_paged(const fg_model_cfg* cfg, const void* q_f16, int64_t q_row_stride, int32_t b,
                                   int32_t topk, const fg_kv_pages* pages, const fg_ragged* seqs,
                                   int32_t rows_bias, void* out_f16, int32_t* kept_rows, void* stream);

/* fg_decode_layer for rows at different steps over a paged cache: row i belongs to sequence
 * seq_ids[i], appends its K/V row at position pos[i] and attends positions 0 .. pos[i]; topk as in
 * fg_decode_layer, per row.  ws >= fg_layer_workspace_bytes(cfg, wts, b). */
int fg_decode_layer_paged(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                          int32_t topk, const fg_kv_pages* pages, const fg_ragged* seqs, void* x_out, void* ws,
                          size_t ws_bytes, void* stream);

/* fg_prefill_layer storing the s K/V rows of sequence seq_ids[i] at positions 0 .. s-1 of its pages
 * (seqs->pos is ignored).  ws >= fg_layer_workspace_bytes(cfg, wts, b*s). */
int fg_prefill_layer_paged(const fg_model_cfg* cfg, const fg_layer_weights* wts, const void* x_in, int32_t b,
                           int32_t s, const fg_kv_pages* pages, const fg_ragged* seqs, void* x_out, void* ws,
                           size_t ws_bytes, void* stream);

/* x0 = E[id] + P[position] with a position per row: ids, positions device int32 [rows]. */
int fg_embed_ragged(const fg_model_cfg* cfg, const void* embed_f16, const void* pos_f16, const int32_t* ids,
                    const int32_t* positions, int64_t rows, void* out_f16, void* stream);

/* Generation in the order of the appendix's diagonal block schedule, for a queue of n_seqs sequences
 * (prompts of s tokens, n generated tokens each) cut into GPU batches of gpu_batch_size: batch g is
 * admitted in iteration g, so in iteration `it` it is at token step it - g.  An iteration runs, layer
 * by layer, the prefill of the admitted batch and ONE decode pass over all rows of the batches still
 * generating (each layer's weights are streamed once for all of them), then emits one token per
 * sequence in flight; n_seqs/gpu_batch_size + n - 1 iterations in all.  A batch is retired after its
 * n-th token and its pages return to the pool; a sequence takes a page when it grows into one.
 * The schedule only reorders independent work: out_ids equals fg_generate's for the same prompts.
 * pages: host array of l pools with the same n_pages >= fg_diagonal_pages_needed(...) (else
 * FG_ERR_WORKSPACE); their contents on entry do not matter.  prompt int32 [n_seqs, s] device; out_ids
 * int32 [n_seqs, n] device.  ws >= fg_diagonal_workspace_bytes(...).  n_seqs % gpu_batch_size == 0.
 * stats (host, may be NULL): decode_s holds the whole run (the phases interleave), prefill_s = 0,
 * tokens = n_seqs * n.  peak_pages (host, may be NULL) receives the largest number of pages in use. */
int fg_generate_diagonal(const fg_model_cfg* cfg, int32_t l, const fg_layer_weights* layers, const void* embed_f16,
                         const void* pos_f16, const void* lnf_g, const void* lnf_b, const int32_t* prompt,
                         int32_t n_seqs, int32_t s, int32_t n, int32_t gpu_batch_size, const fg_kv_pages* pages,
                         int32_t* out_ids, void* ws, size_t ws_bytes, void* stream, fg_stats* stats,
                         int32_t* peak_pages);
size_t fg_diagonal_workspace_bytes(const fg_model_cfg* cfg, const fg_layer_weights* layer0, int32_t n_seqs,
                                   int32_t s, int32_t n, int32_t gpu_batch_size);
/* Pages per layer pool that the schedule above needs at its peak (host arithmetic only; -1 for bad
 * arguments).  The block schedule needs n_seqs * ceil((s + n) / 64). */
int64_t fg_diagonal_pages_needed(int32_t n_seqs, int32_t s, int32_t n, int32_t gpu_batch_size);

/* ---- Per-kernel timing (HIP events on the caller's stream) -----------------------------
 * Between fg_profile_begin and fg_profile_end every kernel launch of the library is bracketed
 * by two events.  fg_profile_end synchronises and accumulates, per kernel class, the summed
 * GPU time and the number of launches; fg_profile_read returns them.  Global, not thread-safe.
 * Classes: GEMM_SMALL_M = projections in the decode shape (up to 320 rows on tiled 4-bit or FP16
 * weights, up to 512 otherwise) and GEMM_SMALL_M_FINISH their partial-sum reduction pass;
 * GEMM_LARGE_M = projections in the prefill shape (reduction pass included);
 * ATTN_DECODE covers the dense and the Top-K decode attention. */
typedef enum {
  FG_K_QUANTIZE = 0, FG_K_DEQUANTIZE, FG_K_LAYERNORM, FG_K_GEMM_SMALL_M, FG_K_GEMM_SMALL_M_FINISH,
  FG_K_GEMM_LARGE_M, FG_K_KV_APPEND, FG_K_ATTN_DECODE, FG_K_ATTN_PREFILL, FG_K_EMBED, FG_K_ARGMAX,
  FG_K_COUNT
} fg_kernel_class;
int fg_profile_begin(void);
/* As fg_profile_begin, but only launches of the classes whose bit (1u << class) is set in class_mask
 * are bracketed; the others run exactly as without profiling (an event pair costs a few microseconds
 * per launch, which matters where a step is a thousand short launches). */
int fg_profile_begin_classes(uint32_t class_mask);
int fg_profile_end(void);
int fg_profile_read(int kernel_class, double* total_ms, int64_t* launches);
const char* fg_kernel_class_name(int kernel_class);

#ifdef __cplusplus
}
#endif
#endif /* FG_H */
