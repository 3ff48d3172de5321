/*
 * energon.h -- C ABI of the padding-free transformer-layer forward for MI355X (gfx950).
 *
 * The library implements the redundant-computation-elimination step of the paper
 * (Sec. 4.3): the valid tokens of a padded batch [B, S, H] are compacted into a dense
 * [T, H] matrix (T = sum of the sequence lengths), the whole decoder block (Sec. 2.2:
 * attention module + MLP module, causal mask) runs on those T rows only, and the padded
 * layout is rebuilt at the end.  Unlike the paper's design, attention also runs on the
 * packed rows (each sequence over its real length), so a stack of L layers packs once
 * and unpacks once.
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are DEVICE pointers, *_host are HOST pointers.  The caller
 *     owns every buffer; the library allocates nothing.  The only state it keeps between calls
 *     is per device and set-once: a flag per kernel that its dynamic-LDS limit has been raised
 *     on that device (first launch there), and the address of the fixed scratch array of
 *     energon_decode_layer_forward_static (first call there).  No result depends on either.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without waiting; two calls on different
 *     streams may run concurrently if their buffers do not overlap.
 *   - Arguments are validated on the host BEFORE anything is enqueued; a call that
 *     returns an error other than ENERGON_ERR_HIP has touched no device memory.
 *   - Matrices are row-major and dense.  Weights are stored [out_features, in_features],
 *     so both GEMM operands are contiguous along the reduction.
 *   - Device pointers must be 16-byte aligned.  For a layer, H, A = n_heads*head_dim and F
 *     must be multiples of 64 (bf16, fp16) or 4 (fp32).
 *   - Sequences are right-padded: the valid tokens of sequence b are positions
 *     0 .. len[b]-1.  0 <= len[b] <= S.  len[b] = 0 and T = 0 are legal.
 *   - Packed order is batch-major then position: packed row cu[b] + s holds padded
 *     position (b, s), where cu is the exclusive prefix sum of the lengths.
 */
#ifndef ENERGON_H_
#define ENERGON_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ENERGON_OK = 0,
  ENERGON_ERR_NULL = -1,        /* a required pointer is NULL                           */
  ENERGON_ERR_SHAPE = -2,       /* a dimension is non-positive or violates divisibility */
  ENERGON_ERR_LENGTH = -3,      /* some len[b] < 0 or > S, or sum(len) != T             */
  ENERGON_ERR_CAPACITY = -4,    /* output / workspace too small                         */
  ENERGON_ERR_ALIGN = -5,       /* a device pointer is not 16-byte aligned              */
  ENERGON_ERR_UNSUPPORTED = -6, /* dtype / head_dim / epilogue not implemented          */
  ENERGON_ERR_HIP = -7          /* the HIP runtime reported an error                    */
} energon_status;

typedef enum {
  ENERGON_F32 = 0,  /* fp32 storage, fp32 arithmetic (vector ALU)                        */
  ENERGON_BF16 = 1, /* bf16 storage, MFMA with fp32 accumulation, fp32 epilogues         */
  ENERGON_F16 = 2   /* fp16 storage (the paper's precision, Sec. 5.1), otherwise as bf16 */
} energon_dtype;

/* Geometry of ONE GPU's share of a layer.  For a tensor-parallel shard (Sec. 4.1.3) pass
 * the local head count and local FFN width; hidden stays the full model width. */
typedef struct {
  int32_t hidden;   /* H  */
  int32_t n_heads;  /* nh : heads on this GPU                     */
  int32_t head_dim; /* d  : 64 or 128                             */
  int32_t ffn;      /* F  : FFN width on this GPU                 */
  float ln_eps;     /* added to the variance inside the sqrt      */
  int32_t dtype;    /* energon_dtype of activations AND weights   */
} EnergonLayerConfig;

/* Device pointers to one layer's parameters, element type = config dtype, read-only.
 * A = nh*d.  w_qkv rows are ordered Q | K | V, head-major inside each third.
 * b_o and b_fc2 may be NULL (row-split shard: the bias belongs after the cross-GPU sum);
 * b_qkv and b_fc1 may be NULL too (no bias). */
typedef struct {
  const void *ln1_g, *ln1_b; /* [H]            */
  const void *w_qkv, *b_qkv; /* [3A, H], [3A]  */
  const void *w_o, *b_o;     /* [H, A],  [H]   */
  const void *ln2_g, *ln2_b; /* [H]            */
  const void *w_fc1, *b_fc1; /* [F, H],  [F]   */
  const void *w_fc2, *b_fc2; /* [H, F],  [H]   */
} EnergonLayerWeights;

/* Epilogues of energon_linear (what is fused after the contraction). */
typedef enum {
  ENERGON_EPI_BIAS = 0,          /* y = x W^T + b                       */
  ENERGON_EPI_BIAS_GELU = 1,     /* y = GeLU(x W^T + b), exact erf form */
  ENERGON_EPI_BIAS_RESIDUAL = 2  /* y = r + x W^T + b                   */
} energon_epilogue;

/* Sub-buffers of the layer workspace, in the order energon_workspace_layout reports them. */
enum {
  ENERGON_WS_U = 0,    /* [T, H]  LayerNorm-1 output          */
  ENERGON_WS_QKV = 1,  /* [T, 3A] Q | K | V                   */
  ENERGON_WS_ATTN = 2, /* [T, A]  attention output            */
  ENERGON_WS_Y1 = 3,   /* [T, H]  x + out-proj                */
  ENERGON_WS_W = 4,    /* [T, H]  LayerNorm-2 output          */
  ENERGON_WS_M = 5,    /* [T, F]  GeLU(FC1)                   */
  ENERGON_WS_COUNT = 6
};

/* Stages timed by energon_layer_forward_profiled, in launch order. */
enum {
  ENERGON_STAGE_LN1 = 0, ENERGON_STAGE_QKV = 1, ENERGON_STAGE_ATTN = 2, ENERGON_STAGE_OUT = 3,
  ENERGON_STAGE_LN2 = 4, ENERGON_STAGE_FC1 = 5, ENERGON_STAGE_FC2 = 6, ENERGON_STAGE_COUNT = 7
};

const char* energon_strerror(int status);

/* Bytes of workspace energon_layer_forward needs for up to max_tokens packed rows: the six
 * intermediates below plus, where the 16-bit contractions would cut tiles along K (see
 * energon_linear_with_scratch), room for the pieces behind them.  A smaller workspace that still
 * holds the intermediates of the actual T is accepted; the contractions then run without cutting.
 * Returns 0 if cfg is NULL/invalid or max_tokens < 0. */
size_t energon_workspace_bytes(const EnergonLayerConfig* cfg, int64_t max_tokens);

/* Byte offsets (offsets_out[ENERGON_WS_COUNT], host) at which a call of
 * energon_layer_forward with exactly `tokens` packed rows places its intermediates inside
 * the workspace; they stay there until the next call (for tests and debugging). */
int energon_workspace_layout(const EnergonLayerConfig* cfg, int64_t tokens, size_t* offsets_out);

/* Remove padding (Sec. 4.3).  Computes on the device, with a wavefront prefix scan,
 * cu_seqlens_dev[B+1] (exclusive prefix sum of lengths, cu[B] = T) and gathers the valid
 * rows:  x_packed[cu[b]+s, :] = x_padded[b, s, :],  token_idx_dev[cu[b]+s] = b*S + s.
 *   x_padded_dev   [B, S, H]   in
 *   lengths_host   [B]         in, host; read before return, reusable afterwards.  The lengths
 *                              travel in the launches' argument blocks, 896 per launch: up to 896
 *                              sequences the call is one kernel launch, beyond that one small scan
 *                              launch per 896 lengths and the gather.  No copy is enqueued and the
 *                              call never waits (capturable in a HIP graph, with these lengths
 *                              baked in).
 *   x_packed_dev   [capacity_tokens, H] out; rows >= T are left untouched
 *   cu_seqlens_dev [B+1] int32 out;  token_idx_dev [capacity_tokens] int32 out (first T)
 *   total_tokens_out           host, optional: T, computed on the host (no device sync)
 * Errors: NULL, SHAPE (B,S,H <= 0, H not a multiple of 8 (4 for fp32), B*S >= 2^31),
 * LENGTH, CAPACITY (T > capacity_tokens), ALIGN, UNSUPPORTED (dtype), HIP. */
int energon_pack(const void* x_padded_dev, const int32_t* lengths_host, int32_t B, int32_t S,
                 int32_t H, int32_t dtype, void* x_packed_dev, int64_t capacity_tokens,
                 int32_t* cu_seqlens_dev, int32_t* token_idx_dev, int64_t* total_tokens_out,
                 void* stream);

/* Rebuild padding (Sec. 4.3).  y_padded[b, s, :] = y_packed[cu[b]+s, :] for s < len[b],
 * exact zeros elsewhere; every element of y_padded is written exactly once.
 *   y_packed_dev [T, H] in; cu_seqlens_dev [B+1] in (as written by energon_pack);
 *   y_padded_dev [B, S, H] out.  T is only used for validation (0 <= T <= B*S). */
int energon_unpack(const void* y_packed_dev, const int32_t* cu_seqlens_dev, int64_t T, int32_t B,
                   int32_t S, int32_t H, int32_t dtype, void* y_padded_dev, void* stream);

/* One pre-LN decoder block (Sec. 2.2) on T packed rows:
 *   u = LN1(x); qkv = u Wqkv^T + bqkv; a = causal attention of each sequence over its own
 *   len[b] tokens; y1 = x + a Wo^T + bo; w = LN2(y1); m = GeLU(w W1^T + b1);
 *   y = y1 + m W2^T + b2.
 *   x_packed_dev [T, H] in; y_packed_dev [T, H] out (may be the same buffer as x);
 *   cu_seqlens_dev [B+1] in; lengths_host [B] in (host; used for validation and launch
 *   shapes only: sum must equal T, each 0 <= len <= max_len);
 *   workspace_dev: at least energon_workspace_bytes(cfg, T) bytes, 256-byte aligned.
 * Errors: NULL, SHAPE (dims <= 0, H/A/F not multiples of 4 (bf16, fp16: of 64)),
 * LENGTH, CAPACITY (workspace), ALIGN, UNSUPPORTED (head_dim not 64/128, dtype, H > 32768
 * (fp32: 16384), A or F >= 2^24), HIP. */
int energon_layer_forward(const EnergonLayerConfig* cfg, const EnergonLayerWeights* weights,
                          const void* x_packed_dev, void* y_packed_dev, int64_t T,
                          const int32_t* cu_seqlens_dev, const int32_t* lengths_host, int32_t B,
                          int32_t max_len, void* workspace_dev, size_t workspace_bytes,
                          void* stream);

/* Same work as energon_layer_forward, with a HIP event recorded on `stream` between the
 * stages; waits for the stream and writes the elapsed milliseconds of each stage to
 * stage_ms_host[ENERGON_STAGE_COUNT].  A measurement aid: it creates and destroys events
 * and blocks the caller. */
int energon_layer_forward_profiled(const EnergonLayerConfig* cfg,
                                   const EnergonLayerWeights* weights, const void* x_packed_dev,
                                   void* y_packed_dev, int64_t T, const int32_t* cu_seqlens_dev,
                                   const int32_t* lengths_host, int32_t B, int32_t max_len,
                                   void* workspace_dev, size_t workspace_bytes, void* stream,
                                   float* stage_ms_host);

/* ---- a stack whose weights do not fit, or are not kept, in device memory ----------------------
 * Sec. 4.4 of the paper keeps the layers that do not fit a GPU in other memory and fetches each
 * over a separate stream while the layer before it computes, checking that the copy has finished
 * before the layer is used.  One GPU's form of that: the L layers' parameters stay in HOST memory
 * (pinned, so that the copies run asynchronously), two device slots of one layer each receive them
 * in turn on `copy_stream`, and `stream` runs layer l from slot l % 2 once an event says its copy has
 * landed; the copy of layer l + 2 into that slot waits, in turn, for an event recorded behind layer
 * l.  Both streams must have the same (default) priority.  The result is bit-identical to L calls of
 * energon_layer_forward on resident weights.
 *   host_layers [L]  structs of HOST pointers (same layouts as EnergonLayerWeights; NULL biases stay NULL)
 *   x_packed_dev [T, H] in and out (every layer runs in place)
 *   slot0_dev, slot1_dev: energon_layer_weights_bytes(cfg) bytes each, 256-byte aligned, distinct
 *   other arguments as energon_layer_forward.  Creates and destroys four events; returns without
 *   waiting.  Errors as energon_layer_forward, plus UNSUPPORTED if both streams are the same. */
size_t energon_layer_weights_bytes(const EnergonLayerConfig* cfg);
int energon_stack_forward_streamed(const EnergonLayerConfig* cfg, const EnergonLayerWeights* host_layers,
                                   int32_t L, void* x_packed_dev, int64_t T, const int32_t* cu_seqlens_dev,
                                   const int32_t* lengths_host, int32_t B, int32_t max_len, void* workspace_dev,
                                   size_t workspace_bytes, void* slot0_dev, void* slot1_dev, size_t slot_bytes,
                                   void* stream, void* copy_stream);

/* ---- the stages on their own (same kernels energon_layer_forward launches) ---------- */

/* Row-wise LayerNorm over H features: y = (x-mean)/sqrt(var+eps)*gamma+beta, biased
 * variance, statistics in fp32.  x_dev, y_dev [T, H]; gamma_dev, beta_dev [H]. */
int energon_layernorm(const void* x_dev, const void* gamma_dev, const void* beta_dev, void* y_dev,
                      int64_t T, int32_t H, float eps, int32_t dtype, void* stream);

/* y[M, N] = epilogue(x[M, K] W[N, K]^T + bias[N]) with residual r[M, N] for
 * ENERGON_EPI_BIAS_RESIDUAL (r may be the same buffer as y).  bias_dev may be NULL.
 * bf16 / fp16: MFMA, fp32 accumulation, epilogue in fp32, one rounding on store;
 * needs K % 64 == 0 and N % 8 == 0.  fp32: N % 4 == 0, K % 4 == 0.  K < 2^24 (else UNSUPPORTED). */
int energon_linear(const void* x_dev, const void* w_dev, const void* bias_dev,
                   const void* residual_dev, void* y_dev, int64_t M, int32_t N, int32_t K,
                   int32_t epilogue, int32_t dtype, void* stream);

/* energon_linear with room for intermediate sums.  For 16-bit problems of at least 192 tiles of
 * 256 x 256 the contraction runs as one persistent workgroup per CU; the tiles beyond the last full
 * round of workgroups would keep only part of the chip busy, so, given scratch, they are cut along
 * K into equal shares, one per workgroup, the fp32 pieces meet in the scratch, and a second kernel
 * adds them in a fixed order and applies the epilogue (same rounding points, a different but fixed
 * order of the fp32 sums for the cut tiles; run-to-run identical).  energon_linear_scratch_bytes
 * returns what a shape needs (0: it would not cut; then scratch may be NULL).  scratch_dev: 256-byte
 * aligned, contents undefined afterwards.  energon_layer_forward does the same inside its
 * workspace.  Other arguments and errors as energon_linear, plus CAPACITY (scratch too small). */
size_t energon_linear_scratch_bytes(int64_t M, int32_t N, int32_t K, int32_t dtype);
int energon_linear_with_scratch(const void* x_dev, const void* w_dev, const void* bias_dev,
                                const void* residual_dev, void* y_dev, int64_t M, int32_t N, int32_t K,
                                int32_t epilogue, int32_t dtype, void* scratch_dev, size_t scratch_bytes,
                                void* stream);

/* Host only, no device is touched: replays, for one 16-bit problem shape, how the persistent
 * contraction kernel deals tiles and pieces of tiles to `workgroups_per_xcd` workgroups on each of
 * the 8 XCDs (32 on MI355X; other values exercise the arithmetic), with or without scratch, and
 * checks that every tile and every slab of K is covered exactly once and that the pieces of a cut
 * tile sit where the second kernel reads them.  Returns 0 if so, a positive code naming the first
 * violated rule otherwise, -1 if that kernel does not take the shape (fewer than 192 tiles of 256 x
 * 256, or K not a multiple of 128).  pieces_out (optional): pieces per cut tile, 1 = no cutting. */
int energon_linear_plan_selfcheck(int64_t M, int32_t N, int32_t K, int32_t workgroups_per_xcd,
                                  int32_t with_scratch, int32_t* pieces_out);

/* Causal attention of every sequence over its real length, on packed rows.
 *   qkv_dev [T, 3A]  (row t: Q | K | V, head h at columns h*d .. (h+1)*d-1 of each third)
 *   out_dev [T, A];  cu_seqlens_dev [B+1];  max_len >= every sequence length.
 * o_i = sum_{j<=i} softmax_j(q_i.k_j / sqrt(d)) v_j with i, j inside one sequence. */
int energon_attention(const void* qkv_dev, void* out_dev, const int32_t* cu_seqlens_dev,
                      int64_t T, int32_t B, int32_t max_len, int32_t n_heads, int32_t head_dim,
                      int32_t dtype, void* stream);

/* ---- the paper's own attention path (Sec. 4.3), kept as a measured comparison point ---------
 * There the attention core stays padded: padding is rebuilt in front of it and removed behind
 * it, each fused with the head transpose ("two kernels that fuse the transpose and pad
 * operations").  bf16 and fp16 (ENERGON_ERR_UNSUPPORTED for fp32); head_dim 64 or 128. */

/* Rebuild padding + head transpose.  qkv_packed_dev [T, 3A] (as energon_attention reads it) ->
 * q_pad_dev, k_pad_dev, v_pad_dev, each [B, n_heads, S, head_dim]:
 *   q_pad[b, h, s, :] = qkv_packed[cu[b]+s, h*d : (h+1)*d]  for s < len[b], exact zeros elsewhere
 * (k, v from the second and last third).  Every output element is written exactly once.
 * qkv_packed_dev may be NULL when T = 0. */
int energon_rebuild_qkv(const void* qkv_packed_dev, const int32_t* cu_seqlens_dev, int64_t T, int32_t B,
                        int32_t S, int32_t n_heads, int32_t head_dim, int32_t dtype, void* q_pad_dev,
                        void* k_pad_dev, void* v_pad_dev, void* stream);

/* Padded attention core on [B, n_heads, S, head_dim] operands: every one of the S queries of
 * every sequence is computed; query i sees keys j with j <= i and j < len[b] (causal and
 * key-padding mask); a sequence of length 0 gives zero rows.  out_pad_dev has the same layout. */
int energon_attention_padded(const void* q_pad_dev, const void* k_pad_dev, const void* v_pad_dev,
                             const int32_t* cu_seqlens_dev, int32_t B, int32_t S, int32_t n_heads,
                             int32_t head_dim, int32_t dtype, void* out_pad_dev, void* stream);

/* Inverse transpose + remove padding:  attn_packed[cu[b]+s, h*d : (h+1)*d] = out_pad[b, h, s, :]
 * for s < len[b].  attn_packed_dev [T, A] (may be NULL when T = 0: nothing is written). */
int energon_remove_attn_padding(const void* out_pad_dev, const int32_t* cu_seqlens_dev, int64_t T, int32_t B,
                                int32_t S, int32_t n_heads, int32_t head_dim, int32_t dtype,
                                void* attn_packed_dev, void* stream);

/* Bytes of the extra buffer energon_layer_forward_drce needs: q, k, v and the attention output
 * in the padded head-major layout, 4 * B * S * A elements.  0 if cfg is invalid. */
size_t energon_drce_workspace_bytes(const EnergonLayerConfig* cfg, int32_t B, int32_t S);

/* energon_layer_forward with the attention stage done the paper's way: rebuild padding
 * (+ transpose), padded attention over all S positions, remove padding (+ transpose).  Same
 * arguments plus pad_workspace_dev (energon_drce_workspace_bytes(cfg, B, max_len) bytes,
 * 256-byte aligned); max_len is the padded length S.  stage_ms_host may be NULL; otherwise
 * the call waits for the stream and reports the stage times as
 * energon_layer_forward_profiled does, the three kernels together as ENERGON_STAGE_ATTN. */
int energon_layer_forward_drce(const EnergonLayerConfig* cfg, const EnergonLayerWeights* weights,
                               const void* x_packed_dev, void* y_packed_dev, int64_t T,
                               const int32_t* cu_seqlens_dev, const int32_t* lengths_host, int32_t B,
                               int32_t max_len, void* workspace_dev, size_t workspace_bytes,
                               void* pad_workspace_dev, size_t pad_workspace_bytes, void* stream,
                               float* stage_ms_host);

/* ---- LayerNorm folded into the linear that follows it (bf16 / fp16) -------------------------
 * Sec. 5.5 of the paper names the fusion of LayerNorm with the QKV contractions and the bias as
 * what the comparison system gains over unfused operators.  Here the fusion is algebraic: with
 * mu, r = mean and 1/sqrt(var + eps) of a row of x,
 *     LayerNorm(x) W^T + b  =  r (x Wf^T - mu c) + bf,
 *     Wf = W gamma (per input feature),  c[n] = sum_k Wf[n,k],  bf = b + W beta,
 * so the contraction reads the un-normalised rows and the normalised matrix is never written.
 * All pointers below are device pointers; fp32 arrays need 16-byte alignment like the rest. */

/* Once per weight matrix: w [N,K], b [N] or NULL, gamma, beta [K] (element type = dtype) ->
 * w_folded [N,K] (same type, may not alias w), colsum [N] and bias_folded [N] in fp32.  colsum is
 * taken from the rounded w_folded.  K % 8 == 0.  ENERGON_ERR_UNSUPPORTED for fp32. */
int energon_fold_layernorm(const void* w, const void* b, const void* gamma, const void* beta, int32_t N, int32_t K,
                           int32_t dtype, void* w_folded, float* colsum, float* bias_folded, void* stream);

/* stats[m] = (mean, 1/sqrt(biased variance + eps)) of row m of x [M,K], fp32 pairs.
 * K % 8 == 0, K <= 32768.  M = 0 is a no-op. */
int energon_row_stats(const void* x, int64_t M, int32_t K, int32_t dtype, float eps, float* stats, void* stream);

/* y [M,N] = act( stats[m].r * (x Wf^T - stats[m].mean * colsum) + bias_folded ), act = GeLU (exact
 * erf form) if gelu != 0, else identity.  Shape rules of energon_linear. */
int energon_linear_ln_folded(const void* x, const void* w_folded, const float* colsum, const float* bias_folded,
                             const float* stats, void* y, int64_t M, int32_t N, int32_t K, int32_t gelu,
                             int32_t dtype, void* stream);

/* Bytes of scratch energon_linear_residual_stats may use: one (sum, squared deviations) pair per
 * row and 128 output columns. */
size_t energon_stats_scratch_bytes(int64_t M, int32_t N);

/* y = residual + x W^T + b as energon_linear does, and stats_out[m] = row statistics (as
 * energon_row_stats) of the ROUNDED y: taken in the contraction's epilogue plus a merge kernel
 * where the launch shape allows (whole 256-column tiles, enough tiles), otherwise by a pass over
 * y.  scratch: energon_stats_scratch_bytes(M, N) bytes, 256-byte aligned, contents undefined
 * afterwards.  N % 8 == 0, N <= 32768. */
int energon_linear_residual_stats(const void* x, const void* w, const void* bias, const void* residual, void* y,
                                  int64_t M, int32_t N, int32_t K, int32_t dtype, float eps, float* stats_out,
                                  void* scratch, size_t scratch_bytes, void* stream);

/* One layer's parameters with both LayerNorms folded (energon_fold_layernorm of w_qkv with
 * ln1 and of w_fc1 with ln2); w_o, b_o, w_fc2, b_fc2 as in EnergonLayerWeights. */
typedef struct {
  const void* wf_qkv;            /* [3A, H] */
  const float *c_qkv, *bf_qkv;   /* [3A]    */
  const void *w_o, *b_o;         /* [H, A], [H] or NULL */
  const void* wf_fc1;            /* [F, H]  */
  const float *c_fc1, *bf_fc1;   /* [F]     */
  const void *w_fc2, *b_fc2;     /* [H, F], [H] or NULL */
} EnergonFoldedLayerWeights;

/* energon_layer_forward on folded weights: row statistics -> QKV (folded) -> attention ->
 * out-proj + residual (statistics from its epilogue) -> FC1 (folded) + GeLU -> FC2 + residual.
 * No normalised activation is written; the workspace (same size and alignment as for
 * energon_layer_forward) holds the statistics in the two regions that path uses for them.
 * stats_in: row statistics of x_packed [T][2] if the caller has them (the previous layer's
 * stats_out), else NULL and they are computed here.  stats_out: if not NULL, receives the row
 * statistics of y_packed for the next layer.  cfg->hidden <= 32768.  bf16 / fp16 only. */
int energon_layer_forward_ln_folded(const EnergonLayerConfig* cfg, const EnergonFoldedLayerWeights* weights,
                                    const void* x_packed_dev, void* y_packed_dev, int64_t T,
                                    const int32_t* cu_seqlens_dev, const int32_t* lengths_host, int32_t B,
                                    int32_t max_len, void* workspace_dev, size_t workspace_bytes,
                                    const float* stats_in, float* stats_out, void* stream);

/* ---- One generation step on cached keys / values (bf16 / fp16) --------------------------------
 * The paper defines the decoder block with a causal mask (Sec. 2.2) and runs it over batches of
 * sequences of different lengths without computing on padding (Sec. 4.3); it does not describe
 * token-by-token generation.  Under a causal mask the K and V rows of earlier tokens never
 * change, so the block's output for a token appended at position p is row p of the block applied
 * to the whole sequence, and needs from the earlier tokens only their K and V rows.  These entry
 * points compute that step for one new token per sequence; every sequence has its own cached
 * length and nothing beyond it is read.
 *
 * Cache layout (per layer, device memory owned by the caller): k_cache, v_cache [B, S_cap, A]
 * row-major, A = n_heads * head_dim, row p of sequence b = K / V of its token at position p.
 * cache_lens_dev [B] int32 on the device: tokens already cached per sequence.  The caller advances
 * it after the last layer of a step; the calls below only read it (so one array serves all layers
 * and nothing is copied from the host: a sequence of these calls can be captured in a HIP graph).
 * A length outside [0, S_cap] is clamped into it; at S_cap the new token still attends the whole
 * cache but its K / V are not stored. */

/* After a prefill: k_cache[b, i] = K row and v_cache[b, i] = V row of token i of sequence b, for
 * every packed row of qkv_packed [T, 3A] (the ENERGON_WS_QKV stage that energon_layer_forward leaves
 * in its workspace).  Positions >= S_cap are not stored; cache rows at and beyond a sequence's
 * length are not touched.  A % 8 == 0. */
int energon_cache_fill(const void* qkv_packed, const int32_t* cu_seqlens_dev, int64_t T, int32_t B, int32_t A,
                       int32_t S_cap, int32_t dtype, void* k_cache, void* v_cache, void* stream);

/* qkv [B, 3A] (q | k | v of the new tokens) -> out [B, A]; also writes row cache_lens[b] of both
 * caches for every sequence.  head_dim 64 or 128. */
int energon_decode_attention(const void* qkv, void* k_cache, void* v_cache, const int32_t* cache_lens_dev, int32_t B,
                             int32_t S_cap, int32_t n_heads, int32_t head_dim, int32_t dtype, void* out,
                             void* stream);

/* Bytes of workspace for energon_decode_layer_forward with batch size B (0 if cfg is invalid). */
size_t energon_decode_workspace_bytes(const EnergonLayerConfig* cfg, int32_t B);

/* One pre-LN decoder block for one new token per sequence: x [B, H] -> y [B, H] (may not alias),
 * same weights and stage order as energon_layer_forward, the attention stage replaced by
 * energon_decode_attention on this layer's caches.  With B <= 64 the four contractions run in a
 * kernel that streams each weight matrix from HBM once.  cache_lens_host may be NULL; if given
 * (a host copy of cache_lens_dev) every length is checked to be in [0, S_cap) before anything is
 * launched (ENERGON_ERR_LENGTH).  workspace: energon_decode_workspace_bytes(cfg, B), 256-byte
 * aligned.  B <= 65535. */
int energon_decode_layer_forward(const EnergonLayerConfig* cfg, const EnergonLayerWeights* weights, const void* x,
                                 void* y, int32_t B, const int32_t* cache_lens_dev, const int32_t* cache_lens_host,
                                 void* k_cache, void* v_cache, int32_t S_cap, void* workspace_dev,
                                 size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels
 * and results as energon_decode_layer_forward, minus the workspace: the intermediates live in a
 * fixed array of ENERGON_STATIC_SCRATCH_BYTES of device memory inside the library (one copy per GPU
 * that loads it, held until the process ends; its address is looked up once per device, on the
 * first call made with that device current).  The call allocates and frees nothing.
 * ENERGON_ERR_CAPACITY if energon_decode_workspace_bytes(cfg, B) exceeds the array (at the
 * hidden-5120 layer of the benchmark: batches up to 160 rows).  All calls on one GPU share the array, which
 * keeps the previous call's contents (nothing in it needs clearing: every stage overwrites what the
 * next one reads): calls on the same GPU must be ordered on one stream or otherwise serialised;
 * two that overlap race. */
#define ENERGON_STATIC_SCRATCH_BYTES (64u << 20)
int energon_decode_layer_forward_static(const EnergonLayerConfig* cfg, const EnergonLayerWeights* weights,
                                        const void* x, void* y, int32_t B, const int32_t* cache_lens_dev,
                                        const int32_t* cache_lens_host, void* k_cache, void* v_cache,
                                        int32_t S_cap, void* stream);

/* ---- The two ends of the model on the packed layout (bf16 / fp16) -----------------------------
 * The paper names the embedding layer (Sec. 2.2) without describing it; learned absolute
 * positions as in the GPT models it runs. */

/* x_packed[t] = wte[ids[t]] + wpe[t - cu_seqlens[b]] for every packed row t of sequence b.
 * ids_dev [T] int32, wte [V, H], wpe [P, H], H % 8 == 0.  Ids outside [0, V) and positions >= P
 * are clamped into the tables. */
int energon_embed_packed(const int32_t* ids_dev, const int32_t* cu_seqlens_dev, int64_t T, int32_t B, const void* wte,
                         int32_t V, const void* wpe, int32_t P, int32_t H, int32_t dtype, void* x_packed,
                         void* stream);

/* x[i] = wte[ids[i]] + wpe[positions[i]] for n rows with explicit positions: the embedding of a
 * generation step (positions_dev = the cached lengths).  Same clamping. */
int energon_embed_at(const int32_t* ids_dev, const int32_t* positions_dev, int64_t n, const void* wte, int32_t V,
                     const void* wpe, int32_t P, int32_t H, int32_t dtype, void* x, void* stream);

/* out[b] = x_packed[cu_seqlens[b+1] - 1], the row of sequence b's last token (zeros if it is
 * empty): what the next-token logits are computed from.  out [B, H]. */
int energon_last_token_rows(const void* x_packed, const int32_t* cu_seqlens_dev, int32_t B, int32_t H, int32_t dtype,
                            void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ENERGON_H_ */
