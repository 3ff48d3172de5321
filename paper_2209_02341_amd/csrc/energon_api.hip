// C ABI of the library (see include/energon.h): argument validation on the host, then
// the kernel launches of each stage, all on the caller's stream.  No allocation, no state.
#include "../../include/energon.h"
#include "common.h"
#include <mutex>

using namespace energon;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool is16(int32_t dt) { return dt == ENERGON_BF16 || dt == ENERGON_F16; }
inline int esize(int32_t dt) { return is16(dt) ? 2 : 4; }
inline int vec_elems(int32_t dt) { return is16(dt) ? 8 : 4; }
inline bool dtype_ok(int32_t dt) { return dt == ENERGON_F32 || dt == ENERGON_BF16 || dt == ENERGON_F16; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }
constexpr int64_t kMaxReduction = (int64_t)1 << 24;   // K of a contraction: 32-bit byte offsets inside a tile
#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return ENERGON_ERR_HIP; } while (0)

int check_cfg(const EnergonLayerConfig* c) {
  if (!c) return ENERGON_ERR_NULL;
  if (!dtype_ok(c->dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (c->hidden <= 0 || c->n_heads <= 0 || c->head_dim <= 0 || c->ffn <= 0) return ENERGON_ERR_SHAPE;
  if (c->head_dim != 64 && c->head_dim != 128) return ENERGON_ERR_UNSUPPORTED;
  const int64_t A = (int64_t)c->n_heads * c->head_dim;
  // LayerNorm keeps a row in the registers of one workgroup (256 threads x 16 vectors of 16 bytes);
  // the contractions address a tile's rows with 32-bit byte offsets (128 rows x K x 2 bytes)
  if (c->hidden > (is16(c->dtype) ? 32768 : 16384)) return ENERGON_ERR_UNSUPPORTED;
  if (A >= kMaxReduction || c->ffn >= kMaxReduction) return ENERGON_ERR_UNSUPPORTED;
  // bf16 / fp16: every reduction dimension (H, A, F) is walked in 64-element slabs by the MFMA GEMM
  const int div = is16(c->dtype) ? 64 : 4;
  if (c->hidden % div || A % div || c->ffn % div) return ENERGON_ERR_SHAPE;
  if (!(c->ln_eps >= 0.f)) return ENERGON_ERR_SHAPE;
  return ENERGON_OK;
}

// T must equal the sum; every length within [0, max_len]
int check_lengths(const int32_t* lengths, int32_t B, int32_t max_len, int64_t* total) {
  int64_t t = 0;
  for (int32_t b = 0; b < B; ++b) {
    if (lengths[b] < 0 || lengths[b] > max_len) return ENERGON_ERR_LENGTH;
    t += lengths[b];
  }
  *total = t;
  return ENERGON_OK;
}

struct WsLayout { size_t off[ENERGON_WS_COUNT]; size_t total; };

WsLayout ws_layout(const EnergonLayerConfig* c, int64_t T) {
  const size_t e = esize(c->dtype), t = (size_t)T;
  const size_t A = (size_t)c->n_heads * c->head_dim, H = c->hidden, F = c->ffn;
  const size_t sizes[ENERGON_WS_COUNT] = {t * H * e, t * 3 * A * e, t * A * e, t * H * e, t * H * e, t * F * e};
  WsLayout l;
  size_t o = 0;
  for (int i = 0; i < ENERGON_WS_COUNT; ++i) { l.off[i] = o; o += round256(sizes[i]); }
  l.total = o;
  return l;
}

// Room behind the six intermediates for the persistent 16-bit contraction kernel to leave the pieces
// of tiles it cuts along K (the largest need of the layer's four contractions; 0 if none cuts).
size_t layer_gemm_scratch_bytes(const EnergonLayerConfig* c, int64_t T) {
  if (!is16(c->dtype) || T <= 0) return 0;
  const int32_t H = c->hidden, A = c->n_heads * c->head_dim, F = c->ffn;
  const int32_t shapes[4][2] = {{3 * A, H}, {H, A}, {F, H}, {H, F}};
  size_t m = 0;
  for (const auto& nk : shapes) {
    const size_t b = gemm_sched_scratch_bytes(T, nk[0], nk[1]);
    m = b > m ? b : m;
  }
  return m;
}

int linear_impl(const void* x, const void* w, const void* bias, const void* res, void* y, int64_t M, int32_t N,
                int32_t K, int32_t epi, int32_t dt, hipStream_t s, const LnFold* fold = nullptr,
                float* split_scratch = nullptr) {
  // split_scratch: room for fp32 partial sums, so that problems with few rows may cut K over workgroups
  if (dt == ENERGON_BF16)
    HIP_TRY(launch_gemm_bf16((const bf16_t*)x, (const bf16_t*)w, (const bf16_t*)bias, (const bf16_t*)res, (bf16_t*)y,
                             M, N, K, epi, s, fold, split_scratch));
  else if (dt == ENERGON_F16)
    HIP_TRY(launch_gemm_f16((const f16_t*)x, (const f16_t*)w, (const f16_t*)bias, (const f16_t*)res, (f16_t*)y, M, N,
                            K, epi, s, fold, split_scratch));
  else if (fold != nullptr)
    return ENERGON_ERR_UNSUPPORTED;
  else
    HIP_TRY(launch_gemm_f32((const float*)x, (const float*)w, (const float*)bias, (const float*)res, (float*)y, M, N,
                            K, epi, s));
  return ENERGON_OK;
}

int attention_impl(const void* qkv, void* out, const int32_t* cu, int32_t B, int32_t max_len, int32_t nh, int32_t d,
                   int32_t dt, hipStream_t s) {
  if (dt == ENERGON_BF16)
    HIP_TRY(launch_attention_bf16((const bf16_t*)qkv, (bf16_t*)out, cu, B, max_len, nh, d, s));
  else if (dt == ENERGON_F16)
    HIP_TRY(launch_attention_f16((const f16_t*)qkv, (f16_t*)out, cu, B, max_len, nh, d, s));
  else
    HIP_TRY(launch_attention_f32((const float*)qkv, (float*)out, cu, B, max_len, nh, d, s));
  return ENERGON_OK;
}

int attention_padded_impl(const void* q, const void* k, const void* v, void* out, const int32_t* cu, int32_t B,
                          int32_t S, int32_t nh, int32_t d, int32_t dt, hipStream_t s) {
  if (dt == ENERGON_BF16)
    HIP_TRY(launch_attention_padded_bf16((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, cu, B, S,
                                         nh, d, s));
  else
    HIP_TRY(launch_attention_padded_f16((const f16_t*)q, (const f16_t*)k, (const f16_t*)v, (f16_t*)out, cu, B, S, nh,
                                        d, s));
  return ENERGON_OK;
}

int check_layer_args(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y, int64_t T,
                     const int32_t* cu, const int32_t* lengths, int32_t B, int32_t max_len, void* ws,
                     size_t ws_bytes) {
  int st = check_cfg(cfg);
  if (st != ENERGON_OK) return st;
  if (!w || !x || !y || !cu || !lengths || !ws) return ENERGON_ERR_NULL;
  if (!w->ln1_g || !w->ln1_b || !w->w_qkv || !w->w_o || !w->ln2_g || !w->ln2_b || !w->w_fc1 || !w->w_fc2)
    return ENERGON_ERR_NULL;
  if (B <= 0 || B > 65535 || max_len <= 0 || T < 0) return ENERGON_ERR_SHAPE;
  // the attention kernels address one sequence's rows with 32-bit byte offsets
  if ((int64_t)max_len * 3 * cfg->n_heads * cfg->head_dim * esize(cfg->dtype) >= ((int64_t)1 << 32)) return ENERGON_ERR_UNSUPPORTED;
  int64_t total = 0;
  st = check_lengths(lengths, B, max_len, &total);
  if (st != ENERGON_OK) return st;
  if (total != T) return ENERGON_ERR_LENGTH;
  if (T >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  const void* ptrs[] = {x, y, ws, w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o, w->b_o,
                        w->ln2_g, w->ln2_b, w->w_fc1, w->b_fc1, w->w_fc2, w->b_fc2};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ENERGON_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return ENERGON_ERR_ALIGN;
  if (ws_bytes < ws_layout(cfg, T).total) return ENERGON_ERR_CAPACITY;
  return ENERGON_OK;
}

// The block itself.  ev == nullptr: plain launches; otherwise ev[0..STAGE_COUNT] are recorded
// around the stages.
// padws == nullptr: variable-length attention on the packed rows; otherwise the paper's path
// (rebuild padding + transpose, padded attention, remove padding + transpose) through padws.
int layer_impl(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y, int64_t T,
               const int32_t* cu, int32_t B, int32_t max_len, void* ws, size_t ws_bytes, hipStream_t s, hipEvent_t* ev,
               void* padws = nullptr) {
  const WsLayout l = ws_layout(cfg, T);
  char* base = static_cast<char*>(ws);
  // scratch of the contractions, if the caller's workspace has it (energon_workspace_bytes plans for it)
  const size_t gs = layer_gemm_scratch_bytes(cfg, T);
  float* const gscratch = gs > 0 && ws_bytes >= l.total + gs ? reinterpret_cast<float*>(base + l.total) : nullptr;
  auto gemm_scratch = [&](int32_t N, int32_t K) { return gscratch && gemm_sched_scratch_bytes(T, N, K) > 0 ? gscratch : nullptr; };
  void* u = base + l.off[ENERGON_WS_U];
  void* qkv = base + l.off[ENERGON_WS_QKV];
  void* att = base + l.off[ENERGON_WS_ATTN];
  void* y1 = base + l.off[ENERGON_WS_Y1];
  void* wn = base + l.off[ENERGON_WS_W];
  void* m = base + l.off[ENERGON_WS_M];
  const int32_t H = cfg->hidden, A = cfg->n_heads * cfg->head_dim, F = cfg->ffn, dt = cfg->dtype;
  int st;
#define MARK(i) do { if (ev) HIP_TRY(hipEventRecord(ev[i], s)); } while (0)
#define STEP(call) do { st = (call); if (st != ENERGON_OK) return st; } while (0)
  MARK(0);
  HIP_TRY(launch_layernorm(x, w->ln1_g, w->ln1_b, u, T, H, cfg->ln_eps, dt, s));
  MARK(1);
  STEP(linear_impl(u, w->w_qkv, w->b_qkv, nullptr, qkv, T, 3 * A, H, ENERGON_EPI_BIAS, dt, s, nullptr, gemm_scratch(3 * A, H)));
  MARK(2);
  if (T > 0 && padws == nullptr) {
    STEP(attention_impl(qkv, att, cu, B, max_len, cfg->n_heads, cfg->head_dim, dt, s));
  } else if (T > 0) {
    const size_t part = (size_t)B * max_len * A * esize(dt);
    char* pb = static_cast<char*>(padws);
    const int32_t hb = cfg->head_dim * esize(dt);
    HIP_TRY(launch_rebuild_qkv(qkv, pb, pb + part, pb + 2 * part, cu, B, max_len, cfg->n_heads, hb, s));
    STEP(attention_padded_impl(pb, pb + part, pb + 2 * part, pb + 3 * part, cu, B, max_len, cfg->n_heads,
                               cfg->head_dim, dt, s));
    HIP_TRY(launch_remove_padding_heads(pb + 3 * part, att, cu, B, max_len, cfg->n_heads, hb, s));
  }
  MARK(3);
  STEP(linear_impl(att, w->w_o, w->b_o, x, y1, T, H, A, ENERGON_EPI_BIAS_RESIDUAL, dt, s, nullptr, gemm_scratch(H, A)));
  MARK(4);
  HIP_TRY(launch_layernorm(y1, w->ln2_g, w->ln2_b, wn, T, H, cfg->ln_eps, dt, s));
  MARK(5);
  STEP(linear_impl(wn, w->w_fc1, w->b_fc1, nullptr, m, T, F, H, ENERGON_EPI_BIAS_GELU, dt, s, nullptr, gemm_scratch(F, H)));
  MARK(6);
  STEP(linear_impl(m, w->w_fc2, w->b_fc2, y1, y, T, H, F, ENERGON_EPI_BIAS_RESIDUAL, dt, s, nullptr, gemm_scratch(H, F)));
  MARK(7);
#undef MARK
#undef STEP
  return ENERGON_OK;
}

// y = res + x W^T + b with the row statistics of the rounded y: from the epilogue's partials where
// the launch can produce them, else by a pass over y.  `partials` holds M * (N / 128) pairs.
int linear_residual_stats(const void* x, const void* w, const void* bias, const void* res, void* y, int64_t M,
                          int32_t N, int32_t K, int32_t dt, float eps, float* stats_out, float* partials,
                          hipStream_t s) {
  if (gemm_emits_row_partials(M, N, K, res == y)) {
    LnFold lf;
    lf.partial = partials;
    const int st = linear_impl(x, w, bias, res, y, M, N, K, ENERGON_EPI_BIAS_RESIDUAL, dt, s, &lf);
    if (st != ENERGON_OK) return st;
    HIP_TRY(launch_merge_partials(partials, M, N / kStatSeg, eps, stats_out, s));
    return ENERGON_OK;
  }
  const int st = linear_impl(x, w, bias, res, y, M, N, K, ENERGON_EPI_BIAS_RESIDUAL, dt, s);
  if (st != ENERGON_OK) return st;
  HIP_TRY(launch_row_stats(y, M, N, eps, dt, stats_out, s));
  return ENERGON_OK;
}

// The block on folded weights (see energon_layer_forward_ln_folded).  The regions of the
// workspace that the unfused path fills with normalised activations hold the partials (U) and
// the two statistics arrays (W) instead.
int layer_folded_impl(const EnergonLayerConfig* cfg, const EnergonFoldedLayerWeights* w, const void* x, void* y,
                      int64_t T, const int32_t* cu, int32_t B, int32_t max_len, void* ws, const float* stats_in,
                      float* stats_out, hipStream_t s) {
  const WsLayout l = ws_layout(cfg, T);
  char* base = static_cast<char*>(ws);
  float* partials = reinterpret_cast<float*>(base + l.off[ENERGON_WS_U]);
  void* qkv = base + l.off[ENERGON_WS_QKV];
  void* att = base + l.off[ENERGON_WS_ATTN];
  void* y1 = base + l.off[ENERGON_WS_Y1];
  float* stats1 = reinterpret_cast<float*>(base + l.off[ENERGON_WS_W]);
  float* stats2 = stats1 + 2 * (size_t)T;
  void* m = base + l.off[ENERGON_WS_M];
  const int32_t H = cfg->hidden, A = cfg->n_heads * cfg->head_dim, F = cfg->ffn, dt = cfg->dtype;
  int st;
#define STEP(call) do { st = (call); if (st != ENERGON_OK) return st; } while (0)
  if (stats_in == nullptr) {
    HIP_TRY(launch_row_stats(x, T, H, cfg->ln_eps, dt, stats1, s));
    stats_in = stats1;
  }
  LnFold f1;
  f1.stats = stats_in; f1.colsum = w->c_qkv; f1.bias = w->bf_qkv;
  STEP(linear_impl(x, w->wf_qkv, nullptr, nullptr, qkv, T, 3 * A, H, EPI_LNFOLD, dt, s, &f1));
  if (T > 0) STEP(attention_impl(qkv, att, cu, B, max_len, cfg->n_heads, cfg->head_dim, dt, s));
  STEP(linear_residual_stats(att, w->w_o, w->b_o, x, y1, T, H, A, dt, cfg->ln_eps, stats2, partials, s));
  LnFold f2;
  f2.stats = stats2; f2.colsum = w->c_fc1; f2.bias = w->bf_fc1;
  STEP(linear_impl(y1, w->wf_fc1, nullptr, nullptr, m, T, F, H, EPI_LNFOLD_GELU, dt, s, &f2));
  if (stats_out != nullptr)
    STEP(linear_residual_stats(m, w->w_fc2, w->b_fc2, y1, y, T, H, F, dt, cfg->ln_eps, stats_out, partials, s));
  else
    STEP(linear_impl(m, w->w_fc2, w->b_fc2, y1, y, T, H, F, ENERGON_EPI_BIAS_RESIDUAL, dt, s));
#undef STEP
  return ENERGON_OK;
}

// layer_impl with a HIP event between the stages; waits for the stream.
int layer_timed(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y, int64_t T,
                const int32_t* cu, int32_t B, int32_t max_len, void* ws, size_t ws_bytes, hipStream_t s, void* padws,
                float* stage_ms) {
  hipEvent_t ev[ENERGON_STAGE_COUNT + 1];
  int made = 0;
  for (; made <= ENERGON_STAGE_COUNT; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) break;
  if (made <= ENERGON_STAGE_COUNT) {
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return ENERGON_ERR_HIP;
  }
  int st = layer_impl(cfg, w, x, y, T, cu, B, max_len, ws, ws_bytes, s, ev, padws);
  if (st == ENERGON_OK && hipEventSynchronize(ev[ENERGON_STAGE_COUNT]) != hipSuccess) st = ENERGON_ERR_HIP;
  if (st == ENERGON_OK)
    for (int i = 0; i < ENERGON_STAGE_COUNT; ++i)
      if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = ENERGON_ERR_HIP;
  if (st != ENERGON_OK) (void)hipStreamSynchronize(s);
  for (int i = 0; i <= ENERGON_STAGE_COUNT; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}

}  // namespace

// Scratch for the entry point that may not allocate (energon_decode_layer_forward_static): the
// layer's intermediates and the partial sums of its contractions live in this array instead of a
// caller's workspace.  Every GPU that loads the library holds its own copy until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address is
// looked up once per device, with that device current, and only that address is ever handed to a
// kernel.  Nothing in it has to start at zero (every stage overwrites what the next one reads).
static __device__ __align__(256) unsigned char scratch[ENERGON_STATIC_SCRATCH_BYTES];

static int static_scratch(void** out) {
  static std::mutex mu;
  static void* addr[32] = {};
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 32) return ENERGON_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return ENERGON_ERR_HIP;
    addr[dev] = p;
  }
  *out = addr[dev];
  return ENERGON_OK;
}

extern "C" {

const char* energon_strerror(int status) {
  switch (status) {
    case ENERGON_OK: return "ok";
    case ENERGON_ERR_NULL: return "a required pointer is NULL";
    case ENERGON_ERR_SHAPE: return "a dimension is non-positive, too large, or violates a divisibility rule";
    case ENERGON_ERR_LENGTH: return "a sequence length is outside [0, S] or the lengths do not sum to T";
    case ENERGON_ERR_CAPACITY: return "an output buffer or the workspace is too small";
    case ENERGON_ERR_ALIGN: return "a device pointer is not aligned as required";
    case ENERGON_ERR_UNSUPPORTED: return "unsupported dtype, head_dim, epilogue or batch size";
    case ENERGON_ERR_HIP: return "the HIP runtime reported an error";
    default: return "unknown status";
  }
}

size_t energon_workspace_bytes(const EnergonLayerConfig* cfg, int64_t max_tokens) {
  if (check_cfg(cfg) != ENERGON_OK || max_tokens < 0) return 0;
  const size_t t = ws_layout(cfg, max_tokens).total + layer_gemm_scratch_bytes(cfg, max_tokens);
  return t ? t : 256;
}

int energon_workspace_layout(const EnergonLayerConfig* cfg, int64_t max_tokens, size_t* offsets_out) {
  const int st = check_cfg(cfg);
  if (st != ENERGON_OK) return st;
  if (!offsets_out) return ENERGON_ERR_NULL;
  if (max_tokens < 0) return ENERGON_ERR_SHAPE;
  const WsLayout l = ws_layout(cfg, max_tokens);
  for (int i = 0; i < ENERGON_WS_COUNT; ++i) offsets_out[i] = l.off[i];
  return ENERGON_OK;
}

int energon_pack(const void* x_padded, const int32_t* lengths, int32_t B, int32_t S, int32_t H, int32_t dtype,
                 void* x_packed, int64_t capacity_tokens, int32_t* cu, int32_t* token_idx, int64_t* total_out,
                 void* stream) {
  if (!x_padded || !lengths || !x_packed || !cu || !token_idx) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (B <= 0 || S <= 0 || H <= 0 || H % vec_elems(dtype) != 0 || capacity_tokens < 0) return ENERGON_ERR_SHAPE;
  if ((int64_t)B * S >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  int64_t T = 0;
  const int st = check_lengths(lengths, B, S, &T);
  if (st != ENERGON_OK) return st;
  if (T > capacity_tokens) return ENERGON_ERR_CAPACITY;
  if (!aligned16(x_padded) || !aligned16(x_packed) || (reinterpret_cast<uintptr_t>(cu) & 3u) ||
      (reinterpret_cast<uintptr_t>(token_idx) & 3u))
    return ENERGON_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (B <= kLensArgMax) {
    // one launch: the lengths ride in the kernel's argument block (copied at launch, so the call
    // neither waits for the stream nor reads lengths after it returns)
    HIP_TRY(launch_pack_scan_rows(x_padded, x_packed, lengths, cu, token_idx, B, S, (int64_t)H * esize(dtype), T, s));
  } else {
    // more lengths than one argument block holds: a scan launch per 896 of them, then the gather
    HIP_TRY(launch_scan_lengths_host(lengths, cu, B, s));
    HIP_TRY(launch_pack_rows(x_padded, x_packed, cu, token_idx, B, S, (int64_t)H * esize(dtype), T, s));
  }
  if (total_out) *total_out = T;
  return ENERGON_OK;
}

int energon_unpack(const void* y_packed, const int32_t* cu, int64_t T, int32_t B, int32_t S, int32_t H,
                   int32_t dtype, void* y_padded, void* stream) {
  if (!y_packed || !cu || !y_padded) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (B <= 0 || S <= 0 || H <= 0 || H % vec_elems(dtype) != 0) return ENERGON_ERR_SHAPE;
  if ((int64_t)B * S >= ((int64_t)1 << 31) || T < 0 || T > (int64_t)B * S) return ENERGON_ERR_SHAPE;
  if (!aligned16(y_packed) || !aligned16(y_padded) || (reinterpret_cast<uintptr_t>(cu) & 3u)) return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_unpack_rows(y_packed, y_padded, cu, B, S, (int64_t)H * esize(dtype), static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_layer_forward(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y,
                          int64_t T, const int32_t* cu, const int32_t* lengths, int32_t B, int32_t max_len, void* ws,
                          size_t ws_bytes, void* stream) {
  const int st = check_layer_args(cfg, w, x, y, T, cu, lengths, B, max_len, ws, ws_bytes);
  if (st != ENERGON_OK) return st;
  return layer_impl(cfg, w, x, y, T, cu, B, max_len, ws, ws_bytes, static_cast<hipStream_t>(stream), nullptr);
}

// ---- a stack whose weights stay in host memory ---------------------------------------------------
namespace {
struct WeightField { const void* EnergonLayerWeights::*ptr; int kind; };   // kind: elements = 0 H, 1 3A*H, 2 3A, 3 H*A, 4 F*H, 5 F, 6 H*F
const WeightField kWeightFields[12] = {
    {&EnergonLayerWeights::ln1_g, 0}, {&EnergonLayerWeights::ln1_b, 0}, {&EnergonLayerWeights::w_qkv, 1},
    {&EnergonLayerWeights::b_qkv, 2}, {&EnergonLayerWeights::w_o, 3},   {&EnergonLayerWeights::b_o, 0},
    {&EnergonLayerWeights::ln2_g, 0}, {&EnergonLayerWeights::ln2_b, 0}, {&EnergonLayerWeights::w_fc1, 4},
    {&EnergonLayerWeights::b_fc1, 5}, {&EnergonLayerWeights::w_fc2, 6}, {&EnergonLayerWeights::b_fc2, 0}};

size_t weight_field_bytes(const EnergonLayerConfig* c, int kind) {
  const size_t H = c->hidden, A = (size_t)c->n_heads * c->head_dim, F = c->ffn, e = esize(c->dtype);
  const size_t n[7] = {H, 3 * A * H, 3 * A, H * A, F * H, F, H * F};
  return n[kind] * e;
}
}  // namespace

size_t energon_layer_weights_bytes(const EnergonLayerConfig* cfg) {
  if (check_cfg(cfg) != ENERGON_OK) return 0;
  size_t t = 0;
  for (const auto& f : kWeightFields) t += round256(weight_field_bytes(cfg, f.kind));
  return t;
}

int energon_stack_forward_streamed(const EnergonLayerConfig* cfg, const EnergonLayerWeights* host_layers, int32_t L,
                                   void* x, int64_t T, const int32_t* cu, const int32_t* lengths, int32_t B,
                                   int32_t max_len, void* ws, size_t ws_bytes, void* slot0, void* slot1,
                                   size_t slot_bytes, void* stream, void* copy_stream) {
  if (!host_layers || !slot0 || !slot1) return ENERGON_ERR_NULL;
  if (L <= 0) return ENERGON_ERR_SHAPE;
  if (stream == copy_stream) return ENERGON_ERR_UNSUPPORTED;   // nothing could overlap
  if ((reinterpret_cast<uintptr_t>(slot0) & 255u) || (reinterpret_cast<uintptr_t>(slot1) & 255u) || slot0 == slot1)
    return ENERGON_ERR_ALIGN;
  {
    const EnergonLayerWeights probe = host_layers[0];
    const int st = check_layer_args(cfg, &probe, x, x, T, cu, lengths, B, max_len, ws, ws_bytes);
    if (st != ENERGON_OK) return st;
  }
  if (slot_bytes < energon_layer_weights_bytes(cfg)) return ENERGON_ERR_CAPACITY;
  for (int32_t l = 0; l < L; ++l) {
    const EnergonLayerWeights& w = host_layers[l];
    if (!w.ln1_g || !w.ln1_b || !w.w_qkv || !w.w_o || !w.ln2_g || !w.ln2_b || !w.w_fc1 || !w.w_fc2) return ENERGON_ERR_NULL;
  }
  hipStream_t cs = static_cast<hipStream_t>(stream), xs = static_cast<hipStream_t>(copy_stream);
  void* slots[2] = {slot0, slot1};
  hipEvent_t ready[2] = {nullptr, nullptr}, released[2] = {nullptr, nullptr};
  int st = ENERGON_OK;
  for (int i = 0; i < 2 && st == ENERGON_OK; ++i)
    if (hipEventCreateWithFlags(&ready[i], hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&released[i], hipEventDisableTiming) != hipSuccess)
      st = ENERGON_ERR_HIP;
  // the copies of layer l into slot l % 2, on the copy stream; fills dev with the device addresses
  auto enqueue_copy = [&](int32_t l, EnergonLayerWeights* dev) -> int {
    char* base = static_cast<char*>(slots[l & 1]);
    size_t off = 0;
    for (const auto& f : kWeightFields) {
      const size_t nbytes = weight_field_bytes(cfg, f.kind);
      const void* src = host_layers[l].*(f.ptr);
      if (src != nullptr) {
        HIP_TRY(hipMemcpyAsync(base + off, src, nbytes, hipMemcpyHostToDevice, xs));
        dev->*(f.ptr) = base + off;
      } else {
        dev->*(f.ptr) = nullptr;
      }
      off += round256(nbytes);
    }
    HIP_TRY(hipEventRecord(ready[l & 1], xs));
    return ENERGON_OK;
  };
  EnergonLayerWeights dev[2];
  // whatever ran on the compute stream before this call may still read the slots
  if (st == ENERGON_OK && (hipEventRecord(released[0], cs) != hipSuccess || hipStreamWaitEvent(xs, released[0], 0) != hipSuccess))
    st = ENERGON_ERR_HIP;
  if (st == ENERGON_OK) st = enqueue_copy(0, &dev[0]);
  for (int32_t l = 0; l < L && st == ENERGON_OK; ++l) {
    if (l + 1 < L) {
      // slot (l + 1) % 2 was last read by layer l - 1: its copy may start once that layer has finished
      if (l >= 1 && hipStreamWaitEvent(xs, released[(l + 1) & 1], 0) != hipSuccess) { st = ENERGON_ERR_HIP; break; }
      st = enqueue_copy(l + 1, &dev[(l + 1) & 1]);
      if (st != ENERGON_OK) break;
    }
    if (hipStreamWaitEvent(cs, ready[l & 1], 0) != hipSuccess) { st = ENERGON_ERR_HIP; break; }
    st = layer_impl(cfg, &dev[l & 1], x, x, T, cu, B, max_len, ws, ws_bytes, cs, nullptr);
    if (st == ENERGON_OK && hipEventRecord(released[l & 1], cs) != hipSuccess) st = ENERGON_ERR_HIP;
  }
  // an event may be destroyed while work that refers to it is pending: the runtime releases it when that completes
  for (int i = 0; i < 2; ++i) {
    if (ready[i]) (void)hipEventDestroy(ready[i]);
    if (released[i]) (void)hipEventDestroy(released[i]);
  }
  return st;
}

int energon_layer_forward_profiled(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x,
                                   void* y, int64_t T, const int32_t* cu, const int32_t* lengths, int32_t B,
                                   int32_t max_len, void* ws, size_t ws_bytes, void* stream, float* stage_ms) {
  if (!stage_ms) return ENERGON_ERR_NULL;
  const int st = check_layer_args(cfg, w, x, y, T, cu, lengths, B, max_len, ws, ws_bytes);
  if (st != ENERGON_OK) return st;
  return layer_timed(cfg, w, x, y, T, cu, B, max_len, ws, ws_bytes, static_cast<hipStream_t>(stream), nullptr, stage_ms);
}

size_t energon_drce_workspace_bytes(const EnergonLayerConfig* cfg, int32_t B, int32_t S) {
  if (check_cfg(cfg) != ENERGON_OK || B <= 0 || S <= 0) return 0;
  return (size_t)4 * B * S * cfg->n_heads * cfg->head_dim * esize(cfg->dtype);
}

static int check_drce_shape(const int32_t* cu, int64_t T, int32_t B, int32_t S, int32_t nh, int32_t d, int32_t dtype) {
  if (!cu) return ENERGON_ERR_NULL;
  if (!is16(dtype) || (d != 64 && d != 128)) return ENERGON_ERR_UNSUPPORTED;
  if (B <= 0 || S <= 0 || nh <= 0 || T < 0 || T > (int64_t)B * S || (int64_t)B * S >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  if ((int64_t)B * nh >= (1 << 24)) return ENERGON_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(cu) & 3u) return ENERGON_ERR_ALIGN;
  return ENERGON_OK;
}

int energon_rebuild_qkv(const void* qkv, const int32_t* cu, int64_t T, int32_t B, int32_t S, int32_t nh, int32_t d,
                        int32_t dtype, void* q, void* k, void* v, void* stream) {
  if ((!qkv && T > 0) || !q || !k || !v) return ENERGON_ERR_NULL;   // T = 0: no packed row is read
  const int st = check_drce_shape(cu, T, B, S, nh, d, dtype);
  if (st != ENERGON_OK) return st;
  if (!aligned16(qkv) || !aligned16(q) || !aligned16(k) || !aligned16(v)) return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_rebuild_qkv(qkv, q, k, v, cu, B, S, nh, d * esize(dtype), static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_attention_padded(const void* q, const void* k, const void* v, const int32_t* cu, int32_t B, int32_t S,
                             int32_t nh, int32_t d, int32_t dtype, void* out, void* stream) {
  if (!q || !k || !v || !out) return ENERGON_ERR_NULL;
  const int st = check_drce_shape(cu, 0, B, S, nh, d, dtype);
  if (st != ENERGON_OK) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return ENERGON_ERR_ALIGN;
  return attention_padded_impl(q, k, v, out, cu, B, S, nh, d, dtype, static_cast<hipStream_t>(stream));
}

int energon_remove_attn_padding(const void* o, const int32_t* cu, int64_t T, int32_t B, int32_t S, int32_t nh,
                                int32_t d, int32_t dtype, void* out, void* stream) {
  if (!o || (!out && T > 0)) return ENERGON_ERR_NULL;
  const int st = check_drce_shape(cu, T, B, S, nh, d, dtype);
  if (st != ENERGON_OK) return st;
  if (!aligned16(o) || !aligned16(out)) return ENERGON_ERR_ALIGN;
  if (T == 0) return ENERGON_OK;
  HIP_TRY(launch_remove_padding_heads(o, out, cu, B, S, nh, d * esize(dtype), static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_layer_forward_drce(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y,
                               int64_t T, const int32_t* cu, const int32_t* lengths, int32_t B, int32_t max_len,
                               void* ws, size_t ws_bytes, void* padws, size_t padws_bytes, void* stream,
                               float* stage_ms) {
  const int st = check_layer_args(cfg, w, x, y, T, cu, lengths, B, max_len, ws, ws_bytes);
  if (st != ENERGON_OK) return st;
  if (!is16(cfg->dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!padws) return ENERGON_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(padws) & 255u) != 0) return ENERGON_ERR_ALIGN;
  if ((int64_t)B * max_len >= ((int64_t)1 << 31) || (int64_t)B * cfg->n_heads >= (1 << 24)) return ENERGON_ERR_SHAPE;
  if (padws_bytes < energon_drce_workspace_bytes(cfg, B, max_len)) return ENERGON_ERR_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!stage_ms) return layer_impl(cfg, w, x, y, T, cu, B, max_len, ws, ws_bytes, s, nullptr, padws);
  return layer_timed(cfg, w, x, y, T, cu, B, max_len, ws, ws_bytes, s, padws, stage_ms);
}

int energon_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t T, int32_t H, float eps,
                      int32_t dtype, void* stream) {
  if (!x || !gamma || !beta || !y) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (T < 0 || T >= ((int64_t)1 << 31) || H <= 0 || H % vec_elems(dtype) != 0 || !(eps >= 0.f)) return ENERGON_ERR_SHAPE;
  if (H / vec_elems(dtype) > 256 * 16) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y)) return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_layernorm(x, gamma, beta, y, T, H, eps, dtype, static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_linear(const void* x, const void* w, const void* bias, const void* residual, void* y, int64_t M,
                   int32_t N, int32_t K, int32_t epilogue, int32_t dtype, void* stream) {
  if (!x || !w || !y) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (epilogue < ENERGON_EPI_BIAS || epilogue > ENERGON_EPI_BIAS_RESIDUAL) return ENERGON_ERR_UNSUPPORTED;
  if (epilogue == ENERGON_EPI_BIAS_RESIDUAL && !residual) return ENERGON_ERR_NULL;
  if (M < 0 || M >= ((int64_t)1 << 31) || N <= 0 || K <= 0) return ENERGON_ERR_SHAPE;
  if (is16(dtype) ? (K % 64 != 0 || N % 8 != 0) : (K % 4 != 0 || N % 4 != 0)) return ENERGON_ERR_SHAPE;
  if (K >= kMaxReduction) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(residual) || !aligned16(y))
    return ENERGON_ERR_ALIGN;
  return linear_impl(x, w, bias, residual, y, M, N, K, epilogue, dtype, static_cast<hipStream_t>(stream));
}

size_t energon_linear_scratch_bytes(int64_t M, int32_t N, int32_t K, int32_t dtype) {
  if (!is16(dtype) || M <= 0 || N <= 0 || K <= 0 || K % 64 != 0 || N % 8 != 0 || K >= kMaxReduction) return 0;
  return round256(gemm_sched_scratch_bytes(M, N, K));
}

int energon_linear_with_scratch(const void* x, const void* w, const void* bias, const void* residual, void* y, int64_t M,
                                int32_t N, int32_t K, int32_t epilogue, int32_t dtype, void* scratch,
                                size_t scratch_bytes, void* stream) {
  if (!x || !w || !y) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (epilogue < ENERGON_EPI_BIAS || epilogue > ENERGON_EPI_BIAS_RESIDUAL) return ENERGON_ERR_UNSUPPORTED;
  if (epilogue == ENERGON_EPI_BIAS_RESIDUAL && !residual) return ENERGON_ERR_NULL;
  if (M < 0 || M >= ((int64_t)1 << 31) || N <= 0 || K <= 0) return ENERGON_ERR_SHAPE;
  if (is16(dtype) ? (K % 64 != 0 || N % 8 != 0) : (K % 4 != 0 || N % 4 != 0)) return ENERGON_ERR_SHAPE;
  if (K >= kMaxReduction) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(residual) || !aligned16(y))
    return ENERGON_ERR_ALIGN;
  const size_t need = energon_linear_scratch_bytes(M, N, K, dtype);
  if (need > 0 && !scratch) return ENERGON_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(scratch) & 255u) != 0) return ENERGON_ERR_ALIGN;
  if (scratch_bytes < need) return ENERGON_ERR_CAPACITY;
  return linear_impl(x, w, bias, residual, y, M, N, K, epilogue, dtype, static_cast<hipStream_t>(stream), nullptr,
                     need > 0 ? static_cast<float*>(scratch) : nullptr);
}

int energon_linear_plan_selfcheck(int64_t M, int32_t N, int32_t K, int32_t workgroups_per_xcd, int32_t with_scratch,
                                  int32_t* pieces_out) {
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 != 0 || workgroups_per_xcd < 1 || workgroups_per_xcd > 1024) return -1;
  return gemm_sched_selfcheck(M, N, K, workgroups_per_xcd, with_scratch, pieces_out);
}

int energon_attention(const void* qkv, void* out, const int32_t* cu, int64_t T, int32_t B, int32_t max_len,
                      int32_t n_heads, int32_t head_dim, int32_t dtype, void* stream) {
  if (!qkv || !out || !cu) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return ENERGON_ERR_UNSUPPORTED;
  if (B <= 0 || max_len <= 0 || n_heads <= 0 || T < 0 || T >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  if (B > 65535 || n_heads > 65535) return ENERGON_ERR_UNSUPPORTED;
  if ((int64_t)max_len * 3 * n_heads * head_dim * esize(dtype) >= ((int64_t)1 << 32)) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(qkv) || !aligned16(out) || (reinterpret_cast<uintptr_t>(cu) & 3u)) return ENERGON_ERR_ALIGN;
  if (T == 0) return ENERGON_OK;
  return attention_impl(qkv, out, cu, B, max_len, n_heads, head_dim, dtype, static_cast<hipStream_t>(stream));
}

int energon_fold_layernorm(const void* w, const void* b, const void* gamma, const void* beta, int32_t N, int32_t K,
                           int32_t dtype, void* w_folded, float* colsum, float* bias_folded, void* stream) {
  if (!w || !gamma || !beta || !w_folded || !colsum || !bias_folded) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (N <= 0 || K <= 0 || K % 8 != 0) return ENERGON_ERR_SHAPE;
  if (w == w_folded) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(w) || !aligned16(gamma) || !aligned16(beta) || !aligned16(w_folded) || !aligned16(colsum) ||
      !aligned16(bias_folded) || (reinterpret_cast<uintptr_t>(b) & 1u))
    return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_fold_weights(w, b, gamma, beta, N, K, dtype, w_folded, colsum, bias_folded,
                              static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_row_stats(const void* x, int64_t M, int32_t K, int32_t dtype, float eps, float* stats, void* stream) {
  if (!x || !stats) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (M < 0 || M >= ((int64_t)1 << 31) || K <= 0 || K % 8 != 0 || !(eps >= 0.f)) return ENERGON_ERR_SHAPE;
  if (K > 32768) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || (reinterpret_cast<uintptr_t>(stats) & 7u)) return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_row_stats(x, M, K, eps, dtype, stats, static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_linear_ln_folded(const void* x, const void* w_folded, const float* colsum, const float* bias_folded,
                             const float* stats, void* y, int64_t M, int32_t N, int32_t K, int32_t gelu,
                             int32_t dtype, void* stream) {
  if (!x || !w_folded || !colsum || !bias_folded || !stats || !y) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (M < 0 || M >= ((int64_t)1 << 31) || N <= 0 || K <= 0) return ENERGON_ERR_SHAPE;
  if (K % 64 != 0 || N % 8 != 0) return ENERGON_ERR_SHAPE;
  if (K >= kMaxReduction) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w_folded) || !aligned16(colsum) || !aligned16(bias_folded) || !aligned16(y) ||
      (reinterpret_cast<uintptr_t>(stats) & 7u))
    return ENERGON_ERR_ALIGN;
  LnFold lf;
  lf.stats = stats; lf.colsum = colsum; lf.bias = bias_folded;
  return linear_impl(x, w_folded, nullptr, nullptr, y, M, N, K, gelu ? EPI_LNFOLD_GELU : EPI_LNFOLD, dtype,
                     static_cast<hipStream_t>(stream), &lf);
}

size_t energon_stats_scratch_bytes(int64_t M, int32_t N) {
  if (M < 0 || N <= 0) return 0;
  const size_t b = round256((size_t)M * (size_t)((N + kStatSeg - 1) / kStatSeg) * 2 * sizeof(float));
  return b ? b : 256;
}

int energon_linear_residual_stats(const void* x, const void* w, const void* bias, const void* residual, void* y,
                                  int64_t M, int32_t N, int32_t K, int32_t dtype, float eps, float* stats_out,
                                  void* scratch, size_t scratch_bytes, void* stream) {
  if (!x || !w || !residual || !y || !stats_out || !scratch) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (M < 0 || M >= ((int64_t)1 << 31) || N <= 0 || K <= 0 || !(eps >= 0.f)) return ENERGON_ERR_SHAPE;
  if (K % 64 != 0 || N % 8 != 0) return ENERGON_ERR_SHAPE;
  if (K >= kMaxReduction) return ENERGON_ERR_UNSUPPORTED;
  if (N > 32768) return ENERGON_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(residual) || !aligned16(y) ||
      (reinterpret_cast<uintptr_t>(stats_out) & 7u) || (reinterpret_cast<uintptr_t>(scratch) & 255u))
    return ENERGON_ERR_ALIGN;
  if (scratch_bytes < energon_stats_scratch_bytes(M, N)) return ENERGON_ERR_CAPACITY;
  return linear_residual_stats(x, w, bias, residual, y, M, N, K, dtype, eps, stats_out, static_cast<float*>(scratch),
                               static_cast<hipStream_t>(stream));
}

int energon_layer_forward_ln_folded(const EnergonLayerConfig* cfg, const EnergonFoldedLayerWeights* w, const void* x,
                                    void* y, int64_t T, const int32_t* cu, const int32_t* lengths, int32_t B,
                                    int32_t max_len, void* ws, size_t ws_bytes, const float* stats_in,
                                    float* stats_out, void* stream) {
  int st = check_cfg(cfg);
  if (st != ENERGON_OK) return st;
  if (!is16(cfg->dtype) || cfg->hidden > 32768) return ENERGON_ERR_UNSUPPORTED;
  if (!w || !x || !y || !cu || !lengths || !ws) return ENERGON_ERR_NULL;
  if (!w->wf_qkv || !w->c_qkv || !w->bf_qkv || !w->w_o || !w->wf_fc1 || !w->c_fc1 || !w->bf_fc1 || !w->w_fc2)
    return ENERGON_ERR_NULL;
  if (B <= 0 || B > 65535 || max_len <= 0 || T < 0) return ENERGON_ERR_SHAPE;
  if ((int64_t)max_len * 3 * cfg->n_heads * cfg->head_dim * esize(cfg->dtype) >= ((int64_t)1 << 32)) return ENERGON_ERR_UNSUPPORTED;
  int64_t total = 0;
  st = check_lengths(lengths, B, max_len, &total);
  if (st != ENERGON_OK) return st;
  if (total != T) return ENERGON_ERR_LENGTH;
  if (T >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  const void* ptrs[] = {x, y, ws, w->wf_qkv, w->c_qkv, w->bf_qkv, w->w_o, w->b_o, w->wf_fc1, w->c_fc1, w->bf_fc1,
                        w->w_fc2, w->b_fc2};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ENERGON_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return ENERGON_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(stats_in) & 7u) || (reinterpret_cast<uintptr_t>(stats_out) & 7u)) return ENERGON_ERR_ALIGN;
  if (ws_bytes < ws_layout(cfg, T).total) return ENERGON_ERR_CAPACITY;
  return layer_folded_impl(cfg, w, x, y, T, cu, B, max_len, ws, stats_in, stats_out, static_cast<hipStream_t>(stream));
}

int energon_decode_attention(const void* qkv, void* k_cache, void* v_cache, const int32_t* cache_lens_dev, int32_t B,
                             int32_t S_cap, int32_t n_heads, int32_t head_dim, int32_t dtype, void* out,
                             void* stream) {
  if (!qkv || !k_cache || !v_cache || !cache_lens_dev || !out) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype) || (head_dim != 64 && head_dim != 128)) return ENERGON_ERR_UNSUPPORTED;
  if (B < 0 || S_cap <= 0 || n_heads <= 0) return ENERGON_ERR_SHAPE;
  if ((int64_t)B * n_heads >= ((int64_t)1 << 31)) return ENERGON_ERR_SHAPE;
  if (!aligned16(qkv) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(cache_lens_dev) & 3u))
    return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_decode_attention(qkv, k_cache, v_cache, cache_lens_dev, B, S_cap, n_heads, head_dim, dtype, out,
                                  static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

// scratch for the partial sums of the few-row contractions of a step (the largest of the four)
static size_t decode_partial_bytes(const EnergonLayerConfig* c, int32_t B) {
  if (!is16(c->dtype) || B < 1) return 0;
  const int32_t H = c->hidden, A = c->n_heads * c->head_dim, F = c->ffn;
  size_t m = 0;
  const int32_t shapes[4][2] = {{3 * A, H}, {H, A}, {F, H}, {H, F}};
  for (const auto& nk : shapes) {
    const size_t b = gemm_skinny_takes(B, nk[0], nk[1], EPI_BIAS) ? gemm_skinny_partial_bytes(B, nk[0], nk[1])
                                                                  : gemm_split_scratch_bytes(B, nk[0], nk[1]);
    m = b > m ? b : m;
  }
  return round256(m);
}

int energon_cache_fill(const void* qkv_packed, const int32_t* cu, int64_t T, int32_t B, int32_t A, int32_t S_cap,
                       int32_t dtype, void* k_cache, void* v_cache, void* stream) {
  if (!cu || !k_cache || !v_cache || (!qkv_packed && T > 0)) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (T < 0 || T >= ((int64_t)1 << 31) || B <= 0 || A <= 0 || A % 8 != 0 || S_cap <= 0) return ENERGON_ERR_SHAPE;
  if (!aligned16(qkv_packed) || !aligned16(k_cache) || !aligned16(v_cache) || (reinterpret_cast<uintptr_t>(cu) & 3u))
    return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_cache_fill(qkv_packed, cu, B, T, (int64_t)A * esize(dtype), S_cap, k_cache, v_cache,
                            static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

size_t energon_decode_workspace_bytes(const EnergonLayerConfig* cfg, int32_t B) {
  if (check_cfg(cfg) != ENERGON_OK || B < 0) return 0;
  const size_t t = ws_layout(cfg, B).total + decode_partial_bytes(cfg, B);
  return t ? t : 256;
}

// Validation and launches of one generation step's layer; `ws` is the caller's workspace or the
// library's static scratch.
static int decode_layer_checked(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y,
                                int32_t B, const int32_t* cache_lens_dev, const int32_t* cache_lens_host,
                                void* k_cache, void* v_cache, int32_t S_cap, void* ws, size_t ws_bytes,
                                bool ws_is_static, void* stream) {
  int st = check_cfg(cfg);
  if (st != ENERGON_OK) return st;
  if (!is16(cfg->dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!w || !x || !y || !cache_lens_dev || !k_cache || !v_cache || (!ws && !ws_is_static)) return ENERGON_ERR_NULL;
  if (!w->ln1_g || !w->ln1_b || !w->w_qkv || !w->w_o || !w->ln2_g || !w->ln2_b || !w->w_fc1 || !w->w_fc2)
    return ENERGON_ERR_NULL;
  if (B < 0 || B > 65535 || S_cap <= 0) return ENERGON_ERR_SHAPE;
  if (x == y) return ENERGON_ERR_UNSUPPORTED;
  if (cache_lens_host)
    for (int32_t b = 0; b < B; ++b)
      if (cache_lens_host[b] < 0 || cache_lens_host[b] >= S_cap) return ENERGON_ERR_LENGTH;
  const void* ptrs[] = {x, y, k_cache, v_cache, w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o, w->b_o,
                        w->ln2_g, w->ln2_b, w->w_fc1, w->b_fc1, w->w_fc2, w->b_fc2};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ENERGON_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(cache_lens_dev) & 3u)) return ENERGON_ERR_ALIGN;
  if (ws_bytes < energon_decode_workspace_bytes(cfg, B)) return ENERGON_ERR_CAPACITY;
  if (ws_is_static) {   // every argument has passed: now, and only now, touch the device
    st = static_scratch(&ws);
    if (st != ENERGON_OK) return st;
  }
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return ENERGON_ERR_ALIGN;
  if (B == 0) return ENERGON_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const WsLayout l = ws_layout(cfg, B);
  char* base = static_cast<char*>(ws);
  void* u = base + l.off[ENERGON_WS_U];
  void* qkv = base + l.off[ENERGON_WS_QKV];
  void* att = base + l.off[ENERGON_WS_ATTN];
  void* y1 = base + l.off[ENERGON_WS_Y1];
  void* wn = base + l.off[ENERGON_WS_W];
  void* m = base + l.off[ENERGON_WS_M];
  const int32_t H = cfg->hidden, A = cfg->n_heads * cfg->head_dim, F = cfg->ffn, dt = cfg->dtype;
  float* part = decode_partial_bytes(cfg, B) ? reinterpret_cast<float*>(base + l.total) : nullptr;
#define STEP(call) do { st = (call); if (st != ENERGON_OK) return st; } while (0)
  HIP_TRY(launch_layernorm(x, w->ln1_g, w->ln1_b, u, B, H, cfg->ln_eps, dt, s));
  STEP(linear_impl(u, w->w_qkv, w->b_qkv, nullptr, qkv, B, 3 * A, H, ENERGON_EPI_BIAS, dt, s, nullptr, part));
  HIP_TRY(launch_decode_attention(qkv, k_cache, v_cache, cache_lens_dev, B, S_cap, cfg->n_heads, cfg->head_dim, dt,
                                  att, s));
  STEP(linear_impl(att, w->w_o, w->b_o, x, y1, B, H, A, ENERGON_EPI_BIAS_RESIDUAL, dt, s, nullptr, part));
  HIP_TRY(launch_layernorm(y1, w->ln2_g, w->ln2_b, wn, B, H, cfg->ln_eps, dt, s));
  STEP(linear_impl(wn, w->w_fc1, w->b_fc1, nullptr, m, B, F, H, ENERGON_EPI_BIAS_GELU, dt, s, nullptr, part));
  STEP(linear_impl(m, w->w_fc2, w->b_fc2, y1, y, B, H, F, ENERGON_EPI_BIAS_RESIDUAL, dt, s, nullptr, part));
#undef STEP
  return ENERGON_OK;
}

int energon_decode_layer_forward(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x, void* y,
                                 int32_t B, const int32_t* cache_lens_dev, const int32_t* cache_lens_host,
                                 void* k_cache, void* v_cache, int32_t S_cap, void* ws, size_t ws_bytes,
                                 void* stream) {
  return decode_layer_checked(cfg, w, x, y, B, cache_lens_dev, cache_lens_host, k_cache, v_cache, S_cap, ws, ws_bytes,
                              false, stream);
}

int energon_decode_layer_forward_static(const EnergonLayerConfig* cfg, const EnergonLayerWeights* w, const void* x,
                                        void* y, int32_t B, const int32_t* cache_lens_dev,
                                        const int32_t* cache_lens_host, void* k_cache, void* v_cache, int32_t S_cap,
                                        void* stream) {
  return decode_layer_checked(cfg, w, x, y, B, cache_lens_dev, cache_lens_host, k_cache, v_cache, S_cap, nullptr,
                              (size_t)ENERGON_STATIC_SCRATCH_BYTES, true, stream);
}

int energon_embed_packed(const int32_t* ids_dev, const int32_t* cu, int64_t T, int32_t B, const void* wte, int32_t V,
                         const void* wpe, int32_t P, int32_t H, int32_t dtype, void* x_packed, void* stream) {
  if (!ids_dev || !cu || !wte || !wpe || !x_packed) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (T < 0 || T >= ((int64_t)1 << 31) || B <= 0 || V <= 0 || P <= 0 || H <= 0 || H % 8 != 0) return ENERGON_ERR_SHAPE;
  if (!aligned16(wte) || !aligned16(wpe) || !aligned16(x_packed) || (reinterpret_cast<uintptr_t>(ids_dev) & 3u) ||
      (reinterpret_cast<uintptr_t>(cu) & 3u))
    return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_embed_packed(ids_dev, cu, nullptr, B, T, wte, V, wpe, P, H, dtype, x_packed,
                              static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_embed_at(const int32_t* ids_dev, const int32_t* positions_dev, int64_t n, const void* wte, int32_t V,
                     const void* wpe, int32_t P, int32_t H, int32_t dtype, void* x, void* stream) {
  if (!ids_dev || !positions_dev || !wte || !wpe || !x) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (n < 0 || n >= ((int64_t)1 << 31) || V <= 0 || P <= 0 || H <= 0 || H % 8 != 0) return ENERGON_ERR_SHAPE;
  if (!aligned16(wte) || !aligned16(wpe) || !aligned16(x) || (reinterpret_cast<uintptr_t>(ids_dev) & 3u) ||
      (reinterpret_cast<uintptr_t>(positions_dev) & 3u))
    return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_embed_packed(ids_dev, nullptr, positions_dev, 1, n, wte, V, wpe, P, H, dtype, x,
                              static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

int energon_last_token_rows(const void* x_packed, const int32_t* cu, int32_t B, int32_t H, int32_t dtype, void* out,
                            void* stream) {
  if (!x_packed || !cu || !out) return ENERGON_ERR_NULL;
  if (!dtype_ok(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (!is16(dtype)) return ENERGON_ERR_UNSUPPORTED;
  if (B < 0 || H <= 0 || H % 8 != 0) return ENERGON_ERR_SHAPE;
  if (!aligned16(x_packed) || !aligned16(out) || (reinterpret_cast<uintptr_t>(cu) & 3u)) return ENERGON_ERR_ALIGN;
  HIP_TRY(launch_last_rows(x_packed, cu, B, (int64_t)H * esize(dtype), out, static_cast<hipStream_t>(stream)));
  return ENERGON_OK;
}

}  // extern "C"
