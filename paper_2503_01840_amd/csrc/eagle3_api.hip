// C ABI (include/eagle3.h): argument checks, workspace carving and the launch sequences of the four
// step calls.  No arithmetic of the method happens on the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/eagle3.h"
#include "../../include/eagle3_measure.h"
#include "common.hpp"
#include "kernels.hpp"

namespace {

thread_local char g_err[512] = "";

int fail_hip(hipError_t e, const char* what) {
  snprintf(g_err, sizeof(g_err), "%s: %s", what, hipGetErrorString(e));
  return EAGLE3_E_HIP;
}
#define CK(expr)                                             \
  do {                                                       \
    hipError_t _e = (expr);                                  \
    if (_e != hipSuccess) return fail_hip(_e, #expr);        \
  } while (0)

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Carver {          // first pass (base == nullptr) measures, second pass hands out pointers
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T> T* take(size_t n) {
    T* p = base ? (T*)(base + off) : nullptr;
    off += align_up(n * sizeof(T));
    return p;
  }
};

}  // namespace

struct eagle3_ctx {
  eagle3_config cfg;
  bool bf16;
  size_t act_size;                      // bytes per activation element
  std::vector<eagle3_layer_weights> layers;
  eagle3_target_weights tw;
  eagle3_draft_weights dw;
  bool has_target = false, has_draft = false;
  void* ws = nullptr;
  size_t ws_bytes = 0, ws_need = 0;

  // optional per-launch timing of the GEMMs
  bool profiling = false;
  struct Stamp { hipEvent_t a, b; double bytes; int kind; };
  std::vector<Stamp> stamps;
  size_t stamps_used = 0;

  int R_max, Md_max, Rall, a_rows, pool_max;
  size_t part_floats, attn_floats;
  // workspace
  float* x; void* act_k; void* act_attn; void* act_h; void* q; float* part; float* attn_scratch;
  int32_t* depth; uint32_t* mask; int32_t* slot; float* cs; SeqInfo* seq;
  float* accept_stats;
  float* z; float* a_buf; int32_t* pos1; float* topk_scratch; DraftState ds;
  int chunk_max;                        // rows per prefill chunk
  int32_t* chain_parent; float* chunk_taps; float* chunk_g;
  int rows1_max;                        // rows per sequence of a chain batch's forward 1
  ChainState cs_chain;

  void carve(void* base) {
    const eagle3_config& c = cfg;
    Carver cv(base);
    const size_t k = c.hidden, I = c.intermediate, Hd = (size_t)c.n_heads * c.head_dim;
    const size_t Rpad = (size_t)(Rall + 63) / 64 * 64;
    x = cv.take<float>((size_t)Rall * k);
    act_k = cv.take<char>(Rpad * 3 * k * act_size);
    act_attn = cv.take<char>(Rpad * Hd * act_size);
    act_h = cv.take<char>(Rpad * I * act_size);
    q = cv.take<char>((size_t)Rall * Hd * act_size);
    part = cv.take<float>(part_floats);
    attn_scratch = cv.take<float>(attn_floats);
    depth = cv.take<int32_t>(Rall);
    mask = cv.take<uint32_t>((size_t)Rall * 4);
    slot = cv.take<int32_t>(Rall);
    cs = cv.take<float>((size_t)Rall * c.head_dim);
    seq = cv.take<SeqInfo>(std::max(c.max_batch, 1));
    accept_stats = cv.take<float>(accept_scratch_floats(R_max, c.vocab));
    const int mb = std::max(c.max_batch, 1);
    z = cv.take<float>((size_t)std::max(Md_max, mb) * c.draft_vocab);
    a_buf = cv.take<float>((size_t)std::max(a_rows, mb * rows1_max) * k);
    pos1 = cv.take<int32_t>(Rall);
    topk_scratch = cv.take<float>(std::max(topk_scratch_floats(c.max_topk, c.draft_vocab, c.max_topk),
                                           topk_scratch_floats(mb, c.draft_vocab, 1)));
    cs_chain.top_val = cv.take<float>(mb);
    cs_chain.top_idx = cv.take<int32_t>(mb);
    cs_chain.row_tok = cv.take<int32_t>(mb);
    cs_chain.row_src = cv.take<int32_t>(mb);
    cs_chain.row_pos = cv.take<int32_t>(mb);
    cs_chain.row_slot = cv.take<int32_t>(mb);
    cs_chain.row_mask = cv.take<uint32_t>((size_t)mb * 4);
    cs_chain.seq = cv.take<SeqInfo>(mb);
    ds.pool_tok = cv.take<int32_t>(pool_max);
    ds.pool_parent = cv.take<int32_t>(pool_max);
    ds.pool_depth = cv.take<int32_t>(pool_max);
    ds.pool_score = cv.take<float>(pool_max);
    ds.pool_mask = cv.take<uint32_t>((size_t)pool_max * 4);
    ds.frontier = cv.take<int32_t>((size_t)c.max_depth * c.max_topk);
    ds.top_val = cv.take<float>((size_t)Md_max * c.max_topk);
    ds.top_idx = cv.take<int32_t>((size_t)Md_max * c.max_topk);
    ds.row_tok = cv.take<int32_t>(c.max_topk);
    ds.row_src = cv.take<int32_t>(c.max_topk);
    ds.row_pos = cv.take<int32_t>(c.max_topk);
    ds.row_slot = cv.take<int32_t>(c.max_topk);
    ds.row_mask = cv.take<uint32_t>((size_t)c.max_topk * 4);
    ds.seq = cv.take<SeqInfo>(1);
    chain_parent = cv.take<int32_t>(64);
    chunk_taps = cv.take<float>((size_t)3 * chunk_max * k);
    chunk_g = cv.take<float>((size_t)chunk_max * k);
    ws_need = cv.off;
  }

  // One projection Y = act W^T.  epi PARTIAL: result (S partial sums) in `part`; *S_out = S.
  // epi SWIGLU: silu(gate)*up lands in act_h.
  int project(const void* act_in, const GemmWeights& W, int M, int N, int K, int epi, int* S_out, hipStream_t st,
              float* direct_out = nullptr) {
    if (bf16 && M > 64) {
      Stamp* sp = profiling && stamps_used < stamps.size() ? &stamps[stamps_used++] : nullptr;
      if (sp) { sp->bytes = 2.0 * N * K; sp->kind = EAGLE3_GEMM_MANY_ROWS; }
      int S = 1;
      void* out = epi == GEMM_EPI_SWIGLU ? act_h : (direct_out ? (void*)direct_out : (void*)part);
      CK(launch_gemm_wide((const bf16_t*)act_in, W, M, N, K, epi, out, direct_out ? 0 : part_floats, &S, st,
                          sp ? sp->a : nullptr, sp ? sp->b : nullptr));
      if (S_out) *S_out = S;
      return EAGLE3_OK;
    }
    if (bf16) {
      int S = epi == GEMM_EPI_SWIGLU ? 1 : gemm_skinny_pick_splits(N, K, M);
      while (S > 1 && ((size_t)S * M * N > part_floats || (K / 128) % S != 0)) --S;   // the next smaller divisor of the stage count
      if (epi == GEMM_EPI_PARTIAL && direct_out == nullptr && (size_t)S * M * N > part_floats) return EAGLE3_E_STATE;
      void* out = epi == GEMM_EPI_SWIGLU ? act_h : (direct_out && S == 1 ? (void*)direct_out : (void*)part);
      Stamp* sp = profiling && stamps_used < stamps.size() ? &stamps[stamps_used++] : nullptr;
      if (sp) {
        sp->bytes = 2.0 * N * K;
        sp->kind = M <= 32 ? EAGLE3_GEMM_FEW_ROWS : gemm_skinny_uses_tile128(W, M, N, S) ? EAGLE3_GEMM_TILE128 : EAGLE3_GEMM_TILE64;
      }
      CK(launch_gemm_skinny((const bf16_t*)act_in, W, M, N, K, S, epi, out, st, sp ? sp->a : nullptr, sp ? sp->b : nullptr));
      if (direct_out && S > 1) CK(launch_reduce_partials(part, S, M, N, direct_out, st));
      if (S_out) *S_out = S;
      return EAGLE3_OK;
    }
    if ((size_t)M * N > part_floats && !direct_out) return EAGLE3_E_STATE;
    float* out = direct_out ? direct_out : part;
    int col = 0;
    for (int i = 0; i < W.nmat; ++i) {
      CK(launch_gemm_f32((const float*)act_in, (const float*)W.w[i], M, W.rows[i], K, out, N, col, st));
      col += W.rows[i];
    }
    if (epi == GEMM_EPI_SWIGLU) CK(launch_swiglu_f32(part, M, N / 2, (float*)act_h, st));
    if (S_out) *S_out = 1;
    return EAGLE3_OK;
  }
};

#define TRY(expr)                  \
  do {                             \
    int _rc = (expr);              \
    if (_rc != EAGLE3_OK) return _rc; \
  } while (0)

extern "C" {

const char* eagle3_strerror(int code) {
  switch (code) {
    case EAGLE3_OK: return "ok";
    case EAGLE3_E_NULL: return "a required pointer is NULL";
    case EAGLE3_E_SHAPE: return "a size is outside what the configuration or the kernels support";
    case EAGLE3_E_STATE: return "weights or workspace not set, or workspace too small";
    case EAGLE3_E_HIP: return "a HIP call failed (see eagle3_last_error)";
    default: return "unknown error code";
  }
}
const char* eagle3_last_error(void) { return g_err; }

int eagle3_create(const eagle3_config* cfg, eagle3_ctx** out) {
  if (!cfg || !out) return EAGLE3_E_NULL;
  const eagle3_config& c = *cfg;
  if (c.hidden <= 0 || c.n_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.intermediate <= 0 || c.vocab <= 0 ||
      c.draft_vocab <= 0 || c.draft_vocab > 512 * 1024 || c.n_layers <= 0 || c.n_heads % c.n_kv_heads != 0)
    return EAGLE3_E_SHAPE;
  if (c.dtype != EAGLE3_BF16 && c.dtype != EAGLE3_FP32) return EAGLE3_E_SHAPE;
  if (c.max_batch < 1 || c.max_nodes < 1 || c.max_nodes > 64 || c.max_depth < 1 || c.max_topk < 1 || c.max_topk > 16 ||
      c.max_new < 1 || c.max_new > 64 || (c.max_depth - 1) * c.max_topk > 128 ||
      1 + c.max_topk + (c.max_depth - 1) * c.max_topk * c.max_topk > DRAFT_MAX_POOL)
    return EAGLE3_E_SHAPE;
  for (int t = 0; t < 3; ++t)
    if (c.tap_layers[t] < 0 || c.tap_layers[t] >= c.n_layers) return EAGLE3_E_SHAPE;
  if (c.dtype == EAGLE3_BF16) {
    if (c.head_dim != 128 || c.hidden % 128 || c.intermediate % 128 || (c.n_heads * c.head_dim) % 128)
      return EAGLE3_E_SHAPE;
    // launches of more than 64 rows go through the many-row GEMM, which stores four outputs at a time
    const long many = std::max((long)c.max_batch * c.max_nodes, (long)c.max_batch * c.max_new);
    if (many > 64 && (c.vocab % 4 || c.draft_vocab % 4)) return EAGLE3_E_SHAPE;
  } else {
    if (c.head_dim % 2 || c.head_dim > 256) return EAGLE3_E_SHAPE;
  }
  if (!(c.rope_theta > 0.f) || !(c.rms_eps >= 0.f)) return EAGLE3_E_SHAPE;
  eagle3_ctx* ctx = new (std::nothrow) eagle3_ctx();
  if (!ctx) return EAGLE3_E_STATE;
  ctx->cfg = c;
  ctx->bf16 = c.dtype == EAGLE3_BF16;
  ctx->act_size = ctx->bf16 ? 2 : 4;
  ctx->R_max = c.max_batch * c.max_nodes;
  ctx->Md_max = std::max(c.max_new, c.max_topk);
  ctx->Rall = std::max(ctx->R_max, ctx->Md_max);
  ctx->a_rows = c.max_new + (c.max_depth - 1) * c.max_topk;
  ctx->chunk_max = std::min(c.max_nodes, c.max_new);
  ctx->rows1_max = std::min(c.max_nodes, c.max_new);
  ctx->pool_max = 1 + c.max_topk + (c.max_depth - 1) * c.max_topk * c.max_topk;
  const size_t widest = std::max<size_t>({(size_t)(c.n_heads + 2 * c.n_kv_heads) * c.head_dim, (size_t)c.hidden,
                                          ctx->bf16 ? (size_t)0 : (size_t)2 * c.intermediate});
  // split-K partial sums: up to 4 slices of the widest projection, 8 of a hidden-sized one
  ctx->part_floats = std::max<size_t>({1024 * widest, 4 * (size_t)ctx->Rall * widest, 8 * (size_t)ctx->Rall * c.hidden});
  size_t af = 0;
  for (int b = 1; b <= c.max_batch; ++b) {
    const int s = attention_pick_splits(b, c.max_nodes, c.n_heads, c.n_kv_heads, 1 << 30);
    af = std::max(af, attention_scratch_floats(b * c.max_nodes, c.n_heads, c.head_dim, s));
  }
  af = std::max(af, attention_scratch_floats(ctx->Md_max, c.n_heads, c.head_dim,
                                             attention_pick_splits(1, ctx->Md_max, c.n_heads, c.n_kv_heads, 1 << 30)));
  ctx->attn_floats = ctx->bf16 ? af : 1;
  ctx->carve(nullptr);
  *out = ctx;
  return EAGLE3_OK;
}

int eagle3_destroy(eagle3_ctx* ctx) {
  if (ctx)
    for (auto& s : ctx->stamps) {
      (void)hipEventDestroy(s.a);
      (void)hipEventDestroy(s.b);
    }
  delete ctx;
  return EAGLE3_OK;
}

int eagle3_workspace_bytes(const eagle3_ctx* ctx, size_t* out) {
  if (!ctx || !out) return EAGLE3_E_NULL;
  *out = ctx->ws_need;
  return EAGLE3_OK;
}

int eagle3_set_workspace(eagle3_ctx* ctx, void* dev, size_t bytes) {
  if (!ctx || !dev) return EAGLE3_E_NULL;
  if (bytes < ctx->ws_need || ((uintptr_t)dev & 255)) return EAGLE3_E_STATE;
  ctx->ws = dev;
  ctx->ws_bytes = bytes;
  ctx->carve(dev);
  return EAGLE3_OK;
}

int eagle3_set_weights(eagle3_ctx* ctx, const eagle3_target_weights* t, const eagle3_draft_weights* d) {
  if (!ctx) return EAGLE3_E_NULL;
  if (t) {
    if (!t->layers || !t->embed || !t->final_norm || !t->lm_head) return EAGLE3_E_NULL;
    for (int l = 0; l < ctx->cfg.n_layers; ++l) {
      const eagle3_layer_weights& w = t->layers[l];
      if (!w.wq || !w.wk || !w.wv || !w.wo || !w.w_gate || !w.w_up || !w.w_down || !w.norm_attn || !w.norm_mlp)
        return EAGLE3_E_NULL;
    }
    ctx->layers.assign(t->layers, t->layers + ctx->cfg.n_layers);
    ctx->tw = *t;
    ctx->tw.layers = ctx->layers.data();
    ctx->has_target = true;
  }
  if (d) {
    const eagle3_layer_weights& w = d->layer;
    if (!d->w_fc || !d->norm_embed || !d->norm_feat || !d->final_norm || !d->lm_head || !d->d2t || !w.wq || !w.wk ||
        !w.wv || !w.wo || !w.w_gate || !w.w_up || !w.w_down || !w.norm_mlp)
      return EAGLE3_E_NULL;
    ctx->dw = *d;
    ctx->has_draft = true;
  }
  return EAGLE3_OK;
}

int eagle3_profile_begin(eagle3_ctx* ctx) {
  if (!ctx) return EAGLE3_E_NULL;
  if (ctx->stamps.empty()) {
    ctx->stamps.resize(8192);
    for (auto& s : ctx->stamps) {
      CK(hipEventCreate(&s.a));
      CK(hipEventCreate(&s.b));
    }
  }
  ctx->stamps_used = 0;
  ctx->profiling = true;
  return EAGLE3_OK;
}

int eagle3_profile_read(eagle3_ctx* ctx, int kind, double* ms_total, int64_t* launches, double* weight_bytes) {
  if (!ctx || !ms_total || !launches || !weight_bytes) return EAGLE3_E_NULL;
  double ms = 0, bytes = 0;
  int64_t n = 0;
  for (size_t i = 0; i < ctx->stamps_used; ++i) {
    auto& s = ctx->stamps[i];
    if (s.kind != kind) continue;
    CK(hipEventSynchronize(s.b));
    float t = 0.f;
    CK(hipEventElapsedTime(&t, s.a, s.b));
    ms += t; bytes += s.bytes; ++n;
  }
  *ms_total = ms; *launches = n; *weight_bytes = bytes;
  return EAGLE3_OK;
}

int eagle3_profile_end(eagle3_ctx* ctx) {
  if (!ctx) return EAGLE3_E_NULL;
  ctx->profiling = false;
  ctx->stamps_used = 0;
  return EAGLE3_OK;
}

static int fuse_rows(eagle3_ctx* ctx, const float* low, const float* mid, const float* high, int M, float* g_out,
                     hipStream_t st);

int eagle3_fuse_features(eagle3_ctx* ctx, const float* low, const float* mid, const float* high, int32_t M,
                         float* g_out, eagle3_stream stream) {
  if (!ctx || !low || !mid || !high || !g_out) return EAGLE3_E_NULL;
  if (!ctx->ws || !ctx->has_draft) return EAGLE3_E_STATE;
  if (M < 1 || M > ctx->cfg.max_new) return EAGLE3_E_SHAPE;
  return fuse_rows(ctx, low, mid, high, M, g_out, (hipStream_t)stream);
}

static int fuse_rows(eagle3_ctx* ctx, const float* low, const float* mid, const float* high, int M, float* g_out,
                     hipStream_t st) {
  const int k = ctx->cfg.hidden;
  CK(launch_pack3(ctx->bf16, low, mid, high, M, k, ctx->act_k, st));
  GemmWeights W = {{ctx->dw.w_fc, nullptr, nullptr}, {k, 0, 0}, 1, 0};
  return ctx->project(ctx->act_k, W, M, k, 3 * k, GEMM_EPI_PARTIAL, nullptr, st, g_out);
}

// attention + output projection + MLP of one layer, shared by the target stack and the draft layer.
// On entry: qkv partial sums are in `part` (S_qkv of them), x holds the residual rows.
// On exit: `part` holds S_down partial sums of the MLP output (to be added to x by the caller).
static int layer_tail(eagle3_ctx* ctx, const eagle3_layer_weights& w, int B, int rows_per_seq, int S_qkv,
                      const int32_t* slot, const float* cs, const uint32_t* mask, const SeqInfo* seq, void* kc, void* vc,
                      int max_len, int* S_down, hipStream_t st) {
  const eagle3_config& c = ctx->cfg;
  const int R = B * rows_per_seq, k = c.hidden, H = c.n_heads, Hkv = c.n_kv_heads, d = c.head_dim, I = c.intermediate;
  CK(launch_rope_kv_write(ctx->bf16, ctx->part, S_qkv, R, H, Hkv, d, cs, slot, ctx->q, kc, vc, st));
  int ns = 1;
  if (ctx->bf16) {
    ns = attention_pick_splits(B, rows_per_seq, H, Hkv, max_len);
    while (ns > 1 && attention_scratch_floats(R, H, d, ns) > ctx->attn_floats) --ns;
  }
  CK(launch_tree_attention(ctx->bf16, ctx->q, kc, vc, seq, mask, B, rows_per_seq, H, Hkv, d, max_len, ns,
                           ctx->attn_scratch, ctx->act_attn, st));
  int S_o = 1;
  GemmWeights Wo = {{w.wo, nullptr, nullptr}, {k, 0, 0}, 1, 0};
  TRY(ctx->project(ctx->act_attn, Wo, R, k, H * d, GEMM_EPI_PARTIAL, &S_o, st));
  CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_o, R, k, w.norm_mlp, c.rms_eps, ctx->act_k, nullptr, st));
  GemmWeights Wgu = {{w.w_gate, w.w_up, nullptr}, {I, I, 0}, 2, 1};
  TRY(ctx->project(ctx->act_k, Wgu, R, 2 * I, k, GEMM_EPI_SWIGLU, nullptr, st));
  GemmWeights Wd = {{w.w_down, nullptr, nullptr}, {k, 0, 0}, 1, 0};
  TRY(ctx->project(ctx->act_h, Wd, R, k, I, GEMM_EPI_PARTIAL, S_down, st));
  return EAGLE3_OK;
}

// Layers [l0, l1) of the target stack over the B*N node rows.  x_in == nullptr: start from the token
// embeddings (requires l0 == 0).  logits != nullptr: finish with the final norm and the LM head (requires
// l1 == n_layers).  x_out (optional) receives the residual stream after layer l1 - 1.
static int verify_layers(eagle3_ctx* ctx, int B, int N, const int32_t* tree_tok, const int32_t* parent,
                         const eagle3_kv* kv, const float* x_in, int l0, int l1, float* x_out, float* logits, float* taps,
                         float* dbg_hidden, hipStream_t st) {
  const eagle3_config& c = ctx->cfg;
  const int R = B * N, k = c.hidden, H = c.n_heads, Hkv = c.n_kv_heads, d = c.head_dim;
  const int max_len = kv->max_prefix_len + N;
  const size_t Rk = (size_t)R * k;

  CK(launch_tree_prep(parent, kv->kv_indptr, kv->prefix_len, B, N, d, c.rope_theta, ctx->depth, ctx->mask, ctx->slot,
                      ctx->cs, ctx->seq, st));
  if (x_in)
    CK(hipMemcpyAsync(ctx->x, x_in, Rk * sizeof(float), hipMemcpyDeviceToDevice, st));
  else
    CK(launch_embed_rows(ctx->bf16, ctx->tw.embed, tree_tok, R, k, c.vocab, ctx->x, st));
  int S_prev = 0;                                   // partial sums of the previous layer's MLP still to be added
  for (int l = l0; l <= l1; ++l) {
    // x becomes the output of layer l-1 here: record taps / debug copies, then norm for what follows
    float* copies[4] = {nullptr, nullptr, nullptr, nullptr};
    if (l > 0 && taps)
      for (int t = 0; t < 3; ++t)
        if (c.tap_layers[t] == l - 1) copies[t] = taps + (size_t)t * Rk;
    if (dbg_hidden) copies[3] = dbg_hidden + (size_t)l * Rk;
    if (l == l1 && x_out) copies[3] = x_out;
    const bool head = l == c.n_layers;
    if (l == l1 && !(head && logits)) {               // the range ends inside the stack: no norm needed
      CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_prev, R, k, nullptr, c.rms_eps, nullptr, copies, st));
      break;
    }
    const void* gain = head ? ctx->tw.final_norm : ctx->layers[l].norm_attn;
    CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_prev, R, k, gain, c.rms_eps, ctx->act_k, copies, st));
    if (l == l1) break;
    const eagle3_layer_weights& w = ctx->layers[l];
    GemmWeights Wqkv = {{w.wq, w.wk, w.wv}, {H * d, Hkv * d, Hkv * d}, 3, 0};
    int S_qkv = 1;
    TRY(ctx->project(ctx->act_k, Wqkv, R, (H + 2 * Hkv) * d, k, GEMM_EPI_PARTIAL, &S_qkv, st));
    TRY(layer_tail(ctx, w, B, N, S_qkv, ctx->slot, ctx->cs, ctx->mask, ctx->seq, kv->k[l], kv->v[l], max_len, &S_prev, st));
  }
  if (l1 == c.n_layers && logits) {
    GemmWeights Wlm = {{ctx->tw.lm_head, nullptr, nullptr}, {c.vocab, 0, 0}, 1, 0};
    return ctx->project(ctx->act_k, Wlm, R, c.vocab, k, GEMM_EPI_PARTIAL, nullptr, st, logits);
  }
  return EAGLE3_OK;
}

static int check_verify_args(eagle3_ctx* ctx, int B, int N, const int32_t* tree_tok, const int32_t* parent,
                             const eagle3_kv* kv, int l0, int l1) {
  if (!ctx || !tree_tok || !parent || !kv) return EAGLE3_E_NULL;
  if (!kv->k || !kv->v || !kv->kv_indptr || !kv->prefix_len) return EAGLE3_E_NULL;
  if (!ctx->ws || !ctx->has_target) return EAGLE3_E_STATE;
  const eagle3_config& c = ctx->cfg;
  if (B < 1 || B > c.max_batch || N < 1 || N > c.max_nodes || kv->max_prefix_len < 0) return EAGLE3_E_SHAPE;
  if (l0 < 0 || l1 < l0 || l1 > c.n_layers) return EAGLE3_E_SHAPE;
  for (int l = l0; l < l1; ++l)
    if (!kv->k[l] || !kv->v[l]) return EAGLE3_E_NULL;
  return EAGLE3_OK;
}

int eagle3_tree_verify(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* parent,
                       const eagle3_kv* kv, float* logits, float* taps, float* dbg_hidden, eagle3_stream stream) {
  if (!logits || !taps) return EAGLE3_E_NULL;
  TRY(check_verify_args(ctx, B, N, tree_tok, parent, kv, 0, ctx ? ctx->cfg.n_layers : 0));
  return verify_layers(ctx, B, N, tree_tok, parent, kv, nullptr, 0, ctx->cfg.n_layers, nullptr, logits, taps, dbg_hidden,
                       (hipStream_t)stream);
}

int eagle3_tree_verify_layers(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* parent,
                              const eagle3_kv* kv, const float* x_in, int32_t layer_begin, int32_t layer_end,
                              float* x_out, float* logits, eagle3_stream stream) {
  TRY(check_verify_args(ctx, B, N, tree_tok, parent, kv, layer_begin, layer_end));
  if (!x_in && layer_begin != 0) return EAGLE3_E_NULL;
  if (!x_out && !logits) return EAGLE3_E_NULL;
  if (logits && layer_end != ctx->cfg.n_layers) return EAGLE3_E_SHAPE;
  return verify_layers(ctx, B, N, tree_tok, parent, kv, x_in, layer_begin, layer_end, x_out, logits, nullptr, nullptr,
                       (hipStream_t)stream);
}

int eagle3_draft_expand(eagle3_ctx* ctx, const float* g_new, const int32_t* tok_new, int32_t n_new,
                        const eagle3_kv* dkv, int32_t depth, int32_t topk, int32_t n_nodes, int32_t* tree_tok,
                        int32_t* parent, int32_t* node_depth, float* cum_logprob, const eagle3_draft_debug* dbg,
                        eagle3_stream stream) {
  if (!ctx || !g_new || !tok_new || !dkv || !tree_tok || !parent || !node_depth || !cum_logprob) return EAGLE3_E_NULL;
  if (!dkv->k || !dkv->v || !dkv->k[0] || !dkv->v[0] || !dkv->kv_indptr || !dkv->prefix_len) return EAGLE3_E_NULL;
  if (!ctx->ws || !ctx->has_draft || !ctx->has_target) return EAGLE3_E_STATE;    // the target's embedding table is used
  const eagle3_config& c = ctx->cfg;
  const int pool = 1 + topk + (depth - 1) * topk * topk;
  if (n_new < 1 || n_new > c.max_new || depth < 1 || depth > c.max_depth || topk < 1 || topk > c.max_topk ||
      n_nodes < 2 || n_nodes > c.max_nodes || n_nodes > pool || dkv->max_prefix_len < 0)
    return EAGLE3_E_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  const int k = c.hidden, H = c.n_heads, Hkv = c.n_kv_heads, d = c.head_dim, Vd = c.draft_vocab, K = topk;
  const eagle3_layer_weights& w = ctx->dw.layer;
  const DraftState& ds = ctx->ds;
  void* kc = dkv->k[0];
  void* vc = dkv->v[0];

  for (int level = 1; level <= depth; ++level) {
    const int M = level == 1 ? n_new : K;
    const int a_row0 = level == 1 ? 0 : n_new + (level - 2) * K;
    const int32_t *pos, *slot;
    const uint32_t* mask;
    const SeqInfo* seq;
    int max_len;
    if (level == 1) {
      CK(launch_draft_prep1(dkv->kv_indptr, dkv->prefix_len, n_new, ctx->pos1, ctx->slot, ctx->mask, ctx->seq, st));
      pos = ctx->pos1; slot = ctx->slot; mask = ctx->mask; seq = ctx->seq;
      max_len = dkv->max_prefix_len + n_new;
      CK(launch_draft_input(ctx->bf16, ctx->tw.embed, c.vocab, tok_new, g_new, nullptr, M, k, ctx->dw.norm_embed,
                            ctx->dw.norm_feat, c.rms_eps, ctx->act_k, ctx->x, pos, d, c.rope_theta, ctx->cs, st));
    } else {
      pos = ds.row_pos; slot = ds.row_slot; mask = ds.row_mask; seq = ds.seq;
      max_len = dkv->max_prefix_len + n_new + (level - 1) * K;
      CK(launch_draft_input(ctx->bf16, ctx->tw.embed, c.vocab, ds.row_tok, ctx->a_buf, ds.row_src, M, k,
                            ctx->dw.norm_embed, ctx->dw.norm_feat, c.rms_eps, ctx->act_k, ctx->x, pos, d, c.rope_theta, ctx->cs,
                            st));
    }
    GemmWeights Wqkv = {{w.wq, w.wk, w.wv}, {H * d, Hkv * d, Hkv * d}, 3, 0};
    int S_qkv = 1, S_down = 1;
    TRY(ctx->project(ctx->act_k, Wqkv, M, (H + 2 * Hkv) * d, 2 * k, GEMM_EPI_PARTIAL, &S_qkv, st));
    TRY(layer_tail(ctx, w, 1, M, S_qkv, slot, ctx->cs, mask, seq, kc, vc, max_len, &S_down, st));
    // a = y1 + MLP(...): keep it for the children, and norm it for the LM head
    float* copies[4] = {ctx->a_buf + (size_t)a_row0 * k, nullptr, nullptr, nullptr};
    CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_down, M, k, ctx->dw.final_norm, c.rms_eps, ctx->act_k, copies, st));
    GemmWeights Wlm = {{ctx->dw.lm_head, nullptr, nullptr}, {Vd, 0, 0}, 1, 0};
    TRY(ctx->project(ctx->act_k, Wlm, M, Vd, k, GEMM_EPI_PARTIAL, nullptr, st, ctx->z));
    const int row0 = level == 1 ? n_new - 1 : 0, n_rows = level == 1 ? 1 : K;
    CK(launch_topk_rows(ctx->z, Vd, row0, n_rows, Vd, K, ctx->topk_scratch, ds.top_val, ds.top_idx, st));
    CK(launch_draft_select(ds, ctx->dw.d2t, dkv->kv_indptr, dkv->prefix_len, level, depth, K, n_new, 0, st));
  }
  CK(launch_draft_rerank(ds, ctx->dw.d2t, tok_new, n_new, depth, K, n_nodes, tree_tok, parent, node_depth, cum_logprob,
                         dbg ? dbg->chosen : nullptr, st));
  if (dbg) {
    const size_t pb = (size_t)pool * 4;
    if (dbg->pool_tok) CK(hipMemcpyAsync(dbg->pool_tok, ds.pool_tok, pb, hipMemcpyDeviceToDevice, st));
    if (dbg->pool_parent) CK(hipMemcpyAsync(dbg->pool_parent, ds.pool_parent, pb, hipMemcpyDeviceToDevice, st));
    if (dbg->pool_score) CK(hipMemcpyAsync(dbg->pool_score, ds.pool_score, pb, hipMemcpyDeviceToDevice, st));
    if (dbg->frontier && depth > 1)
      CK(hipMemcpyAsync(dbg->frontier, ds.frontier, (size_t)(depth - 1) * K * 4, hipMemcpyDeviceToDevice, st));
  }
  return EAGLE3_OK;
}

int eagle3_accept(eagle3_ctx* ctx, int32_t B, int32_t N, const float* logits, const int32_t* tree_tok,
                  const int32_t* parent, float temperature, const float* uniforms, int32_t* accept_len, int32_t* path,
                  int32_t* bonus_tok, eagle3_stream stream) {
  if (!ctx || !logits || !tree_tok || !parent || !accept_len || !path || !bonus_tok) return EAGLE3_E_NULL;
  if (temperature > 0.f && !uniforms) return EAGLE3_E_NULL;
  if (!ctx->ws) return EAGLE3_E_STATE;
  if (B < 1 || B > ctx->cfg.max_batch || N < 1 || N > ctx->cfg.max_nodes || !(temperature >= 0.f)) return EAGLE3_E_SHAPE;
  CK(launch_accept(logits, tree_tok, parent, B, N, ctx->cfg.vocab, temperature, uniforms, ctx->accept_stats, accept_len,
                   path, bonus_tok, (hipStream_t)stream));
  return EAGLE3_OK;
}

int eagle3_draft_chain(eagle3_ctx* ctx, int32_t B, const float* g_new, const int32_t* tok_new, const int32_t* n_new,
                       int32_t rows1, const eagle3_kv* dkv, int32_t length, int32_t* chain_tok, float* chain_logp,
                       eagle3_stream stream) {
  if (!ctx || !g_new || !tok_new || !n_new || !dkv || !chain_tok || !chain_logp) return EAGLE3_E_NULL;
  if (!dkv->k || !dkv->v || !dkv->k[0] || !dkv->v[0] || !dkv->kv_indptr || !dkv->prefix_len) return EAGLE3_E_NULL;
  if (!ctx->ws || !ctx->has_draft || !ctx->has_target) return EAGLE3_E_STATE;
  const eagle3_config& c = ctx->cfg;
  if (B < 1 || B > c.max_batch || rows1 < 1 || rows1 > ctx->rows1_max || length < 1 || length > c.max_depth ||
      dkv->max_prefix_len < 0)
    return EAGLE3_E_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  const int k = c.hidden, H = c.n_heads, Hkv = c.n_kv_heads, d = c.head_dim, Vd = c.draft_vocab;
  const eagle3_layer_weights& w = ctx->dw.layer;
  const ChainState& cs = ctx->cs_chain;
  void* kc = dkv->k[0];
  void* vc = dkv->v[0];
  for (int level = 1; level <= length; ++level) {
    const int rps = level == 1 ? rows1 : 1, M = B * rps;
    const int32_t *pos, *slot;
    const uint32_t* mask;
    const SeqInfo* seq;
    if (level == 1) {
      CK(launch_chain_prep1(dkv->kv_indptr, dkv->prefix_len, B, rows1, ctx->pos1, ctx->slot, ctx->mask, ctx->seq, st));
      pos = ctx->pos1; slot = ctx->slot; mask = ctx->mask; seq = ctx->seq;
      CK(launch_draft_input(ctx->bf16, ctx->tw.embed, c.vocab, tok_new, g_new, nullptr, M, k, ctx->dw.norm_embed,
                            ctx->dw.norm_feat, c.rms_eps, ctx->act_k, ctx->x, pos, d, c.rope_theta, ctx->cs, st));
    } else {
      pos = cs.row_pos; slot = cs.row_slot; mask = cs.row_mask; seq = cs.seq;
      CK(launch_draft_input(ctx->bf16, ctx->tw.embed, c.vocab, cs.row_tok, ctx->a_buf, cs.row_src, M, k, ctx->dw.norm_embed,
                            ctx->dw.norm_feat, c.rms_eps, ctx->act_k, ctx->x, pos, d, c.rope_theta, ctx->cs, st));
    }
    const int max_len = dkv->max_prefix_len + rows1 + level;
    GemmWeights Wqkv = {{w.wq, w.wk, w.wv}, {H * d, Hkv * d, Hkv * d}, 3, 0};
    int S_qkv = 1, S_down = 1;
    TRY(ctx->project(ctx->act_k, Wqkv, M, (H + 2 * Hkv) * d, 2 * k, GEMM_EPI_PARTIAL, &S_qkv, st));
    TRY(layer_tail(ctx, w, B, rps, S_qkv, slot, ctx->cs, mask, seq, kc, vc, max_len, &S_down, st));
    if (level == 1 && rows1 > 1) {
      // a = y1 + MLP(...) for every row, then the row of each sequence's last real position moves to row b
      CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_down, M, k, nullptr, c.rms_eps, nullptr, nullptr, st));
      CK(launch_chain_gather(ctx->x, n_new, B, rows1, k, ctx->a_buf, st));
      CK(hipMemcpyAsync(ctx->x, ctx->a_buf, (size_t)B * k * sizeof(float), hipMemcpyDeviceToDevice, st));
      CK(launch_add_norm(ctx->bf16, ctx->x, nullptr, 0, B, k, ctx->dw.final_norm, c.rms_eps, ctx->act_k, nullptr, st));
    } else {
      float* copies[4] = {ctx->a_buf, nullptr, nullptr, nullptr};
      CK(launch_add_norm(ctx->bf16, ctx->x, ctx->part, S_down, B, k, ctx->dw.final_norm, c.rms_eps, ctx->act_k, copies, st));
    }
    GemmWeights Wlm = {{ctx->dw.lm_head, nullptr, nullptr}, {Vd, 0, 0}, 1, 0};
    TRY(ctx->project(ctx->act_k, Wlm, B, Vd, k, GEMM_EPI_PARTIAL, nullptr, st, ctx->z));
    CK(launch_topk_rows(ctx->z, Vd, 0, B, Vd, 1, ctx->topk_scratch, cs.top_val, cs.top_idx, st));
    CK(launch_chain_select(cs, ctx->dw.d2t, dkv->kv_indptr, dkv->prefix_len, n_new, tok_new, B, rows1, level, length,
                           chain_tok, chain_logp, st));
  }
  return EAGLE3_OK;
}

int eagle3_prefill(eagle3_ctx* ctx, const int32_t* tokens, int32_t T, const eagle3_kv* kv, const eagle3_kv* dkv,
                   float* g_last, float* logits_last, eagle3_stream stream) {
  if (!ctx || !tokens || !kv || !dkv || !g_last || !logits_last) return EAGLE3_E_NULL;
  if (!kv->k || !kv->v || !kv->kv_indptr || !kv->prefix_len) return EAGLE3_E_NULL;
  if (!dkv->k || !dkv->v || !dkv->k[0] || !dkv->v[0] || !dkv->kv_indptr || !dkv->prefix_len) return EAGLE3_E_NULL;
  if (!ctx->ws || !ctx->has_target || !ctx->has_draft) return EAGLE3_E_STATE;
  const eagle3_config& c = ctx->cfg;
  if (T < 1 || kv->max_prefix_len < 0 || dkv->max_prefix_len < 0) return EAGLE3_E_SHAPE;
  for (int l = 0; l < c.n_layers; ++l)
    if (!kv->k[l] || !kv->v[l]) return EAGLE3_E_NULL;
  hipStream_t st = (hipStream_t)stream;
  const int k = c.hidden, H = c.n_heads, Hkv = c.n_kv_heads, d = c.head_dim, C = ctx->chunk_max;
  const eagle3_layer_weights& w = ctx->dw.layer;
  CK(launch_chain_parent(ctx->chain_parent, std::min(C, 64), st));
  int done_draft = 0;
  for (int c0 = 0; c0 < T; c0 += C) {
    const int n = std::min(C, T - c0);
    const bool last = c0 + n == T;
    // target: the chunk as a chain on top of everything cached so far; features of every position recorded
    eagle3_kv kvc = *kv;
    kvc.max_prefix_len = kv->max_prefix_len + c0;
    const size_t nk = (size_t)n * k;
    TRY(verify_layers(ctx, 1, n, tokens + c0, ctx->chain_parent, &kvc, nullptr, 0, c.n_layers, nullptr, nullptr,
                      ctx->chunk_taps, nullptr, st));
    CK(launch_advance_lengths((int32_t*)kv->prefix_len, 1, n, st));
    if (last) {                                       // next-token logits of the last position only
      CK(launch_add_norm(ctx->bf16, ctx->x + (size_t)(n - 1) * k, nullptr, 0, 1, k, ctx->tw.final_norm, c.rms_eps, ctx->act_k,
                         nullptr, st));
      GemmWeights Wlm = {{ctx->tw.lm_head, nullptr, nullptr}, {c.vocab, 0, 0}, 1, 0};
      TRY(ctx->project(ctx->act_k, Wlm, 1, c.vocab, k, GEMM_EPI_PARTIAL, nullptr, st, logits_last));
    }
    // fused features of the chunk's positions; the draft cache rows of those whose next token is known
    TRY(fuse_rows(ctx, ctx->chunk_taps, ctx->chunk_taps + nk, ctx->chunk_taps + 2 * nk, n, ctx->chunk_g, st));
    if (last) CK(hipMemcpyAsync(g_last, ctx->chunk_g + (size_t)(n - 1) * k, (size_t)k * sizeof(float), hipMemcpyDeviceToDevice, st));
    const int m = last ? n - 1 : n;
    if (m > 0) {
      CK(launch_draft_prep1(dkv->kv_indptr, dkv->prefix_len, m, ctx->pos1, ctx->slot, ctx->mask, ctx->seq, st));
      CK(launch_draft_input(ctx->bf16, ctx->tw.embed, c.vocab, tokens + c0 + 1, ctx->chunk_g, nullptr, m, k, ctx->dw.norm_embed,
                            ctx->dw.norm_feat, c.rms_eps, ctx->act_k, ctx->x, ctx->pos1, d, c.rope_theta, ctx->cs, st));
      GemmWeights Wqkv = {{w.wq, w.wk, w.wv}, {H * d, Hkv * d, Hkv * d}, 3, 0};
      int S_qkv = 1;
      TRY(ctx->project(ctx->act_k, Wqkv, m, (H + 2 * Hkv) * d, 2 * k, GEMM_EPI_PARTIAL, &S_qkv, st));
      CK(launch_rope_kv_write(ctx->bf16, ctx->part, S_qkv, m, H, Hkv, d, ctx->cs, ctx->slot, ctx->q, dkv->k[0], dkv->v[0], st));
      CK(launch_advance_lengths((int32_t*)dkv->prefix_len, 1, m, st));
      done_draft += m;
    }
  }
  (void)done_draft;
  return EAGLE3_OK;
}

int eagle3_ttt_attention(int32_t dtype, int32_t T, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, int32_t step,
                         const void* q, const void* k_steps, const void* v_steps, float* out, eagle3_stream stream) {
  if (!q || !k_steps || !v_steps || !out) return EAGLE3_E_NULL;
  if (dtype != EAGLE3_BF16 && dtype != EAGLE3_FP32) return EAGLE3_E_SHAPE;
  if (T < 1 || n_heads < 1 || n_kv_heads < 1 || n_heads % n_kv_heads || step < 0 || head_dim < 1) return EAGLE3_E_SHAPE;
  if (dtype == EAGLE3_BF16 ? head_dim != 128 : (head_dim > 1024 || (size_t)(T + step) * 4 > 60 * 1024)) return EAGLE3_E_SHAPE;
  CK(launch_ttt_attention(dtype == EAGLE3_BF16, q, k_steps, v_steps, T, n_heads, n_kv_heads, head_dim, step, out,
                          (hipStream_t)stream));
  return EAGLE3_OK;
}

int eagle3_commit(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* path,
                  const int32_t* accept_len, const int32_t* bonus_tok, const eagle3_kv* kv, int32_t* prefix_len,
                  const float* taps, int32_t rows, float* taps_new, int32_t* tok_new, int32_t* n_new,
                  int32_t* draft_prefix_len, int32_t draft_rows, eagle3_stream stream) {
  if (!ctx || !tree_tok || !path || !accept_len || !bonus_tok || !kv || !prefix_len || !taps || !tok_new || !n_new)
    return EAGLE3_E_NULL;
  if (!kv->k || !kv->v || !kv->kv_indptr) return EAGLE3_E_NULL;
  const eagle3_config& c = ctx->cfg;
  if (B < 1 || B > c.max_batch || N < 1 || N > c.max_nodes || rows < 1 || draft_rows < 0) return EAGLE3_E_SHAPE;
  for (int l = 0; l < c.n_layers; ++l)
    if (!kv->k[l] || !kv->v[l]) return EAGLE3_E_NULL;
  CK(launch_commit(kv->k, kv->v, c.n_layers, kv->kv_indptr, prefix_len, tree_tok, path, accept_len, bonus_tok, taps, B, N,
                   c.hidden, (int)(c.n_kv_heads * c.head_dim * ctx->act_size), rows, taps_new, tok_new, n_new,
                   draft_prefix_len, draft_rows, (hipStream_t)stream));
  return EAGLE3_OK;
}

}  // extern "C"
