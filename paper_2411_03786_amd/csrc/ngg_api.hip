// C ABI of libngg (declared in include/ngg.h): context, argument checks, the launch sequence of
// one verify step and the decode loop.  Host logic only; every step of the path runs in kernels.
#include "ngg.h"
#include "ngg_internal.h"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace ngg;

// Scratch memory of ngg_context_drafts_static: match list, (count, last start) pairs and the grouping
// table of the context matcher for up to NGG_STATIC_MAX_TOKENS tokens.  Every GPU the library runs on
// holds its own copy until the process ends.
constexpr int kStaticSlots = 2 * NGG_STATIC_MAX_TOKENS;                       // a power of two
constexpr size_t kStaticInts = (size_t)NGG_STATIC_MAX_TOKENS * 3 + (size_t)3 * kStaticSlots;
static __device__ __align__(256) int32_t scratch[kStaticInts];

namespace {

// Prompt tokens per forward pass of ngg_prefill.  16-bit models: up to 2048, which the wide GEMM kernel takes as
// row tiles of 256 that share the weights through the L2 (one sweep of the weights from HBM per 2048 tokens instead
// of per 256); fp32 models: 256 (two 128-row passes of the skinny kernel).
constexpr int kPrefillChunk16 = 2048, kPrefillChunk32 = 256;
thread_local std::string g_create_error = "";

struct ProfSpan { int cls; hipEvent_t e0, e1; };

}  // namespace

struct ngg_ctx {
  ngg_model_desc d{};
  ngg_weights w{};
  std::vector<ngg_layer_weights> layers;
  hipStream_t stream = nullptr;
  int esize = 2;          // bytes per weight / KV element
  int Spad = 0, Mcap = 0, max_splits = 0, unembed_tiles = 0;
  int prefill_chunk = 0;           // prompt tokens per forward pass of ngg_prefill
  // One decode step (drafts, block forward, acceptance, commit) captured as a HIP graph: its kernels read the
  // context length from n_dev, so the same graph replays step after step (a replayed launch costs the GPU
  // 1.6-1.75 us against 2.4 us for a stream launch, measured on MI355X with chains of 320 small kernels).
  int32_t *n_dev = nullptr;        // [1] context length as the captured kernels see it
  int32_t n_dev_value = -1;        // what n_dev holds (-1: unknown)
  int32_t n_upload = 0;            // staging for the copy to n_dev
  int graph_mode = 2;              // ngg_step_graphs: 0 never, 1 whenever a step qualifies, 2 where it measures faster
  // mode 2: per step shape, three steps launched on the stream and three replayed are timed (host clock around the
  // step, which ends in a synchronisation either way); the faster way is kept until the shape changes
  int tune_key[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int tune_count = 0, tune_choice = -1;
  double tune_ms[2] = {0.0, 0.0};
  bool graph_broken = false;       // a capture or instantiation failed: stay with stream launches
  int32_t graph_captures = 0, graph_replays = 0;
  hipGraphExec_t step_graph = nullptr;
  hipStream_t cap_stream = nullptr;   // the step is recorded on a stream of the library's own (the caller's may be the default
                                      // stream, which cannot be captured) and replayed on the caller's
  int graph_key[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // k, w, k_ctx_max, q_min, q_max, attention slices, draft source, 1
  int eager_key[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // the same of the last step launched on the stream (its kernels are loaded)
  size_t part_rows = 0;            // rows (slices x block rows rounded to 128) the attention partial buffers hold per head
  // device buffers
  int32_t *hist = nullptr, *drafts = nullptr, *block_tok = nullptr, *res = nullptr, *next1 = nullptr;
  int32_t *mlist = nullptr, *reps = nullptr, *gtab = nullptr, *ctx_rows = nullptr, *n_ctx = nullptr;
  int gtab_slots = 0;              // slots of the matcher's grouping table: a power of two >= 2 * Spad
  int32_t *bg_table = nullptr, *bg_tok = nullptr;   // full-model bigram table [vocab][bg_K]; token ids of one build pass
  int bg_K = 0;
  bool bg_use = false;             // bigram rows from the table instead of the U.E[x] sweep
  int32_t *uni_top = nullptr;      // tokens by ascending unigram distance, uni_K of them
  int uni_K = 0;
  bool uni_use = false;            // model rows start with the unigram's tokens
  int8_t *row_src = nullptr;
  void *kcache = nullptr, *vcache = nullptr, *kscr = nullptr, *vscr = nullptr;
  float *h = nullptr, *hpart = nullptr, *part_o = nullptr, *part_ml = nullptr, *pmax_val = nullptr, *z = nullptr, *logits = nullptr;
  float *rope_cos = nullptr, *rope_sin = nullptr;
  float *row_ss = nullptr;         // [Mcap][kNormSegs] sums of squares of the rows the last RMSNorm wrote
  int *pmax_idx = nullptr, *cand_idx = nullptr;
  float *cand_val = nullptr;
  void *xn = nullptr, *q = nullptr, *attn = nullptr, *act = nullptr;
  // the library's own operand-order copies of every matrix it multiplies with
  void *wtiled = nullptr;          // one allocation
  struct LayerT { const void *wqkv, *wo, *wgu, *wdown; float s_qkv, s_o, s_gu, s_down; };   // s_*: power-of-two scale of the stored copy
  std::vector<LayerT> lt;
  const void *unemb_t = nullptr;
  float unemb_scale = 1.0f;        // the operand-order copy of the output embedding holds the stored values times this
  float emb_scale = 1.0f;          // rows of the input embedding are multiplied by this when they become a 16-bit operand
  int32_t *res_host = nullptr;     // pinned
  // host state
  std::vector<int32_t> tokens;     // committed history mirror
  int n = 0;                       // context length (0 = no prefill yet)
  bool have_verify = false;
  int last_k = 0, last_w = 0;
  int32_t attn_layout[4] = {0, 0, 0, 0};   // last forward: key-list slices per head, attention workgroups, block rows, cached positions
  bool drafts_on_device = false;
  int drafts_k = 0, drafts_w = 0;
  // row allocation between the strategies inside the library's decode loop (ngg_allocation)
  int alloc_mode = NGG_ALLOC_FIXED, alloc_coverage = 90, alloc_warmup = 8;
  int64_t ctx_rank_wins[32] = {};  // since the last prefill: calls won, with an accepted draft, by the r-th context row
  std::string err;
  // profiling
  int prof_mask = 0;               // bit i: record events around kernels of class i
  int prof_every = 1;              // ... around one launch in every prof_every of a class
  int64_t prof_seen[NGG_PROF_COUNT] = {};
  std::vector<ProfSpan> spans;
  std::vector<hipEvent_t> free_events;
};

namespace {

ngg_status fail(ngg_ctx *c, ngg_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  else g_create_error = buf;
  return st;
}

#define NGG_HIP(c, call)                                                                                  \
  do {                                                                                                    \
    hipError_t e_ = (call);                                                                               \
    if (e_ != hipSuccess) return fail((c), NGG_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));      \
  } while (0)

inline size_t rup(size_t x, size_t m) { return (x + m - 1) / m * m; }

struct ProfScope {
  ngg_ctx *c;
  ProfSpan sp{};
  bool on;
  ProfScope(ngg_ctx *ctx, int cls) : c(ctx), on(((ctx->prof_mask >> cls) & 1) != 0) {
    if (!on) return;
    if (c->prof_seen[cls]++ % c->prof_every != 0) { on = false; return; }
    sp.cls = cls;
    for (hipEvent_t *e : {&sp.e0, &sp.e1}) {
      if (!c->free_events.empty()) { *e = c->free_events.back(); c->free_events.pop_back(); }
      else if (hipEventCreate(e) != hipSuccess) { on = false; return; }
    }
    (void)hipEventRecord(sp.e0, c->stream);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(sp.e1, c->stream);
    c->spans.push_back(sp);
  }
};

template <typename P>
ngg_status dev_alloc(ngg_ctx *c, P **p, size_t bytes, bool zero) {
  void *v = nullptr;
  hipError_t e = hipMalloc(&v, bytes ? bytes : 16);
  if (e != hipSuccess) return fail(c, NGG_ENOMEM, "hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
  *p = (P *)v;
  if (zero) NGG_HIP(c, hipMemsetAsync(v, 0, bytes ? bytes : 16, c->stream));
  return NGG_OK;
}

// One forward over a block of R rows x C columns sitting at positions P .. P+C-1 on a cached
// context of P tokens (Section 3).  Leaves this block's keys/values in the scratch, and, when
// `unembed` is set, the per-tile argmax partials (and optional logits) of every block position.
ngg_status forward(ngg_ctx *c, int R, int C, int P, bool from_hist, int w, bool unembed, bool want_logits,
                   const int32_t *tok_src = nullptr,     // tok_src: from_hist reads its tokens here instead of the history
                   bool last_row_only = false,           // unembedding of the block's last token alone (it becomes row 0 of the partials)
                   bool kv_direct = false,               // a prefill piece at a tile boundary writes its keys/values straight into the cache
                   const int32_t *n_dev = nullptr) {     // the kernels take P = *n_dev - 1 (a captured step); P here still sets the launch shapes
  const ngg_model_desc &d = c->d;
  // a verify block keeps one copy of the column every row shares (the uncached last context token): 1 + R*w tokens
  const int shared0 = (!from_hist && C >= 2) ? 1 : 0;
  const int M = block_tokens(R, C, shared0);
  (void)w;
  const int dt = d.dtype;
  const int dq = d.n_heads * d.head_dim;
  hipStream_t s = c->stream;
  {
    ProfScope ps(c, NGG_PROF_OTHER);
    launch_embed(dt, c->w.tok_emb, tok_src ? tok_src : c->hist, c->drafts, c->block_tok, c->h, d.d_model, M,
                 tok_src ? 0 : P, from_hist ? 1 : (shared0 ? 0 : 2), s, n_dev);
  }
  const int n_splits = attention_splits(dt, d.head_dim, d.n_heads, M, P, c->max_splits);
  c->attn_layout[0] = n_splits; c->attn_layout[1] = attention_workgroups(dt, d.head_dim, d.n_heads, M, n_splits);
  c->attn_layout[2] = M; c->attn_layout[3] = P;
  const int Mpart = (M + 127) / 128 * 128;
  if ((size_t)n_splits * Mpart > c->part_rows)
    return fail(c, NGG_ECAPACITY, "attention partials: %d slices of %d rows exceed the %zu rows allocated", n_splits, Mpart, c->part_rows);
  const size_t part_stride = (size_t)c->Mcap * d.d_model;
  const int ks_o = gemm_residual_splits(dt, M, d.d_model, dq), ks_down = gemm_residual_splits(dt, M, d.d_model, d.d_ffn);
  const int ss_segs = rmsnorm_segments(d.d_model);
  int pending = 0;                                   // residual partials the next RMSNorm has to add
  for (int l = 0; l < d.n_layers; ++l) {
    const ngg_layer_weights &lw = c->layers[l];
    const size_t kv_layer = (size_t)l * d.n_kv_heads;
    char *kscr_l = (char *)c->kscr + kv_layer * c->Mcap * d.head_dim * c->esize;
    char *vscr_l = (char *)c->vscr + kv_layer * d.head_dim * c->Mcap * c->esize;
    int kv_rows = c->Mcap;
    if (kv_direct) {                                 // the block's tiles are the cache's tiles P / 32 ..
      kscr_l = (char *)c->kcache + (kv_layer * c->Spad + P) * d.head_dim * c->esize;
      vscr_l = (char *)c->vcache + (kv_layer * c->Spad + P) * d.head_dim * c->esize;
      kv_rows = c->Spad;
    }
    { ProfScope ps(c, NGG_PROF_NORM); launch_rmsnorm(dt, c->h, c->hpart, pending, part_stride, lw.attn_norm, c->xn, d.d_model, M, c->Mcap, c->row_ss, s); }
    {
      ProfScope ps(c, NGG_PROF_GEMM_QKV);
      GemmArgs g{};
      g.X = c->xn; g.W0 = c->lt[l].wqkv;
      g.M = M; g.N = dq + 2 * d.n_kv_heads * d.head_dim; g.K = d.d_model;
      g.q = c->q; g.kscr = kscr_l; g.vscr = vscr_l; g.kv_rows = kv_rows;
      g.H = d.n_heads; g.Hkv = d.n_kv_heads; g.hd = d.head_dim; g.Mcap = c->Mcap; g.C = C; g.P = P; g.shared0 = shared0;
      g.n_dev = n_dev;
      g.rope_cos = c->rope_cos; g.rope_sin = c->rope_sin;
      g.row_ss = c->row_ss; g.ss_segs = ss_segs; g.ss_eps = d.rms_eps;
      g.out_scale = 1.0f / c->lt[l].s_qkv;
      launch_gemm(dt, EPI_QKV, g, s);
    }
    {
      ProfScope ps(c, NGG_PROF_ATTENTION);
      AttnArgs a{};
      a.q = c->q;
      a.kcache = (char *)c->kcache + kv_layer * c->Spad * d.head_dim * c->esize;
      a.vcache = (char *)c->vcache + kv_layer * d.head_dim * c->Spad * c->esize;
      a.kscr = kscr_l; a.vscr = vscr_l; a.kv_rows = kv_rows;
      a.part_o = c->part_o; a.part_ml = c->part_ml; a.out = c->attn;
      a.H = d.n_heads; a.Hkv = d.n_kv_heads; a.Mcap = c->Mcap; a.Spad = c->Spad; a.M = M; a.C = C; a.P = P;
      a.n_splits = n_splits; a.shared0 = shared0; a.Mpart = Mpart; a.n_dev = n_dev;
      a.scale = 1.0f / std::sqrt((float)d.head_dim);
      launch_attention(dt, d.head_dim, a, s);
    }
    {
      ProfScope ps(c, NGG_PROF_GEMM_O);
      GemmArgs g{};
      g.X = c->attn; g.W0 = c->lt[l].wo; g.M = M; g.N = d.d_model; g.K = dq;
      g.hpart = c->hpart; g.KS = ks_o; g.Mcap = c->Mcap;
      g.out_scale = 1.0f / c->lt[l].s_o;
      launch_gemm(dt, EPI_RESIDUAL, g, s);
    }
    { ProfScope ps(c, NGG_PROF_NORM); launch_rmsnorm(dt, c->h, c->hpart, ks_o, part_stride, lw.mlp_norm, c->xn, d.d_model, M, c->Mcap, c->row_ss, s); }
    {
      ProfScope ps(c, NGG_PROF_GEMM_GATEUP);
      GemmArgs g{};
      g.X = c->xn; g.W0 = c->lt[l].wgu; g.M = M; g.N = d.d_ffn; g.K = d.d_model;
      g.act = c->act; g.Mcap = c->Mcap;
      g.row_ss = c->row_ss; g.ss_segs = ss_segs; g.ss_eps = d.rms_eps;
      g.out_scale = 1.0f / c->lt[l].s_gu;
      launch_gemm(dt, EPI_GATEUP, g, s);
    }
    {
      ProfScope ps(c, NGG_PROF_GEMM_DOWN);
      GemmArgs g{};
      g.X = c->act; g.W0 = c->lt[l].wdown; g.M = M; g.N = d.d_model; g.K = d.d_ffn;
      g.hpart = c->hpart; g.KS = ks_down; g.Mcap = c->Mcap;
      g.out_scale = 1.0f / c->lt[l].s_down;
      launch_gemm(dt, EPI_RESIDUAL, g, s);
    }
    pending = ks_down;
  }
  if (unembed) {
    { ProfScope ps(c, NGG_PROF_NORM); launch_rmsnorm(dt, c->h, c->hpart, pending, part_stride, c->w.final_norm, c->xn, d.d_model, M, c->Mcap, c->row_ss, s); }
    ProfScope ps(c, NGG_PROF_GEMM_UNEMBED);
    GemmArgs g{};
    g.X = c->xn; g.W0 = c->unemb_t; g.M = M; g.N = d.vocab; g.K = d.d_model;
    g.logits = want_logits ? c->logits : nullptr;
    g.pmax_val = c->pmax_val; g.pmax_idx = c->pmax_idx; g.Mcap = c->Mcap;
    g.row_ss = c->row_ss; g.ss_segs = ss_segs; g.ss_eps = d.rms_eps;
    if (last_row_only) {                               // rows of the activation layout lie one chunk row apart in every chunk
      const int kc = dt == 1 ? KChunk<half_t>::value : KChunk<float>::value;
      g.X = (const char *)c->xn + (size_t)(M - 1) * kc * c->esize;
      g.row_ss = c->row_ss + (size_t)(M - 1) * kNormSegs;
      g.M = 1;
    }
    g.out_scale = 1.0f / c->unemb_scale;
    launch_gemm(dt, EPI_UNEMBED, g, s);
  }
  NGG_HIP(c, hipGetLastError());
  return NGG_OK;
}

ngg_status ensure_logits(ngg_ctx *c) {
  if (c->logits) return NGG_OK;
  return dev_alloc(c, &c->logits, (size_t)c->Mcap * c->d.vocab * sizeof(float), false);
}

ngg_status build_next1(ngg_ctx *c) {
  // next1[x] = argmax_v <unemb[v], tok_emb[x]>: the unembedding GEMM applied to rows of the input
  // embedding (no normalisation), 256 vocabulary entries per pass over the output embedding (16-bit models: one
  // pass of the wide kernel; with 64 per pass a 128K vocabulary cost 2004 sweeps of 788 MB) or 64 (fp32).
  const ngg_model_desc &d = c->d;
  const int rows = d.dtype == NGG_BF16 ? 256 : 64;       // Mcap >= 256
  for (int x0 = 0; x0 < d.vocab; x0 += rows) {
    const int M = std::min(rows, d.vocab - x0);
    launch_pack_rows(d.dtype, (const char *)c->w.tok_emb + (size_t)x0 * d.d_model * c->esize, c->xn, d.d_model, M, c->Mcap,
                     c->stream, c->emb_scale);
    GemmArgs g{};
    g.X = c->xn;
    g.W0 = c->unemb_t; g.M = M; g.N = d.vocab; g.K = d.d_model;
    g.pmax_val = c->pmax_val; g.pmax_idx = c->pmax_idx; g.Mcap = c->Mcap;
    g.out_scale = 1.0f / (c->unemb_scale * c->emb_scale);
    launch_gemm(d.dtype, EPI_UNEMBED, g, c->stream);
    launch_next1_finish(c->pmax_val, c->pmax_idx, c->unembed_tiles, c->Mcap, M, c->next1 + x0, c->stream);
  }
  NGG_HIP(c, hipGetLastError());
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  return NGG_OK;
}

// Power of two that brings a matrix whose largest magnitude is `amax` to [2^13, 2^14) (fp16 holds up to
// 65504): the 16-bit copy then keeps every bit of a bf16 value down to 2^-31 of the maximum.
float operand_scale(int dtype, float amax) {
  if (dtype != NGG_BF16 || !(amax > 0.0f) || !std::isfinite(amax)) return 1.0f;
  int e = 0;
  (void)std::frexp(amax, &e);                              // amax = m * 2^e, 0.5 <= m < 1
  return std::ldexp(1.0f, 14 - e);
}

// Copies every matrix the step multiplies with into operand order (one-off, at create); 16-bit models:
// scaled by a power of two per matrix (q, k, v share one, gate and up share one) and rounded to fp16.
ngg_status tile_all_weights(ngg_ctx *c) {
  const ngg_model_desc &d = c->d;
  const size_t dq = (size_t)d.n_heads * d.head_dim, dkv = (size_t)d.n_kv_heads * d.head_dim;
  const size_t e_qkv = (dq + 2 * dkv) * d.d_model, e_o = (size_t)d.d_model * dq, e_gu = (size_t)2 * d.d_ffn * d.d_model,
               e_down = (size_t)d.d_model * d.d_ffn, e_layer = e_qkv + e_o + e_gu + e_down;
  const size_t total = e_layer * d.n_layers + (size_t)d.vocab * d.d_model;
  ngg_status st = dev_alloc(c, &c->wtiled, total * c->esize, false);
  if (st != NGG_OK) return st;
  // largest magnitude per stored copy: 4 per layer, then the output and the input embedding
  const int n_max = 4 * d.n_layers + 2;
  unsigned *amax_dev = nullptr;
  st = dev_alloc(c, &amax_dev, (size_t)n_max * sizeof(unsigned), true);
  if (st != NGG_OK) return st;
  std::vector<unsigned> amax_bits((size_t)n_max, 0u);
  if (d.dtype == NGG_BF16) {
    for (int l = 0; l < d.n_layers; ++l) {
      const ngg_layer_weights &lw = c->layers[l];
      unsigned *a = amax_dev + 4 * l;
      launch_absmax(d.dtype, lw.wq, dq * d.d_model, a + 0, c->stream);
      launch_absmax(d.dtype, lw.wk, dkv * d.d_model, a + 0, c->stream);
      launch_absmax(d.dtype, lw.wv, dkv * d.d_model, a + 0, c->stream);
      launch_absmax(d.dtype, lw.wo, e_o, a + 1, c->stream);
      launch_absmax(d.dtype, lw.w_gate, e_gu / 2, a + 2, c->stream);
      launch_absmax(d.dtype, lw.w_up, e_gu / 2, a + 2, c->stream);
      launch_absmax(d.dtype, lw.w_down, e_down, a + 3, c->stream);
    }
    launch_absmax(d.dtype, c->w.unemb, (size_t)d.vocab * d.d_model, amax_dev + 4 * d.n_layers, c->stream);
    launch_absmax(d.dtype, c->w.tok_emb, (size_t)d.vocab * d.d_model, amax_dev + 4 * d.n_layers + 1, c->stream);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(amax_bits.data(), amax_dev, (size_t)n_max * sizeof(unsigned), hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) { (void)hipFree(amax_dev); return fail(c, NGG_EHIP, "ngg_create: weight range scan failed: %s", hipGetErrorString(e)); }
  }
  (void)hipFree(amax_dev);
  auto scale_of = [&](int i) {
    float amax;
    memcpy(&amax, &amax_bits[(size_t)i], sizeof amax);
    return operand_scale(d.dtype, amax);
  };
  char *base = (char *)c->wtiled;
  c->lt.resize(d.n_layers);
  for (int l = 0; l < d.n_layers; ++l) {
    const ngg_layer_weights &lw = c->layers[l];
    char *p = base + (size_t)l * e_layer * c->esize;
    char *qkv = p, *o = qkv + e_qkv * c->esize, *gu = o + e_o * c->esize, *down = gu + e_gu * c->esize;
    const float s_qkv = scale_of(4 * l), s_o = scale_of(4 * l + 1), s_gu = scale_of(4 * l + 2), s_down = scale_of(4 * l + 3);
    // q, k, v: every 16-row fragment holds 8 pairs (i, i + hd/2) of one head; gate/up: gate and up of 8 features
    launch_tile_weights(d.dtype, lw.wq, qkv, (int)dq, d.d_model, 0, c->stream, s_qkv, 1, d.head_dim / 2);
    launch_tile_weights(d.dtype, lw.wk, qkv, (int)dkv, d.d_model, (int)dq, c->stream, s_qkv, 1, d.head_dim / 2);
    launch_tile_weights(d.dtype, lw.wv, qkv, (int)dkv, d.d_model, (int)(dq + dkv), c->stream, s_qkv, 1, d.head_dim / 2);
    launch_tile_weights(d.dtype, lw.wo, o, d.d_model, (int)dq, 0, c->stream, s_o);
    launch_tile_weights(d.dtype, lw.w_gate, gu, d.d_ffn, d.d_model, 0, c->stream, s_gu, 2);
    launch_tile_weights(d.dtype, lw.w_up, gu, d.d_ffn, d.d_model, 0, c->stream, s_gu, 3);
    launch_tile_weights(d.dtype, lw.w_down, down, d.d_model, d.d_ffn, 0, c->stream, s_down);
    c->lt[l] = {qkv, o, gu, down, s_qkv, s_o, s_gu, s_down};
  }
  char *ue = base + e_layer * d.n_layers * c->esize;
  c->unemb_scale = scale_of(4 * d.n_layers);
  c->emb_scale = scale_of(4 * d.n_layers + 1);
  launch_tile_weights(d.dtype, c->w.unemb, ue, d.vocab, d.d_model, 0, c->stream, c->unemb_scale);
  c->unemb_t = ue;
  NGG_HIP(c, hipGetLastError());
  return NGG_OK;
}

double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace

extern "C" {

const char *ngg_last_error(const ngg_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

ngg_status ngg_destroy(ngg_ctx *c) {
  if (!c) return NGG_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  void *bufs[] = {c->hist, c->drafts, c->block_tok, c->res, c->next1, c->mlist, c->reps, c->gtab, c->ctx_rows, c->n_ctx,
                  c->row_src, c->hpart, c->wtiled, c->cand_val, c->cand_idx, c->kcache, c->vcache, c->kscr, c->vscr, c->h, c->part_o, c->part_ml, c->pmax_val, c->z,
                  c->logits, c->rope_cos, c->rope_sin, c->pmax_idx, c->xn, c->q, c->attn, c->act, c->bg_table, c->bg_tok, c->uni_top, c->row_ss, c->n_dev};
  for (void *b : bufs)
    if (b) (void)hipFree(b);
  if (c->step_graph) (void)hipGraphExecDestroy(c->step_graph);
  if (c->cap_stream) (void)hipStreamDestroy(c->cap_stream);
  if (c->res_host) (void)hipHostFree(c->res_host);
  for (auto &sp : c->spans) { (void)hipEventDestroy(sp.e0); (void)hipEventDestroy(sp.e1); }
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  delete c;
  return NGG_OK;
}

ngg_status ngg_create(const ngg_model_desc *desc, const ngg_weights *weights, void *hip_stream, ngg_ctx **out) {
  if (!desc || !weights || !out) return fail(nullptr, NGG_EINVAL, "ngg_create: null argument");
  *out = nullptr;
  const ngg_model_desc &d = *desc;
  if (d.dtype != NGG_F32 && d.dtype != NGG_BF16) return fail(nullptr, NGG_EINVAL, "ngg_create: dtype must be NGG_F32 or NGG_BF16");
  if (d.n_layers < 1 || d.d_model < 32 || d.n_heads < 1 || d.n_kv_heads < 1 || d.d_ffn < 32 || d.vocab < 16)
    return fail(nullptr, NGG_EINVAL, "ngg_create: non-positive model dimension");
  if (d.head_dim != 32 && d.head_dim != 64 && d.head_dim != 128)
    return fail(nullptr, NGG_EINVAL, "ngg_create: head_dim %d not in {32, 64, 128}", d.head_dim);
  if (d.d_model % 32 || d.d_ffn % 32 || (d.n_heads * d.head_dim) % 32)
    return fail(nullptr, NGG_EINVAL, "ngg_create: d_model, d_ffn and n_heads*head_dim must be multiples of 32");
  if (d.d_model > 16384 || d.d_ffn > 65536)
    return fail(nullptr, NGG_EINVAL, "ngg_create: d_model %d / d_ffn %d beyond the supported 16384 / 65536", d.d_model, d.d_ffn);
  if (d.vocab % 32) return fail(nullptr, NGG_EINVAL, "ngg_create: vocab must be a multiple of 32");
  if (d.n_heads % d.n_kv_heads) return fail(nullptr, NGG_EINVAL, "ngg_create: n_heads must be a multiple of n_kv_heads");
  if (d.max_k < 1 || d.max_k > 32 || d.max_w < 0 || d.max_w > 32)
    return fail(nullptr, NGG_EINVAL, "ngg_create: need 1 <= max_k <= 32 and 0 <= max_w <= 32");
  if (d.max_seq < 2) return fail(nullptr, NGG_EINVAL, "ngg_create: max_seq must be at least 2");
  if (!(d.rms_eps >= 0.0f) || !(d.rope_theta > 0.0f)) return fail(nullptr, NGG_EINVAL, "ngg_create: bad rms_eps / rope_theta");
  if (!weights->tok_emb || !weights->unemb || !weights->final_norm || !weights->layers)
    return fail(nullptr, NGG_EINVAL, "ngg_create: null weight pointer");
  for (int l = 0; l < d.n_layers; ++l) {
    const ngg_layer_weights &lw = weights->layers[l];
    if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.mlp_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
      return fail(nullptr, NGG_EINVAL, "ngg_create: null weight pointer in layer %d", l);
  }

  ngg_ctx *c = new (std::nothrow) ngg_ctx;
  if (!c) return fail(nullptr, NGG_ENOMEM, "ngg_create: out of host memory");
  c->d = d;
  c->w = *weights;
  c->layers.assign(weights->layers, weights->layers + d.n_layers);
  c->w.layers = c->layers.data();
  c->stream = (hipStream_t)hip_stream;
  c->esize = d.dtype == NGG_BF16 ? 2 : 4;
  c->Spad = (int)rup((size_t)d.max_seq + 1, 32);
  // whole GEMM row tiles: 64 rows, or 128-row tiles once a block has more than 64 rows
  c->prefill_chunk = d.dtype == NGG_BF16 ? std::min(kPrefillChunk16, (int)rup((size_t)d.max_seq, 256)) : kPrefillChunk32;
  c->Mcap = (int)rup((size_t)std::max(d.max_k * (d.max_w + 1), c->prefill_chunk), 64);
  if (c->Mcap > 64) c->Mcap = (int)rup((size_t)c->Mcap, 128);
  c->max_splits = 32;
  c->unembed_tiles = d.vocab / 32;

  const size_t kv_elems = (size_t)d.n_layers * d.n_kv_heads * d.head_dim;
  const int dq = d.n_heads * d.head_dim;
  ngg_status st = NGG_OK;
#define TRY(x) do { if (st == NGG_OK) st = (x); } while (0)
  TRY(dev_alloc(c, &c->hist, (size_t)c->Spad * 4, true));
  TRY(dev_alloc(c, &c->drafts, (size_t)d.max_k * std::max(1, d.max_w) * 4, true));
  TRY(dev_alloc(c, &c->block_tok, (size_t)c->Mcap * 4, true));
  TRY(dev_alloc(c, &c->res, (size_t)(res_greedy_off(d.max_k) + c->Mcap) * 4, true));
  TRY(dev_alloc(c, &c->next1, (size_t)d.vocab * 4, true));
  TRY(dev_alloc(c, &c->mlist, (size_t)c->Spad * 4, true));
  TRY(dev_alloc(c, &c->reps, (size_t)c->Spad * 8, true));
  c->gtab_slots = 128;
  while (c->gtab_slots < 2 * c->Spad) c->gtab_slots <<= 1;
  TRY(dev_alloc(c, &c->gtab, (size_t)3 * c->gtab_slots * 4, true));
  TRY(dev_alloc(c, &c->ctx_rows, (size_t)d.max_k * std::max(1, d.max_w) * 4, true));
  TRY(dev_alloc(c, &c->n_ctx, 16, true));
  TRY(dev_alloc(c, &c->row_src, (size_t)d.max_k, true));
  TRY(dev_alloc(c, &c->kcache, kv_elems * c->Spad * c->esize, true));
  TRY(dev_alloc(c, &c->vcache, kv_elems * c->Spad * c->esize, true));
  TRY(dev_alloc(c, &c->kscr, kv_elems * c->Mcap * c->esize, true));
  TRY(dev_alloc(c, &c->vscr, kv_elems * c->Mcap * c->esize, true));
  TRY(dev_alloc(c, &c->h, (size_t)c->Mcap * d.d_model * 4, true));
  TRY(dev_alloc(c, &c->n_dev, 16, true));
  // (+ 16 rows: the unembedding of a piece's last token alone starts its row tile at that row)
  TRY(dev_alloc(c, &c->row_ss, (size_t)(c->Mcap + 16) * kNormSegs * 4, true));
  TRY(dev_alloc(c, &c->hpart, (size_t)kMaxResidualSplits * c->Mcap * d.d_model * 4, true));
  TRY(dev_alloc(c, &c->xn, act_elems(d.dtype, c->Mcap, d.d_model) * c->esize, true));
  TRY(dev_alloc(c, &c->q, (size_t)c->Mcap * dq * c->esize, true));
  TRY(dev_alloc(c, &c->attn, act_elems(d.dtype, c->Mcap, dq) * c->esize, true));
  TRY(dev_alloc(c, &c->act, act_elems(d.dtype, c->Mcap, d.d_ffn) * c->esize, true));
  // attention partials, [head][slice][rows]: slices x rows is at most 32 x 128 for blocks of up to 64 tokens, and
  // (two workgroups per CU) x 128 rows per workgroup, shared among the heads, above that (attention_splits)
  c->part_rows = std::max({(size_t)(c->Mcap + 127) / 128 * 128, (size_t)65536 / d.n_heads + 128, (size_t)(c->max_splits + 1) * 128});
  TRY(dev_alloc(c, &c->part_o, (size_t)d.n_heads * c->part_rows * d.head_dim * 4, true));
  TRY(dev_alloc(c, &c->part_ml, (size_t)d.n_heads * c->part_rows * 2 * 4, true));
  TRY(dev_alloc(c, &c->pmax_val, (size_t)c->unembed_tiles * c->Mcap * 4, true));
  TRY(dev_alloc(c, &c->pmax_idx, (size_t)c->unembed_tiles * c->Mcap * 4, true));
  TRY(dev_alloc(c, &c->z, (size_t)d.vocab * 4, true));
  TRY(dev_alloc(c, &c->cand_val, (size_t)256 * 32 * 4, true));
  TRY(dev_alloc(c, &c->cand_idx, (size_t)256 * 32 * 4, true));
  const int half = d.head_dim / 2;
  TRY(dev_alloc(c, &c->rope_cos, (size_t)c->Spad * half * 4, false));
  TRY(dev_alloc(c, &c->rope_sin, (size_t)c->Spad * half * 4, false));
#undef TRY
  if (st == NGG_OK && hipHostMalloc((void **)&c->res_host, (size_t)(res_greedy_off(d.max_k) + c->Mcap) * 4) != hipSuccess)
    st = fail(c, NGG_ENOMEM, "ngg_create: hipHostMalloc failed");
  if (st == NGG_OK) {
    // rotary table in double on the host: angle = pos * theta^(-2i/head_dim)
    std::vector<float> cs((size_t)c->Spad * half), sn((size_t)c->Spad * half);
    for (int i = 0; i < half; ++i) {
      const double inv = std::pow((double)d.rope_theta, -2.0 * i / d.head_dim);
      for (int p = 0; p < c->Spad; ++p) {
        cs[(size_t)p * half + i] = (float)std::cos(p * inv);
        sn[(size_t)p * half + i] = (float)std::sin(p * inv);
      }
    }
    hipError_t e = hipMemcpy(c->rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) st = fail(c, NGG_EHIP, "ngg_create: rotary table upload failed: %s", hipGetErrorString(e));
  }
  if (st == NGG_OK) st = tile_all_weights(c);
  if (st == NGG_OK) st = build_next1(c);
  if (st != NGG_OK) {
    g_create_error = c->err;
    ngg_destroy(c);
    return st;
  }
  c->tokens.reserve(d.max_seq);
  *out = c;
  return NGG_OK;
}

ngg_status ngg_prefill(ngg_ctx *c, const int32_t *prompt, int32_t n_prompt) {
  if (!c) return NGG_EINVAL;
  if (!prompt || n_prompt < 1) return fail(c, NGG_EINVAL, "ngg_prefill: need a prompt of at least one token");
  if (n_prompt + 1 > c->d.max_seq) return fail(c, NGG_ECAPACITY, "ngg_prefill: prompt of %d tokens exceeds max_seq %d", n_prompt, c->d.max_seq);
  for (int i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->d.vocab) return fail(c, NGG_EINVAL, "ngg_prefill: token %d at %d out of range", prompt[i], i);
  c->n = 0;
  c->have_verify = false;
  c->drafts_on_device = false;
  for (auto &r : c->ctx_rank_wins) r = 0;
  c->tokens.assign(prompt, prompt + n_prompt);
  NGG_HIP(c, hipMemcpyAsync(c->hist, prompt, (size_t)n_prompt * 4, hipMemcpyHostToDevice, c->stream));
  const ngg_model_desc &d = c->d;
  for (int p0 = 0; p0 < n_prompt; p0 += c->prefill_chunk) {
    const int C = std::min(c->prefill_chunk, n_prompt - p0);
    const bool last = p0 + C == n_prompt;
    // pieces start at multiples of 256 positions: their key/value tiles are cache tiles, written in place (no commit copy)
    ngg_status st = forward(c, 1, C, p0, true, 0, last, false, nullptr, true, true);   // the last piece predicts the first new token
    if (st != NGG_OK) return st;
    ProfScope ps(c, NGG_PROF_ACCEPT_COMMIT);
    if (last)
      launch_argmax_accept(c->pmax_val, c->pmax_idx, c->unembed_tiles, c->Mcap, 1, 0, 1, 0, nullptr, nullptr, nullptr, c->res,
                           res_greedy_off(d.max_k), c->stream);

  }
  // first generated token = greedy prediction after the last prompt token
  int32_t first = 0;
  NGG_HIP(c, hipMemcpyAsync(&first, c->res + res_greedy_off(d.max_k), 4, hipMemcpyDeviceToHost, c->stream));
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  NGG_HIP(c, hipMemcpyAsync(c->hist + n_prompt, &first, 4, hipMemcpyHostToDevice, c->stream));
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  c->tokens.push_back(first);
  c->n = n_prompt + 1;
  return NGG_OK;
}

// the draft kernels of one step (n_dev: they take the context length from the device)
static void queue_drafts(ngg_ctx *c, const ngg_draft_cfg *cfg, const int32_t *n_dev) {
  DraftArgs a{};
  a.hist = c->hist; a.n = c->n; a.n_dev = n_dev; a.k = cfg->k; a.w = cfg->w; a.k_ctx_max = cfg->k_ctx_max; a.q_min = cfg->q_min; a.q_max = cfg->q_max;
  a.mlist = c->mlist; a.reps = c->reps; a.gtab = c->gtab; a.gtab_slots = c->gtab_slots; a.ctx_rows = c->ctx_rows; a.n_ctx = c->n_ctx;
  a.tok_emb = c->w.tok_emb; a.emb_scale = c->emb_scale; a.unemb_t = c->unemb_t; a.unemb_scale = c->unemb_scale; a.d = c->d.d_model; a.vocab = c->d.vocab; a.z = c->z; a.cand_val = c->cand_val; a.cand_idx = c->cand_idx; a.next1 = c->next1;
  a.drafts = c->drafts; a.row_src = c->row_src;
  if (c->bg_use) { a.bg_table = c->bg_table; a.bg_K = c->bg_K; }
  if (c->uni_use) a.uni_top = c->uni_top;
  launch_build_drafts(c->d.dtype, a, c->stream);
}

ngg_status ngg_build_drafts(ngg_ctx *c, const ngg_draft_cfg *cfg, int32_t *drafts, int8_t *row_src, int32_t *n_ctx_rows) {
  if (!c) return NGG_EINVAL;
  if (!cfg) return fail(c, NGG_EINVAL, "ngg_build_drafts: null cfg");
  if (c->n < 1) return fail(c, NGG_ESTATE, "ngg_build_drafts: no context (call ngg_prefill first)");
  if (cfg->k < 1 || cfg->w < 0) return fail(c, NGG_EINVAL, "ngg_build_drafts: need k >= 1 and w >= 0");
  if (cfg->k > c->d.max_k || cfg->w > c->d.max_w) return fail(c, NGG_ECAPACITY, "ngg_build_drafts: k=%d w=%d exceed max_k=%d max_w=%d", cfg->k, cfg->w, c->d.max_k, c->d.max_w);
  if (cfg->k_ctx_max < 0 || cfg->q_min < 1 || cfg->q_max < cfg->q_min || cfg->q_max > 64)
    return fail(c, NGG_EINVAL, "ngg_build_drafts: need k_ctx_max >= 0 and 1 <= q_min <= q_max <= 64");
  if (cfg->k > c->d.vocab) return fail(c, NGG_EINVAL, "ngg_build_drafts: k exceeds the vocabulary");
  if (c->bg_use && cfg->k > c->bg_K) return fail(c, NGG_ECAPACITY, "ngg_build_drafts: k=%d exceeds the %d ranks kept in the bigram table", cfg->k, c->bg_K);
  if (c->uni_use && cfg->k > c->uni_K) return fail(c, NGG_ECAPACITY, "ngg_build_drafts: k=%d exceeds the %d unigram tokens kept", cfg->k, c->uni_K);
  {
    ProfScope ps(c, NGG_PROF_DRAFTS);
    queue_drafts(c, cfg, nullptr);
  }
  NGG_HIP(c, hipGetLastError());
  c->drafts_on_device = true;
  c->drafts_k = cfg->k;
  c->drafts_w = cfg->w;
  if (drafts || row_src || n_ctx_rows) {
    if (drafts && cfg->w > 0) NGG_HIP(c, hipMemcpyAsync(drafts, c->drafts, (size_t)cfg->k * cfg->w * 4, hipMemcpyDeviceToHost, c->stream));
    if (row_src) NGG_HIP(c, hipMemcpyAsync(row_src, c->row_src, (size_t)cfg->k, hipMemcpyDeviceToHost, c->stream));
    if (n_ctx_rows) NGG_HIP(c, hipMemcpyAsync(n_ctx_rows, c->n_ctx, 4, hipMemcpyDeviceToHost, c->stream));
    NGG_HIP(c, hipStreamSynchronize(c->stream));
  }
  return NGG_OK;
}

ngg_status ngg_verify_step(ngg_ctx *c, const int32_t *drafts, int32_t k, int32_t w, ngg_verify_out *out) {
  if (!c) return NGG_EINVAL;
  if (!out) return fail(c, NGG_EINVAL, "ngg_verify_step: null out");
  if (c->n < 1) return fail(c, NGG_ESTATE, "ngg_verify_step: no context (call ngg_prefill first)");
  if (k < 1 || w < 0) return fail(c, NGG_EINVAL, "ngg_verify_step: need k >= 1 and w >= 0");
  if (k > c->d.max_k || w > c->d.max_w) return fail(c, NGG_ECAPACITY, "ngg_verify_step: k=%d w=%d exceed max_k=%d max_w=%d", k, w, c->d.max_k, c->d.max_w);
  if (c->n + w > c->d.max_seq) return fail(c, NGG_ECAPACITY, "ngg_verify_step: n=%d + w=%d exceeds max_seq=%d", c->n, w, c->d.max_seq);
  const ngg_model_desc &d = c->d;
  if (drafts) {
    for (int i = 0; i < k * w; ++i)
      if (drafts[i] < 0 || drafts[i] >= d.vocab) return fail(c, NGG_EINVAL, "ngg_verify_step: draft token %d out of range", drafts[i]);
    if (w > 0) NGG_HIP(c, hipMemcpyAsync(c->drafts, drafts, (size_t)k * w * 4, hipMemcpyHostToDevice, c->stream));
    c->drafts_on_device = true;
    c->drafts_k = k;
    c->drafts_w = w;
  } else if (w > 0 && (!c->drafts_on_device || c->drafts_k != k || c->drafts_w != w)) {
    return fail(c, NGG_ESTATE, "ngg_verify_step: no device drafts of shape (%d, %d); call ngg_build_drafts or pass drafts", k, w);
  }
  if (out->logits) { ngg_status st = ensure_logits(c); if (st != NGG_OK) return st; }
  const int C = w + 1, M = k * C;                       // M: entries of the (k, w+1) grid the caller sees
  const int shared0 = C >= 2 ? 1 : 0;                  // the block itself holds 1 + k*w tokens (forward)
  ngg_status st = forward(c, k, C, c->n - 1, false, w, true, out->logits != nullptr);
  if (st != NGG_OK) return st;
  const int goff = res_greedy_off(d.max_k);
  {
    ProfScope ps(c, NGG_PROF_ACCEPT_COMMIT);
    launch_argmax_accept(c->pmax_val, c->pmax_idx, c->unembed_tiles, c->Mcap, k, k, C, shared0, c->drafts, c->row_src, c->n_ctx,
                         c->res, goff, c->stream);
  }
  NGG_HIP(c, hipGetLastError());
  NGG_HIP(c, hipMemcpyAsync(c->res_host, c->res, (size_t)(goff + M) * 4, hipMemcpyDeviceToHost, c->stream));
  if (out->logits) {
    // device logits are per block token; the caller's [k][w+1][vocab] grid repeats the shared column in every row
    const size_t row = (size_t)d.vocab * 4;
    for (int r = 0; r < k; ++r) {
      char *dst = (char *)out->logits + (size_t)r * C * row;
      NGG_HIP(c, hipMemcpyAsync(dst, c->logits + (size_t)block_index(r, 0, C, shared0) * d.vocab, row, hipMemcpyDeviceToHost, c->stream));
      if (w > 0)
        NGG_HIP(c, hipMemcpyAsync(dst + row, c->logits + (size_t)block_index(r, 1, C, shared0) * d.vocab, (size_t)w * row,
                                  hipMemcpyDeviceToHost, c->stream));
    }
  }
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  out->k = k; out->w = w;
  out->winner = c->res_host[RES_WINNER];
  out->n_accept = c->res_host[RES_NACCEPT];
  out->n_new = c->res_host[RES_NNEW];
  if (out->greedy) memcpy(out->greedy, c->res_host + goff, (size_t)M * 4);
  if (out->accept_len) memcpy(out->accept_len, c->res_host + RES_ACCEPT, (size_t)k * 4);
  if (out->new_tokens) memcpy(out->new_tokens, c->res_host + RES_NEWTOK, (size_t)out->n_new * 4);
  c->have_verify = true;
  c->last_k = k;
  c->last_w = w;
  return NGG_OK;
}

ngg_status ngg_commit(ngg_ctx *c, int32_t max_new, int32_t *n_committed) {
  if (!c) return NGG_EINVAL;
  if (max_new <= 0) return fail(c, NGG_EINVAL, "ngg_commit: max_new must be positive");
  if (!c->have_verify) return fail(c, NGG_ESTATE, "ngg_commit: no verify call to commit");
  const ngg_model_desc &d = c->d;
  if (c->n >= d.max_seq) return fail(c, NGG_ECAPACITY, "ngg_commit: the context is full (n = max_seq = %d)", d.max_seq);
  max_new = std::min(max_new, d.max_seq - c->n);       // a fully accepted block at n + w == max_seq loses its last token
  const int n_new = std::min(c->res_host[RES_NNEW], max_new);
  {
    ProfScope ps(c, NGG_PROF_ACCEPT_COMMIT);
    launch_commit(d.dtype, c->kcache, c->vcache, c->kscr, c->vscr, d.n_layers, d.n_kv_heads, d.head_dim, c->Spad, c->Mcap,
                  c->last_w + 1, c->last_w >= 1 ? 1 : 0, c->n - 1, c->res, 0, 0, max_new, c->hist, c->stream);
  }
  NGG_HIP(c, hipGetLastError());
  for (int i = 0; i < n_new; ++i) c->tokens.push_back(c->res_host[RES_NEWTOK + i]);
  c->n += n_new;
  c->have_verify = false;
  c->drafts_on_device = false;
  if (n_committed) *n_committed = n_new;
  return NGG_OK;
}

// Rows the context strategy may take in the next call.  Fixed: the configured cap.  Adaptive (the ablation of
// Section 5.2 finds the context strategy's wins concentrated in its first rows, with diminishing returns from
// more, while it is often handed the whole batch): the smallest number of leading context rows that held
// `coverage` percent of the context strategy's wins so far, once `warmup` such wins were seen; the rows
// this frees go to the bigram.  Integer arithmetic only: the oracle takes the same decision.
static int context_row_cap(const ngg_ctx *c, int configured) {
  if (c->alloc_mode != NGG_ALLOC_ADAPTIVE) return configured;
  int64_t total = 0;
  for (int64_t r : c->ctx_rank_wins) total += r;
  if (total < c->alloc_warmup) return configured;
  int64_t seen = 0;
  int cap = 32;
  for (int r = 0; r < 32; ++r) {
    seen += c->ctx_rank_wins[r];
    if (100 * seen >= (int64_t)c->alloc_coverage * total) { cap = r + 1; break; }
  }
  return std::min(configured, std::max(1, cap));
}

constexpr double kGraphLaunchMs = 0.006;   // per kernel launch; steps slower than this are never captured in mode 2

// What fixes the launch shapes and constant arguments of a decode step: a captured step is replayed only while
// these stay the same (the number of attention slices moves with the context length)
static void step_key(const ngg_ctx *c, const ngg_draft_cfg &s, int key[8]) {
  const ngg_model_desc &d = c->d;
  const int C = s.w + 1, M = block_tokens(s.k, C, C >= 2 ? 1 : 0);
  key[0] = s.k; key[1] = s.w; key[2] = s.k_ctx_max; key[3] = s.q_min; key[4] = s.q_max;
  key[5] = attention_splits(d.dtype, d.head_dim, d.n_heads, M, c->n - 1, c->max_splits);
  key[6] = (c->bg_use ? 1 : 0) | (c->uni_use ? 2 : 0);
  key[7] = 1;
}

// One decode step as a graph replay: the kernels of ngg_build_drafts, ngg_verify_step (without logits) and
// ngg_commit, in the same shapes and order, with the context length read from n_dev, which the last node advances.
// Returns NGG_OK with *done = false when the step has to be launched on the stream instead (capture failed).
static ngg_status graph_step(ngg_ctx *c, const ngg_draft_cfg &step, const int key[8], ngg_verify_out &vo, int32_t *n_new_out,
                             bool *done) {
  *done = false;
  const ngg_model_desc &d = c->d;
  const int k = step.k, w = step.w, C = w + 1, shared0 = C >= 2 ? 1 : 0, M = k * C, goff = res_greedy_off(d.max_k);
  if (!c->step_graph || memcmp(key, c->graph_key, sizeof c->graph_key) != 0) {
    if (c->step_graph) { (void)hipGraphExecDestroy(c->step_graph); c->step_graph = nullptr; }
    if (!c->cap_stream && hipStreamCreateWithFlags(&c->cap_stream, hipStreamNonBlocking) != hipSuccess) {
      (void)hipGetLastError(); c->cap_stream = nullptr; c->graph_broken = true; return NGG_OK;
    }
    hipError_t eb = hipStreamBeginCapture(c->cap_stream, hipStreamCaptureModeThreadLocal);
    if (eb != hipSuccess) {
      c->err = std::string("step graph not captured: ") + hipGetErrorString(eb);
      (void)hipGetLastError(); c->graph_broken = true; return NGG_OK;
    }
    hipStream_t callers = c->stream;
    c->stream = c->cap_stream;                           // everything below is recorded, not run
    queue_drafts(c, &step, c->n_dev);
    const ngg_status st = forward(c, k, C, c->n - 1, false, w, true, false, nullptr, false, false, c->n_dev);
    if (st == NGG_OK) {
      launch_argmax_accept(c->pmax_val, c->pmax_idx, c->unembed_tiles, c->Mcap, k, k, C, shared0, c->drafts, c->row_src, c->n_ctx,
                           c->res, goff, c->stream);
      launch_commit(d.dtype, c->kcache, c->vcache, c->kscr, c->vscr, d.n_layers, d.n_kv_heads, d.head_dim, c->Spad, c->Mcap,
                    C, shared0, c->n - 1, c->res, 0, 0, w + 1, c->hist, c->stream, c->n_dev);
      launch_advance(c->n_dev, c->res, w + 1, c->stream);
    }
    hipGraph_t g = nullptr;
    hipError_t e = hipStreamEndCapture(c->cap_stream, &g);
    c->stream = callers;
    if (st == NGG_OK && e == hipSuccess) e = hipGraphInstantiate(&c->step_graph, g, nullptr, nullptr, 0);
    if (g) (void)hipGraphDestroy(g);
    if (st != NGG_OK || e != hipSuccess) {
      if (e != hipSuccess) c->err = std::string("step graph not captured: ") + hipGetErrorString(e);
      (void)hipGetLastError();
      c->step_graph = nullptr;
      c->graph_broken = true;
      return NGG_OK;
    }
    memcpy(c->graph_key, key, sizeof c->graph_key);
    c->graph_captures += 1;
  }
  if (c->n_dev_value != c->n) {                          // the device copy follows the steps it runs itself; anything else sets it here
    c->n_upload = c->n;
    NGG_HIP(c, hipMemcpyAsync(c->n_dev, &c->n_upload, 4, hipMemcpyHostToDevice, c->stream));
  }
  NGG_HIP(c, hipGraphLaunch(c->step_graph, c->stream));
  c->graph_replays += 1;
  NGG_HIP(c, hipMemcpyAsync(c->res_host, c->res, (size_t)(goff + M) * 4, hipMemcpyDeviceToHost, c->stream));
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  vo.k = k; vo.w = w;
  vo.winner = c->res_host[RES_WINNER];
  vo.n_accept = c->res_host[RES_NACCEPT];
  vo.n_new = c->res_host[RES_NNEW];
  const int n_new = std::min(vo.n_new, w + 1);
  for (int i = 0; i < n_new; ++i) c->tokens.push_back(c->res_host[RES_NEWTOK + i]);
  c->n += n_new;
  c->n_dev_value = c->n;
  c->have_verify = false;
  c->drafts_on_device = false;
  c->last_k = k; c->last_w = w;
  *n_new_out = n_new;
  *done = true;
  return NGG_OK;
}

// (build_drafts, verify_step, commit) until n_gen tokens were appended after position n0 or max_calls
// verify calls were made
static ngg_status decode_loop(ngg_ctx *c, int n0, int n_gen, int64_t max_calls, const ngg_draft_cfg *cfg, ngg_stats &st) {
  int64_t calls = 0;
  while (c->n - n0 < n_gen && calls < max_calls) {
    // drafts wider than the remaining budget are pointless, and n + w must stay within max_seq
    ngg_draft_cfg step = *cfg;
    const int left = n_gen - (c->n - n0);
    step.w = std::min(step.w, std::max(0, std::min(left - 1, c->d.max_seq - c->n)));
    step.k_ctx_max = context_row_cap(c, step.k_ctx_max);
    double t0 = now_ms();
    ngg_verify_out vo{};
    int32_t n_new = 0;
    ngg_status rc = NGG_OK;
    // A step whose shapes equal the previous step's (so every kernel has been launched once), with nothing that
    // needs the stream (profiling brackets) and no clamp on what it may commit, is replayed from a captured graph
    int key[8];
    step_key(c, step, key);
    bool replayed = false;
    const bool qualifies = c->graph_mode != 0 && !c->graph_broken && c->prof_mask == 0 && left >= step.w + 1 &&
                           c->n + step.w + 1 <= c->d.max_seq;
    bool tuning = false;
    if (qualifies && c->graph_mode == 2) {
      if (memcmp(key, c->tune_key, sizeof key) != 0) {
        memcpy(c->tune_key, key, sizeof key);
        c->tune_count = 0; c->tune_choice = -1; c->tune_ms[0] = c->tune_ms[1] = 1e30;
      }
      tuning = c->tune_choice < 0;
    }
    const bool want_graph = qualifies && (c->graph_mode == 1 || c->tune_choice == 1 || (tuning && c->tune_count >= 3));
    if (want_graph && memcmp(key, c->eager_key, sizeof key) == 0) {
      rc = graph_step(c, step, key, vo, &n_new, &replayed);
      if (rc != NGG_OK) return rc;
      if (replayed) st.ms_verify += now_ms() - t0;
    }
    if (!replayed) {
      // nothing is fetched here, so the forward pass is queued while the drafts are still being built; the
      // accept kernel hands the builder's row bookkeeping back with the result
      rc = ngg_build_drafts(c, &step, nullptr, nullptr, nullptr);
      if (rc != NGG_OK) return rc;
      double t1 = now_ms();
      rc = ngg_verify_step(c, nullptr, step.k, step.w, &vo);
      if (rc != NGG_OK) return rc;
      double t2 = now_ms();
      rc = ngg_commit(c, left, &n_new);
      if (rc != NGG_OK) return rc;
      double t3 = now_ms();
      st.ms_drafts += t1 - t0; st.ms_verify += t2 - t1; st.ms_commit += t3 - t2;
      memcpy(c->eager_key, key, sizeof key);
    }
    if (tuning) {
      const int which = c->tune_count < 3 ? 0 : 1;
      if (which == 1 && !replayed) c->tune_choice = 0;       // no graph to be had
      else {
        c->tune_ms[which] = std::min(c->tune_ms[which], now_ms() - t0);
        ++c->tune_count;
        // A step that takes more than kGraphLaunchMs per kernel it launches (ten per layer, a dozen around them) is
        // bound by the device, not by its launches (the host queues one in about 2.5 us): replay cannot win, so
        // the capture (milliseconds for a 32-layer step) is not paid either.
        if (c->tune_count == 3 && c->tune_ms[0] > kGraphLaunchMs * (10 * c->d.n_layers + 12)) c->tune_choice = 0;
        else if (c->tune_count == 6) c->tune_choice = c->tune_ms[1] < 0.98 * c->tune_ms[0] ? 1 : 0;
      }
    }
    st.calls += 1;
    st.tokens += n_new;
    st.new_hist[n_new] += 1;
    const int n_ctx = c->res_host[RES_NCTX];
    const int ws = c->res_host[RES_WINSRC] ? 1 : 0;
    st.winner_src[ws] += 1;
    st.ctx_rows += n_ctx;
    st.accept_hist[ws][vo.n_accept] += 1;
    if (vo.n_accept > 0) st.rank_hist[ws][ws ? vo.winner - n_ctx : vo.winner] += 1;
    if (vo.n_accept > 0 && ws == 0) c->ctx_rank_wins[vo.winner] += 1;
    st.alloc_hist[n_ctx] += 1;
    ++calls;
  }
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  return NGG_OK;
}

ngg_status ngg_greedy_decode(ngg_ctx *c, const int32_t *prompt, int32_t n_prompt, int32_t n_gen, const ngg_draft_cfg *cfg,
                             int32_t *out_tokens, ngg_stats *stats) {
  if (!c) return NGG_EINVAL;
  if (!out_tokens || n_gen < 1) return fail(c, NGG_EINVAL, "ngg_greedy_decode: need out_tokens and n_gen >= 1");
  if ((long)n_prompt + n_gen > c->d.max_seq) return fail(c, NGG_ECAPACITY, "ngg_greedy_decode: %d + %d tokens exceed max_seq=%d", n_prompt, n_gen, c->d.max_seq);
  ngg_draft_cfg plain{1, 0, 0, 1, 1};
  if (!cfg) cfg = &plain;
  ngg_stats st{};
  double t0 = now_ms();
  ngg_status rc = ngg_prefill(c, prompt, n_prompt);
  if (rc != NGG_OK) return rc;
  st.ms_prefill = now_ms() - t0;
  rc = decode_loop(c, n_prompt, n_gen, INT64_MAX, cfg, st);
  if (rc != NGG_OK) return rc;
  st.tokens = n_gen;
  memcpy(out_tokens, c->tokens.data() + n_prompt, (size_t)n_gen * 4);
  if (stats) *stats = st;
  return NGG_OK;
}

ngg_status ngg_decode_more(ngg_ctx *c, int32_t n_gen, int32_t max_calls, const ngg_draft_cfg *cfg, int32_t *out_tokens,
                           int32_t *n_out, ngg_stats *stats) {
  if (!c) return NGG_EINVAL;
  if (c->n < 1) return fail(c, NGG_ESTATE, "ngg_decode_more: no context (call ngg_prefill first)");
  if (n_gen < 1 || max_calls < 1) return fail(c, NGG_EINVAL, "ngg_decode_more: need n_gen >= 1 and max_calls >= 1");
  if ((long)c->n + n_gen > c->d.max_seq) return fail(c, NGG_ECAPACITY, "ngg_decode_more: %d + %d tokens exceed max_seq=%d", c->n, n_gen, c->d.max_seq);
  ngg_draft_cfg plain{1, 0, 0, 1, 1};
  if (!cfg) cfg = &plain;
  ngg_stats st{};
  const int n0 = c->n;
  ngg_status rc = decode_loop(c, n0, n_gen, max_calls, cfg, st);
  if (rc != NGG_OK) return rc;
  const int made = c->n - n0;
  if (out_tokens) memcpy(out_tokens, c->tokens.data() + n0, (size_t)made * 4);
  if (n_out) *n_out = made;
  if (stats) *stats = st;
  return NGG_OK;
}

ngg_status ngg_get_tokens(const ngg_ctx *c, int32_t *dst, int32_t cap, int32_t *n) {
  if (!c || !n) return NGG_EINVAL;
  *n = c->n;
  if (dst && cap > 0) memcpy(dst, c->tokens.data(), (size_t)std::min(cap, c->n) * 4);
  return NGG_OK;
}

ngg_status ngg_profile_enable(ngg_ctx *c, int32_t class_mask) {
  if (!c) return NGG_EINVAL;
  c->prof_mask = class_mask;
  return NGG_OK;
}

ngg_status ngg_profile_sample(ngg_ctx *c, int32_t every) {
  if (!c) return NGG_EINVAL;
  if (every < 1) return fail(c, NGG_EINVAL, "ngg_profile_sample: every must be >= 1");
  c->prof_every = every;
  return NGG_OK;
}

ngg_status ngg_profile_reset(ngg_ctx *c) {
  if (!c) return NGG_EINVAL;
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  for (auto &sp : c->spans) { c->free_events.push_back(sp.e0); c->free_events.push_back(sp.e1); }
  c->spans.clear();
  for (auto &n : c->prof_seen) n = 0;
  return NGG_OK;
}

ngg_status ngg_profile_read(ngg_ctx *c, double *ms, int64_t *launches) {
  if (!c || !ms || !launches) return NGG_EINVAL;
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < NGG_PROF_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  for (auto &sp : c->spans) {
    float t = 0.0f;
    NGG_HIP(c, hipEventElapsedTime(&t, sp.e0, sp.e1));
    ms[sp.cls] += t;
    launches[sp.cls] += 1;
  }
  return NGG_OK;
}

ngg_status ngg_profile_bracket_overhead(ngg_ctx *c, double *us) {
  if (!c || !us) return NGG_EINVAL;
  // brackets queued back to back, as they are inside a step (a bracket on an idle stream also
  // pays the wake-up of the queue); the first 8 warm up
  constexpr int kReps = 64, kWarm = 8;
  std::vector<hipEvent_t> ev(2 * (kReps + kWarm));
  for (auto &e : ev) NGG_HIP(c, hipEventCreate(&e));
  for (int i = 0; i < kReps + kWarm; ++i) {
    NGG_HIP(c, hipEventRecord(ev[2 * i], c->stream));
    launch_noop(c->stream);
    NGG_HIP(c, hipEventRecord(ev[2 * i + 1], c->stream));
  }
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  double sum = 0.0;
  for (int i = kWarm; i < kReps + kWarm; ++i) {
    float t = 0.0f;
    NGG_HIP(c, hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1]));
    sum += t;
  }
  for (auto &e : ev) (void)hipEventDestroy(e);
  *us = sum * 1e3 / kReps;
  return NGG_OK;
}

ngg_status ngg_profile_read_bandwidth(ngg_ctx *c, double *gbps) {
  if (!c || !gbps) return NGG_EINVAL;
  // one sweep over the library's own operand-order copy of the weights (read-only here), timed with events on the
  // context's stream: 4 repetitions after one warm-up, the best one reported
  const ngg_model_desc &d = c->d;
  const size_t dq = (size_t)d.n_heads * d.head_dim, dkv = (size_t)d.n_kv_heads * d.head_dim;
  const size_t bytes = (((dq + 2 * dkv) * d.d_model + (size_t)d.d_model * dq + (size_t)3 * d.d_ffn * d.d_model) * d.n_layers +
                        (size_t)d.vocab * d.d_model) * c->esize / 16 * 16;
  constexpr int kBlocks = 2048, kReps = 4;
  unsigned *sink = nullptr;
  ngg_status st = dev_alloc(c, &sink, kBlocks * sizeof(unsigned), true);
  if (st != NGG_OK) return st;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t err = hipEventCreate(&e0);
  if (err == hipSuccess) err = hipEventCreate(&e1);
  double best_ms = 1e30;
  for (int r = 0; r <= kReps && err == hipSuccess; ++r) {
    err = hipEventRecord(e0, c->stream);
    launch_read_probe(c->wtiled, bytes, sink, kBlocks, c->stream);
    if (err == hipSuccess) err = hipEventRecord(e1, c->stream);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    if (r > 0 && ms < best_ms) best_ms = ms;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  if (err != hipSuccess) return fail(c, NGG_EHIP, "ngg_profile_read_bandwidth: %s", hipGetErrorString(err));
  *gbps = (double)bytes / (best_ms * 1e-3) / 1e9;
  return NGG_OK;
}

ngg_status ngg_bigram_table_build(ngg_ctx *c, int32_t top_k) {
  if (!c) return NGG_EINVAL;
  const ngg_model_desc &d = c->d;
  if (top_k < 1 || top_k > 64 || top_k > d.vocab) return fail(c, NGG_EINVAL, "ngg_bigram_table_build: need 1 <= top_k <= min(64, vocab)");
  if (top_k < d.max_k) return fail(c, NGG_EINVAL, "ngg_bigram_table_build: top_k=%d is below max_k=%d (a step may ask for max_k bigram rows)", top_k, d.max_k);
  c->graph_key[7] = 0;                                  // a captured step may hold the old table's address
  if (c->bg_table) { (void)hipFree(c->bg_table); c->bg_table = nullptr; c->bg_use = false; }
  ngg_status st = dev_alloc(c, &c->bg_table, (size_t)d.vocab * top_k * 4, true);
  if (st != NGG_OK) return st;
  if (!c->bg_tok) { st = dev_alloc(c, &c->bg_tok, (size_t)c->Mcap * 4, true); if (st != NGG_OK) return st; }
  st = ensure_logits(c);
  if (st != NGG_OK) return st;
  c->bg_K = top_k;
  // p_M(. | x) for every token x: the whole model on the one-token context x.  Mcap contexts per
  // pass: a block of Mcap rows of width 1 on an empty cache (a token attends to itself only).
  c->have_verify = false;                              // the block scratch no longer holds the last verify call
  for (int x0 = 0; x0 < d.vocab; x0 += c->Mcap) {
    const int M = std::min(c->Mcap, d.vocab - x0);
    launch_iota(c->bg_tok, x0, M, c->stream);
    st = forward(c, M, 1, 0, true, 0, true, true, c->bg_tok);
    if (st != NGG_OK) return st;
    launch_row_topk(c->logits, M, d.vocab, top_k, c->bg_table + (size_t)x0 * top_k, c->stream);
  }
  NGG_HIP(c, hipGetLastError());
  NGG_HIP(c, hipStreamSynchronize(c->stream));
  return NGG_OK;
}

ngg_status ngg_unigram_build(ngg_ctx *c, int32_t top_k) {
  if (!c) return NGG_EINVAL;
  const ngg_model_desc &d = c->d;
  if (top_k < 1 || top_k > 64 || top_k > d.vocab) return fail(c, NGG_EINVAL, "ngg_unigram_build: need 1 <= top_k <= min(64, vocab)");
  if (top_k < d.max_k) return fail(c, NGG_EINVAL, "ngg_unigram_build: top_k=%d is below max_k=%d (a step may ask for max_k rows)", top_k, d.max_k);
  c->graph_key[7] = 0;                                  // a captured step may hold the old list's address
  if (c->uni_top) { (void)hipFree(c->uni_top); c->uni_top = nullptr; c->uni_use = false; }
  ngg_status st = dev_alloc(c, &c->uni_top, (size_t)top_k * 4, true);
  if (st != NGG_OK) return st;
  st = ensure_logits(c);
  if (st != NGG_OK) return st;
  // scratch of this build only: the input embedding in operand order (the "weight" of the GEMM below),
  // the mean output embedding, and the negated squared distance of every token
  void *emb_t = nullptr;
  float *mean = nullptr, *negd2 = nullptr;
  st = dev_alloc(c, &emb_t, (size_t)d.vocab * d.d_model * c->esize, false);
  if (st == NGG_OK) st = dev_alloc(c, &mean, (size_t)d.d_model * 4, false);
  if (st == NGG_OK) st = dev_alloc(c, &negd2, (size_t)d.vocab * 4, false);
  if (st == NGG_OK) {
    launch_tile_weights(d.dtype, c->w.tok_emb, emb_t, d.vocab, d.d_model, 0, c->stream, c->emb_scale);
    const float row_scale = d.dtype == NGG_BF16 ? 0.5f * c->unemb_scale : 1.0f;   // a centred row is at most twice the largest entry
    launch_column_mean(d.dtype, c->w.unemb, d.vocab, d.d_model, mean, c->stream);
    c->have_verify = false;                            // the activation buffers are reused
    // d(x)^2 = sum_y ((u_x - u_mean) . v_y)^2: rows u_x - u_mean through the GEMM against the input
    // embedding, Mcap tokens per pass, then the sum of squares of every output row
    for (int x0 = 0; x0 < d.vocab; x0 += c->Mcap) {
      const int M = std::min(c->Mcap, d.vocab - x0);
      launch_pack_rows(d.dtype, (const char *)c->w.unemb + (size_t)x0 * d.d_model * c->esize, c->xn, d.d_model, M, c->Mcap,
                       c->stream, row_scale, mean);
      GemmArgs g{};
      g.X = c->xn;
      g.W0 = emb_t; g.M = M; g.N = d.vocab; g.K = d.d_model;
      g.logits = c->logits; g.pmax_val = c->pmax_val; g.pmax_idx = c->pmax_idx; g.Mcap = c->Mcap;
      g.out_scale = 1.0f / (c->emb_scale * row_scale);
      launch_gemm(d.dtype, EPI_UNEMBED, g, c->stream);
      launch_neg_row_sumsq(c->logits, M, d.vocab, negd2 + x0, c->stream);
    }
    launch_row_topk(negd2, 1, d.vocab, top_k, c->uni_top, c->stream);     // nearest first, ties to the lower id
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) st = fail(c, NGG_EHIP, "ngg_unigram_build: %s", hipGetErrorString(e));
  }
  if (emb_t) (void)hipFree(emb_t);
  if (mean) (void)hipFree(mean);
  if (negd2) (void)hipFree(negd2);
  if (st != NGG_OK) return st;
  c->uni_K = top_k;
  return NGG_OK;
}

ngg_status ngg_allocation(ngg_ctx *c, int32_t mode, int32_t coverage_percent, int32_t warmup_wins) {
  if (!c) return NGG_EINVAL;
  if (mode != NGG_ALLOC_FIXED && mode != NGG_ALLOC_ADAPTIVE) return fail(c, NGG_EINVAL, "ngg_allocation: unknown mode %d", mode);
  if (mode == NGG_ALLOC_ADAPTIVE && (coverage_percent < 1 || coverage_percent > 100 || warmup_wins < 1))
    return fail(c, NGG_EINVAL, "ngg_allocation: need 1 <= coverage_percent <= 100 and warmup_wins >= 1");
  c->alloc_mode = mode;
  if (mode == NGG_ALLOC_ADAPTIVE) { c->alloc_coverage = coverage_percent; c->alloc_warmup = warmup_wins; }
  return NGG_OK;
}

ngg_status ngg_step_graphs(ngg_ctx *c, int32_t on) {
  if (!c) return NGG_EINVAL;
  if (on < 0 || on > 2) return fail(c, NGG_EINVAL, "ngg_step_graphs: mode must be 0, 1 or 2");
  c->graph_mode = on;
  c->tune_choice = -1; c->tune_count = 0; c->tune_key[7] = 0;
  return NGG_OK;
}

ngg_status ngg_bigram_source(ngg_ctx *c, int32_t source) {
  if (!c) return NGG_EINVAL;
  if (source != NGG_BIGRAM_DIRECT && source != NGG_BIGRAM_TABLE && source != NGG_UNIGRAM)
    return fail(c, NGG_EINVAL, "ngg_bigram_source: unknown source %d", source);
  if (source == NGG_BIGRAM_TABLE && !c->bg_table) return fail(c, NGG_ESTATE, "ngg_bigram_source: no table (call ngg_bigram_table_build first)");
  if (source == NGG_UNIGRAM && !c->uni_top) return fail(c, NGG_ESTATE, "ngg_bigram_source: no unigram (call ngg_unigram_build first)");
  c->bg_use = source == NGG_BIGRAM_TABLE;
  c->uni_use = source == NGG_UNIGRAM;
  c->drafts_on_device = false;
  return NGG_OK;
}

ngg_status ngg_context_drafts_static(const int32_t *tokens, int32_t n, int32_t w, int32_t k_ctx_max, int32_t q_min,
                                     int32_t q_max, int32_t *rows, int32_t *n_rows, void *hip_stream) {
  static_assert((kStaticSlots & (kStaticSlots - 1)) == 0, "the grouping table needs a power-of-two slot count");
  if (!tokens || !rows || !n_rows) return fail(nullptr, NGG_EINVAL, "ngg_context_drafts_static: null pointer");
  if (n < 1 || n > NGG_STATIC_MAX_TOKENS)
    return fail(nullptr, NGG_ECAPACITY, "ngg_context_drafts_static: n=%d outside 1 .. %d (the static scratch holds no more)", n,
                NGG_STATIC_MAX_TOKENS);
  if (w < 1 || w > 32 || k_ctx_max < 1 || k_ctx_max > 32)
    return fail(nullptr, NGG_EINVAL, "ngg_context_drafts_static: need 1 <= w <= 32 and 1 <= k_ctx_max <= 32");
  if (q_min < 1 || q_max < q_min || q_max > 64)
    return fail(nullptr, NGG_EINVAL, "ngg_context_drafts_static: need 1 <= q_min <= q_max <= 64");
  // the array's device address, looked up once per device (each GPU has its own copy at its own address)
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static int32_t *base[kMaxDevices] = {};
  int dev = -1;
  NGG_HIP(nullptr, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, NGG_EINVAL, "ngg_context_drafts_static: device %d not supported", dev);
  int32_t *ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!base[dev]) {
      void *p = nullptr;
      NGG_HIP(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      base[dev] = (int32_t *)p;
    }
    ptr = base[dev];
  }
  DraftArgs a{};
  a.hist = tokens; a.n = n; a.k = k_ctx_max; a.w = w; a.k_ctx_max = k_ctx_max; a.q_min = q_min; a.q_max = q_max;
  a.mlist = ptr;
  a.reps = ptr + NGG_STATIC_MAX_TOKENS;
  a.gtab = ptr + (size_t)3 * NGG_STATIC_MAX_TOKENS;
  a.gtab_slots = kStaticSlots;
  a.ctx_rows = rows; a.n_ctx = n_rows;
  launch_ctx_match(a, (hipStream_t)hip_stream);      // clears the part of the table it uses itself: nothing to reset here
  NGG_HIP(nullptr, hipGetLastError());
  return NGG_OK;
}

ngg_status ngg_debug_peek(ngg_ctx *c, const char *name, void *dst, int64_t cap, int64_t *bytes, int32_t *stride) {
  if (!c || !name || !bytes) return NGG_EINVAL;
  const ngg_model_desc &d = c->d;
  const void *src = nullptr;
  size_t sz = 0;
  const size_t kv = (size_t)d.n_layers * d.n_kv_heads * d.head_dim * c->Spad * c->esize;
  const std::string nm(name);
  if (nm == "h") { src = c->h; sz = (size_t)c->Mcap * d.d_model * 4; }
  else if (nm == "z") { src = c->z; sz = (size_t)d.vocab * 4; }
  else if (nm == "next1") { src = c->next1; sz = (size_t)d.vocab * 4; }
  else if (nm == "bg_table" && c->bg_table) { src = c->bg_table; sz = (size_t)d.vocab * c->bg_K * 4; }
  else if (nm == "uni_top" && c->uni_top) { src = c->uni_top; sz = (size_t)c->uni_K * 4; }
  else if (nm == "hist") { src = c->hist; sz = (size_t)c->Spad * 4; }
  else if (nm == "block_tok") { src = c->block_tok; sz = (size_t)c->Mcap * 4; }
  else if (nm == "kcache") { src = c->kcache; sz = kv; }
  else if (nm == "vcache") { src = c->vcache; sz = kv; }
  else if (nm == "attn") { src = c->attn; sz = act_elems(d.dtype, c->Mcap, d.n_heads * d.head_dim) * c->esize; }
  else if (nm == "attn_layout") {                       // host-side record, no device copy
    *bytes = (int64_t)sizeof c->attn_layout;
    if (dst && cap > 0) memcpy(dst, c->attn_layout, std::min((size_t)cap, sizeof c->attn_layout));
    return NGG_OK;
  }
  else if (nm == "step_graphs") {                       // host-side record: on, broken, captures, replays
    const int32_t v[4] = {c->graph_mode, c->graph_broken ? 1 : 0, c->graph_captures, c->graph_replays};
    *bytes = (int64_t)sizeof v;
    if (dst && cap > 0) memcpy(dst, v, std::min((size_t)cap, sizeof v));
    return NGG_OK;
  }
  else return fail(c, NGG_EINVAL, "ngg_debug_peek: unknown buffer '%s'", name);
  *bytes = (int64_t)sz;
  if (stride) *stride = c->Spad;
  if (dst && cap > 0) {
    NGG_HIP(c, hipMemcpyAsync(dst, src, std::min((size_t)cap, sz), hipMemcpyDeviceToHost, c->stream));
    NGG_HIP(c, hipStreamSynchronize(c->stream));
  }
  return NGG_OK;
}

}  // extern "C"
