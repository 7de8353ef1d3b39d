// Host side of libtsd: argument validation, arena carving, weight loading, and the sequencing of
// kernel launches that make up prefill, draft proposal, single-pass verification, acceptance and
// the target-only baseline step.  Nothing here allocates device memory.
#include <chrono>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <random>

#include "tsd_internal.h"

using namespace tsd;

namespace {

thread_local std::string g_err;  // errors of calls that have no handle

struct Layer {
  char *Wqkv, *Wo, *W1, *W2;  // routed FFN: W1 = [E][F][D], W2 = [E][D][F]
  float* Wr;                  // routed FFN: router [E][D], fp32 (NULL for a dense FFN)
};
struct ModelDev {
  tsd_model_cfg c;
  int hd;
  int mfma_attn;     // attention on the matrix cores (bf16, head_dim 64, pages of at least 8 tokens)
  char* W_e;
  char* W_h;
  std::vector<Layer> layers;
  // second copy in MFMA-fragment order for the one-launch draft phase (draft only, NULL otherwise)
  char* fW_e = nullptr;
  char* fW_h = nullptr;
  std::vector<Layer> flayers;
  float *rope_cos, *rope_sin;
  char* kv_pool;
  size_t layer_pool_bytes;
  bool loaded;
};

struct Plan {  // byte offsets into the arena
  size_t total;
};

}  // namespace

struct tsd_ctx {
  tsd_config cfg;
  int es;  // bytes per element of the compute dtype
  char* arena;
  size_t arena_bytes;
  ModelDev model[2];
  int pages_per_series, n_pages;
  int* page_table;
  int *len, *committed, *round, *active, *n_acc;
  float *mean, *sdev, *pending, *prev, *forecast, *znorm;
  long long* stat;
  float *X, *mu_q, *mu_p, *ell, *logu;
  float* diag;  // [3P + 1]: 1/(2 s_p^2), 1/(2 s_q^2), s_q, then the log-det scalar (diagonal surrogate)
  bool diag_on = false;
  float diag_min_sp = 0.f;
  float* x;   // residual stream, fp32
  char* xb;   // its bf16 shadow (GEMM A operand in bf16 mode)
  char *qbuf, *abuf, *hbuf;
  int rows_max;
  bool fused_draft = false;  // tsd_draft_propose is one launch (see draft_fused.hip)
  long long* trace_buf = nullptr;  // [kTraceMax] stage stamps of tsd_trace_draft
  bool trace_on = false;
  int skinny;  // all decode passes have at most 32 rows: they take the skinny GEMM (fixed per handle so that a
               // series' bits never depend on how many other series are still active)
  int* moe_ids;
  int* route_tap[2] = {nullptr, nullptr};  // caller-owned parity tap per model (tsd_set_route_tap), NULL = off
  float* moe_gates;
  int *moe_src, *moe_slot;
  char* moe_tmap;
  float* moe_Y;
  char* moe_h;
  int* count_out;
  // Pinned host words {active series, most patches still needed, launch number} that the compaction kernel
  // writes itself (NULL when pinned memory could not be had: then the counts are copied back instead).
  int* host_counts = nullptr;
  int seq_launched = 0;          // compaction launches enqueued so far (the device keeps the same count)
  bool seq_ready = false;        // the device-side launch counter has been zeroed
  bool compact_pending = false;  // the last tsd_round already enqueued the compaction tsd_num_active wants
  int* act_list;   // series still decoding, ascending (device)
  int* act_list_next;  // handles whose passes are sized on the host: the buffer every compaction writes (see compact_target)
  int n_act;       // host copy of its length; -1 = unknown (use the full batch)
  long long* stats_out;
  // forecast in flight
  bool prefilled;
  int B, N, T, H;
  bool injected;  // next accept reads mu_q from its own buffer
  float alpha_override;
  std::vector<int> host_pt;
  // captured launch sequences of tsd_round / tsd_target_step (rebuilt when anything they bake in changes)
  // one round graph per number of positions and per size class of the active list (the launches of a graph are
  // sized, and their kernels chosen, for a fixed number of series; the device-side count caps the work below that)
  hipGraphExec_t graph_round[17][8] = {}, graph_step = nullptr;
  bool capturing = false;  // a graph capture of this handle's launches is in progress
  int capture_rows = 0;    // series the launches being captured are sized for
  int seq_floor = 0;       // deliveries of the counts up to this launch number describe an earlier decode
  int k_round = 0;  // positions the next round proposes: min(K, most patches any active series still needs)
  int need_lb = 0;  // lower bound on the most patches any series still needs (0 = unknown)
  // measurement tap: event pairs around every launch of one kernel family
  int* refill_list = nullptr;      // device copy of the slots of the last tsd_refill
  std::vector<int> host_refill;
  int K_max = 0;  // K the handle was created with: buffers, pages and the skinny decision are sized for it
  int prof_class = -1;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
  std::vector<tsd_launch_rec> prof_recs;  // one per bracketed launch of the current / last measurement
  size_t prof_used = 0;
  double prof_work = 0;
  std::string err;
};

namespace {

int fail(tsd_ctx* ctx, int code, const std::string& msg) {
  if (ctx)
    ctx->err = msg;
  else
    g_err = msg;
  return code;
}

#define HIP_TRY(ctx, expr)                                                                        \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(ctx, TSD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int check_model(const tsd_model_cfg& m, const char* name, std::string& why) {
  auto bad = [&](const char* w) {
    why = std::string(name) + ": " + w;
    return TSD_E_INVALID_ARG;
  };
  if (m.n_layers < 1 || m.n_layers > 256) return bad("n_layers must be in 1..256");
  if (m.d_model < 16 || m.d_model % 8) return bad("d_model must be a positive multiple of 8");
  if (m.n_heads < 1 || m.d_model % m.n_heads) return bad("n_heads must divide d_model");
  int hd = m.d_model / m.n_heads;
  if (hd != 16 && hd != 32 && hd != 64) return bad("head_dim must be 16, 32 or 64");
  if (m.d_ff < 8 || m.d_ff % 8) return bad("d_ff must be a positive multiple of 8");
  if (m.n_experts != 0) {
    if (m.n_experts < 2 || m.n_experts > 16) return bad("n_experts must be 0 (dense) or in 2..16");
    if (m.top_k < 1 || m.top_k > 4 || m.top_k > m.n_experts) return bad("top_k must be in 1..min(4, n_experts)");
    if (m.d_model % 4) return bad("d_model must be a multiple of 4");
  }
  return TSD_OK;
}

int check_config(const tsd_config* c, std::string& why) {
  if (!c) {
    why = "cfg is NULL";
    return TSD_E_INVALID_ARG;
  }
  auto bad = [&](const char* w) {
    why = w;
    return TSD_E_INVALID_ARG;
  };
  int rc;
  if ((rc = check_model(c->target, "target", why))) return rc;
  if ((rc = check_model(c->draft, "draft", why))) return rc;
  if (c->patch < 8 || c->patch % 8 || c->patch > 1024) return bad("patch must be a multiple of 8 in 8..1024");
  if (c->K < 1 || c->K > 16) return bad("K must be in 1..16");
  if (c->max_batch < 1 || c->max_batch > (1 << 20)) return bad("max_batch out of range");
  if (c->max_tokens < c->K + 3 || c->max_tokens > 1024) return bad("max_tokens must be in K+3..1024");
  if (c->dtype != TSD_F32 && c->dtype != TSD_BF16) return bad("dtype must be TSD_F32 or TSD_BF16");
  if (!is_pow2(c->page_tokens) || c->page_tokens > 64) return bad("page_tokens must be a power of two <= 64");
  if (!(c->sigma_p > 0.f) || !(c->sigma_q > 0.f) || !std::isfinite(c->sigma_p) || !std::isfinite(c->sigma_q))
    return bad("sigma_p and sigma_q must be positive and finite");
  if (!(c->fallback_r >= 0.f) || c->fallback_r > c->sigma_p) return bad("fallback_r must lie in [0, sigma_p]");
  if (c->flags & ~(TSD_FLAG_SCRAMBLE_PAGES | TSD_FLAG_NO_TEMPERING | TSD_FLAG_NO_GRAPH | TSD_FLAG_NO_COMPACT | TSD_FLAG_NO_SKINNY | TSD_FLAG_SAMPLE_PROPOSALS |
                   TSD_FLAG_NAIVE_VERIFY | TSD_FLAG_THRESHOLD_RULE | TSD_FLAG_BATCH_SYNC | TSD_FLAG_NO_PINNED_COUNTS |
                   TSD_FLAG_NO_FUSED_DRAFT | TSD_FLAG_FUSED_DRAFT | TSD_FLAG_NO_WIDE_GEMM))
    return bad("unknown flag bits");
  if ((c->flags & TSD_FLAG_NO_FUSED_DRAFT) && (c->flags & TSD_FLAG_FUSED_DRAFT))
    return bad("TSD_FLAG_FUSED_DRAFT and TSD_FLAG_NO_FUSED_DRAFT exclude each other");
  if ((c->max_tokens + c->page_tokens - 1) / c->page_tokens > 64)
    return bad("max_tokens / page_tokens must not exceed 64 pages per series");
  for (const tsd_model_cfg* m : {&c->target, &c->draft})
    if (m->n_experts > 0 && (size_t)std::max((long)c->max_batch * (c->K + 1), (long)c->max_tokens) * m->top_k > 144 * 1024)
      return bad("max_batch * (K + 1) * top_k too large for the expert sort (one byte per assignment in 144 KB of LDS)");
  for (const tsd_model_cfg* m : {&c->target, &c->draft})
    if (attention_lds_bytes(c->dtype, m->d_model / m->n_heads, c->max_tokens, c->page_tokens) > 160 * 1024)
      return bad("max_tokens too large: one head's K and V rows must fit the 160 KB of LDS");
  return TSD_OK;
}

constexpr int kTraceMax = 512;  // stage stamps tsd_trace_draft can return

struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    size_t r = off;
    off += bytes;
    return r;
  }
};

// The whole draft phase as one kernel.  Supported: dense bf16 draft with head_dim 64 on the matrix-core
// attention, widths in whole MFMA k-steps and column blocks, and everything it keeps in LDS
// fits.  Chosen by default where it was measured to win: every workgroup streams all draft weights per
// step, which beats a chain of launch-bound kernels only while those weights are small (at most 4 MiB, in
// 8-step chunks) and the batch neither so small that the kernel-per-stage path runs its skinny products
// (passes of at most 32 rows) nor so large that its tiled products fill the chip (wins measured from 8 to
// 512 series; at 1024 series with a larger draft it loses).  TSD_FLAG_FUSED_DRAFT selects it wherever it is supported,
// TSD_FLAG_NO_FUSED_DRAFT never.
bool fused_draft_ok(const tsd_config& c) {
  const tsd_model_cfg& d = c.draft;
  const bool supported = c.dtype == TSD_BF16 && d.n_experts == 0 &&
                         d.d_model == 64 * d.n_heads && c.page_tokens >= 8 && d.d_model % 32 == 0 && d.d_ff % 32 == 0 &&
                         c.patch % 16 == 0 && d.n_layers <= kDraftFusedMaxLayers &&
                         draft_fused_lds_bytes(d.d_model, d.d_ff, c.patch) <= 160 * 1024;
  if (!supported || (c.flags & TSD_FLAG_NO_FUSED_DRAFT)) return false;
  if (c.flags & TSD_FLAG_FUSED_DRAFT) return true;
  const size_t wbytes = (size_t)d.n_layers * (4 * (size_t)d.d_model * d.d_model + 2 * (size_t)d.d_model * d.d_ff) * 2;
  return draft_fused_chunk(d.d_model, d.d_ff) == 8 && wbytes <= ((size_t)4 << 20) && (size_t)c.max_batch * (c.K + 1) > 32 &&
         c.max_batch <= 512;
}

// Lays out everything the handle needs inside the arena.  With ctx == nullptr only sizes it.
size_t carve(const tsd_config& c, tsd_ctx* ctx) {
  Carver cv;
  char* base = ctx ? ctx->arena : nullptr;
  const size_t es = c.dtype == TSD_BF16 ? 2 : 4;
  const int P = c.patch, B = c.max_batch, K = c.K;
  const int pps = (c.max_tokens + c.page_tokens - 1) / c.page_tokens;
  const size_t n_pages = (size_t)B * pps;
  auto at = [&](size_t off) { return base ? base + off : nullptr; };
  for (int w = 0; w < 2; ++w) {
    const tsd_model_cfg& m = w == 0 ? c.target : c.draft;
    const size_t D = m.d_model, F = m.d_ff;
    const int hd = m.d_model / m.n_heads;
    ModelDev* md = ctx ? &ctx->model[w] : nullptr;
    size_t o = cv.take(P * D * es);
    if (md) {
      md->c = m;
      md->hd = hd;
      md->mfma_attn = (c.dtype == TSD_BF16 && hd == 64 && c.page_tokens >= 8) ? 1 : 0;
      md->W_e = at(o);
      md->layers.resize(m.n_layers);
      md->loaded = false;
    }
    const size_t nE = m.n_experts > 0 ? m.n_experts : 1;
    for (int l = 0; l < m.n_layers; ++l) {
      size_t oq = cv.take(3 * D * D * es), oo = cv.take(D * D * es), o1 = cv.take(nE * D * F * es), o2 = cv.take(nE * F * D * es);
      size_t orr = m.n_experts > 0 ? cv.take(nE * D * 4) : 0;
      if (md) md->layers[l] = Layer{at(oq), at(oo), at(o1), at(o2), m.n_experts > 0 ? (float*)at(orr) : nullptr};
    }
    o = cv.take(D * P * es);
    if (md) md->W_h = at(o);
    if (w == 1 && fused_draft_ok(c)) {
      const int ch = draft_fused_chunk((int)D, (int)F);
      auto frag = [&](size_t N, size_t K) { return cv.take(draft_fused_packed_elems((int)N, (int)K, ch) * 2); };
      size_t fe = frag(D, P), fh = frag(P, D);
      if (md) {
        md->fW_e = at(fe);
        md->fW_h = at(fh);
        md->flayers.resize(m.n_layers);
      }
      for (int l = 0; l < m.n_layers; ++l) {
        size_t fq = frag(3 * D, D), fo = frag(D, D), f1 = frag(F, D), f2 = frag(D, F);
        if (md) md->flayers[l] = Layer{at(fq), at(fo), at(f1), at(f2), nullptr};
      }
    }
    size_t oc = cv.take((size_t)c.max_tokens * (hd / 2) * 4), os = cv.take((size_t)c.max_tokens * (hd / 2) * 4);
    if (md) {
      md->rope_cos = (float*)at(oc);
      md->rope_sin = (float*)at(os);
    }
    const size_t layer_pool = n_pages * 2 * c.page_tokens * D * es;
    o = cv.take(layer_pool * m.n_layers);
    if (md) {
      md->kv_pool = at(o);
      md->layer_pool_bytes = layer_pool;
    }
  }
  size_t o_pt = cv.take(n_pages * 4);
  size_t o_len = cv.take(B * 4), o_com = cv.take(B * 4), o_rnd = cv.take(B * 4), o_act = cv.take(B * 4), o_nacc = cv.take(B * 4);
  size_t o_mean = cv.take(B * 4), o_sdev = cv.take(B * 4);
  size_t o_pend = cv.take((size_t)B * P * 4), o_prev = cv.take((size_t)B * P * 4);
  size_t o_fc = cv.take((size_t)B * c.max_tokens * P * 4), o_zn = cv.take((size_t)B * c.max_tokens * P * 4);
  size_t o_stat = cv.take((size_t)B * 5 * 8);
  size_t o_X = cv.take((size_t)B * K * P * 4), o_mq = cv.take((size_t)B * K * P * 4), o_mp = cv.take((size_t)B * (K + 1) * P * 4);
  size_t o_ell = cv.take((size_t)B * K * 4), o_logu = cv.take((size_t)B * K * 4);
  size_t o_diag = cv.take((size_t)(3 * P + 1) * 4);
  const size_t Dm = std::max(c.target.d_model, c.draft.d_model), Fm = std::max(c.target.d_ff, c.draft.d_ff);
  const size_t rows = std::max((size_t)B * (K + 1), (size_t)c.max_tokens);
  size_t o_xb = cv.take(rows * Dm * es);
  size_t o_x = cv.take(rows * Dm * 4), o_q = cv.take(rows * Dm * es), o_a = cv.take(rows * Dm * es), o_h = cv.take(rows * Fm * es);
  size_t o_trace = cv.take(kTraceMax * 8);
  size_t o_cnt = cv.take(256), o_so = cv.take(256), o_alist = cv.take((size_t)B * 4), o_rlist = cv.take((size_t)B * 4);
  size_t o_alist2 = cv.take((size_t)B * 4);
  // routed FFN scratch: one slot per (token, chosen expert)
  const size_t topk = std::max(c.target.n_experts > 0 ? c.target.top_k : 0, c.draft.n_experts > 0 ? c.draft.top_k : 0);
  const size_t slots = rows * topk, nEmax = std::max(c.target.n_experts, c.draft.n_experts);
  size_t o_ids = 0, o_gates = 0, o_src = 0, o_slot = 0, o_tmap = 0, o_Y = 0, o_hx = 0;
  if (topk) {
    o_ids = cv.take(slots * 4);
    o_gates = cv.take(slots * 4);
    o_src = cv.take(slots * 4);
    o_slot = cv.take(slots * 4);
    o_tmap = cv.take((slots / 64 + nEmax + 2) * 16);
    o_Y = cv.take(slots * Dm * 4);
    o_hx = cv.take(slots * Fm * es);
  }
  if (ctx) {
    ctx->es = (int)es;
    ctx->pages_per_series = pps;
    ctx->n_pages = (int)n_pages;
    ctx->page_table = (int*)at(o_pt);
    ctx->len = (int*)at(o_len);
    ctx->committed = (int*)at(o_com);
    ctx->round = (int*)at(o_rnd);
    ctx->active = (int*)at(o_act);
    ctx->n_acc = (int*)at(o_nacc);
    ctx->mean = (float*)at(o_mean);
    ctx->sdev = (float*)at(o_sdev);
    ctx->pending = (float*)at(o_pend);
    ctx->prev = (float*)at(o_prev);
    ctx->forecast = (float*)at(o_fc);
    ctx->znorm = (float*)at(o_zn);
    ctx->stat = (long long*)at(o_stat);
    ctx->X = (float*)at(o_X);
    ctx->mu_q = (float*)at(o_mq);
    ctx->mu_p = (float*)at(o_mp);
    ctx->ell = (float*)at(o_ell);
    ctx->logu = (float*)at(o_logu);
    ctx->diag = (float*)at(o_diag);
    ctx->x = (float*)at(o_x);
    ctx->xb = at(o_xb);
    ctx->qbuf = at(o_q);
    ctx->abuf = at(o_a);
    ctx->hbuf = at(o_h);
    ctx->rows_max = (int)rows;
    ctx->K_max = K;
    ctx->skinny = (c.dtype == TSD_BF16 && !(c.flags & TSD_FLAG_NO_SKINNY) && (size_t)B * (K + 1) <= 32) ? 1 : 0;
    ctx->fused_draft = fused_draft_ok(c);
    ctx->trace_buf = (long long*)at(o_trace);
    ctx->count_out = (int*)at(o_cnt);
    ctx->act_list = (int*)at(o_alist);
    ctx->act_list_next = (int*)at(o_alist2);
    ctx->refill_list = (int*)at(o_rlist);
    ctx->moe_ids = topk ? (int*)at(o_ids) : nullptr;
    ctx->moe_gates = (float*)at(o_gates);
    ctx->moe_src = (int*)at(o_src);
    ctx->moe_slot = (int*)at(o_slot);
    ctx->moe_tmap = at(o_tmap);
    ctx->moe_Y = (float*)at(o_Y);
    ctx->moe_h = at(o_hx);
    ctx->stats_out = (long long*)at(o_so);
  }
  return (cv.off + 255) & ~(size_t)255;
}

size_t weights_count(const tsd_model_cfg& m, int P) {
  size_t D = m.d_model, F = m.d_ff, E = m.n_experts;
  size_t per_layer = D + 4 * D * D + D + (E > 0 ? D * E + E * 2 * D * F : 2 * D * F);
  return (size_t)P * D + per_layer * m.n_layers + D + D * P;
}

// What a bracketed launch was: the model it belongs to, the GEMM kernel chosen (gemm_variant) and the product's shape.
struct Shape {
  int model = -1, tile = 0, M = 0, N = 0, K = 0;
};
Shape shape_of(const tsd_ctx* ctx, int which, int amode, int epi, const GemmP& g) {
  return Shape{which, gemm_variant(ctx->cfg.dtype, amode, epi, g), g.M, g.N, g.K};
}

// Launches `fn` on `st`; if kernel family `cls` is being profiled (or all are), brackets it with two events.
template <typename F>
hipError_t timed_launch(tsd_ctx* ctx, int cls, double work, hipStream_t st, F fn, Shape sh = Shape()) {
  if (ctx->prof_class != cls && ctx->prof_class != TSD_K_COUNT) return fn();
  if (ctx->prof_used == ctx->prof_events.size()) {
    hipEvent_t a, b;
    hipError_t e = hipEventCreate(&a);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&b);
    if (e != hipSuccess) return e;
    ctx->prof_events.emplace_back(a, b);
  }
  auto& ev = ctx->prof_events[ctx->prof_used++];
  ctx->prof_recs.push_back(tsd_launch_rec{cls, sh.model, sh.tile, sh.M, sh.N, sh.K, 0.f, work});
  hipError_t e = hipEventRecord(ev.first, st);
  if (e != hipSuccess) return e;
  e = fn();
  if (e != hipSuccess) return e;
  ctx->prof_work += work;
  return hipEventRecord(ev.second, st);
}

struct Pass {
  int which;
  int B, s0, nq;
  const int* act;  // compacted pass over B listed series (NULL: series s0 .. s0+B-1)
  const int* n_dev;  // device-side count of listed series (NULL: B)
  const int* base_pos;
  int pos_off;
  const float *src0, *src1;
  long stride0, stride1;
  int n0;
  float* out;  // NULL = skip the head
  long out_stride_b;
  int t_skip;
};

// One causal pass of `nq` new tokens per series through a model, against its paged KV cache.
int run_pass(tsd_ctx* ctx, const Pass& ps, hipStream_t st) {
  const tsd_config& c = ctx->cfg;
  ModelDev& md = ctx->model[ps.which];
  const int D = md.c.d_model, F = md.c.d_ff, P = c.patch, M = ps.B * ps.nq;
  if (M > ctx->rows_max) return fail(ctx, TSD_E_OUT_OF_RANGE, "pass exceeds the activation workspace");
  GemmP g;
  std::memset(&g, 0, sizeof(g));
  g.allow_skinny = ctx->skinny;
  g.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
  g.M = M;
  g.nq = ps.nq;
  // patch embedding
  g.N = D;
  g.K = P;
  g.src0 = ps.src0;
  g.src1 = ps.src1;
  g.stride0 = ps.stride0;
  g.stride1 = ps.stride1;
  g.n0 = ps.n0;
  g.act = ps.act;
  g.n_dev = ps.n_dev;
  g.W = md.W_e;
  g.Cf = ctx->x;
  g.Cb = ctx->xb;
  const void* xin = c.dtype == TSD_BF16 ? (const void*)ctx->xb : (const void*)ctx->x;  // A operand of the norm-fused GEMMs
  HIP_TRY(ctx, timed_launch(ctx, TSD_K_EMBED, 2.0 * M * D * P, st, [&] { return launch_gemm(c.dtype, A_TOK, EP_STORE, g, st); }, shape_of(ctx, ps.which, A_TOK, EP_STORE, g)));
  for (int l = 0; l < md.c.n_layers; ++l) {
    char* pool = md.kv_pool + (size_t)l * md.layer_pool_bytes;
    GemmP q;
    std::memset(&q, 0, sizeof(q));
    q.allow_skinny = ctx->skinny;
    q.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
    q.M = M;
    q.nq = ps.nq;
    q.N = 3 * D;
    q.K = D;
    q.A = xin;
    q.W = md.layers[l].Wqkv;
    q.q_out = ctx->qbuf;
    q.kv_pool = pool;
    q.page_table = ctx->page_table;
    q.pt_stride = ctx->pages_per_series;
    q.base_pos = ps.base_pos;
    q.pos_off = ps.pos_off;
    q.s0 = ps.s0;
    q.act = ps.act;
    q.n_dev = ps.n_dev;
    q.rope_cos = md.rope_cos;
    q.rope_sin = md.rope_sin;
    q.D = D;
    q.Hh = md.c.n_heads;
    q.hd = md.hd;
    q.PT = c.page_tokens;
    q.pt_shift = __builtin_ctz(c.page_tokens);
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_QKV, 6.0 * M * D * D, st, [&] { return launch_gemm(c.dtype, A_NORM, EP_QKV, q, st); }, shape_of(ctx, ps.which, A_NORM, EP_QKV, q)));
    AttnP a;
    std::memset(&a, 0, sizeof(a));
    a.q = ctx->qbuf;
    a.out = ctx->abuf;
    a.kv_pool = pool;
    a.page_table = ctx->page_table;
    a.pt_stride = ctx->pages_per_series;
    a.base_pos = ps.base_pos;
    a.pos_off = ps.pos_off;
    a.s0 = ps.s0;
    a.act = ps.act;
    a.n_dev = ps.n_dev;
    a.nq = ps.nq;
    a.B = ps.B;
    a.Hh = md.c.n_heads;
    a.hd = md.hd;
    a.D = D;
    a.PT = c.page_tokens;
    a.pt_shift = __builtin_ctz(c.page_tokens);
    a.mfma = md.mfma_attn;
    a.model = ps.which;
    a.scale = 1.0f / std::sqrt((float)md.hd);
    // K and V rows of the shortest history this pass can see (N-1 cached tokens + the new ones), q and output rows
    const double attn_bytes = (double)ps.B * D * ctx->es * (2.0 * (ctx->N - 1 + ps.nq + (ps.base_pos ? ps.pos_off : 1 - ctx->N)) + 2.0 * ps.nq);
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_ATTN, attn_bytes, st, [&] { return launch_attention(c.dtype, a, c.max_tokens, st); }, Shape{ps.which, 0, M, D, 0}));
    GemmP o;
    std::memset(&o, 0, sizeof(o));
    o.allow_skinny = ctx->skinny;
    o.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
    o.M = M;
    o.nq = ps.nq;
    o.n_dev = ps.n_dev;
    o.N = D;
    o.K = D;
    o.A = ctx->abuf;
    o.W = md.layers[l].Wo;
    o.Cf = ctx->x;
    o.Cb = ctx->xb;
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_RESID, 2.0 * M * D * D, st, [&] { return launch_gemm(c.dtype, A_ACT, EP_RESID, o, st); }, shape_of(ctx, ps.which, A_ACT, EP_RESID, o)));
    if (md.c.n_experts > 0) {
      // routed FFN: router -> stable sort of (token, choice) by expert -> grouped up/down GEMMs -> gated combine
      const int E = md.c.n_experts, topk = md.c.top_k, slots = M * topk;
      int bm = gemm_row_tile(c.dtype, slots, F, 0);
      if (bm == 128 && F >= kQuarterK) {
        // the experts' second product is a long contraction of activations: at 128-row tiles only the wide-tile
        // kernels take it (they keep the running sum of its four runs); where they do not apply, 64-row tiles
        GemmP probe;
        std::memset(&probe, 0, sizeof(probe));
        probe.M = slots;
        probe.N = D;
        probe.K = F;
        probe.tile_map = ctx->moe_tmap;
        probe.force_bm = 128;
        probe.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
        if (gemm_wide_bm(c.dtype, A_ACT, EP_STORE, probe) != 128) bm = 64;
      }
      const int n_mtiles = (slots + bm - 1) / bm + E;
      HIP_TRY(ctx, timed_launch(ctx, TSD_K_ROUTE, 4.0 * M * D, st, [&] {
        return launch_router(ctx->x, md.layers[l].Wr, M, D, E, topk, ctx->moe_ids, ctx->moe_gates, st);
      }, Shape{ps.which, 1, M, E, D}));
      if (ctx->route_tap[ps.which])
        HIP_TRY(ctx, launch_route_tap(ctx->moe_ids, ctx->route_tap[ps.which], l, M, ps.nq, ps.act, ps.s0, ps.base_pos, ps.pos_off,
                                      c.max_batch, c.max_tokens, topk, st));
      HIP_TRY(ctx, timed_launch(ctx, TSD_K_ROUTE, 12.0 * slots, st, [&] {
        return launch_permute(ctx->moe_ids, slots, topk, E, bm, n_mtiles, ctx->moe_src, ctx->moe_slot, ctx->moe_tmap, st);
      }, Shape{ps.which, 2, slots, E, 0}));
      GemmP f1;
      std::memset(&f1, 0, sizeof(f1));
      f1.M = slots;
      f1.nq = ps.nq;
      f1.N = F;
      f1.K = D;
      f1.A = xin;
      f1.W = md.layers[l].W1;
      f1.Ct = ctx->moe_h;
      f1.tile_map = ctx->moe_tmap;
      f1.src_row = ctx->moe_src;
      f1.w_stride = (long)F * D;
      f1.n_mtiles = n_mtiles;
      f1.force_bm = bm;
      f1.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
      HIP_TRY(ctx, timed_launch(ctx, TSD_K_GELU, 2.0 * slots * D * F, st, [&] { return launch_gemm(c.dtype, A_NORM, EP_GELU, f1, st); },
                                shape_of(ctx, ps.which, A_NORM, EP_GELU, f1)));
      GemmP f2;
      std::memset(&f2, 0, sizeof(f2));
      f2.M = slots;
      f2.nq = ps.nq;
      f2.N = D;
      f2.K = F;
      f2.A = ctx->moe_h;
      f2.W = md.layers[l].W2;
      f2.Cf = ctx->moe_Y;
      f2.tile_map = ctx->moe_tmap;
      f2.w_stride = (long)D * F;
      f2.n_mtiles = n_mtiles;
      f2.force_bm = bm;
      f2.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
      HIP_TRY(ctx, timed_launch(ctx, TSD_K_RESID, 2.0 * slots * D * F, st, [&] { return launch_gemm(c.dtype, A_ACT, EP_STORE, f2, st); },
                                shape_of(ctx, ps.which, A_ACT, EP_STORE, f2)));
      HIP_TRY(ctx, timed_launch(ctx, TSD_K_ROUTE, 4.0 * D * (2.0 * M + slots), st, [&] {
        return launch_combine(c.dtype, ctx->moe_Y, ctx->moe_slot, ctx->moe_gates, ctx->x, c.dtype == TSD_BF16 ? ctx->xb : nullptr, M, D, topk, st);
      }, Shape{ps.which, 3, M, D, topk}));
      continue;
    }
    GemmP f1;
    std::memset(&f1, 0, sizeof(f1));
    f1.allow_skinny = ctx->skinny;
    f1.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
    f1.M = M;
    f1.nq = ps.nq;
    f1.n_dev = ps.n_dev;
    f1.N = F;
    f1.K = D;
    f1.A = xin;
    f1.W = md.layers[l].W1;
    f1.Ct = ctx->hbuf;
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_GELU, 2.0 * M * D * F, st, [&] { return launch_gemm(c.dtype, A_NORM, EP_GELU, f1, st); },
                              shape_of(ctx, ps.which, A_NORM, EP_GELU, f1)));
    GemmP f2;
    std::memset(&f2, 0, sizeof(f2));
    f2.allow_skinny = ctx->skinny;
    f2.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
    f2.M = M;
    f2.nq = ps.nq;
    f2.n_dev = ps.n_dev;
    f2.N = D;
    f2.K = F;
    f2.A = ctx->hbuf;
    f2.W = md.layers[l].W2;
    f2.Cf = ctx->x;
    f2.Cb = ctx->xb;
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_RESID, 2.0 * M * D * F, st, [&] { return launch_gemm(c.dtype, A_ACT, EP_RESID, f2, st); },
                              shape_of(ctx, ps.which, A_ACT, EP_RESID, f2)));
  }
  if (ps.out) {
    GemmP h;
    std::memset(&h, 0, sizeof(h));
    h.allow_skinny = ctx->skinny;
    h.no_wide = (c.flags & TSD_FLAG_NO_WIDE_GEMM) ? 1 : 0;
    h.M = M;
    h.nq = ps.nq;
    h.N = P;
    h.K = D;
    h.A = ctx->x;  // the head reads the fp32 residual
    h.W = md.W_h;
    h.out = ps.out;
    h.out_stride_b = ps.out_stride_b;
    h.t_skip = ps.t_skip;
    h.act = ps.act;
    h.n_dev = ps.n_dev;
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_HEAD, 2.0 * M * D * P, st, [&] { return launch_gemm(c.dtype, A_NORM32, EP_HEAD, h, st); },
                              shape_of(ctx, ps.which, A_NORM32, EP_HEAD, h)));
  }
  return TSD_OK;
}

// Series a pass has to cover: the compacted active list when tsd_num_active has built one since
// the last prefill/reset (it stays a superset of the active set as series finish), else everyone.
struct Cover {
  const int* act;
  int n;
  const int* n_dev;  // launches being captured into a graph: the count is read on the device at replay
};
// Dense models can replay a graph however many series are still active: its launches are sized for
// a size class of the active list (see class_rows) and every kernel caps its work by the device-side
// count that the compaction maintains (the routed FFN sizes its expert runs on the host, so it cannot).
bool device_counts(const tsd_ctx* ctx) {
  return !(ctx->cfg.flags & TSD_FLAG_NO_COMPACT) && ctx->cfg.target.n_experts == 0 && ctx->cfg.draft.n_experts == 0 &&
         ctx->B > 1;
}
// The compaction that ends every tsd_round rewrites the list on the device, while the host's copy of its
// length is refreshed only by tsd_num_active.  A launch that pairs an older (larger) host count with the newer
// list must not read the list's stale tail (it can repeat series that are still active: two workgroups would
// then commit for one series).  Handles that follow the device-side count therefore ALWAYS cap their work by
// it, captured or not: list and count are rewritten together, in stream order.  Handles whose passes are sized
// on the host (routed FFN, one series, ...) keep two list buffers instead: compactions always write the second one
// (a fixed address, so captured launch sequences may contain them), and tsd_num_active copies it over the list the
// passes read when it takes delivery of the matching count.
Cover cover(const tsd_ctx* ctx) {
  if (ctx->capturing && device_counts(ctx)) return Cover{ctx->act_list, ctx->capture_rows, ctx->count_out};
  if (ctx->n_act >= 0 && ctx->n_act < ctx->B) return Cover{ctx->act_list, ctx->n_act, device_counts(ctx) ? ctx->count_out : nullptr};
  return Cover{nullptr, ctx->B, nullptr};
}
// The list buffer a compaction may write now.
int* compact_target(const tsd_ctx* ctx) { return device_counts(ctx) ? ctx->act_list : ctx->act_list_next; }

void drop_graphs(tsd_ctx* ctx) {
  for (auto& row : ctx->graph_round)
    for (hipGraphExec_t& g : row)
      if (g) {
        (void)hipGraphExecDestroy(g);
        g = nullptr;
      }
  if (ctx->graph_step) {
    (void)hipGraphExecDestroy(ctx->graph_step);
    ctx->graph_step = nullptr;
  }
}

// Size classes of the active list for graph replay: the launches of a captured round are sized for class_rows(i)
// series, the smallest class that still holds every series the host knows to be active.  (The kernels a launch
// picks give the same bits whatever the class, so the class only decides how much of the chip a late round wastes.)
constexpr int kSizeClasses = 8;
int class_rows(const tsd_ctx* ctx, int i) {
  static const int num[kSizeClasses] = {32, 24, 16, 12, 8, 4, 2, 1};  // 32nds of the batch
  return std::max(1, (int)(((long)ctx->B * num[i] + 31) / 32));
}
int size_class(const tsd_ctx* ctx) {
  const int n = (ctx->n_act >= 0 && ctx->n_act < ctx->B) ? ctx->n_act : ctx->B;
  int i = 0;
  while (i + 1 < kSizeClasses && class_rows(ctx, i + 1) >= n) ++i;
  return i;
}

// A look at the pinned count words without waiting: if a compaction of the current decode has delivered since the
// last look, the host's upper bounds on the active series and on the patches still needed follow it.  Counts only
// fall during a decode, so a delivery that is not the latest is still a valid bound.
void peek_counts(tsd_ctx* ctx) {
  if (!ctx->host_counts || !ctx->seq_ready || !device_counts(ctx)) return;
  const int s1 = __atomic_load_n(&ctx->host_counts[2], __ATOMIC_ACQUIRE);
  if (s1 <= ctx->seq_floor) return;
  const int c0 = __atomic_load_n(&ctx->host_counts[0], __ATOMIC_RELAXED), c1 = __atomic_load_n(&ctx->host_counts[1], __ATOMIC_RELAXED);
  if (__atomic_load_n(&ctx->host_counts[2], __ATOMIC_ACQUIRE) != s1) return;  // a delivery in progress: next time
  if (c0 < 0 || c0 > ctx->B || c1 < 0) return;
  if (ctx->n_act < 0 || c0 < ctx->n_act) ctx->n_act = c0;
  if (c1 >= 1 && (ctx->k_round < 1 || c1 < ctx->k_round)) ctx->k_round = c1;
}

// Runs `body` (a sequence of kernel launches on `st`) through a HIP graph: captured on first use,
// replayed afterwards.  Falls back to plain launches on the NULL stream, when the caller is
// itself capturing `st`, or when graphs are switched off.
template <typename F>
int run_graphed(tsd_ctx* ctx, hipGraphExec_t* slot, hipStream_t st, F body, bool counts = true) {
  if ((ctx->cfg.flags & TSD_FLAG_NO_GRAPH) || st == nullptr || ctx->prof_class >= 0) return body();
  if (cover(ctx).act && !(counts && device_counts(ctx))) return body();  // host-sized compacted passes cannot be replayed
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  HIP_TRY(ctx, hipStreamIsCapturing(st, &cs));
  if (cs != hipStreamCaptureStatusNone) return body();
  if (!*slot) {
    HIP_TRY(ctx, hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    ctx->capturing = counts;
    int rc = body();
    ctx->capturing = false;
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(st, &graph);
    if (rc) {
      if (graph) (void)hipGraphDestroy(graph);
      return rc;
    }
    if (e != hipSuccess) return fail(ctx, TSD_E_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    e = hipGraphInstantiate(slot, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) {
      *slot = nullptr;
      return fail(ctx, TSD_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e));
    }
  }
  HIP_TRY(ctx, hipGraphLaunch(*slot, st));
  return TSD_OK;
}

// Positions the next round proposes and verifies.  A series with r patches left tests min(K, r)
// positions (the acceptance kernel applies that per series); when tsd_num_active has reported
// that no active series needs K more patches, the passes themselves shrink to the largest need.
int round_positions(const tsd_ctx* ctx) {
  const int K = ctx->cfg.K;
  return (ctx->k_round >= 1 && ctx->k_round < K) ? ctx->k_round : K;
}

int require_ready(tsd_ctx* ctx, bool need_prefill) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (need_prefill) {
    if (!ctx->model[0].loaded || !ctx->model[1].loaded) return fail(ctx, TSD_E_BAD_STATE, "weights of both models must be loaded first");
    if (!ctx->prefilled) return fail(ctx, TSD_E_BAD_STATE, "tsd_prefill has not been called");
  }
  return TSD_OK;
}

int accept_commit_impl(tsd_ctx* ctx, const int32_t* forced, int K, hipStream_t st) {
  const tsd_config& c = ctx->cfg;
  AcceptP a;
  std::memset(&a, 0, sizeof(a));
  a.X = ctx->X;
  const bool sampled = (c.flags & TSD_FLAG_SAMPLE_PROPOSALS) != 0;
  a.mu_q = (ctx->injected || sampled) ? ctx->mu_q : ctx->X;  // mean-propagating scheme: x_i = mu_q^(i)
  a.mu_p = ctx->mu_p;
  a.forced = forced;
  a.pending = ctx->pending;
  a.prev = ctx->prev;
  a.forecast = ctx->forecast;
  a.len = ctx->len;
  a.committed = ctx->committed;
  a.round = ctx->round;
  a.active = ctx->active;
  a.n_acc = ctx->n_acc;
  a.ell = ctx->ell;
  a.logu = ctx->logu;
  a.stat = ctx->stat;
  const Cover cv = cover(ctx);
  if (cv.n == 0) return TSD_OK;
  a.B = cv.n;
  a.act = cv.act;
  a.n_dev = cv.n_dev;
  a.K = K;
  a.P = c.patch;
  a.T = ctx->T;
  a.inv2sp2 = 1.0f / (2.0f * c.sigma_p * c.sigma_p);
  a.inv2sq2 = 1.0f / (2.0f * c.sigma_q * c.sigma_q);
  a.logdet = 0.5f * std::log((c.sigma_q * c.sigma_q) / (c.sigma_p * c.sigma_p));
  a.temper = (c.flags & TSD_FLAG_NO_TEMPERING) ? (float)c.patch : 1.0f;
  a.log_alpha_override = ctx->alpha_override > 0.f ? std::log(ctx->alpha_override) : 1.0f;
  a.fallback_r = K > 0 ? c.fallback_r : 0.f;  // the target-only step commits the target mean
  if (ctx->diag_on) {
    a.inv2sp2_vec = ctx->diag;
    a.inv2sq2_vec = ctx->diag + c.patch;
    a.logdet_dev = ctx->diag + 3 * c.patch;
  }
  a.key0 = (unsigned)(c.seed & 0xFFFFFFFFull);
  a.key1 = (unsigned)(c.seed >> 32);
  a.threshold = (c.flags & TSD_FLAG_THRESHOLD_RULE) ? 1 : 0;
  if ((c.flags & TSD_FLAG_BATCH_SYNC) && K > 0) {
    // the series' own counts first (their minimum lands in the sync word), then the commit
    a.sync = ctx->count_out + 8;
    HIP_TRY(ctx, launch_fill_int(a.sync, INT_MAX, 1, st));
    a.mode = 1;
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_ACCEPT, 4.0 * ctx->B * c.patch * (2.0 * K + 2), st, [&] { return launch_accept(a, st); }, Shape{-1, 0, cv.n, K, c.patch}));
    a.mode = 2;
  }
  HIP_TRY(ctx, timed_launch(ctx, TSD_K_ACCEPT, 4.0 * ctx->B * c.patch * (2.0 * K + 2), st, [&] { return launch_accept(a, st); }, Shape{-1, 0, cv.n, K, c.patch}));
  ctx->injected = false;
  ctx->compact_pending = false;  // whatever compaction was enqueued before describes an older state
  ctx->need_lb = 0;              // ... and so does the last count of patches still needed
  return TSD_OK;
}

}  // namespace

namespace tsd {
int fail_no_handle(int code, const std::string& msg) { return fail(nullptr, code, msg); }
}  // namespace tsd

extern "C" {

int tsd_abi_version(void) { return 1; }

const char* tsd_last_error(tsd_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int tsd_workspace_bytes(const tsd_config* cfg, size_t* bytes_host) {
  std::string why;
  int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  if (!bytes_host) return fail(nullptr, TSD_E_INVALID_ARG, "bytes_host is NULL");
  *bytes_host = carve(*cfg, nullptr);
  return TSD_OK;
}

int tsd_weights_count(const tsd_config* cfg, int which, size_t* n_floats_host) {
  std::string why;
  int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  if (which != TSD_TARGET && which != TSD_DRAFT) return fail(nullptr, TSD_E_INVALID_ARG, "which must be TSD_TARGET or TSD_DRAFT");
  if (!n_floats_host) return fail(nullptr, TSD_E_INVALID_ARG, "n_floats_host is NULL");
  *n_floats_host = weights_count(which == TSD_TARGET ? cfg->target : cfg->draft, cfg->patch);
  return TSD_OK;
}

int tsd_create(const tsd_config* cfg, void* arena_dev, size_t arena_bytes, tsd_ctx** out) {
  std::string why;
  int rc = check_config(cfg, why);
  if (rc) return fail(nullptr, rc, why);
  if (!out) return fail(nullptr, TSD_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (!arena_dev) return fail(nullptr, TSD_E_INVALID_ARG, "arena_dev is NULL");
  if ((uintptr_t)arena_dev & 255) return fail(nullptr, TSD_E_INVALID_ARG, "arena_dev must be 256-byte aligned");
  size_t need = carve(*cfg, nullptr);
  if (arena_bytes < need) return fail(nullptr, TSD_E_INVALID_ARG, "arena smaller than tsd_workspace_bytes");
  tsd_ctx* ctx = new (std::nothrow) tsd_ctx();
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "out of host memory");
  ctx->cfg = *cfg;
  ctx->arena = (char*)arena_dev;
  ctx->arena_bytes = arena_bytes;
  ctx->prefilled = false;
  ctx->injected = false;
  ctx->alpha_override = -1.f;
  ctx->n_act = -1;
  ctx->B = ctx->N = ctx->T = ctx->H = 0;
  carve(*cfg, ctx);
  // rotary tables: angle(pos, i) = pos * base^(-2 i / hd), computed in double
  for (int w = 0; w < 2; ++w) {
    ModelDev& md = ctx->model[w];
    const int half = md.hd / 2;
    std::vector<float> cs((size_t)cfg->max_tokens * half), sn(cs.size());
    for (int pos = 0; pos < cfg->max_tokens; ++pos)
      for (int i = 0; i < half; ++i) {
        double ang = (double)pos * std::pow(kRopeBase, -2.0 * i / md.hd);
        cs[(size_t)pos * half + i] = (float)std::cos(ang);
        sn[(size_t)pos * half + i] = (float)std::sin(ang);
      }
    hipError_t e = hipMemcpy(md.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(md.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      std::string msg = std::string("copying rotary tables: ") + hipGetErrorString(e);
      delete ctx;
      return fail(nullptr, TSD_E_HIP, msg);
    }
  }
  {
    // a few pinned host words for the active-series counts, and the device-side launch counter that numbers
    // their deliveries; without them tsd_num_active copies the counts back and waits on the stream
    int* hc = nullptr;
    if (!(cfg->flags & TSD_FLAG_NO_PINNED_COUNTS) && hipHostMalloc((void**)&hc, 64, hipHostMallocDefault) == hipSuccess && hc) {
      hc[0] = hc[1] = hc[2] = 0;
      if (hipMemset(ctx->count_out + 4, 0, 4) == hipSuccess) {
        ctx->host_counts = hc;
        ctx->seq_ready = true;
      } else {
        (void)hipHostFree(hc);
      }
    }
    (void)hipGetLastError();
  }
  if (cfg->target.n_experts > 0 || cfg->draft.n_experts > 0) {
    hipError_t e = prepare_moe();
    if (e != hipSuccess) {
      std::string msg = std::string("raising the expert-sort kernel's LDS limit: ") + hipGetErrorString(e);
      delete ctx;
      return fail(nullptr, TSD_E_HIP, msg);
    }
  }
  {
    hipError_t e = prepare_gemm(cfg->dtype);
    if (e != hipSuccess) {
      std::string msg = std::string("raising the GEMM kernels' LDS limit: ") + hipGetErrorString(e);
      delete ctx;
      return fail(nullptr, TSD_E_HIP, msg);
    }
  }
  if (ctx->fused_draft) {
    hipError_t e = prepare_draft_fused();
    if (e != hipSuccess) {
      std::string msg = std::string("raising the fused draft kernel's LDS limit: ") + hipGetErrorString(e);
      delete ctx;
      return fail(nullptr, TSD_E_HIP, msg);
    }
  }
  for (int w = 0; w < 2; ++w) {
    hipError_t e = prepare_attention(cfg->dtype, ctx->model[w].hd, cfg->max_tokens, cfg->page_tokens);
    if (e != hipSuccess) {
      std::string msg = std::string("raising the attention kernel's LDS limit: ") + hipGetErrorString(e);
      delete ctx;
      return fail(nullptr, TSD_E_HIP, msg);
    }
  }
  *out = ctx;
  return TSD_OK;
}

int tsd_destroy(tsd_ctx* ctx) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  hipError_t e = hipDeviceSynchronize();
  drop_graphs(ctx);
  if (ctx->host_counts) (void)hipHostFree(ctx->host_counts);
  for (auto& ev : ctx->prof_events) {
    (void)hipEventDestroy(ev.first);
    (void)hipEventDestroy(ev.second);
  }
  delete ctx;
  if (e != hipSuccess) return fail(nullptr, TSD_E_HIP, std::string("hipDeviceSynchronize: ") + hipGetErrorString(e));
  return TSD_OK;
}

int tsd_load_weights(tsd_ctx* ctx, int which, const float* blob_dev, size_t n_floats, void* stream) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (which != TSD_TARGET && which != TSD_DRAFT) return fail(ctx, TSD_E_INVALID_ARG, "which must be TSD_TARGET or TSD_DRAFT");
  if (!blob_dev) return fail(ctx, TSD_E_INVALID_ARG, "blob_dev is NULL");
  ModelDev& md = ctx->model[which];
  const tsd_config& c = ctx->cfg;
  if (n_floats != weights_count(md.c, c.patch)) return fail(ctx, TSD_E_INVALID_ARG, "n_floats does not match tsd_weights_count");
  hipStream_t st = (hipStream_t)stream;
  drop_graphs(ctx);
  const size_t D = md.c.d_model, F = md.c.d_ff, P = c.patch, es = ctx->es;
  const float* w = blob_dev;
  auto pack = [&](const float* W, const float* gain, void* out, int K, int N) {
    PackP p{W, gain, out, K, N};
    return launch_pack(c.dtype, p, st);
  };
  HIP_TRY(ctx, pack(w, nullptr, md.W_e, (int)P, (int)D));
  w += P * D;
  for (int l = 0; l < md.c.n_layers; ++l) {
    const float* g1 = w;
    w += D;
    for (int j = 0; j < 3; ++j) {  // W_q, W_k, W_v stacked as rows of one [3D][D] matrix
      HIP_TRY(ctx, pack(w, g1, md.layers[l].Wqkv + (size_t)j * D * D * es, (int)D, (int)D));
      w += D * D;
    }
    HIP_TRY(ctx, pack(w, nullptr, md.layers[l].Wo, (int)D, (int)D));
    w += D * D;
    const float* g2 = w;
    w += D;
    if (md.c.n_experts > 0) {
      const size_t E = md.c.n_experts;
      PackP pr{w, g2, md.layers[l].Wr, (int)D, (int)E};  // router stays fp32
      HIP_TRY(ctx, launch_pack(TSD_F32, pr, st));
      w += D * E;
      for (size_t e = 0; e < E; ++e) {
        HIP_TRY(ctx, pack(w, g2, md.layers[l].W1 + e * F * D * es, (int)D, (int)F));
        w += D * F;
        HIP_TRY(ctx, pack(w, nullptr, md.layers[l].W2 + e * D * F * es, (int)F, (int)D));
        w += F * D;
      }
    } else {
      HIP_TRY(ctx, pack(w, g2, md.layers[l].W1, (int)D, (int)F));
      w += D * F;
      HIP_TRY(ctx, pack(w, nullptr, md.layers[l].W2, (int)F, (int)D));
      w += F * D;
    }
  }
  const float* gf = w;
  w += D;
  HIP_TRY(ctx, pack(w, gf, md.W_h, (int)D, (int)P));
  if (which == TSD_DRAFT && ctx->fused_draft) {
    auto frag = [&](const char* src, char* dst, size_t N, size_t K, int heads) {
      return launch_repack_fragments(src, dst, (int)N, (int)K, draft_fused_chunk((int)D, (int)F), heads, (int)D, st);
    };
    HIP_TRY(ctx, frag(md.W_e, md.fW_e, D, P, 0));
    HIP_TRY(ctx, frag(md.W_h, md.fW_h, P, D, 0));
    for (int l = 0; l < md.c.n_layers; ++l) {
      HIP_TRY(ctx, frag(md.layers[l].Wqkv, md.flayers[l].Wqkv, 3 * D, D, md.c.n_heads));
      HIP_TRY(ctx, frag(md.layers[l].Wo, md.flayers[l].Wo, D, D, 0));
      HIP_TRY(ctx, frag(md.layers[l].W1, md.flayers[l].W1, F, D, 0));
      HIP_TRY(ctx, frag(md.layers[l].W2, md.flayers[l].W2, D, F, 0));
    }
  }
  md.loaded = true;
  return TSD_OK;
}

int tsd_prefill(tsd_ctx* ctx, const float* series_dev, int32_t B, int32_t n_ctx_patches, int32_t horizon_steps, void* stream) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (!ctx->model[0].loaded || !ctx->model[1].loaded) return fail(ctx, TSD_E_BAD_STATE, "weights of both models must be loaded first");
  if (!series_dev) return fail(ctx, TSD_E_INVALID_ARG, "series_dev is NULL");
  const tsd_config& c = ctx->cfg;
  if (B < 1 || n_ctx_patches < 2 || horizon_steps < 1) return fail(ctx, TSD_E_INVALID_ARG, "need B >= 1, n_ctx_patches >= 2, horizon_steps >= 1");
  if (B > c.max_batch) return fail(ctx, TSD_E_OUT_OF_RANGE, "B exceeds max_batch");
  const int P = c.patch, N = n_ctx_patches, T = (horizon_steps + P - 1) / P;
  if ((long)N + T + ctx->K_max > c.max_tokens) return fail(ctx, TSD_E_OUT_OF_RANGE, "n_ctx_patches + ceil(horizon/P) + K exceeds max_tokens");
  hipStream_t st = (hipStream_t)stream;
  ctx->prefilled = false;
  ctx->n_act = -1;
  ctx->seq_floor = ctx->seq_launched;
  ctx->compact_pending = false;
  ctx->k_round = 0;
  ctx->need_lb = T;  // every series needs all T patches
  drop_graphs(ctx);  // batch size, context length and horizon are baked into the captured launches
  // page table: every series reserves the pages its whole forecast can touch
  const int need = (N + T + ctx->K_max + c.page_tokens - 1) / c.page_tokens;
  std::vector<int> perm;
  if (c.flags & TSD_FLAG_SCRAMBLE_PAGES) {
    perm.resize(ctx->n_pages);
    for (int i = 0; i < ctx->n_pages; ++i) perm[i] = i;
    std::mt19937_64 rng(c.seed ^ 0x5bd1e995u);
    for (int i = ctx->n_pages - 1; i > 0; --i) std::swap(perm[i], perm[(size_t)(rng() % (uint64_t)(i + 1))]);
  }
  ctx->host_pt.assign((size_t)B * ctx->pages_per_series, 0);
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < need; ++j) {
      int phys = j * B + b;  // pages handed out position-major across the batch
      ctx->host_pt[(size_t)b * ctx->pages_per_series + j] = perm.empty() ? phys : perm[phys];
    }
  HIP_TRY(ctx, hipMemcpyAsync(ctx->page_table, ctx->host_pt.data(), ctx->host_pt.size() * 4, hipMemcpyHostToDevice, st));
  PrefillP pp{series_dev, ctx->znorm, ctx->mean, ctx->sdev, ctx->pending, ctx->prev, ctx->len, ctx->committed,
              ctx->round, ctx->active, ctx->stat, B, N, P, nullptr, 0, ctx->act_list, ctx->count_out, B, T};
  HIP_TRY(ctx, launch_prefill_stats(pp, st));
  ctx->B = B;
  ctx->N = N;
  ctx->T = T;
  ctx->H = horizon_steps;
  // context patches 0..N-2 through both models, in chunks of series that fit the workspace
  const int nq = N - 1;
  const int chunk = std::max(1, ctx->rows_max / nq);
  for (int which = 0; which < 2; ++which)
    for (int s0 = 0; s0 < B; s0 += chunk) {
      Pass ps;
      std::memset(&ps, 0, sizeof(ps));
      ps.which = which;
      ps.B = std::min(chunk, B - s0);
      ps.s0 = s0;
      ps.nq = nq;
      ps.base_pos = nullptr;
      ps.pos_off = 0;
      ps.src0 = ctx->znorm + (size_t)s0 * N * P;
      ps.stride0 = (long)N * P;
      ps.n0 = nq;
      ps.out = nullptr;
      int rc = run_pass(ctx, ps, st);
      if (rc) return rc;
    }
  ctx->prefilled = true;
  return TSD_OK;
}

int tsd_refill(tsd_ctx* ctx, const int32_t* slots_host, int32_t n, const float* series_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!slots_host || !series_dev) return fail(ctx, TSD_E_INVALID_ARG, "slots_host and series_dev must not be NULL");
  if (n < 1 || n > ctx->B) return fail(ctx, TSD_E_OUT_OF_RANGE, "n must be in 1..B of the running forecast");
  std::vector<char> seen((size_t)ctx->B, 0);
  for (int j = 0; j < n; ++j) {
    const int b = slots_host[j];
    if (b < 0 || b >= ctx->B) return fail(ctx, TSD_E_OUT_OF_RANGE, "slot index outside 0..B-1");
    if (seen[(size_t)b]) return fail(ctx, TSD_E_INVALID_ARG, "a slot is listed twice");
    seen[(size_t)b] = 1;
  }
  hipStream_t st = (hipStream_t)stream;
  const tsd_config& c = ctx->cfg;
  const int N = ctx->N, P = c.patch;
  HIP_TRY(ctx, hipStreamSynchronize(st));  // an earlier refill's list may still be in use
  ctx->host_refill.assign(slots_host, slots_host + n);
  HIP_TRY(ctx, hipMemcpyAsync(ctx->refill_list, ctx->host_refill.data(), (size_t)n * 4, hipMemcpyHostToDevice, st));
  PrefillP pp{series_dev, ctx->znorm, ctx->mean, ctx->sdev, ctx->pending, ctx->prev, ctx->len, ctx->committed,
              ctx->round, ctx->active, ctx->stat, n, N, P, ctx->refill_list, 1, nullptr, nullptr, 0, 0};
  HIP_TRY(ctx, launch_prefill_stats(pp, st));
  // every slot may be active again: identity list until the next tsd_num_active
  HIP_TRY(ctx, launch_identity_list(ctx->act_list, ctx->count_out, ctx->B, ctx->T, st));
  const int nq = N - 1;
  const int chunk = std::max(1, ctx->rows_max / nq);
  for (int which = 0; which < 2; ++which)
    for (int s0 = 0; s0 < n; s0 += chunk) {
      Pass ps;
      std::memset(&ps, 0, sizeof(ps));
      ps.which = which;
      ps.B = std::min(chunk, n - s0);
      ps.act = ctx->refill_list + s0;
      ps.nq = nq;
      ps.base_pos = nullptr;
      ps.pos_off = 0;
      ps.src0 = ctx->znorm;  // rows are gathered by slot
      ps.stride0 = (long)N * P;
      ps.n0 = nq;
      ps.out = nullptr;
      if ((rc = run_pass(ctx, ps, st))) return rc;
    }
  ctx->n_act = -1;  // the active list is stale until the next tsd_num_active
  ctx->seq_floor = ctx->seq_launched;
  ctx->compact_pending = false;
  ctx->k_round = 0;
  ctx->need_lb = 0;
  return TSD_OK;
}

int tsd_reset_decode(tsd_ctx* ctx, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  PrefillP pp{nullptr, ctx->znorm, ctx->mean, ctx->sdev, ctx->pending, ctx->prev, ctx->len, ctx->committed,
              ctx->round, ctx->active, ctx->stat, ctx->B, ctx->N, ctx->cfg.patch, nullptr, 0, ctx->act_list,
              ctx->count_out, ctx->B, ctx->T};
  HIP_TRY(ctx, launch_reset(pp, (hipStream_t)stream));
  ctx->n_act = -1;  // every series is active again
  ctx->seq_floor = ctx->seq_launched;
  ctx->compact_pending = false;
  ctx->k_round = 0;
  ctx->need_lb = ctx->T;  // every series needs all T patches again
  return TSD_OK;
}

int tsd_draft_propose(tsd_ctx* ctx, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  const tsd_config& c = ctx->cfg;
  const int P = c.patch, K = c.K;      // K: layout of the round tensors
  const int Kr = round_positions(ctx);  // positions proposed this round
  hipStream_t st = (hipStream_t)stream;
  ctx->injected = false;
  // Step 1 ingests two tokens per series: the token just before the pending one and the pending
  // one.  After a fully accepted round the draft cache lacks the former (it proposed x_K but
  // never consumed it); for the other series the rewrite stores identical values.
  const Cover cv = cover(ctx);
  if (cv.n == 0) return TSD_OK;
  if (ctx->fused_draft) {
    const ModelDev& md = ctx->model[TSD_DRAFT];
    DraftFusedP f;
    std::memset(&f, 0, sizeof(f));
    f.W_e = reinterpret_cast<const bf16*>(md.fW_e);
    f.W_h = reinterpret_cast<const bf16*>(md.fW_h);
    for (int l = 0; l < md.c.n_layers; ++l) {
      f.Wqkv[l] = reinterpret_cast<const bf16*>(md.flayers[l].Wqkv);
      f.Wo[l] = reinterpret_cast<const bf16*>(md.flayers[l].Wo);
      f.W1[l] = reinterpret_cast<const bf16*>(md.flayers[l].W1);
      f.W2[l] = reinterpret_cast<const bf16*>(md.flayers[l].W2);
    }
    f.kv_pool = reinterpret_cast<bf16*>(md.kv_pool);
    f.layer_pool_elems = md.layer_pool_bytes / 2;
    f.rope_cos = md.rope_cos;
    f.rope_sin = md.rope_sin;
    f.page_table = ctx->page_table;
    f.pt_stride = ctx->pages_per_series;
    f.len = ctx->len;
    f.act = cv.act;
    f.n_dev = cv.n_dev;
    f.n = cv.n;
    f.prev = ctx->prev;
    f.pending = ctx->pending;
    f.X = ctx->X;
    f.x_stride = (long)K * P;
    if (c.flags & TSD_FLAG_SAMPLE_PROPOSALS) {
      f.mu_q = ctx->mu_q;
      f.round = ctx->round;
      f.sigma_q = c.sigma_q;
      f.sigma_q_vec = ctx->diag_on ? ctx->diag + 2 * P : nullptr;
      f.key0 = (unsigned)(c.seed & 0xFFFFFFFFull);
      f.key1 = (unsigned)(c.seed >> 32);
    }
    f.Kr = Kr;
    f.L = md.c.n_layers;
    f.D = md.c.d_model;
    f.F = md.c.d_ff;
    f.Hh = md.c.n_heads;
    f.P = P;
    f.PT = c.page_tokens;
    f.pt_shift = __builtin_ctz(c.page_tokens);
    f.scale = 1.0f / std::sqrt((float)md.hd);
    f.chunk = draft_fused_chunk(f.D, f.F);
    f.trace = ctx->trace_on ? ctx->trace_buf : nullptr;
    f.trace_max = kTraceMax;
    // series per workgroup: two keep a workgroup's attention stage to one (series, head) pair per wavefront
    // at 4 heads; beyond 512 series more per workgroup keep the grid near one workgroup per compute unit.
    // (From the batch the handle was created for: a series' bits do not depend on who else is active.)
    f.spw = c.max_batch == 1 ? 1 : c.max_batch <= 512 ? 2 : c.max_batch <= 1024 ? 4 : 8;
    // work: the flops of the Kr + 1 token passes it replaces
    const double D = f.D, tok = (double)cv.n * (Kr + 1);
    const double flops = 2.0 * tok * (2.0 * P * D + f.L * (4.0 * D * D + 2.0 * D * f.F));
    HIP_TRY(ctx, timed_launch(ctx, TSD_K_DRAFT, flops, st, [&] { return launch_draft_fused(f, st); }, Shape{TSD_DRAFT, 0, cv.n, Kr, 0}));
    return TSD_OK;
  }
  Pass ps;
  std::memset(&ps, 0, sizeof(ps));
  ps.which = TSD_DRAFT;
  ps.B = cv.n;
  ps.act = cv.act;
  ps.n_dev = cv.n_dev;
  ps.nq = 2;
  ps.base_pos = ctx->len;
  ps.pos_off = -1;
  ps.src0 = ctx->prev;
  ps.stride0 = P;
  ps.n0 = 1;
  ps.src1 = ctx->pending;
  ps.stride1 = P;
  // Sampled proposals: the head writes mu_q^(i) to its own buffer and a small kernel adds
  // sigma_q * eps into X, which the next step (and the target) then consume.
  const bool sampled = (c.flags & TSD_FLAG_SAMPLE_PROPOSALS) != 0;
  float* head_out = sampled ? ctx->mu_q : ctx->X;
  auto draw = [&](int i) -> int {
    if (!sampled) return TSD_OK;
    SampleP sp;
    std::memset(&sp, 0, sizeof(sp));
    sp.mu_q = ctx->mu_q;
    sp.X = ctx->X;
    sp.act = cv.act;
    sp.n_dev = cv.n_dev;
    sp.round = ctx->round;
    sp.n = cv.n;
    sp.K = K;
    sp.P = P;
    sp.i = i;
    sp.sigma_q = c.sigma_q;
    sp.sigma_q_vec = ctx->diag_on ? ctx->diag + 2 * P : nullptr;
    sp.key0 = (unsigned)(c.seed & 0xFFFFFFFFull);
    sp.key1 = (unsigned)(c.seed >> 32);
    HIP_TRY(ctx, launch_sample(sp, st));
    return TSD_OK;
  };
  ps.out = head_out;
  ps.out_stride_b = (long)K * P;
  ps.t_skip = 1;
  if ((rc = run_pass(ctx, ps, st))) return rc;
  if ((rc = draw(1))) return rc;
  for (int i = 2; i <= Kr; ++i) {  // step i consumes x_{i-1} at position len + i - 1, emits x_i
    std::memset(&ps, 0, sizeof(ps));
    ps.which = TSD_DRAFT;
    ps.B = cv.n;
    ps.act = cv.act;
    ps.n_dev = cv.n_dev;
    ps.nq = 1;
    ps.base_pos = ctx->len;
    ps.pos_off = i - 1;
    ps.src0 = ctx->X + (size_t)(i - 2) * P;
    ps.stride0 = (long)K * P;
    ps.n0 = 1;
    ps.out = head_out + (size_t)(i - 1) * P;
    ps.out_stride_b = (long)K * P;
    ps.t_skip = 0;
    if ((rc = run_pass(ctx, ps, st))) return rc;
    if ((rc = draw(i))) return rc;
  }
  return TSD_OK;
}

int tsd_target_verify(tsd_ctx* ctx, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  const tsd_config& c = ctx->cfg;
  const int P = c.patch, K = c.K;
  const int Kr = round_positions(ctx);  // boundaries beyond Kr + 1 belong to patches no active series can commit
  const Cover cv = cover(ctx);
  if (cv.n == 0) return TSD_OK;
  Pass ps;
  std::memset(&ps, 0, sizeof(ps));
  ps.which = TSD_TARGET;
  ps.B = cv.n;
  ps.act = cv.act;
  ps.n_dev = cv.n_dev;
  ps.nq = Kr + 1;
  ps.base_pos = ctx->len;
  ps.pos_off = 0;
  ps.src0 = ctx->pending;
  ps.stride0 = P;
  ps.n0 = 1;
  ps.src1 = ctx->X;
  ps.stride1 = (long)K * P;
  ps.out = ctx->mu_p;
  ps.out_stride_b = (long)(K + 1) * P;
  ps.t_skip = 0;
  if (c.flags & TSD_FLAG_NAIVE_VERIFY) {
    // Ablation "w/o single-pass verification": every prefix [pending, x_1..x_{i-1}] is encoded by
    // a pass of its own and only its last boundary is read, so a round costs (K+1)(K+2)/2 target
    // tokens instead of K+1.  (Each pass rewrites the same KV entries with the same values.)
    for (int i = 1; i <= Kr + 1; ++i) {
      ps.nq = i;
      ps.t_skip = i - 1;
      ps.out = ctx->mu_p + (size_t)(i - 1) * P;
      if ((rc = run_pass(ctx, ps, (hipStream_t)stream))) return rc;
    }
    return TSD_OK;
  }
  return run_pass(ctx, ps, (hipStream_t)stream);
}

int tsd_accept_commit(tsd_ctx* ctx, const int32_t* forced_len_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  return accept_commit_impl(ctx, forced_len_dev, ctx->cfg.K, (hipStream_t)stream);
}

int tsd_round(tsd_ctx* ctx, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  // With pinned host words at hand the round ends with the compaction tsd_num_active would otherwise have to
  // launch, copy back and wait for: the caller's next tsd_num_active only watches the host words.
  const bool deliver = ctx->host_counts && ctx->seq_ready;
  const int need_before = ctx->need_lb;  // a round commits at most K + 1 patches per series
  if (!(ctx->cfg.flags & TSD_FLAG_NO_COMPACT)) peek_counts(ctx);
  const int cls = device_counts(ctx) ? size_class(ctx) : 0;
  ctx->capture_rows = class_rows(ctx, cls);
  rc = run_graphed(ctx, &ctx->graph_round[round_positions(ctx)][cls], (hipStream_t)stream, [&]() {
    int r;
    if ((r = tsd_draft_propose(ctx, stream))) return r;
    if ((r = tsd_target_verify(ctx, stream))) return r;
    if ((r = tsd_accept_commit(ctx, nullptr, stream))) return r;
    if (deliver)
      HIP_TRY(ctx, launch_compact_active(ctx->active, ctx->committed, ctx->T, ctx->B, compact_target(ctx), ctx->count_out,
                                         ctx->host_counts, (hipStream_t)stream));
    return (int)TSD_OK;
  });
  if (rc == TSD_OK) {
    // (a replayed graph does not pass through accept_commit_impl: keep the bound on the patches still needed honest here)
    ctx->need_lb = std::max(0, need_before - (ctx->cfg.K + 1));
    if (deliver) {
      ctx->seq_launched++;
      ctx->compact_pending = true;
    }
  }
  return rc;
}

int tsd_target_step(tsd_ctx* ctx, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  const int P = ctx->cfg.patch;
  return run_graphed(ctx, &ctx->graph_step, (hipStream_t)stream, [&]() {
    Pass ps;
    std::memset(&ps, 0, sizeof(ps));
    const Cover cv = cover(ctx);
    if (cv.n == 0) return TSD_OK;
    ps.which = TSD_TARGET;
    ps.B = cv.n;
    ps.act = cv.act;
    ps.n_dev = cv.n_dev;
    ps.nq = 1;
    ps.base_pos = ctx->len;
    ps.pos_off = 0;
    ps.src0 = ctx->pending;
    ps.stride0 = P;
    ps.n0 = 1;
    ps.out = ctx->mu_p;
    ps.out_stride_b = P;
    ps.t_skip = 0;
    int r = run_pass(ctx, ps, (hipStream_t)stream);
    if (r) return r;
    return accept_commit_impl(ctx, nullptr, 0, (hipStream_t)stream);  // K = 0: commit the target's mean
  }, /*counts=*/false);  // target-only decoding finishes every series in the same step: nothing to compact
}

int tsd_num_active(tsd_ctx* ctx, int32_t* out_host, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!out_host) return fail(ctx, TSD_E_INVALID_ARG, "out_host is NULL");
  hipStream_t st = (hipStream_t)stream;
  int32_t both[2] = {0, 0};
  if (ctx->host_counts && ctx->seq_ready) {
    if (!ctx->compact_pending) {
      HIP_TRY(ctx, launch_compact_active(ctx->active, ctx->committed, ctx->T, ctx->B, compact_target(ctx), ctx->count_out,
                                         ctx->host_counts, st));
      ctx->seq_launched++;
    }
    ctx->compact_pending = false;
    // Watch the pinned words for this launch's number (stored last by the kernel); a wait on the stream
    // is the fallback if it does not show up within a second.
    const auto t0 = std::chrono::steady_clock::now();
    bool seen = false;
    for (unsigned spins = 0;; ++spins) {
      if (__atomic_load_n(&ctx->host_counts[2], __ATOMIC_ACQUIRE) == ctx->seq_launched) {
        seen = true;
        break;
      }
      if ((spins & 1023) == 1023 && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(1)) break;
      __builtin_ia32_pause();
    }
    if (!seen) {
      HIP_TRY(ctx, hipStreamSynchronize(st));
      if (__atomic_load_n(&ctx->host_counts[2], __ATOMIC_ACQUIRE) != ctx->seq_launched)
        return fail(ctx, TSD_E_HIP, "the active-series count was not delivered");
    }
    both[0] = ctx->host_counts[0];
    both[1] = ctx->host_counts[1];
  } else {
    HIP_TRY(ctx, launch_compact_active(ctx->active, ctx->committed, ctx->T, ctx->B, compact_target(ctx), ctx->count_out, nullptr, st));
    HIP_TRY(ctx, hipMemcpyAsync(both, ctx->count_out, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
  }
  // the list that belongs to these counts is the one the last compaction wrote: it becomes the list the passes read
  // (enqueued behind everything that still reads the old one)
  if (!device_counts(ctx))
    HIP_TRY(ctx, launch_copy(ctx->act_list, ctx->act_list_next, ((size_t)ctx->B * 4 + 15) & ~(size_t)15, st));
  *out_host = both[0];
  if (!(ctx->cfg.flags & TSD_FLAG_NO_COMPACT)) {
    ctx->n_act = both[0];    // later passes cover only these series ...
    ctx->k_round = both[1];  // ... and only the positions one of them can still commit
  }
  ctx->need_lb = both[1];
  return TSD_OK;
}

int tsd_run_rounds(tsd_ctx* ctx, int32_t max_rounds, int32_t* rounds_host, int32_t* active_host, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (max_rounds < 1) return fail(ctx, TSD_E_INVALID_ARG, "max_rounds must be at least 1");
  int32_t rounds = 0, active = -1;
  while (rounds < max_rounds) {
    if ((rc = tsd_round(ctx, stream))) return rc;  // lowers need_lb (a bound on the most patches any series still needs) by K + 1
    ++rounds;
    // (handles whose passes are sized on the host need every count: it is what shrinks their passes)
    // (a running measurement asks every time, so that the rows it books for a launch are the rows the launch runs)
    if (ctx->need_lb > 0 && rounds < max_rounds && device_counts(ctx) && ctx->prof_class < 0) continue;  // somebody still needs patches: no need to ask
    if ((rc = tsd_num_active(ctx, &active, stream))) return rc;
    if (active == 0) break;
  }
  if (rounds_host) *rounds_host = rounds;
  if (active_host) *active_host = active;
  return TSD_OK;
}

int tsd_get_forecast(tsd_ctx* ctx, float* out_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!out_dev) return fail(ctx, TSD_E_INVALID_ARG, "out_dev is NULL");
  HIP_TRY(ctx, launch_forecast_out(ctx->forecast, ctx->mean, ctx->sdev, ctx->committed, out_dev, ctx->B, ctx->cfg.patch,
                                   ctx->T, ctx->H, (hipStream_t)stream));
  return TSD_OK;
}

int tsd_get_round_io(tsd_ctx* ctx, float* X_dev, float* mu_q_dev, float* mu_p_dev, int32_t* n_acc_dev, float* ell_dev,
                     float* logu_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const size_t B = ctx->B, K = ctx->cfg.K, P = ctx->cfg.patch;
  auto cp = [&](void* dst, const void* src, size_t bytes) {
    return dst ? hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) : hipSuccess;
  };
  HIP_TRY(ctx, cp(X_dev, ctx->X, B * K * P * 4));
  // mean proposals: x_i = mu_q^(i), one buffer; sampled proposals keep the means beside the draws
  HIP_TRY(ctx, cp(mu_q_dev, (ctx->cfg.flags & TSD_FLAG_SAMPLE_PROPOSALS) ? ctx->mu_q : ctx->X, B * K * P * 4));
  HIP_TRY(ctx, cp(mu_p_dev, ctx->mu_p, B * (K + 1) * P * 4));
  HIP_TRY(ctx, cp(n_acc_dev, ctx->n_acc, B * 4));
  HIP_TRY(ctx, cp(ell_dev, ctx->ell, B * K * 4));
  HIP_TRY(ctx, cp(logu_dev, ctx->logu, B * K * 4));
  return TSD_OK;
}

int tsd_set_round_io(tsd_ctx* ctx, const float* X_dev, const float* mu_q_dev, const float* mu_p_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!X_dev || !mu_q_dev || !mu_p_dev) return fail(ctx, TSD_E_INVALID_ARG, "X_dev, mu_q_dev and mu_p_dev are all required");
  hipStream_t st = (hipStream_t)stream;
  const size_t B = ctx->B, K = ctx->cfg.K, P = ctx->cfg.patch;
  HIP_TRY(ctx, hipMemcpyAsync(ctx->X, X_dev, B * K * P * 4, hipMemcpyDeviceToDevice, st));
  HIP_TRY(ctx, hipMemcpyAsync(ctx->mu_q, mu_q_dev, B * K * P * 4, hipMemcpyDeviceToDevice, st));
  HIP_TRY(ctx, hipMemcpyAsync(ctx->mu_p, mu_p_dev, B * (K + 1) * P * 4, hipMemcpyDeviceToDevice, st));
  ctx->injected = true;
  return TSD_OK;
}

int tsd_get_state(tsd_ctx* ctx, int32_t* len_dev, int32_t* committed_dev, float* pending_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const size_t B = ctx->B, P = ctx->cfg.patch;
  if (len_dev) HIP_TRY(ctx, hipMemcpyAsync(len_dev, ctx->len, B * 4, hipMemcpyDeviceToDevice, st));
  if (committed_dev) HIP_TRY(ctx, hipMemcpyAsync(committed_dev, ctx->committed, B * 4, hipMemcpyDeviceToDevice, st));
  if (pending_dev) HIP_TRY(ctx, hipMemcpyAsync(pending_dev, ctx->pending, B * P * 4, hipMemcpyDeviceToDevice, st));
  return TSD_OK;
}

int tsd_get_stats(tsd_ctx* ctx, tsd_stats* out_host, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!out_host) return fail(ctx, TSD_E_INVALID_ARG, "out_host is NULL");
  hipStream_t st = (hipStream_t)stream;
  long long h[5];
  HIP_TRY(ctx, launch_sum_stats(ctx->stat, ctx->B, ctx->stats_out, st));
  HIP_TRY(ctx, hipMemcpyAsync(h, ctx->stats_out, sizeof(h), hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipStreamSynchronize(st));
  out_host->rounds = h[0];
  out_host->tested = h[1];
  out_host->accepted = h[2];
  out_host->committed = h[3];
  out_host->near_ties = h[4];
  return TSD_OK;
}

int tsd_get_series_stats(tsd_ctx* ctx, int64_t* out_dev, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!out_dev) return fail(ctx, TSD_E_INVALID_ARG, "out_dev is NULL");
  static_assert(sizeof(long long) == sizeof(int64_t), "counter width");
  HIP_TRY(ctx, hipMemcpyAsync(out_dev, ctx->stat, (size_t)ctx->B * 5 * sizeof(int64_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return TSD_OK;
}

int tsd_set_route_tap(tsd_ctx* ctx, int which, int32_t* ids_dev, size_t n_ints) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (which != TSD_TARGET && which != TSD_DRAFT) return fail(ctx, TSD_E_INVALID_ARG, "which must be TSD_TARGET or TSD_DRAFT");
  const tsd_model_cfg& m = ctx->model[which].c;
  if (ids_dev) {
    if (m.n_experts == 0) return fail(ctx, TSD_E_BAD_STATE, "this model has a dense FFN: there are no routing choices to record");
    const size_t need = (size_t)m.n_layers * ctx->cfg.max_batch * ctx->cfg.max_tokens * m.top_k;
    if (n_ints < need) return fail(ctx, TSD_E_INVALID_ARG, "ids_dev must hold n_layers * max_batch * max_tokens * top_k int32");
  }
  ctx->route_tap[which] = ids_dev;
  drop_graphs(ctx);  // the captured launch sequences do not contain the tap's copies
  return TSD_OK;
}

int tsd_profile_begin(tsd_ctx* ctx, int kernel_class) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (kernel_class < -1 || kernel_class > TSD_K_COUNT) return fail(ctx, TSD_E_INVALID_ARG, "kernel_class must be a TSD_K_* value, TSD_K_COUNT (every family) or -1");
  ctx->prof_class = kernel_class;
  ctx->prof_used = 0;
  ctx->prof_work = 0;
  ctx->prof_recs.clear();
  return TSD_OK;
}

int tsd_profile_end(tsd_ctx* ctx, int64_t* launches_host, double* ms_host, double* work_host, void* stream) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (!launches_host || !ms_host || !work_host) return fail(ctx, TSD_E_INVALID_ARG, "output pointers must not be NULL");
  if (ctx->prof_class < 0) return fail(ctx, TSD_E_BAD_STATE, "tsd_profile_begin has not selected a kernel class");
  ctx->prof_class = -1;
  HIP_TRY(ctx, hipStreamSynchronize((hipStream_t)stream));
  double ms = 0;
  for (size_t i = 0; i < ctx->prof_used; ++i) {
    float t = 0;
    HIP_TRY(ctx, hipEventElapsedTime(&t, ctx->prof_events[i].first, ctx->prof_events[i].second));
    ms += t;
    if (i < ctx->prof_recs.size()) ctx->prof_recs[i].ms = t;
  }
  *launches_host = (int64_t)ctx->prof_used;
  *ms_host = ms;
  *work_host = ctx->prof_work;
  ctx->prof_used = 0;
  return TSD_OK;
}

int tsd_profile_launches(tsd_ctx* ctx, tsd_launch_rec* out_host, int32_t max_records, int32_t* n_host) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (!n_host || (max_records > 0 && !out_host) || max_records < 0) return fail(ctx, TSD_E_INVALID_ARG, "need n_host, and out_host for max_records > 0");
  if (ctx->prof_class >= 0) return fail(ctx, TSD_E_BAD_STATE, "a measurement is still running: call tsd_profile_end first");
  *n_host = (int32_t)ctx->prof_recs.size();
  for (size_t i = 0; i < ctx->prof_recs.size() && i < (size_t)max_records; ++i) out_host[i] = ctx->prof_recs[i];
  return TSD_OK;
}

int tsd_bench_gemm(int dtype, int variant, int M, int N, int K, const void* A_dev, const void* Wt_dev, void* C_dev,
                   void* stream) {
  const int no_wide = (variant & 8) ? 1 : 0;  // + 8: never the wide-tile kernels
  variant &= ~8;
  if (variant < 0 || variant > 3) return fail(nullptr, TSD_E_INVALID_ARG, "variant must be 0, 1, 2 or 3 (+ 8)");
  if (variant == 3 && dtype != TSD_BF16) return fail(nullptr, TSD_E_INVALID_ARG, "variant 3 is bf16 only");
  if (dtype != TSD_F32 && dtype != TSD_BF16) return fail(nullptr, TSD_E_INVALID_ARG, "dtype must be TSD_F32 or TSD_BF16");
  if (M < 1 || N < 4 || K < 8 || (K % 8) || (N % 4)) return fail(nullptr, TSD_E_INVALID_ARG, "need M >= 1, N a multiple of 4, K a multiple of 8");
  if (!A_dev || !Wt_dev || !C_dev) return fail(nullptr, TSD_E_INVALID_ARG, "device pointers must not be NULL");
  static bool prepared = false;
  if (!prepared) {
    HIP_TRY(nullptr, prepare_gemm(TSD_BF16));
    prepared = true;
  }
  GemmP g;
  std::memset(&g, 0, sizeof(g));
  g.allow_skinny = 1;  // products of at most 32 rows take the skinny kernel, as in a small-batch handle
  g.no_wide = no_wide;
  g.M = M;
  g.N = N;
  g.K = K;
  g.nq = 1;
  g.A = A_dev;
  g.W = Wt_dev;
  g.Cf = reinterpret_cast<float*>(C_dev);
  if (variant == 3) {  // the FFN-up product as the passes run it: fused norm, GELU, result in the compute dtype
    g.Cf = nullptr;
    g.Ct = C_dev;
    HIP_TRY(nullptr, launch_gemm(dtype, A_NORM, EP_GELU, g, (hipStream_t)stream));
    return TSD_OK;
  }
  HIP_TRY(nullptr, launch_gemm(dtype, variant == 1 ? A_NORM : A_ACT, variant == 2 ? EP_RESID : EP_STORE, g, (hipStream_t)stream));
  return TSD_OK;
}

int tsd_bench_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev) return fail(nullptr, TSD_E_INVALID_ARG, "device pointers must not be NULL");
  if (bytes == 0 || (bytes % 16) || ((uintptr_t)dst_dev % 16) || ((uintptr_t)src_dev % 16))
    return fail(nullptr, TSD_E_INVALID_ARG, "bytes and both pointers must be non-zero multiples of 16");
  HIP_TRY(nullptr, launch_copy(dst_dev, src_dev, bytes, (hipStream_t)stream));
  return TSD_OK;
}

int tsd_trace_draft(tsd_ctx* ctx, int64_t* ticks_host, int32_t max_ticks, int32_t* n_host, void* stream) {
  int rc = require_ready(ctx, true);
  if (rc) return rc;
  if (!ticks_host || !n_host) return fail(ctx, TSD_E_INVALID_ARG, "ticks_host and n_host must not be NULL");
  if (max_ticks < 1) return fail(ctx, TSD_E_INVALID_ARG, "max_ticks must be positive");
  if (!ctx->fused_draft) return fail(ctx, TSD_E_BAD_STATE, "this handle runs the draft phase kernel by kernel: there are no stages to stamp");
  hipStream_t st = (hipStream_t)stream;
  static_assert(sizeof(long long) == 2 * sizeof(int), "the stamp buffer is cleared as ints");
  HIP_TRY(ctx, launch_fill_int(reinterpret_cast<int*>(ctx->trace_buf), 0, 2 * kTraceMax, st));
  ctx->trace_on = true;
  rc = tsd_draft_propose(ctx, stream);
  ctx->trace_on = false;
  if (rc) return rc;
  std::vector<long long> h(kTraceMax);
  HIP_TRY(ctx, hipMemcpyAsync(h.data(), ctx->trace_buf, sizeof(long long) * kTraceMax, hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipStreamSynchronize(st));
  int n = 0;
  while (n < kTraceMax && h[n] != 0) ++n;
  *n_host = n;
  for (int i = 0; i < n && i < max_ticks; ++i) ticks_host[i] = h[i];
  return TSD_OK;
}

int tsd_bench_mfma(int32_t blocks, int32_t iters, float* sink_dev, void* stream) {
  if (!sink_dev) return fail(nullptr, TSD_E_INVALID_ARG, "sink_dev must not be NULL");
  if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24))
    return fail(nullptr, TSD_E_INVALID_ARG, "need 1..65536 blocks and 1..2^24 iters");
  HIP_TRY(nullptr, launch_mfma_peak(blocks, iters, sink_dev, (hipStream_t)stream));
  return TSD_OK;
}

int tsd_set_accept_override(tsd_ctx* ctx, float alpha) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (alpha > 1.f || alpha == 0.f || std::isnan(alpha)) return fail(ctx, TSD_E_INVALID_ARG, "alpha must be in (0, 1], or negative to disable");
  ctx->alpha_override = alpha < 0.f ? -1.f : alpha;
  drop_graphs(ctx);
  return TSD_OK;
}

int tsd_set_block_size(tsd_ctx* ctx, int32_t K) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (K < 1 || K > ctx->K_max) return fail(ctx, TSD_E_OUT_OF_RANGE, "K must be in 1..K of tsd_create");
  if (K != ctx->cfg.K) {
    ctx->cfg.K = K;
    ctx->k_round = 0;
    ctx->injected = false;  // injected round tensors were laid out for the old K
    drop_graphs(ctx);
  }
  return TSD_OK;
}

int tsd_set_sigma(tsd_ctx* ctx, float sigma_p, float sigma_q) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (!(sigma_p > 0.f) || !(sigma_q > 0.f) || !std::isfinite(sigma_p) || !std::isfinite(sigma_q))
    return fail(ctx, TSD_E_INVALID_ARG, "sigma_p and sigma_q must be positive and finite");
  if (ctx->cfg.fallback_r > sigma_p) return fail(ctx, TSD_E_INVALID_ARG, "sigma_p must not fall below fallback_r");
  ctx->cfg.sigma_p = sigma_p;
  ctx->cfg.sigma_q = sigma_q;
  ctx->diag_on = false;
  drop_graphs(ctx);
  return TSD_OK;
}

int tsd_set_sigma_diag(tsd_ctx* ctx, const float* sigma_p_dev, const float* sigma_q_dev, void* stream) {
  if (!ctx) return fail(nullptr, TSD_E_INVALID_ARG, "ctx is NULL");
  if (!sigma_p_dev || !sigma_q_dev) return fail(ctx, TSD_E_INVALID_ARG, "sigma_p_dev and sigma_q_dev are both required");
  const int P = ctx->cfg.patch;
  hipStream_t st = (hipStream_t)stream;
  std::vector<float> sp(P), sq(P), pack(3 * (size_t)P + 1);
  HIP_TRY(ctx, hipMemcpyAsync(sp.data(), sigma_p_dev, (size_t)P * 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipMemcpyAsync(sq.data(), sigma_q_dev, (size_t)P * 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipStreamSynchronize(st));
  double logdet = 0.0;
  float min_sp = INFINITY;
  for (int e = 0; e < P; ++e) {
    if (!(sp[e] > 0.f) || !(sq[e] > 0.f) || !std::isfinite(sp[e]) || !std::isfinite(sq[e]))
      return fail(ctx, TSD_E_INVALID_ARG, "every per-dimension scale must be positive and finite");
    pack[e] = (float)(1.0 / (2.0 * (double)sp[e] * sp[e]));
    pack[P + e] = (float)(1.0 / (2.0 * (double)sq[e] * sq[e]));
    pack[2 * P + e] = sq[e];
    logdet += std::log((double)sq[e] * sq[e]) - std::log((double)sp[e] * sp[e]);
    min_sp = std::min(min_sp, sp[e]);
  }
  if (ctx->cfg.fallback_r > min_sp) return fail(ctx, TSD_E_INVALID_ARG, "no target scale may fall below fallback_r");
  pack[3 * (size_t)P] = (float)(logdet / (2.0 * P));
  HIP_TRY(ctx, hipMemcpy(ctx->diag, pack.data(), pack.size() * 4, hipMemcpyHostToDevice));
  ctx->diag_on = true;
  drop_graphs(ctx);
  return TSD_OK;
}

}  // extern "C"
