// C ABI of libpass_hip.so: context, arena layout, paged K/V bookkeeping, the step schedule and
// Algorithm 1's loop.  All arithmetic of the method runs in the kernels this file launches.
#include <limits.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <map>
#include <string>
#include <tuple>
#include <vector>

#include "pass_internal.h"

using namespace pass;

namespace {

struct Arena {
  char *base;
  size_t off;
  template <typename T>
  T *take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T *p = base ? (T *)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

struct LayerW {
  void *attn_norm, *wqkv, *wo, *ffn_norm, *wgu, *wdown;
};

struct Slot {
  int state = 0;  // 0 empty, 1 ready for draft, 2 ready for verify
  int kv_len = 0, n_gen = 0;
  uint32_t seq_id = 0;
  uint32_t iteration = 0;  // iterations of Algorithm 1 / 2 completed (mirror of the device counter)
  std::vector<int> pages;
};

// Workspace of the look-ahead embedding training (caller's memory, carved by carve_train)
struct TrainWs {
  bool on = false;
  bool mfma = false;  // the context runs on the matrix-core path: packed transposes of the weights, gradients as tiles
  int64_t step = 0;   // optimiser steps taken (AdamW's bias correction)
  float *master, *m1, *m2, *grad;                    // [k][d] fp32: trained values, AdamW moments, last gradient
  // what the backward pass needs of every layer, [L][kMaxRows][..]: the residual stream before the two norms (d each),
  // the layer's q | k | v workspace (3D; the rotated queries are what is used), the attention output (D) and the
  // ln-sum-exp of its rows (H), the gate | up pre-activations (2F).  The forward pass writes them in place: its
  // workspace pointers are set to the layer's area.
  float *save_h0, *save_h1, *save_qkv, *save_attn, *save_lse, *save_gu;
  float *save_hl;                                    // [kMaxRows][d] residual stream before the final norm
  float *logits;                                     // [kMaxRows][V] logits, then d loss / d logits
  float *dh, *dxn, *dattn, *dqkv, *dact, *dgu;       // gradients of the rows' activations
  float *part;                                       // [kTrainSplits][kMaxRows][max(d, D, F)] slice sums of a transposed projection
  float *dq_part;                                    // [kTrainAttnSplits][kMaxRows][D] the key chunks' shares of dq
  // matrix-core path: the weights' transposes in packed tiles (dx = W^T dy is then the forward pass's own product),
  // and the (hi, lo) tiles of the gradient that is the next product's input [2 * kMaxRows * max(V, 2F, 3D, d)]
  void *lm_head_t = nullptr;
  std::vector<LayerW> layers_t;  // wqkv, wo, wgu, wdown: the transposes; the norm gains are unused
  uint16_t *x = nullptr;
  float *row_loss;                                   // [kMaxRows]
  int32_t *targets;                                  // [kMaxRows] target token of a row, -1 = no loss
};

constexpr int kReportStride = 4 + kMaxK + kMaxK + 1 + 1;  // ... and the slot's iteration counter

// Scratch of pass_draft_static: the attention partials (running maximum, sum and accumulator of
// every (row, head, split)) of one call, for callers that may not allocate.  One copy per GPU,
// held until the process ends; its contents are whatever the last call left.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
unsigned char *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, set by pass_create

// bytes of attention partials a call of M rows needs: [M][H][kMaxSplits] triples (m, l, acc[hd])
size_t partials_bytes(const pass_config &c, int M) {
  return (size_t)M * c.n_heads * kMaxSplits * (c.head_dim + 2) * sizeof(float);
}

}  // namespace

struct pass_ctx {
  pass_config cfg;
  hipStream_t stream;
  Params P;
  size_t esz;  // bytes per model element
  // weights (arena)
  void *tok_emb, *lm_head, *final_norm, *lookahead, *staging;
  size_t staging_bytes;
  std::vector<LayerW> layers;
  bool weights_loaded = false;
  bool use_mfma = false;  // matrix-core path active (set by pass_load_weights)
  int opt_graph = 0, opt_path = 0, opt_attn = 0;
  // device scratch
  int32_t *prompt_buf;
  // host
  std::vector<Slot> slots;
  std::vector<int> free_pages;
  int32_t *report_host = nullptr;       // pinned, written by the report kernel; two reports (one may be in flight)
  int32_t *block_table_host = nullptr;  // pinned mirror of P.block_table
  hipEvent_t ev[3];
  hipEvent_t ev2[2][4];  // run_iterations: per in-flight iteration, start / middle / end of the calls and report landed
  int kv_slack = 0;      // positions an unreported iteration may have added to every running slot
  int device = 0;        // the GPU the context lives on (current when pass_create ran)
  bool static_scratch = false;  // this call keeps its attention partials in the library's static array (pass_draft_static)
  // optional timing of the dominant kernel (the gate/up GEMM): one event pair per layer
  // captured (model call + epilogue) graphs, keyed by everything that is baked into the launches:
  // mode, batch, attention grid width, sampling arguments
  typedef std::tuple<int, int, int, uint32_t, uint32_t, uint32_t, int, int, int, int, int> GraphKey;
  int row_base = 0;  // SampleArgs::row_base of the calls issued now (pass_sps_iteration's drafting steps)
  std::map<GraphKey, hipGraphExec_t> graphs;
  int opt_kernel_timing = 0;
  GemmTuning tuning;
  TrainWs train;
  float *train_loss_host = nullptr;  // pinned [kMaxRows]  // launch shapes of the decode GEMMs (captured graphs carry them: cleared when it changes)
  int opt_prefill_chunk = 64;
  int opt_prefill_tiled = -1;  // -1: prompts of more than 2 * kMaxRows rows take the tiled pass; 0 never; 1 always
  Params PP;                   // P with the row buffers of the tiled prompt pass
  PrefillWs pws;
  std::vector<hipEvent_t> kev;
  double kernel_ms = 0;
  int64_t kernel_launches = 0;
  std::string err;
};

namespace {

std::string g_create_error;  // message of the last failed pass_create (no context exists yet)

int fail(pass_ctx *c, int code, const char *fmt, ...) {
  if (c) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    c->err = buf;
  }
  return code;
}

#define HIP_TRY(c, call)                                                                         \
  do {                                                                                           \
    hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess) return fail((c), PASS_EDEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

bool config_ok(const pass_config *c, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return false; };
  if (!c) return bad("null config");
  if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->d_ffn < 8 || c->vocab < 2) return bad("bad shape");
  if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (c->d_model % 8 || c->d_ffn % 8) return bad("d_model and d_ffn must be multiples of 8");
  if (c->dtype != PASS_F32 && c->dtype != PASS_BF16) return bad("dtype must be PASS_F32 or PASS_BF16");
  if (c->k < 0 || c->k > kMaxK) return bad("k out of range");
  if (c->max_slots < 1 || (1 + c->k) * c->max_slots > kMaxRows) return bad("(1+k)*max_slots exceeds PASS_MAX_ROWS");
  if (c->max_seq_len < 2 + c->k) return bad("max_seq_len too small");
  if (c->max_seq_len > 65536) return bad("max_seq_len above 65536");
  if (c->page_size < 16 || (c->page_size & (c->page_size - 1))) return bad("page_size must be a power of two >= 16");
  if (c->n_pages < 0) return bad("n_pages negative");
  if (!(c->rms_eps > 0) || !(c->rope_base > 1)) return bad("rms_eps / rope_base");
  return true;
}

int pages_per_seq(const pass_config &c) { return (c.max_seq_len + c.page_size - 1) / c.page_size; }
int pool_pages(const pass_config &c) { return c.n_pages ? c.n_pages : c.max_slots * pages_per_seq(c); }

// Carve the arena.  With base == nullptr only the size is computed.
size_t carve(const pass_config &c, char *base, pass_ctx *ctx) {
  Arena A{base, 0};
  const size_t esz = c.dtype == PASS_F32 ? 4 : 2;
  const size_t d = c.d_model, D = (size_t)c.n_heads * c.head_dim, F = c.d_ffn, V = c.vocab, S = c.max_slots;
  const size_t M = kMaxRows;
  const int pps = pages_per_seq(c);
  const int np = pool_pages(c);
  Params P;
  memset(&P, 0, sizeof P);
  P.L = c.n_layers; P.d = c.d_model; P.H = c.n_heads; P.hd = c.head_dim; P.D = (int)D; P.F = c.d_ffn; P.V = c.vocab;
  P.k = c.k; P.k_act = c.k; P.la_token = -1; P.max_slots = c.max_slots; P.max_seq_len = c.max_seq_len; P.page_size = c.page_size;
  P.page_shift = __builtin_ctz(c.page_size); P.n_pages = np; P.pages_per_seq = pps;
  P.gen_cap = c.max_seq_len + kMaxK + 2;
  P.eps = c.rms_eps; P.rope_base = c.rope_base;

  P.kv_len = A.take<int32_t>(S); P.pending = A.take<int32_t>(S); P.first = A.take<int32_t>(S);
  P.drafts = A.take<int32_t>(S * kMaxK); P.n_gen = A.take<int32_t>(S); P.n_acc = A.take<int32_t>(S);
  P.frozen = A.take<int32_t>(S); P.gen_limit = A.take<int32_t>(S);
  P.iter = A.take<uint32_t>(S); P.seq_id = A.take<uint32_t>(S);
  P.last_out = A.take<int32_t>(S * (kMaxK + 1));
  P.gen = A.take<int32_t>(S * P.gen_cap);
  P.logz_d = A.take<float>(S * (kMaxK + 1)); P.logz_p = A.take<float>(S * (kMaxK + 1));
  P.argmax_p = A.take<int32_t>(S * (kMaxK + 1));
  P.flt_key_d = A.take<uint32_t>(S * (kMaxK + 1)); P.flt_key_p = A.take<uint32_t>(S * (kMaxK + 1));
  P.flt_tie_d = A.take<int32_t>(S * (kMaxK + 1)); P.flt_tie_p = A.take<int32_t>(S * (kMaxK + 1));
  P.fallbacks = A.take<int32_t>(1);
  P.block_table = A.take<int32_t>(S * pps);
  P.draft_logits = A.take<float>(S * (1 + c.k) * V);
  P.verify_logits = A.take<float>(S * (1 + c.k) * V);
  P.step_slots = A.take<int32_t>(M);
  P.row_pos = A.take<int32_t>(M); P.row_slot = A.take<int32_t>(M); P.row_out = A.take<int32_t>(M);
  P.rope_cos = A.take<float>(M * c.head_dim / 2); P.rope_sin = A.take<float>(M * c.head_dim / 2);
  P.rope_theta = A.take<double>(c.head_dim / 2);
  P.h = A.take<float>(M * d); P.xn = A.take<float>(M * d); P.qkv = A.take<float>(M * 3 * D);
  P.attn = A.take<float>(M * D); P.gu = A.take<float>(M * 2 * F); P.act = A.take<float>(M * F);
  P.attn_x = A.take<uint16_t>(2 * M * D); P.act_x = A.take<uint16_t>(2 * M * F); P.xg = A.take<uint16_t>(2 * M * d);
  P.ssq = A.take<float>((d / 16 + 1) * M);
  P.part_acc = A.take<float>(M * c.n_heads * kMaxSplits * c.head_dim);
  P.part_m = A.take<float>(M * c.n_heads * kMaxSplits); P.part_l = A.take<float>(M * c.n_heads * kMaxSplits);
  size_t pool_elems = (size_t)c.n_layers * np * c.n_heads * c.page_size * c.head_dim;
  P.k_pool = A.take<char>(pool_elems * esz); P.v_pool = A.take<char>(pool_elems * esz);
  int32_t *prompt_buf = A.take<int32_t>(std::max(c.max_seq_len, kPrefillRows));

  void *tok_emb = A.take<char>(V * d * esz), *lm_head = A.take<char>(V * d * esz);
  void *final_norm = A.take<char>(d * esz), *lookahead = A.take<char>((size_t)(c.k ? c.k : 1) * d * esz);
  std::vector<LayerW> layers(c.n_layers);
  for (auto &l : layers) {
    l.attn_norm = A.take<char>(d * esz); l.ffn_norm = A.take<char>(d * esz);
    l.wqkv = A.take<char>(3 * D * d * esz); l.wo = A.take<char>(d * D * esz);
    l.wgu = A.take<char>(2 * F * d * esz); l.wdown = A.take<char>(d * F * esz);
  }
  size_t stage = V * d;
  if (F * d > stage) stage = F * d;
  if (D * d > stage) stage = D * d;
  size_t stage_bytes = stage * esz;
  // The staging area doubles as the row buffers of the tiled prompt pass (weights are staged only
  // while they are loaded): h, (hi, lo) of the normed rows, q, (hi, lo) of the attention output and
  // of silu(gate) * up, partial sums of h^2, rotary table.
  PrefillWs W;
  memset(&W, 0, sizeof W);
  W.rows = std::min(kPrefillRows, (c.max_seq_len + 127) / 128 * 128);
  W.np = (int)(d / 16);  // most partial sums of h^2 a row can have (one per strip)
  const size_t R = W.rows;
  const size_t ws_bytes = R * 4 * (d + d + D + D + F + W.np + c.head_dim) + 8 * 256;
  if (ws_bytes > stage_bytes) stage_bytes = ws_bytes;
  void *staging = A.take<char>(stage_bytes);
  if (ctx) {
    ctx->P = P; ctx->esz = esz; ctx->prompt_buf = prompt_buf;
    ctx->tok_emb = tok_emb; ctx->lm_head = lm_head; ctx->final_norm = final_norm; ctx->lookahead = lookahead;
    ctx->layers = layers; ctx->staging = staging; ctx->staging_bytes = stage_bytes;
    Arena S2{(char *)staging, 0};
    Params PP = P;
    PP.h = S2.take<float>(R * d); PP.xg = S2.take<uint16_t>(2 * R * d);
    W.q = S2.take<float>(R * D); PP.attn_x = S2.take<uint16_t>(2 * R * D); PP.act_x = S2.take<uint16_t>(2 * R * F);
    PP.ssq = S2.take<float>(R * W.np);
    PP.rope_cos = S2.take<float>(R * c.head_dim / 2); PP.rope_sin = S2.take<float>(R * c.head_dim / 2);
    ctx->PP = PP; ctx->pws = W;
  }
  return (A.off + 255) & ~(size_t)255;
}

size_t carve_train(const pass_config &c, bool mfma, char *base, TrainWs *out) {
  Arena A{base, 0};
  const size_t d = c.d_model, D = (size_t)c.n_heads * c.head_dim, F = c.d_ffn, V = c.vocab, L = c.n_layers, M = kMaxRows;
  const size_t kd = (size_t)(c.k ? c.k : 1) * d;
  TrainWs T;
  T.master = A.take<float>(kd); T.m1 = A.take<float>(kd); T.m2 = A.take<float>(kd); T.grad = A.take<float>(kd);
  T.save_h0 = A.take<float>(L * M * d); T.save_h1 = A.take<float>(L * M * d);
  T.save_qkv = A.take<float>(L * M * 3 * D); T.save_attn = A.take<float>(L * M * D); T.save_lse = A.take<float>(L * M * c.n_heads);
  T.save_gu = A.take<float>(L * M * 2 * F);
  T.save_hl = A.take<float>(M * d);
  T.logits = A.take<float>(M * V);
  T.dh = A.take<float>(M * d); T.dxn = A.take<float>(M * d); T.dattn = A.take<float>(M * D); T.dqkv = A.take<float>(M * 3 * D);
  T.dact = A.take<float>(M * F); T.dgu = A.take<float>(M * 2 * F);
  T.part = A.take<float>((size_t)kTrainSplits * M * std::max(std::max(d, D), F));
  T.dq_part = A.take<float>((size_t)kTrainAttnSplits * M * D);
  T.row_loss = A.take<float>(M);
  T.targets = A.take<int32_t>(M);
  T.mfma = mfma;
  if (mfma) {
    T.x = A.take<uint16_t>(2 * M * std::max(std::max(V, 2 * F), std::max(3 * D, d)));
    T.lm_head_t = A.take<uint16_t>(V * d);
    T.layers_t.resize(L);
    for (auto &l : T.layers_t) {
      l.attn_norm = l.ffn_norm = nullptr;
      l.wqkv = A.take<uint16_t>(3 * D * d); l.wo = A.take<uint16_t>(d * D);
      l.wgu = A.take<uint16_t>(2 * F * d); l.wdown = A.take<uint16_t>(d * F);
    }
  }
  if (out) *out = T;
  return (A.off + 255) & ~(size_t)255;
}

__global__ void gather_report_kernel(Params p, int B, int32_t *out) {
  int b = threadIdx.x;
  if (b >= B) return;
  int slot = p.step_slots[b];
  int32_t *o = out + b * kReportStride;
  o[0] = p.kv_len[slot]; o[1] = p.n_gen[slot]; o[2] = p.n_acc[slot]; o[3] = p.first[slot];
  for (int t = 0; t < kMaxK; ++t) o[4 + t] = p.drafts[slot * kMaxK + t];
  for (int t = 0; t <= kMaxK; ++t) o[4 + kMaxK + t] = p.last_out[slot * (kMaxK + 1) + t];
  o[kReportStride - 1] = (int32_t)p.iter[slot];
}

int poke(pass_ctx *c, std::vector<int32_t *> &ptrs, std::vector<int32_t> &vals) {
  for (size_t i = 0; i < ptrs.size(); i += 16) {
    int n = (int)std::min<size_t>(16, ptrs.size() - i);
    launch_poke(ptrs.data() + i, vals.data() + i, n, c->stream);
  }
  ptrs.clear();
  vals.clear();
  HIP_TRY(c, hipGetLastError());
  return PASS_OK;
}

void release_pages(pass_ctx *c, int slot) {
  Slot &s = c->slots[slot];
  for (int pg : s.pages) c->free_pages.push_back(pg);
  s.pages.clear();
}

// Make sure `slot` has pages for positions [0, n_pos).
int ensure_pages(pass_ctx *c, int slot, int n_pos) {
  Slot &s = c->slots[slot];
  const int ps = c->cfg.page_size, pps = c->P.pages_per_seq;
  int need = (n_pos + ps - 1) / ps;
  if (need > pps) return fail(c, PASS_ECAPACITY, "slot %d: %d positions exceed max_seq_len", slot, n_pos);
  int have = (int)s.pages.size();
  if (need <= have) return PASS_OK;
  if ((int)c->free_pages.size() < need - have) return fail(c, PASS_ECAPACITY, "K/V page pool exhausted");
  for (int i = have; i < need; ++i) {
    int pg = c->free_pages.back();
    c->free_pages.pop_back();
    s.pages.push_back(pg);
    c->block_table_host[(size_t)slot * pps + i] = pg;
  }
  // entries are only ever appended while a sequence lives, so an in-flight copy of this row can
  // at worst see a newer value of an entry no running kernel reads
  HIP_TRY(c, hipMemcpyAsync(c->P.block_table + (size_t)slot * pps + have, c->block_table_host + (size_t)slot * pps + have,
                            sizeof(int32_t) * (need - have), hipMemcpyHostToDevice, c->stream));
  return PASS_OK;
}

int set_step_slots(pass_ctx *c, const int32_t *slots, int B) {
  std::vector<int32_t *> ptrs;
  std::vector<int32_t> vals;
  for (int b = 0; b < B; ++b) { ptrs.push_back(c->P.step_slots + b); vals.push_back(slots[b]); }
  return poke(c, ptrs, vals);
}

int choose_splits(const pass_ctx *c, int B, int R, int max_keys) {
  // grid width only: each row group cuts its own keys by a rule of its own length (split_plan in
  // the attention kernel); workgroups beyond a group's split count exit at once
  (void)B; (void)R;
  if (c->P.v_transposed)  // the most splits any group of at most max_keys keys can have (the plan is not monotone)
    return max_splits_mfma(std::max(1, max_keys), c->P.H);
  return std::max(1, std::min(kMaxSplits, (max_keys + 63) / 64));
}

// One model call on B*R rows.  logits_base == nullptr: no LM head (prefill).
int run_step(pass_ctx *c, int mode, int B, int R, float *logits_base, int max_keys, const int32_t *prefill_ids) {
  Params P = c->P;
  P.prefill_ids = const_cast<int32_t *>(prefill_ids);
  const int dt = c->cfg.dtype, M = B * R;
  if (c->static_scratch) {  // same layout as in the arena: [M][H][kMaxSplits] accumulators, then maxima, then sums
    float *base = (float *)g_scratch_ptr[c->device];
    const size_t triples = (size_t)M * P.H * kMaxSplits;
    P.part_acc = base;
    P.part_m = base + triples * P.hd;
    P.part_l = P.part_m + triples;
  }
  hipStream_t s = c->stream;
  const int S = choose_splits(c, B, R, max_keys);
  const bool timing = c->opt_kernel_timing && mode != MODE_PREFILL;
  if (timing && c->kev.empty()) {
    c->kev.resize(2);
    for (auto &e : c->kev) HIP_TRY(c, hipEventCreate(&e));
  }
  if (c->use_mfma) {
    launch_assemble_mfma(P, c->tok_emb, c->lookahead, c->layers[0].attn_norm, mode, B, R, s);
    for (int l = 0; l < P.L; ++l) {
      const LayerW &w = c->layers[l];
      launch_gemm_qkv(P, c->tuning, w.wqkv, l, M, s);
      launch_attention(P, dt, l, B, R, S, 1, s);
      launch_gemm_resid(P, c->tuning, w.wo, P.attn_x, P.D, w.ffn_norm, M, s);
      launch_gemm_gateup(P, c->tuning, w.wgu, M, s);
      launch_gemm_resid(P, c->tuning, w.wdown, P.act_x, P.F,
                        l + 1 < P.L ? c->layers[l + 1].attn_norm : c->final_norm, M, s);
    }
    if (logits_base) launch_gemm_logits(P, c->tuning, c->lm_head, logits_base, M, s);
  } else {
  launch_assemble(P, dt, c->tok_emb, c->lookahead, mode, B, R, s);
  for (int l = 0; l < P.L; ++l) {
    const LayerW &w = c->layers[l];
    launch_rmsnorm(P, dt, P.h, w.attn_norm, P.xn, M, s);
    launch_gemm_generic(dt, P.xn, w.wqkv, P.qkv, M, 3 * P.D, P.d, 3 * P.D, nullptr, 0, s);
    launch_rope_kv(P, dt, l, M, s);
    launch_attention(P, dt, l, B, R, S, 0, s);
    launch_gemm_generic(dt, P.attn, w.wo, P.h, M, P.d, P.D, P.d, nullptr, 1, s);
    launch_rmsnorm(P, dt, P.h, w.ffn_norm, P.xn, M, s);
    launch_gemm_generic(dt, P.xn, w.wgu, P.gu, M, 2 * P.F, P.d, 2 * P.F, nullptr, 0, s);
    launch_silu_mul(P, M, s);
    launch_gemm_generic(dt, P.act, w.wdown, P.h, M, P.d, P.F, P.d, nullptr, 1, s);
  }
  if (logits_base) {
    launch_rmsnorm(P, dt, P.h, c->final_norm, P.xn, M, s);
    launch_gemm_generic(dt, P.xn, c->lm_head, logits_base, M, P.V, P.d, P.V, P.row_out, 0, s);
  }
  }
  HIP_TRY(c, hipGetLastError());
  if (timing) {
    // The dominant kernel on its own: the gate/up GEMM of every layer (each with its own weights,
    // on this call's rows) launched back to back between two events.  Its outputs are workspaces
    // the step has already consumed, so nothing changes for the caller.
    HIP_TRY(c, hipEventRecord(c->kev[0], s));
    for (int l = 0; l < P.L; ++l) {
      if (c->use_mfma)
        launch_gemm_gateup(P, c->tuning, c->layers[l].wgu, M, s);
      else
        launch_gemm_generic(dt, P.xn, c->layers[l].wgu, P.gu, M, 2 * P.F, P.d, 2 * P.F, nullptr, 0, s);
    }
    HIP_TRY(c, hipEventRecord(c->kev[1], s));
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(s));
    float ms = 0;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->kev[0], c->kev[1]));
    c->kernel_ms += ms;
    c->kernel_launches += P.L;
  }
  return PASS_OK;
}

// One tiled pass over the weights: the rows `segs` describes (M rows including padding, M <= pws.rows), token
// ids of all M rows at `ids` (device).  Attention runs per sequence on its own rows of the pass (row_base:
// multiples of 128, so a sequence's rows are whole 8-row groups of the (hi, lo) tiles).
// No LM head: the last prompt token stays pending and goes through the first draft call.
struct PassSeg { int slot, pos0, rows, row_base; };

// How pass_prefill_batch packs prompts into tiled passes of at most `cap` rows (a multiple of 128): prompt b has
// lens[b] - 1 rows to cache; its rows start on a block of 128 rows of a pass; what does not fit goes on in the next
// pass.  Segments come out in launch order: rows [pos0, pos0 + rows) of `prompt` at rows row_base .. of pass `pass`.
struct PlanSeg { int pass, prompt, pos0, rows, row_base; };
std::vector<PlanSeg> plan_prefill(int cap, const int32_t *lens, int n) {
  std::vector<PlanSeg> out;
  int pass = 0, cur = 0;
  for (int b = 0; b < n; ++b) {
    const int rows = lens[b] - 1;
    for (int done = 0; done < rows;) {
      if (cur >= cap) { ++pass; cur = 0; }
      const int take = std::min(rows - done, cap - cur);
      out.push_back(PlanSeg{pass, b, done, take, cur});
      done += take;
      cur = (cur + take + kPrefillBlockRows - 1) / kPrefillBlockRows * kPrefillBlockRows;
    }
  }
  return out;
}
int run_prefill_pass(pass_ctx *c, const std::vector<PassSeg> &parts, int M, const int32_t *ids) {
  Params P = c->P;
  const Params &B = c->PP;
  P.h = B.h; P.xg = B.xg; P.attn_x = B.attn_x; P.act_x = B.act_x; P.ssq = B.ssq;
  P.rope_cos = B.rope_cos; P.rope_sin = B.rope_sin;
  P.prefill_ids = const_cast<int32_t *>(ids);
  PrefillWs W = c->pws;
  W.resid_strips = W.resid_strips_opt ? W.resid_strips_opt : prefill_resid_strips(P, M);
  W.np = (P.d / 16 + W.resid_strips - 1) / W.resid_strips;
  PrefillSegs segs;
  memset(&segs, 0, sizeof segs);
  segs.n_blocks = (M + kPrefillBlockRows - 1) / kPrefillBlockRows;
  for (const PassSeg &g : parts)
    for (int done = 0; done < g.rows; done += kPrefillBlockRows) {
      const int b = (g.row_base + done) / kPrefillBlockRows;
      segs.slot[b] = g.slot;
      segs.pos[b] = g.pos0 + done;
      segs.rows[b] = std::min(kPrefillBlockRows, g.rows - done);
    }
  hipStream_t s = c->stream;
  launch_assemble_prefill_segs(P, c->tok_emb, c->layers[0].attn_norm, segs, M, W.np, W.rows, s);
  for (int l = 0; l < P.L; ++l) {
    const LayerW &w = c->layers[l];
    launch_prefill_qkv(P, W, w.wqkv, l, segs, M, s);
    for (const PassSeg &g : parts) {
      Params Pg = P;
      PrefillWs Wg = W;
      Pg.attn_x = P.attn_x + (size_t)g.row_base * 2 * P.D;  // 8-row groups of 16 * D elements
      Wg.q = W.q + (size_t)g.row_base * P.D;
      launch_prefill_attention(Pg, Wg, l, g.slot, g.pos0, g.rows, s);
    }
    launch_prefill_resid(P, W, w.wo, P.attn_x, P.D, w.ffn_norm, M, s);
    launch_prefill_gateup(P, W, w.wgu, M, s);
    launch_prefill_resid(P, W, w.wdown, P.act_x, P.F, l + 1 < P.L ? c->layers[l + 1].attn_norm : c->final_norm, M, s);
  }
  HIP_TRY(c, hipGetLastError());
  return PASS_OK;
}

// Prompt rows [pos0, pos0 + R) of one slot, R <= pws.rows
int run_prefill_tiled(pass_ctx *c, int slot, int pos0, int R, const int32_t *ids) {
  return run_prefill_pass(c, {PassSeg{slot, pos0, R, 0}}, R, ids);
}

int check_slots(pass_ctx *c, const int32_t *slots, int n_slots, int want_state) {
  if (!slots || n_slots < 1 || n_slots > c->cfg.max_slots) return fail(c, PASS_EINVAL, "bad slot list");
  for (int i = 0; i < n_slots; ++i) {
    int s = slots[i];
    if (s < 0 || s >= c->cfg.max_slots) return fail(c, PASS_EINVAL, "slot %d out of range", s);
    for (int j = 0; j < i; ++j)
      if (slots[j] == s) return fail(c, PASS_EINVAL, "slot %d listed twice", s);
    if (c->slots[s].state != want_state)
      return fail(c, PASS_ESTATE, "slot %d is in state %d, call needs state %d", s, c->slots[s].state, want_state);
  }
  return PASS_OK;
}

int check_sampling(pass_ctx *c, const pass_sampling *sp) {
  if (!sp) return fail(c, PASS_EINVAL, "null sampling parameters");
  if (!(sp->temperature >= 0.f) || !isfinite(sp->temperature)) return fail(c, PASS_EINVAL, "temperature must be >= 0");
  if (sp->top_k < 0) return fail(c, PASS_EINVAL, "top_k must be >= 0 (0 = no filter)");
  return PASS_OK;
}

SampleArgs sample_args(const pass_sampling *sp, int commit) {
  SampleArgs a;
  a.temperature = sp->temperature;
  a.seed_lo = (uint32_t)sp->seed;
  a.seed_hi = (uint32_t)(sp->seed >> 32);
  a.commit = commit;
  a.top_k = sp->top_k;
  a.row_base = 0;
  a.stats_only = 0;
  return a;
}

int fetch_report(pass_ctx *c, int B) {
  // the kernel stores straight into the pinned (device-visible, coherent) host buffer: no copy
  gather_report_kernel<<<1, 64, 0, c->stream>>>(c->P, B, c->report_host);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PASS_OK;
}

int max_keys_of(pass_ctx *c, const int32_t *slots, int B, int extra) {
  int mk = 1;
  for (int b = 0; b < B; ++b) mk = std::max(mk, c->slots[slots[b]].kv_len + c->kv_slack + extra);
  return mk;
}

// the two halves of an iteration, without host synchronisation
int issue_call_eager(pass_ctx *c, int mode, const int32_t *slots, int B, const pass_sampling *sp, int commit) {
  const int R = 1 + c->P.k_act;
  const bool draft = mode == MODE_DRAFT;
  int rc = run_step(c, mode, B, R, draft ? c->P.draft_logits : c->P.verify_logits,
                    max_keys_of(c, slots, B, draft ? R : R + 1), nullptr);
  if (rc) return rc;
  if (draft) {
    SampleArgs a = sample_args(sp, commit);
    a.row_base = c->row_base;
    launch_draft_epilogue(c->P, a, B, R, c->stream);
  } else
    launch_verify_epilogue(c->P, sample_args(sp, commit), B, R, c->stream);
  HIP_TRY(c, hipGetLastError());
  return PASS_OK;
}

// One model call plus its sampling epilogue.  With the "graph" option the launches are captured
// once per (mode, batch, attention grid width, sampling arguments) and replayed: every kernel
// reads positions, slots and tokens from device memory, so a replay needs no new arguments.
int issue_call(pass_ctx *c, int mode, const int32_t *slots, int B, const pass_sampling *sp, int commit) {
  // the null stream cannot be captured: graphs need a stream of their own
  if (!c->opt_graph || c->opt_kernel_timing || c->stream == nullptr || c->static_scratch)
    return issue_call_eager(c, mode, slots, B, sp, commit);
  const int R = 1 + c->P.k_act;
  const int S = choose_splits(c, B, R, max_keys_of(c, slots, B, mode == MODE_DRAFT ? R : R + 1));
  uint32_t tbits;
  memcpy(&tbits, &sp->temperature, 4);
  pass_ctx::GraphKey key(mode, B, S, tbits, (uint32_t)sp->seed, (uint32_t)(sp->seed >> 32), commit, sp->top_k, c->P.k_act, c->P.la_token, c->row_base);
  auto it = c->graphs.find(key);
  if (it == c->graphs.end()) {
    if (c->graphs.size() >= 64) {  // bound the cache: drop everything, recapture on demand
      for (auto &g : c->graphs) (void)hipGraphExecDestroy(g.second);
      c->graphs.clear();
    }
    hipGraph_t graph = nullptr;
    HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
    int rc = issue_call_eager(c, mode, slots, B, sp, commit);
    hipError_t e = hipStreamEndCapture(c->stream, &graph);
    if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess) return fail(c, PASS_EDEVICE, "hipStreamEndCapture: %s", hipGetErrorString(e));
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return fail(c, PASS_EDEVICE, "hipGraphInstantiate: %s", hipGetErrorString(e));
    it = c->graphs.emplace(key, exec).first;
  }
  HIP_TRY(c, hipGraphLaunch(it->second, c->stream));
  return PASS_OK;
}

int issue_draft(pass_ctx *c, const int32_t *slots, int B, const pass_sampling *sp, int commit) {
  return issue_call(c, MODE_DRAFT, slots, B, sp, commit);
}

int issue_verify(pass_ctx *c, const int32_t *slots, int B, const pass_sampling *sp, int commit) {
  return issue_call(c, MODE_VERIFY, slots, B, sp, commit);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

size_t pass_arena_bytes(const pass_config *cfg) {
  if (!config_ok(cfg, nullptr)) return 0;
  return carve(*cfg, nullptr, nullptr);
}

int pass_create(const pass_config *cfg, void *hip_stream, void *device_arena, size_t arena_bytes, pass_ctx **out) {
  if (!out) return PASS_EINVAL;
  *out = nullptr;
  std::string why;
  if (!config_ok(cfg, &why)) { g_create_error = "pass_create: " + why; return PASS_EINVAL; }
  if (!device_arena || ((uintptr_t)device_arena & 255)) { g_create_error = "pass_create: arena null or misaligned"; return PASS_EINVAL; }
  if (arena_bytes < carve(*cfg, nullptr, nullptr)) { g_create_error = "pass_create: arena too small"; return PASS_EINVAL; }
  pass_ctx *c = new pass_ctx();
  c->cfg = *cfg;
  c->stream = (hipStream_t)hip_stream;
  carve(*cfg, (char *)device_arena, c);
  // the static scratch array of pass_draft_static: its device address on this GPU, looked up once
  if (hipGetDevice(&c->device) != hipSuccess || c->device < 0 || c->device >= kMaxDevices) {
    g_create_error = "pass_create: cannot tell the current device";
    delete c;
    return PASS_EDEVICE;
  }
  if (!g_scratch_ptr[c->device]) {
    void *sp = nullptr;
    hipError_t es = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
    if (es != hipSuccess || !sp) {
      g_create_error = std::string("pass_create: hipGetSymbolAddress(scratch): ") + hipGetErrorString(es);
      delete c;
      return PASS_EDEVICE;
    }
    g_scratch_ptr[c->device] = (unsigned char *)sp;
  }
  c->slots.resize(cfg->max_slots);
  for (int i = pool_pages(*cfg) - 1; i >= 0; --i) c->free_pages.push_back(i);
  const size_t S = cfg->max_slots;
  auto die = [&](hipError_t e) {
    g_create_error = std::string("pass_create: ") + hipGetErrorString(e);
    if (c->report_host) (void)hipHostFree(c->report_host);
    if (c->block_table_host) (void)hipHostFree(c->block_table_host);
    delete c;
    return PASS_EDEVICE;
  };
  hipError_t e = hipHostMalloc((void **)&c->report_host, sizeof(int32_t) * 2 * S * kReportStride, hipHostMallocDefault);
  if (e != hipSuccess) return die(e);
  e = hipHostMalloc((void **)&c->block_table_host, sizeof(int32_t) * S * c->P.pages_per_seq, hipHostMallocDefault);
  if (e != hipSuccess) return die(e);
  memset(c->block_table_host, 0, sizeof(int32_t) * S * c->P.pages_per_seq);
  for (auto &ev : c->ev) {
    e = hipEventCreate(&ev);
    if (e != hipSuccess) return die(e);
  }
  for (auto &set : c->ev2)
    for (auto &ev : set) {
      e = hipEventCreate(&ev);
      if (e != hipSuccess) return die(e);
    }
  // per-slot state starts at zero; block table at page 0 (valid memory, never read before set)
  size_t state_ints = (size_t)((char *)c->P.gen - (char *)c->P.kv_len) / 4;
  launch_fill_i32(c->P.kv_len, 0, state_ints, c->stream);
  launch_fill_i32(c->P.block_table, 0, S * c->P.pages_per_seq, c->stream);
  launch_fill_i32(c->P.fallbacks, 0, 1, c->stream);
  {
    // K/V pools start as zeros: positions that are masked out of an attention tile are still
    // multiplied (by probability 0) in the matrix-core kernel and must never hold NaN patterns
    size_t pool_bytes = (size_t)cfg->n_layers * c->P.n_pages * cfg->n_heads * cfg->page_size * cfg->head_dim * c->esz;
    launch_fill_i32((int32_t *)c->P.k_pool, 0, pool_bytes / 4, c->stream);
    launch_fill_i32((int32_t *)c->P.v_pool, 0, pool_bytes / 4, c->stream);
  }
  launch_fill_i32(c->P.gen_limit, INT_MAX, S, c->stream);
  launch_fill_i32(c->P.step_slots, 0, kMaxRows, c->stream);
  // row tables: entries past a call's row count are never meant to be read, but start in bounds
  launch_fill_i32(c->P.row_pos, 0, kMaxRows, c->stream);
  launch_fill_i32(c->P.row_slot, 0, kMaxRows, c->stream);
  launch_fill_i32(c->P.row_out, 0, kMaxRows, c->stream);
  // rotary frequencies theta_i = base^(-2i/hd), in double (the angle pos * theta_i is formed in double too)
  std::vector<double> theta(cfg->head_dim / 2);
  for (int i = 0; i < cfg->head_dim / 2; ++i) theta[i] = pow((double)cfg->rope_base, -2.0 * i / (double)cfg->head_dim);
  e = hipMemcpyAsync(c->P.rope_theta, theta.data(), theta.size() * sizeof(double), hipMemcpyHostToDevice, c->stream);
  if (e != hipSuccess) return die(e);
  e = hipGetLastError();
  if (e != hipSuccess) return die(e);
  e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return die(e);
  *out = c;
  return PASS_OK;
}

int pass_load_weights(pass_ctx *c, const pass_weights *w, int on_device) {
  if (!c) return PASS_EINVAL;
  if (!w || !w->tok_emb || !w->lm_head || !w->final_norm || (c->cfg.k > 0 && !w->lookahead) || !w->attn_norm ||
      !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
    return fail(c, PASS_EINVAL, "null weight pointer");
  const size_t e = c->esz, d = c->P.d, D = c->P.D, F = c->P.F, V = c->P.V;
  c->train.on = false;  // a training set-up belongs to the weights it was made from (their packed transposes)
  const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
  auto cp = [&](void *dst, const void *src, size_t elems) -> int {
    if (!src) return fail(c, PASS_EINVAL, "null weight pointer");
    HIP_TRY(c, hipMemcpyAsync(dst, src, elems * e, kind, c->stream));
    return PASS_OK;
  };
  int rc = PASS_OK;
  c->use_mfma = c->opt_path != 1 && c->cfg.dtype == PASS_BF16 && d % 32 == 0 && D % 32 == 0 && F % 32 == 0 &&
                V % 16 == 0;
  // matrix-core attention: transposed V pages (nothing is cached yet, so the layout can still be chosen)
  c->P.v_transposed = c->use_mfma && c->opt_attn != 1 && c->cfg.head_dim == 128 && c->cfg.page_size % 32 == 0;
  if (c->use_mfma) {
    // matrices go through the tile packer; on_device = 0 stages each tensor in the arena first
    auto pack = [&](void *dst, const void *src, size_t N, size_t K, int strip_off, int strip_stride) -> int {
      if (!src) return fail(c, PASS_EINVAL, "null weight pointer");
      const void *dev_src = src;
      if (!on_device) {
        HIP_TRY(c, hipMemcpyAsync(c->staging, src, N * K * e, hipMemcpyHostToDevice, c->stream));
        dev_src = c->staging;
      }
      launch_pack_tiles((const uint16_t *)dev_src, (uint16_t *)dst, (int)N, (int)K, strip_off, strip_stride, c->stream);
      HIP_TRY(c, hipGetLastError());
      return PASS_OK;
    };
    if ((rc = cp(c->tok_emb, w->tok_emb, V * d))) return rc;
    if ((rc = pack(c->lm_head, w->lm_head, V, d, 0, 1))) return rc;
    if ((rc = cp(c->final_norm, w->final_norm, d))) return rc;
    if (c->cfg.k > 0 && (rc = cp(c->lookahead, w->lookahead, (size_t)c->cfg.k * d))) return rc;
    for (int l = 0; l < c->P.L; ++l) {
      LayerW &lw = c->layers[l];
      if ((rc = cp(lw.attn_norm, w->attn_norm[l], d))) return rc;
      if ((rc = cp(lw.ffn_norm, w->ffn_norm[l], d))) return rc;
      const int ds = (int)(D / 16);
      if ((rc = pack(lw.wqkv, w->wq[l], D, d, 0, 1))) return rc;
      if ((rc = pack(lw.wqkv, w->wk[l], D, d, ds, 1))) return rc;
      if ((rc = pack(lw.wqkv, w->wv[l], D, d, 2 * ds, 1))) return rc;
      if ((rc = pack(lw.wo, w->wo[l], d, D, 0, 1))) return rc;
      if ((rc = pack(lw.wgu, w->w_gate[l], F, d, 0, 2))) return rc;  // gate strips at even positions
      if ((rc = pack(lw.wgu, w->w_up[l], F, d, 1, 2))) return rc;    // up strips at odd positions
      if ((rc = pack(lw.wdown, w->w_down[l], d, F, 0, 1))) return rc;
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->weights_loaded = true;
    return PASS_OK;
  }
  if ((rc = cp(c->tok_emb, w->tok_emb, V * d))) return rc;
  if ((rc = cp(c->lm_head, w->lm_head, V * d))) return rc;
  if ((rc = cp(c->final_norm, w->final_norm, d))) return rc;
  if (c->cfg.k > 0 && (rc = cp(c->lookahead, w->lookahead, (size_t)c->cfg.k * d))) return rc;
  for (int l = 0; l < c->P.L; ++l) {
    LayerW &lw = c->layers[l];
    if ((rc = cp(lw.attn_norm, w->attn_norm[l], d))) return rc;
    if ((rc = cp(lw.ffn_norm, w->ffn_norm[l], d))) return rc;
    if ((rc = cp(lw.wqkv, w->wq[l], D * d))) return rc;
    if ((rc = cp((char *)lw.wqkv + D * d * e, w->wk[l], D * d))) return rc;
    if ((rc = cp((char *)lw.wqkv + 2 * D * d * e, w->wv[l], D * d))) return rc;
    if ((rc = cp(lw.wo, w->wo[l], d * D))) return rc;
    if ((rc = cp(lw.wgu, w->w_gate[l], F * d))) return rc;
    if ((rc = cp((char *)lw.wgu + F * d * e, w->w_up[l], F * d))) return rc;
    if ((rc = cp(lw.wdown, w->w_down[l], d * F))) return rc;
  }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->weights_loaded = true;
  return PASS_OK;
}

int pass_release(pass_ctx *c, int slot) {
  if (!c) return PASS_EINVAL;
  if (slot < 0 || slot >= c->cfg.max_slots) return fail(c, PASS_EINVAL, "slot %d out of range", slot);
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  release_pages(c, slot);
  c->slots[slot] = Slot();
  return PASS_OK;
}

// what pass_prefill does before and after the prompt's rows go through the model
static int prefill_begin(pass_ctx *c, int slot, uint32_t seq_id, const int32_t *prompt, int n) {
  if (slot < 0 || slot >= c->cfg.max_slots) return fail(c, PASS_EINVAL, "slot %d out of range", slot);
  if (!prompt || n < 1) return fail(c, PASS_EINVAL, "prompt must hold at least one token");
  for (int i = 0; i < n; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->cfg.vocab) return fail(c, PASS_EINVAL, "prompt[%d] = %d outside the vocabulary", i, prompt[i]);
  if (n - 1 + 1 + c->cfg.k > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "prompt of %d tokens does not fit max_seq_len", n);
  int rc = pass_release(c, slot);
  if (rc) return rc;
  if ((rc = ensure_pages(c, slot, n - 1 + 1 + c->cfg.k))) return rc;
  c->slots[slot].seq_id = seq_id;
  const Params &P = c->P;
  std::vector<int32_t *> ptrs = {P.kv_len + slot, P.pending + slot, P.n_gen + slot, (int32_t *)P.iter + slot,
                                 (int32_t *)P.seq_id + slot, P.gen_limit + slot, P.frozen + slot, P.n_acc + slot};
  std::vector<int32_t> vals = {0, prompt[n - 1], 0, 0, (int32_t)seq_id, INT_MAX, 0, 0};
  return poke(c, ptrs, vals);
}
static int prefill_end(pass_ctx *c, int slot, int n) {  // after the stream has been synchronised
  Slot &s = c->slots[slot];
  s.kv_len = n - 1;
  s.n_gen = 0;
  s.iteration = 0;
  s.state = 1;
  return PASS_OK;
}

int pass_prefill(pass_ctx *c, int slot, uint32_t seq_id, const int32_t *prompt, int n) {
  if (!c) return PASS_EINVAL;
  if (!c->weights_loaded) return fail(c, PASS_ESTATE, "weights not loaded");
  int rc = prefill_begin(c, slot, seq_id, prompt, n);
  if (rc) return rc;
  const Params &P = c->P;
  std::vector<int32_t *> ptrs = {P.step_slots};
  std::vector<int32_t> vals = {slot};
  if ((rc = poke(c, ptrs, vals))) return rc;
  if (n > 1) {
    HIP_TRY(c, hipMemcpyAsync(c->prompt_buf, prompt, sizeof(int32_t) * (n - 1), hipMemcpyHostToDevice, c->stream));
    // long prompts on the matrix-core path: tiled kernels, up to pws.rows rows per pass over the
    // weights; otherwise the decode kernels, prefill_chunk rows per pass.  A tiled pass costs about
    // as much as two passes of the decode kernels however few rows it carries (a workgroup walks
    // all of K whatever the row count), so it takes over above two chunks.
    const bool tiled = c->use_mfma && c->P.v_transposed &&
                       (c->opt_prefill_tiled == 1 || (c->opt_prefill_tiled < 0 && n - 1 > 2 * kMaxRows));
    const int chunk = tiled ? c->pws.rows : c->opt_prefill_chunk;
    for (int done = 0; done < n - 1; done += chunk) {
      int R = std::min(chunk, n - 1 - done);
      ptrs = {P.kv_len + slot};
      vals = {done};
      if ((rc = poke(c, ptrs, vals))) return rc;
      if (tiled)
        rc = run_prefill_tiled(c, slot, done, R, c->prompt_buf + done);
      else
        rc = run_step(c, MODE_PREFILL, 1, R, nullptr, done + R, c->prompt_buf + done);
      if (rc) return rc;
    }
    ptrs = {P.kv_len + slot};
    vals = {n - 1};
    if ((rc = poke(c, ptrs, vals))) return rc;
  }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return prefill_end(c, slot, n);
}

int pass_prefill_batch(pass_ctx *c, const int32_t *slots, const uint32_t *seq_ids, const int32_t *prompts, const int32_t *lens,
                       int n_slots) {
  if (!c) return PASS_EINVAL;
  if (!c->weights_loaded) return fail(c, PASS_ESTATE, "weights not loaded");
  if (!slots || !seq_ids || !prompts || !lens || n_slots < 1 || n_slots > c->cfg.max_slots) return fail(c, PASS_EINVAL, "bad slot list");
  long total = 0;
  for (int b = 0; b < n_slots; ++b) {
    for (int j = 0; j < b; ++j)
      if (slots[j] == slots[b]) return fail(c, PASS_EINVAL, "slot %d listed twice", slots[b]);
    if (lens[b] < 1) return fail(c, PASS_EINVAL, "prompt must hold at least one token");
    total += lens[b] - 1;
  }
  // the tiled kernels take rows of several sequences through one pass over the weights; where they do not
  // apply (generic path, untransposed V pages, switched off, or too few rows to pay for a tiled pass) the
  // prompts go one by one
  const bool tiled = c->use_mfma && c->P.v_transposed &&
                     (c->opt_prefill_tiled == 1 || (c->opt_prefill_tiled < 0 && total > 2 * kMaxRows));
  int rc;
  if (!tiled) {
    const int32_t *pr = prompts;
    for (int b = 0; b < n_slots; pr += lens[b], ++b)
      if ((rc = pass_prefill(c, slots[b], seq_ids[b], pr, lens[b]))) return rc;
    return PASS_OK;
  }
  {
    const int32_t *pr = prompts;
    for (int b = 0; b < n_slots; pr += lens[b], ++b)
      if ((rc = prefill_begin(c, slots[b], seq_ids[b], pr, lens[b]))) return rc;
  }
  // passes: a sequence's rows start on a block of 128 rows; a prompt that does not fit goes on in the next pass
  const std::vector<PlanSeg> plan = plan_prefill(c->pws.rows, lens, n_slots);
  std::vector<size_t> first_token(n_slots, 0);  // where prompt b starts in `prompts`
  for (int b = 1; b < n_slots; ++b) first_token[b] = first_token[b - 1] + lens[b - 1];
  std::vector<std::vector<int32_t>> keep;  // the passes' token ids, alive until the stream has been synchronised
  for (size_t i0 = 0; i0 < plan.size();) {
    size_t i1 = i0;
    while (i1 < plan.size() && plan[i1].pass == plan[i0].pass) ++i1;
    const int M = plan[i1 - 1].row_base + plan[i1 - 1].rows;
    std::vector<PassSeg> parts;
    std::vector<int32_t> ids(M, 0);  // padding rows carry token 0
    for (size_t i = i0; i < i1; ++i) {
      const PlanSeg &g = plan[i];
      parts.push_back(PassSeg{slots[g.prompt], g.pos0, g.rows, g.row_base});
      std::copy(prompts + first_token[g.prompt] + g.pos0, prompts + first_token[g.prompt] + g.pos0 + g.rows, ids.begin() + g.row_base);
    }
    keep.push_back(std::move(ids));
    HIP_TRY(c, hipMemcpyAsync(c->prompt_buf, keep.back().data(), sizeof(int32_t) * M, hipMemcpyHostToDevice, c->stream));
    if ((rc = run_prefill_pass(c, parts, M, c->prompt_buf))) return rc;
    i0 = i1;
  }
  std::vector<int32_t *> ptrs;
  std::vector<int32_t> vals;
  for (int b = 0; b < n_slots; ++b) {
    ptrs.push_back(c->P.kv_len + slots[b]);
    vals.push_back(lens[b] - 1);
  }
  if ((rc = poke(c, ptrs, vals))) return rc;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int b = 0; b < n_slots; ++b) prefill_end(c, slots[b], lens[b]);
  return PASS_OK;
}

static int draft_call(pass_ctx *c, const int32_t *slots, int n_slots, const pass_sampling *sp, int32_t *out_first,
                      int32_t *out_drafts) {
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 1))) return rc;
  if ((rc = check_sampling(c, sp))) return rc;
  const int k = c->cfg.k;
  for (int b = 0; b < n_slots; ++b) {
    if (c->slots[slots[b]].kv_len + 1 + k > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "slot %d is full", slots[b]);
    if ((rc = ensure_pages(c, slots[b], c->slots[slots[b]].kv_len + 1 + k))) return rc;
  }
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  if ((rc = issue_draft(c, slots, n_slots, sp, 1))) return rc;
  if ((rc = fetch_report(c, n_slots))) return rc;
  for (int b = 0; b < n_slots; ++b) {
    const int32_t *r = c->report_host + b * kReportStride;
    Slot &s = c->slots[slots[b]];
    s.kv_len = r[0];
    s.n_gen = r[1];
    s.state = 2;
    if (out_first) out_first[b] = r[3];
    if (out_drafts)
      for (int t = 0; t < k; ++t) out_drafts[b * k + t] = t < c->P.k_act ? r[4 + t] : -1;
  }
  return PASS_OK;
}

int pass_draft(pass_ctx *c, const int32_t *slots, int n_slots, const pass_sampling *sp, int32_t *out_first,
               int32_t *out_drafts) {
  if (!c) return PASS_EINVAL;
  return draft_call(c, slots, n_slots, sp, out_first, out_drafts);
}

int pass_draft_static(pass_ctx *c, const int32_t *slots, int n_slots, const pass_sampling *sp, int32_t *out_first,
                      int32_t *out_drafts) {
  if (!c) return PASS_EINVAL;
  if (n_slots < 1 || n_slots > c->cfg.max_slots) return fail(c, PASS_EINVAL, "bad slot list");
  const size_t need = partials_bytes(c->cfg, n_slots * (1 + c->P.k_act));
  if (need > kStaticScratchBytes)
    return fail(c, PASS_ECAPACITY, "pass_draft_static: %d rows x %d heads x %d dims need %zu bytes of attention partials, the "
                "static scratch holds %zu", n_slots * (1 + c->P.k_act), c->cfg.n_heads, c->cfg.head_dim, need, kStaticScratchBytes);
  if (!g_scratch_ptr[c->device]) return fail(c, PASS_EDEVICE, "pass_draft_static: no scratch address for device %d", c->device);
  c->static_scratch = true;  // launched eagerly (no graph is built), partials in the static array
  const int rc = draft_call(c, slots, n_slots, sp, out_first, out_drafts);
  c->static_scratch = false;
  return rc;
}

int pass_verify(pass_ctx *c, const int32_t *slots, int n_slots, const pass_sampling *sp, int32_t *out_n_accepted,
                int32_t *out_tokens) {
  if (!c) return PASS_EINVAL;
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 2))) return rc;
  if ((rc = check_sampling(c, sp))) return rc;
  const int k = c->cfg.k;
  for (int b = 0; b < n_slots; ++b) {
    if (c->slots[slots[b]].kv_len + 1 + k > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "slot %d is full", slots[b]);
    if ((rc = ensure_pages(c, slots[b], c->slots[slots[b]].kv_len + 1 + k))) return rc;
  }
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  if ((rc = issue_verify(c, slots, n_slots, sp, 1))) return rc;
  if ((rc = fetch_report(c, n_slots))) return rc;
  for (int b = 0; b < n_slots; ++b) {
    const int32_t *r = c->report_host + b * kReportStride;
    Slot &s = c->slots[slots[b]];
    s.kv_len = r[0];
    s.n_gen = r[1];
    s.iteration = (uint32_t)r[kReportStride - 1];
    s.state = 1;
    int a = r[2];
    if (out_n_accepted) out_n_accepted[b] = a;
    if (out_tokens)
      for (int t = 0; t <= k; ++t) out_tokens[b * (k + 1) + t] = t <= a ? r[4 + kMaxK + t] : -1;
  }
  return PASS_OK;
}

// One drafting-model call of Algorithm 2 on B slots of the drafter context: a single-row call whose
// token is drawn with the random stream of draft row `row` of the target's iteration (the drafter
// slots' iteration counters were set to the targets').  Host mirrors are updated; slots stay in
// state 1 (a drafter never verifies).
static int sps_drafter_step(pass_ctx *d, const int32_t *slots, int B, const pass_sampling *sp, int row) {
  int rc;
  for (int b = 0; b < B; ++b) {
    Slot &s = d->slots[slots[b]];
    if (s.kv_len + 1 > d->cfg.max_seq_len) return fail(d, PASS_ECAPACITY, "drafter slot %d is full", slots[b]);
    if ((rc = ensure_pages(d, slots[b], s.kv_len + 1))) return rc;
  }
  if ((rc = set_step_slots(d, slots, B))) return rc;
  d->row_base = row;
  rc = issue_call(d, MODE_DRAFT, slots, B, sp, 1);
  d->row_base = 0;
  if (rc) return rc;
  for (int b = 0; b < B; ++b) d->slots[slots[b]].kv_len += 1;  // the drafting epilogue appends its token
  return PASS_OK;
}

int pass_sps_iteration(pass_ctx *t, pass_ctx *d, const int32_t *t_slots, const int32_t *d_slots, int n_slots,
                       const pass_sampling *sp, int32_t *out_drafts, int32_t *out_n_accepted, int32_t *out_tokens) {
  if (!t || !d) return PASS_EINVAL;
  int rc;
  if ((rc = check_slots(t, t_slots, n_slots, 1))) return rc;
  if ((rc = check_slots(d, d_slots, n_slots, 1))) { fail(t, rc, "drafter: %s", d->err.c_str()); return rc; }
  if ((rc = check_sampling(t, sp))) return rc;
  if (t == d) return fail(t, PASS_EINVAL, "target and drafter must be two contexts");
  if (d->P.k_act != 0) return fail(t, PASS_EINVAL, "the drafter context must run single-row calls (k = 0 or lookahead_rows = 0)");
  if (d->cfg.vocab != t->cfg.vocab) return fail(t, PASS_EINVAL, "target and drafter vocabularies differ");
  const int L = t->P.k_act, k = t->cfg.k, V = t->cfg.vocab;
  std::vector<int32_t *> ptrs;
  std::vector<int32_t> vals;
  for (int b = 0; b < n_slots; ++b) {
    const Slot &ts = t->slots[t_slots[b]], &ds = d->slots[d_slots[b]];
    if (ts.kv_len != ds.kv_len || ts.seq_id != ds.seq_id)
      return fail(t, PASS_ESTATE, "slot pair %d: target and drafter do not hold the same sequence", b);
    if (ts.kv_len + 1 + k > t->cfg.max_seq_len) return fail(t, PASS_ECAPACITY, "slot %d is full", t_slots[b]);
    if (ds.kv_len + 1 + L > d->cfg.max_seq_len) return fail(t, PASS_ECAPACITY, "drafter slot %d is full", d_slots[b]);
    if ((rc = ensure_pages(t, t_slots[b], ts.kv_len + 1 + k))) return rc;
    ptrs.push_back((int32_t *)d->P.iter + d_slots[b]);  // the drafter draws with the target's iteration counter
    vals.push_back((int32_t)ts.iteration);
  }
  if ((rc = poke(d, ptrs, vals))) { fail(t, rc, "drafter: %s", d->err.c_str()); return rc; }
  // drafting: L sequential single-row calls of the drafter; each call's logits row and token go straight
  // into the target's draft state (row t of the slot's draft logits, draft t - 1), on the drafter's stream
  for (int row = 1; row <= L; ++row) {
    if ((rc = sps_drafter_step(d, d_slots, n_slots, sp, row))) { fail(t, rc, "drafter: %s", d->err.c_str()); return rc; }
    for (int b = 0; b < n_slots; ++b) {
      HIP_TRY(t, hipMemcpyAsync(t->P.draft_logits + ((size_t)t_slots[b] * (1 + k) + row) * V,
                                d->P.draft_logits + (size_t)d_slots[b] * (1 + d->cfg.k) * V, sizeof(float) * V,
                                hipMemcpyDeviceToDevice, d->stream));
      HIP_TRY(t, hipMemcpyAsync(t->P.drafts + (size_t)t_slots[b] * kMaxK + (row - 1), d->P.first + d_slots[b], sizeof(int32_t),
                                hipMemcpyDeviceToDevice, d->stream));
    }
  }
  HIP_TRY(t, hipStreamSynchronize(d->stream));  // the target's stream may now read what the drafter's stream wrote
  // validation: filter and ln-sum-exp of the drafted rows, then Algorithm 1's validation call unchanged
  if ((rc = set_step_slots(t, t_slots, n_slots))) return rc;
  if (L > 0) {
    SampleArgs a = sample_args(sp, 0);
    a.stats_only = 1;
    launch_draft_epilogue(t->P, a, n_slots, 1 + L, t->stream);
    HIP_TRY(t, hipGetLastError());
  }
  if ((rc = issue_verify(t, t_slots, n_slots, sp, 1))) return rc;
  if ((rc = fetch_report(t, n_slots))) return rc;
  std::vector<int32_t> again;  // drafter slots whose every draft was accepted: the row of draft L is still to be made
  for (int b = 0; b < n_slots; ++b) {
    const int32_t *r = t->report_host + b * kReportStride;
    Slot &ts = t->slots[t_slots[b]];
    ts.kv_len = r[0];
    ts.n_gen = r[1];
    ts.iteration = (uint32_t)r[kReportStride - 1];
    const int a = r[2];
    if (out_n_accepted) out_n_accepted[b] = a;
    if (out_drafts)
      for (int i = 0; i < k; ++i) out_drafts[b * k + i] = i < L ? r[4 + i] : -1;
    if (out_tokens)
      for (int i = 0; i <= k; ++i) out_tokens[b * (k + 1) + i] = i <= a ? r[4 + kMaxK + i] : -1;
    if (a == L) again.push_back(d_slots[b]);
  }
  if (!again.empty() && (rc = sps_drafter_step(d, again.data(), (int)again.size(), sp, L + 1))) {
    fail(t, rc, "drafter: %s", d->err.c_str());
    return rc;
  }
  // the drafter follows the target: rows of rejected drafts are dead, the last token is the target's
  ptrs.clear();
  vals.clear();
  for (int b = 0; b < n_slots; ++b) {
    const int32_t *r = t->report_host + b * kReportStride;
    Slot &ds = d->slots[d_slots[b]];
    ds.kv_len = r[0];
    ds.n_gen = r[1];
    ds.iteration = t->slots[t_slots[b]].iteration;
    ptrs.push_back(d->P.kv_len + d_slots[b]);
    vals.push_back(r[0]);
    ptrs.push_back(d->P.n_gen + d_slots[b]);  // (the drafter's own token buffer holds drafts: only its count follows)
    vals.push_back(std::min(r[1], d->P.gen_cap));
    ptrs.push_back(d->P.pending + d_slots[b]);
    vals.push_back(r[4 + kMaxK + r[2]]);
  }
  if ((rc = poke(d, ptrs, vals))) { fail(t, rc, "drafter: %s", d->err.c_str()); return rc; }
  HIP_TRY(t, hipStreamSynchronize(d->stream));
  return PASS_OK;
}

// Algorithm 1's loop, pipelined: iteration i + 1 is issued before the report of iteration i (36 ints per
// slot, stored by a small kernel straight into pinned host memory) has been read, so the device never
// waits for the host.  Until a report lands the host only knows an upper bound of every sequence's
// length (an iteration adds at most k + 2 positions): pages are provided and the attention grid is
// sized for that bound; the exact lengths live on the device.
// target < 0: exactly n_iters iterations.  target >= 0: until every slot has made `target` tokens
// since start[b]; the next iteration is issued blind only while some slot needs it even if the
// iteration in flight yields all k + 2 tokens, otherwise the report is read first, so no iteration
// runs that Algorithm 1 would not run.  Slots that have reached the target are frozen on the device.
static int run_pipeline(pass_ctx *c, const int32_t *slots, int n_slots, int n_iters, int target, const int *start,
                        const pass_sampling *sp, pass_stats &st) {
  const int k = c->cfg.k;
  const size_t rep_ints = (size_t)c->cfg.max_slots * kReportStride;
  const int grow = c->P.k_act + 2;
  auto retire = [&](int par) -> int {
    HIP_TRY(c, hipEventSynchronize(c->ev2[par][3]));
    float ms_d = 0, ms_v = 0;
    HIP_TRY(c, hipEventElapsedTime(&ms_d, c->ev2[par][0], c->ev2[par][1]));
    HIP_TRY(c, hipEventElapsedTime(&ms_v, c->ev2[par][1], c->ev2[par][2]));
    st.draft_ms += ms_d;
    st.verify_ms += ms_v;
    for (int b = 0; b < n_slots; ++b) {
      const int32_t *r = c->report_host + par * rep_ints + b * kReportStride;
      Slot &s = c->slots[slots[b]];
      if (target < 0 || r[1] != s.n_gen) {  // the slot was live in this iteration (a frozen one adds nothing)
        st.iterations += 1;
        st.drafts_proposed += c->P.k_act;
        st.drafts_accepted += r[2];
      }
      if (target < 0) st.tokens_out += r[1] - s.n_gen;
      s.kv_len = r[0];
      s.n_gen = r[1];
      s.iteration = (uint32_t)r[kReportStride - 1];
    }
    return PASS_OK;
  };
  int pending = -1;  // parity of the iteration whose report has not been read, or -1
  auto loop = [&]() -> int {
    for (int it = 0; target >= 0 || it < n_iters; ++it) {
      const int par = it & 1;
      int rc2;
      if (target >= 0) {
        bool all_done = true, certain = false;
        for (int b = 0; b < n_slots; ++b) {
          const int made = c->slots[slots[b]].n_gen - start[b];
          all_done &= made >= target;
          certain |= made + (pending >= 0 ? grow : 0) < target;
        }
        if (pending >= 0 && !certain) {  // the iteration in flight may be the last: look before going on
          const int was = pending;
          pending = -1;
          if ((rc2 = retire(was))) return rc2;
          --it;
          continue;
        }
        if (pending < 0 && all_done) return PASS_OK;
      }
      bool again = false;
      for (int b = 0; b < n_slots; ++b) {
        Slot &s = c->slots[slots[b]];
        const bool done = target >= 0 && s.n_gen - start[b] >= target;  // frozen on the device: needs no room
        if (!done && pending >= 0 && s.kv_len + grow + 2 + k > c->cfg.max_seq_len) {  // the bound no longer fits: use exact lengths
          const int was = pending;
          pending = -1;
          if ((rc2 = retire(was))) return rc2;
          again = target >= 0;  // the report may have finished the slot, or all of them
          if (again) break;
        }
        const int ub = s.kv_len + (!done && pending >= 0 ? grow : 0);  // a finished slot's length is exact and stays
        if (!done && ub + 2 + k > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "slot %d is full", slots[b]);
        // rows of a finished slot beyond its capacity are dead (row_is_dead): pages up to the capacity suffice
        if ((rc2 = ensure_pages(c, slots[b], std::min(ub + (done ? 1 : 2) + k, c->cfg.max_seq_len)))) return rc2;
      }
      if (again) { --it; continue; }
      c->kv_slack = pending >= 0 ? grow : 0;
      HIP_TRY(c, hipEventRecord(c->ev2[par][0], c->stream));
      if ((rc2 = issue_draft(c, slots, n_slots, sp, 1))) return rc2;
      HIP_TRY(c, hipEventRecord(c->ev2[par][1], c->stream));
      if ((rc2 = issue_verify(c, slots, n_slots, sp, 1))) return rc2;
      HIP_TRY(c, hipEventRecord(c->ev2[par][2], c->stream));
      gather_report_kernel<<<1, 64, 0, c->stream>>>(c->P, n_slots, c->report_host + par * rep_ints);
      HIP_TRY(c, hipGetLastError());
      HIP_TRY(c, hipEventRecord(c->ev2[par][3], c->stream));
      const int was = pending;
      pending = par;
      if (was >= 0 && (rc2 = retire(was))) return rc2;
    }
    return PASS_OK;
  };
  int rc = loop();
  // whatever happened, leave the host's view of the slots exact
  if (pending >= 0) {
    int rc2 = retire(pending);
    if (!rc) rc = rc2;
  }
  c->kv_slack = 0;
  return rc;
}

int pass_generate(pass_ctx *c, const int32_t *slots, int n_slots, int max_new, const pass_sampling *sp,
                  int32_t *out_tokens, pass_stats *out_stats) {
  if (!c) return PASS_EINVAL;
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 1))) return rc;
  if ((rc = check_sampling(c, sp))) return rc;
  if (max_new < 0 || (max_new > 0 && !out_tokens)) return fail(c, PASS_EINVAL, "bad max_new / out_tokens");
  const int k = c->cfg.k;
  pass_stats st;
  memset(&st, 0, sizeof st);
  std::vector<int> start(n_slots);
  std::vector<int32_t *> ptrs;
  std::vector<int32_t> vals;
  for (int b = 0; b < n_slots; ++b) {
    start[b] = c->slots[slots[b]].n_gen;
    if (start[b] + max_new + k + 1 > c->P.gen_cap) return fail(c, PASS_ECAPACITY, "slot %d: token buffer too small", slots[b]);
    ptrs.push_back(c->P.gen_limit + slots[b]);
    vals.push_back(start[b] + max_new);
  }
  if ((rc = poke(c, ptrs, vals))) return rc;
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  rc = run_pipeline(c, slots, n_slots, 0, max_new, start.data(), sp, st);
  if (!rc)
    for (int b = 0; b < n_slots; ++b) {
      if (max_new > 0)
        HIP_TRY(c, hipMemcpyAsync(out_tokens + (size_t)b * max_new, c->P.gen + (size_t)slots[b] * c->P.gen_cap + start[b],
                                  sizeof(int32_t) * max_new, hipMemcpyDeviceToHost, c->stream));
      st.tokens_out += max_new;
    }
  // the token targets go away with the call
  for (int b = 0; b < n_slots; ++b) { ptrs.push_back(c->P.gen_limit + slots[b]); vals.push_back(INT_MAX); }
  const int r2 = poke(c, ptrs, vals);
  (void)hipStreamSynchronize(c->stream);
  if (!rc) rc = r2;
  if (!rc && out_stats) *out_stats = st;
  return rc;
}

int pass_run_iterations(pass_ctx *c, const int32_t *slots, int n_slots, int n_iters, const pass_sampling *sp,
                        pass_stats *out_stats) {
  if (!c) return PASS_EINVAL;
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 1))) return rc;
  if ((rc = check_sampling(c, sp))) return rc;
  if (n_iters < 0) return fail(c, PASS_EINVAL, "n_iters negative");
  pass_stats st;
  memset(&st, 0, sizeof st);
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  rc = run_pipeline(c, slots, n_slots, n_iters, -1, nullptr, sp, st);
  if (!rc && out_stats) *out_stats = st;
  return rc;
}

int pass_kernel_time(pass_ctx *c, double *total_ms, int64_t *launches) {
  if (!c || !total_ms || !launches) return PASS_EINVAL;
  *total_ms = c->kernel_ms;
  *launches = c->kernel_launches;
  return PASS_OK;
}

int pass_plain_read(pass_ctx *c, size_t bytes, int iters, double *out_us) {
  if (!c) return PASS_EINVAL;
  if (!c->weights_loaded) return fail(c, PASS_ESTATE, "weights not loaded");
  // the model's tensors lie back to back in the arena, from the embedding table to the staging area
  const char *base = (const char *)c->tok_emb;
  const size_t span = (size_t)((const char *)c->staging - base);
  if (!out_us || iters < 1 || bytes == 0 || bytes % 16 || bytes > span) return fail(c, PASS_EINVAL, "bad argument");
  HIP_TRY(c, hipEventRecord(c->ev[0], c->stream));
  size_t off = 0;
  for (int i = 0; i < iters; ++i) {
    if (off + bytes > span) off = 0;
    launch_plain_read(base + off, bytes, (uint32_t *)c->P.fallbacks, c->stream);
    off += bytes;
  }
  HIP_TRY(c, hipEventRecord(c->ev[1], c->stream));
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  float ms = 0;
  HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[0], c->ev[1]));
  *out_us = (double)ms * 1e3 / iters;
  return PASS_OK;
}

int pass_rng_uniforms(pass_ctx *c, uint64_t seed, uint32_t seq_id, uint32_t iteration, uint32_t row, uint32_t purpose,
                      uint32_t first, size_t n, float *out) {
  if (!c) return PASS_EINVAL;
  if (!out || row > 255u || purpose > 3u || first % 4u || (uint64_t)first + n > ((uint64_t)1 << 32))
    return fail(c, PASS_EINVAL, "bad argument");
  // staged through the validation call's logits, in pieces of that buffer's size
  const size_t cap = ((size_t)c->cfg.max_slots * (1 + c->cfg.k) * c->cfg.vocab) & ~(size_t)3;
  if (cap == 0) return fail(c, PASS_ECAPACITY, "no staging room");
  for (size_t done = 0; done < n;) {
    const size_t m = std::min(cap, n - done);
    launch_rng_uniforms(c->P.verify_logits, first + (uint32_t)done, (int)m, seed, seq_id, iteration, row, purpose, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemcpyAsync(out + done, c->P.verify_logits, m * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    done += m;
  }
  return PASS_OK;
}

int pass_get_logits(pass_ctx *c, int slot, int which, float *out) {
  if (!c) return PASS_EINVAL;
  if (slot < 0 || slot >= c->cfg.max_slots || !out || (which != 0 && which != 1)) return fail(c, PASS_EINVAL, "bad argument");
  size_t n = (size_t)(1 + c->cfg.k) * c->cfg.vocab;
  const float *src = (which ? c->P.verify_logits : c->P.draft_logits) + (size_t)slot * n;
  HIP_TRY(c, hipMemcpyAsync(out, src, n * sizeof(float), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PASS_OK;
}

int pass_get_tokens(pass_ctx *c, int slot, int first, int n, int32_t *out) {
  if (!c) return PASS_EINVAL;
  if (slot < 0 || slot >= c->cfg.max_slots || first < 0 || n < 0 || !out) return fail(c, PASS_EINVAL, "bad argument");
  if (c->slots[slot].state == 0) return fail(c, PASS_ESTATE, "slot %d is empty", slot);
  if ((int64_t)first + n > c->slots[slot].n_gen)
    return fail(c, PASS_ECAPACITY, "slot %d has generated %d tokens", slot, c->slots[slot].n_gen);
  if (n == 0) return PASS_OK;
  HIP_TRY(c, hipMemcpyAsync(out, c->P.gen + (size_t)slot * c->P.gen_cap + first, sizeof(int32_t) * n,
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PASS_OK;
}

size_t pass_train_bytes(pass_ctx *c) {
  if (!c || !c->weights_loaded || c->cfg.k < 1) return 0;
  return carve_train(c->cfg, c->use_mfma, nullptr, nullptr);
}

int pass_train_begin(pass_ctx *c, void *device_workspace, size_t bytes, int32_t init_token) {
  if (!c) return PASS_EINVAL;
  if (!c->weights_loaded) return fail(c, PASS_ESTATE, "weights not loaded");
  if (c->use_mfma && (c->P.d % 64 || c->P.D % 64 || c->P.F % 64 || c->P.V % 32))
    return fail(c, PASS_ESTATE, "training on the matrix-core path needs d_model, n_heads * head_dim and d_ffn in multiples of 64 and the "
                                "vocabulary in multiples of 32: load the model with the \"path\" option at 1");
  if (c->cfg.k < 1) return fail(c, PASS_EINVAL, "the model has no look-ahead embeddings (k = 0)");
  if (c->P.d > 8192 || c->P.d % 4) return fail(c, PASS_ESTATE, "training takes models of d_model up to 8192, in multiples of 4");
  if (!device_workspace || ((uintptr_t)device_workspace & 255) || bytes < carve_train(c->cfg, c->use_mfma, nullptr, nullptr))
    return fail(c, PASS_EINVAL, "training workspace null, misaligned or smaller than pass_train_bytes");
  if (init_token >= c->cfg.vocab) return fail(c, PASS_EINVAL, "init_token outside the vocabulary");
  carve_train(c->cfg, c->use_mfma, (char *)device_workspace, &c->train);
  if (c->use_mfma) {
    const int d = c->P.d, D = c->P.D, F = c->P.F, V = c->P.V;
    launch_transpose_packed(c->lm_head, c->train.lm_head_t, V, d, c->stream);
    for (int l = 0; l < c->P.L; ++l) {
      const LayerW &w = c->layers[l], &t = c->train.layers_t[l];
      launch_transpose_packed(w.wqkv, t.wqkv, 3 * D, d, c->stream);
      launch_transpose_packed(w.wo, t.wo, d, D, c->stream);
      launch_transpose_packed(w.wgu, t.wgu, 2 * F, d, c->stream);
      launch_transpose_packed(w.wdown, t.wdown, d, F, c->stream);
    }
    HIP_TRY(c, hipGetLastError());
  }
  if (!c->train_loss_host) HIP_TRY(c, hipHostMalloc((void **)&c->train_loss_host, sizeof(float) * kMaxRows, hipHostMallocDefault));
  launch_lookahead_init(c->cfg.dtype, c->tok_emb, c->lookahead, init_token, c->cfg.k, c->P.d, c->train.master, c->train.m1,
                        c->train.m2, c->stream);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->train.on = true;
  c->train.step = 0;
  return PASS_OK;
}

int pass_train_step(pass_ctx *c, const int32_t *slots, int n_slots, const int32_t *targets, const pass_adamw *opt, float *out_loss) {
  if (!c) return PASS_EINVAL;
  if (!c->train.on) return fail(c, PASS_ESTATE, "pass_train_begin has not been called");
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 1))) return rc;
  if (!targets || !opt || !(opt->lr >= 0.f) || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) ||
      !(opt->eps > 0.f) || !(opt->weight_decay >= 0.f))
    return fail(c, PASS_EINVAL, "bad targets / optimiser parameters");
  const int k = c->cfg.k, R = 1 + k, M = n_slots * R;
  if (c->P.k_act != k || c->P.la_token >= 0)
    return fail(c, PASS_ESTATE, "training uses all k look-ahead embeddings (\"lookahead_rows\" = k, \"lookahead_token\" = -1)");
  int max_keys = 1;
  std::vector<int32_t> tg(M);
  for (int b = 0; b < n_slots; ++b) {
    const Slot &s = c->slots[slots[b]];
    if (s.kv_len + R > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "slot %d is full", slots[b]);
    if (s.kv_len + R > kTrainMaxKeys) return fail(c, PASS_ECAPACITY, "slot %d: a training step takes at most %d keys", slots[b], kTrainMaxKeys);
    if ((rc = ensure_pages(c, slots[b], s.kv_len + R))) return rc;
    max_keys = std::max(max_keys, s.kv_len + R);
    tg[b * R] = -1;  // the row of w_T predicts w_{T+1}: no loss there
    for (int i = 0; i < k; ++i) {
      const int32_t t = targets[b * k + i];
      if (t < 0 || t >= c->cfg.vocab) return fail(c, PASS_EINVAL, "target %d of slot %d outside the vocabulary", i, slots[b]);
      tg[b * R + 1 + i] = t;
    }
  }
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  TrainWs &T = c->train;
  Params P = c->P;
  const int dt = c->cfg.dtype;
  hipStream_t s = c->stream;
  const size_t d = P.d, D = P.D, F = P.F, V = P.V, H = P.H;
  HIP_TRY(c, hipMemcpyAsync(T.targets, tg.data(), sizeof(int32_t) * M, hipMemcpyHostToDevice, s));
  const int S = choose_splits(c, n_slots, R, max_keys);
  const float loss_scale = 1.0f / (float)(n_slots * k);
  if (T.mfma) {
    // ---- forward: the drafting call's own kernels (the gate/up product also keeps its pre-activations); each
    // layer's q, attention output and ln-sum-exp land in that layer's area ----
    launch_assemble_train_mfma(P, c->tok_emb, T.master, c->layers[0].attn_norm, n_slots, R, s);
    for (int l = 0; l < P.L; ++l) {
      const LayerW &w = c->layers[l];
      P.qkv = T.save_qkv + (size_t)l * kMaxRows * 3 * D;
      P.attn_x = (uint16_t *)(T.save_attn + (size_t)l * kMaxRows * D);
      P.lse = T.save_lse + (size_t)l * kMaxRows * H;
      HIP_TRY(c, hipMemcpyAsync(T.save_h0 + (size_t)l * kMaxRows * d, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
      launch_gemm_qkv(P, c->tuning, w.wqkv, l, M, s);
      launch_attention(P, dt, l, n_slots, R, S, 1, s);
      launch_gemm_resid(P, c->tuning, w.wo, P.attn_x, P.D, w.ffn_norm, M, s);
      HIP_TRY(c, hipMemcpyAsync(T.save_h1 + (size_t)l * kMaxRows * d, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
      launch_gemm_gateup_save(P, w.wgu, T.save_gu + (size_t)l * kMaxRows * 2 * F, M, s);
      launch_gemm_resid(P, c->tuning, w.wdown, P.act_x, P.F, l + 1 < P.L ? c->layers[l + 1].attn_norm : c->final_norm, M, s);
    }
    HIP_TRY(c, hipMemcpyAsync(T.save_hl, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
    launch_gemm_logits(P, c->tuning, c->lm_head, T.logits, M, s);
    // ---- backward: every dx = W^T dy is a matrix-core product with the packed transpose; its input travels as
    // (hi, lo) tiles (T.x), its output as slices over the contraction (T.part) that the consumer adds up ----
    const size_t rows = kMaxRows;
    launch_ce_grad(T.logits, T.targets, loss_scale, T.row_loss, M, P.V, T.x, s);
    int KS = launch_gemm_plain(P, T.lm_head_t, T.x, M, (int)d, (int)V, T.part, s);
    launch_rmsnorm_bwd(P, dt, T.save_hl, c->final_norm, T.part, KS, rows * d, T.dh, M, 0, T.x, s);
    for (int l = P.L - 1; l >= 0; --l) {
      const LayerW &w = c->layers[l], &t = T.layers_t[l];
      KS = launch_gemm_plain(P, t.wdown, T.x, M, (int)F, (int)d, T.part, s);
      launch_swiglu_bwd_tiles(P, T.save_gu + (size_t)l * kMaxRows * 2 * F, T.part, KS, rows * F, T.x, M, s);
      KS = launch_gemm_plain(P, t.wgu, T.x, M, (int)d, (int)(2 * F), T.part, s);
      launch_rmsnorm_bwd(P, dt, T.save_h1 + (size_t)l * kMaxRows * d, w.ffn_norm, T.part, KS, rows * d, T.dh, M, 1, T.x, s);
      KS = launch_gemm_plain(P, t.wo, T.x, M, (int)D, (int)d, T.part, s);
      launch_attn_bwd(P, dt, l, n_slots, R, max_keys, T.save_qkv + (size_t)l * kMaxRows * 3 * D, (int)(3 * D), nullptr,
                      (const uint16_t *)(T.save_attn + (size_t)l * kMaxRows * D), T.save_lse + (size_t)l * kMaxRows * H, T.part, KS,
                      rows * D, T.dq_part, T.dqkv, T.x, s);
      KS = launch_gemm_plain(P, t.wqkv, T.x, M, (int)d, (int)(3 * D), T.part, s);
      launch_rmsnorm_bwd(P, dt, T.save_h0 + (size_t)l * kMaxRows * d, w.attn_norm, T.part, KS, rows * d, T.dh, M, 1, T.x, s);
    }
  } else {
    // ---- forward: the drafting call on the generic kernels, look-ahead rows from the master values; each layer
    // works in its own area of the workspace, so what the backward pass needs is simply left there ----
    launch_assemble_train(P, dt, c->tok_emb, T.master, n_slots, R, s);
    for (int l = 0; l < P.L; ++l) {
      const LayerW &w = c->layers[l];
      P.qkv = T.save_qkv + (size_t)l * kMaxRows * 3 * D;
      P.attn = T.save_attn + (size_t)l * kMaxRows * D;
      P.lse = T.save_lse + (size_t)l * kMaxRows * H;
      P.gu = T.save_gu + (size_t)l * kMaxRows * 2 * F;
      HIP_TRY(c, hipMemcpyAsync(T.save_h0 + (size_t)l * kMaxRows * d, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
      launch_rmsnorm(P, dt, P.h, w.attn_norm, P.xn, M, s);
      launch_gemm_generic(dt, P.xn, w.wqkv, P.qkv, M, 3 * P.D, P.d, 3 * P.D, nullptr, 0, s);
      launch_rope_kv(P, dt, l, M, s);
      launch_attention(P, dt, l, n_slots, R, S, 0, s);
      launch_gemm_generic(dt, P.attn, w.wo, P.h, M, P.d, P.D, P.d, nullptr, 1, s);
      HIP_TRY(c, hipMemcpyAsync(T.save_h1 + (size_t)l * kMaxRows * d, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
      launch_rmsnorm(P, dt, P.h, w.ffn_norm, P.xn, M, s);
      launch_gemm_generic(dt, P.xn, w.wgu, P.gu, M, 2 * P.F, P.d, 2 * P.F, nullptr, 0, s);
      launch_silu_mul(P, M, s);
      launch_gemm_generic(dt, P.act, w.wdown, P.h, M, P.d, P.F, P.d, nullptr, 1, s);
    }
    HIP_TRY(c, hipMemcpyAsync(T.save_hl, P.h, sizeof(float) * M * d, hipMemcpyDeviceToDevice, s));
    launch_rmsnorm(P, dt, P.h, c->final_norm, P.xn, M, s);
    launch_gemm_generic(dt, P.xn, c->lm_head, T.logits, M, P.V, P.d, P.V, nullptr, 0, s);
    // ---- loss on the look-ahead rows and its gradient, back through the frozen model ----
    launch_ce_grad(T.logits, T.targets, loss_scale, T.row_loss, M, P.V, nullptr, s);
    launch_gemm_t(dt, T.logits, (int)V, c->lm_head, T.part, T.dxn, (int)d, M, (int)V, (int)d, s);
    launch_rmsnorm_bwd(P, dt, T.save_hl, c->final_norm, T.dxn, 1, 0, T.dh, M, 0, nullptr, s);
    for (int l = P.L - 1; l >= 0; --l) {
      const LayerW &w = c->layers[l];
      launch_gemm_t(dt, T.dh, (int)d, w.wdown, T.part, T.dact, (int)F, M, (int)d, (int)F, s);
      launch_swiglu_bwd(P, T.save_gu + (size_t)l * kMaxRows * 2 * F, T.dact, T.dgu, M, s);
      launch_gemm_t(dt, T.dgu, (int)(2 * F), w.wgu, T.part, T.dxn, (int)d, M, (int)(2 * F), (int)d, s);
      launch_rmsnorm_bwd(P, dt, T.save_h1 + (size_t)l * kMaxRows * d, w.ffn_norm, T.dxn, 1, 0, T.dh, M, 1, nullptr, s);
      launch_gemm_t(dt, T.dh, (int)d, w.wo, T.part, T.dattn, (int)D, M, (int)d, (int)D, s);
      launch_attn_bwd(P, dt, l, n_slots, R, max_keys, T.save_qkv + (size_t)l * kMaxRows * 3 * D, (int)(3 * D),
                      T.save_attn + (size_t)l * kMaxRows * D, nullptr, T.save_lse + (size_t)l * kMaxRows * H, T.dattn, 1, 0,
                      T.dq_part, T.dqkv, nullptr, s);
      launch_gemm_t(dt, T.dqkv, (int)(3 * D), w.wqkv, T.part, T.dxn, (int)d, M, (int)(3 * D), (int)d, s);
      launch_rmsnorm_bwd(P, dt, T.save_h0 + (size_t)l * kMaxRows * d, w.attn_norm, T.dxn, 1, 0, T.dh, M, 1, nullptr, s);
    }
  }
  // ---- AdamW on the look-ahead embeddings; the model's own tensor follows in its storage type ----
  T.step += 1;
  const float bc1 = (float)(1.0 - pow((double)opt->beta1, (double)T.step)), bc2 = (float)(1.0 - pow((double)opt->beta2, (double)T.step));
  launch_lookahead_adamw(dt, T.dh, n_slots, R, P.d, T.grad, T.master, T.m1, T.m2, c->lookahead, opt->lr, opt->beta1, opt->beta2,
                         opt->eps, opt->weight_decay, bc1, bc2, s);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipMemcpyAsync(c->train_loss_host, T.row_loss, sizeof(float) * M, hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  if (out_loss) {
    double sum = 0;
    for (int m = 0; m < M; ++m) sum += c->train_loss_host[m];
    *out_loss = (float)(sum / (n_slots * k));
  }
  return PASS_OK;
}

int pass_train_read(pass_ctx *c, int what, float *out) {
  if (!c) return PASS_EINVAL;
  if (!c->train.on) return fail(c, PASS_ESTATE, "pass_train_begin has not been called");
  if (!out || what < 0 || what > 3) return fail(c, PASS_EINVAL, "bad argument");
  const float *src[4] = {c->train.master, c->train.grad, c->train.m1, c->train.m2};
  HIP_TRY(c, hipMemcpyAsync(out, src[what], sizeof(float) * c->cfg.k * c->P.d, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PASS_OK;
}

int pass_train_resume(pass_ctx *c, const float *master, const float *m1, const float *m2, int64_t steps) {
  if (!c) return PASS_EINVAL;
  if (!c->train.on) return fail(c, PASS_ESTATE, "pass_train_begin has not been called");
  if (steps < 0 || steps > (int64_t)1 << 40) return fail(c, PASS_EINVAL, "bad step count");
  const size_t bytes = sizeof(float) * c->cfg.k * c->P.d;
  const float *src[3] = {master, m1, m2};
  float *dst[3] = {c->train.master, c->train.m1, c->train.m2};
  for (int i = 0; i < 3; ++i)  // pageable host memory: the copy has left the caller's array when the call returns
    if (src[i]) HIP_TRY(c, hipMemcpyAsync(dst[i], src[i], bytes, hipMemcpyHostToDevice, c->stream));
  if (master) {
    launch_lookahead_store(c->cfg.dtype, c->train.master, c->cfg.k, c->P.d, c->lookahead, c->stream);
    HIP_TRY(c, hipGetLastError());
  }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->train.step = steps;
  return PASS_OK;
}

int pass_prefill_plan(int rows_per_pass, const int32_t *lens, int n, int max_segs, int32_t *out_segs, int *n_segs) {
  if (rows_per_pass < kPrefillBlockRows || rows_per_pass % kPrefillBlockRows || !lens || n < 1 || !n_segs || (max_segs > 0 && !out_segs))
    return PASS_EINVAL;
  for (int b = 0; b < n; ++b)
    if (lens[b] < 1) return PASS_EINVAL;
  const std::vector<PlanSeg> plan = plan_prefill(rows_per_pass, lens, n);
  *n_segs = (int)plan.size();
  if ((int)plan.size() > max_segs) return PASS_ECAPACITY;
  for (size_t i = 0; i < plan.size(); ++i) {
    int32_t *o = out_segs + 5 * i;
    o[0] = plan[i].pass; o[1] = plan[i].prompt; o[2] = plan[i].pos0; o[3] = plan[i].rows; o[4] = plan[i].row_base;
  }
  return PASS_OK;
}

int pass_attention_plan(int n_heads, int n_keys, int *n_splits, int *chunk_keys, int *grid_splits) {
  if (n_heads < 1 || n_keys < 1) return PASS_EINVAL;
  int ns, ch;
  split_plan_mfma(n_keys, n_heads, ns, ch);
  if (n_splits) *n_splits = ns;
  if (chunk_keys) *chunk_keys = ch;
  if (grid_splits) *grid_splits = max_splits_mfma(n_keys, n_heads);
  return PASS_OK;
}

int pass_seq_len(pass_ctx *c, int slot, int32_t *kv_len, int32_t *n_generated) {
  if (!c) return PASS_EINVAL;
  if (slot < 0 || slot >= c->cfg.max_slots) return fail(c, PASS_EINVAL, "slot %d out of range", slot);
  if (c->slots[slot].state == 0) return fail(c, PASS_ESTATE, "slot %d is empty", slot);
  if (kv_len) *kv_len = c->slots[slot].kv_len;
  if (n_generated) *n_generated = c->slots[slot].n_gen;
  return PASS_OK;
}

int pass_set_option(pass_ctx *c, const char *name, int value) {
  if (!c || !name) return PASS_EINVAL;
  if (!strcmp(name, "graph")) { c->opt_graph = value; return PASS_OK; }
  // "tune.*": sweep knobs for development, not part of the stable interface (listed here only)
  //   tune.gemm_cfg       launch shape of the decode-sized matrix-core GEMMs of this context:
  //                       kind * 10000 + wavefronts * 100 + unroll (kind 0 QKV, 1 Wo, 2 gate/up, 3 LM head, 4 down;
  //                       wavefronts 4/8/16; unroll 1/2/4); calls with more than 8 rows: 1000000 + kind * 10000 +
  //                       wavefronts * 100 + blocks (strips of 16 output features per workgroup, 0..4);
  //                       2000000 + K slices of the split residual GEMM (0 = never split)
  //   tune.prefill_rows   prompt rows per pass of the tiled prompt pass (a multiple of 128)
  //   tune.prefill_tile   query rows per attention workgroup of the tiled prompt pass (0, 16, 32, 128)
  //   tune.prefill_block  tiles along the features * 100 + tiles along the rows of the block of GEMM tiles one die
  //                       works on at a time (0 = default 8 x 8)
  //   tune.prefill_strips strips of 16 features per wavefront in the tiled GEMMs (0 = by row count, 1, 2, 4)
  if (!strcmp(name, "tune.gemm_cfg")) {
    if (value >= 2000000) {
      if (c->tuning.set_split(value - 2000000)) return fail(c, PASS_EINVAL, "tune.gemm_cfg (split residual GEMM): 0 .. 8 slices of K");
    } else if (value >= 1000000) {
      int v = value - 1000000;
      if (c->tuning.set_big(v / 10000, (v / 100) % 100, v % 100))
        return fail(c, PASS_EINVAL, "tune.gemm_cfg (more than 8 rows): kind 0..4, wavefronts 4/8/16, blocks 0..4");
    } else if (c->tuning.set(value / 10000, (value / 100) % 100, value % 100))
      return fail(c, PASS_EINVAL, "tune.gemm_cfg: kind 0..4, wavefronts 4/8/16, unroll 1/2/4");
    for (auto &g : c->graphs) (void)hipGraphExecDestroy(g.second);  // captured launches carry the old shape
    c->graphs.clear();
    return PASS_OK;
  }
  if (!strcmp(name, "lookahead_rows") || !strcmp(name, "lookahead_token")) {
    for (const Slot &s : c->slots)
      if (s.state == 2) return fail(c, PASS_ESTATE, "%s cannot change between a drafting and a validation call", name);
    if (!strcmp(name, "lookahead_rows")) {
      if (value < 0 || value > c->cfg.k) return fail(c, PASS_EINVAL, "lookahead_rows: 0 .. k (%d)", c->cfg.k);
      c->P.k_act = value;
    } else {
      if (value < -1 || value >= c->cfg.vocab) return fail(c, PASS_EINVAL, "lookahead_token: -1 (embeddings) or a token id");
      c->P.la_token = value;
    }
    return PASS_OK;
  }
  if (!strcmp(name, "prefill_chunk")) {
    if (value < 1 || value > kMaxRows) return fail(c, PASS_EINVAL, "prefill_chunk: 1 .. %d", kMaxRows);
    c->opt_prefill_chunk = value;
    return PASS_OK;
  }
  if (!strcmp(name, "prefill_tiled")) {
    if (value < -1 || value > 1) return fail(c, PASS_EINVAL, "prefill_tiled: -1 (by prompt length), 0 (never) or 1 (always)");
    c->opt_prefill_tiled = value;
    return PASS_OK;
  }
  if (!strcmp(name, "tune.prefill_rows")) {
    const int cap = std::min(kPrefillRows, (c->cfg.max_seq_len + 127) / 128 * 128);
    if (value < 128 || value > cap || value % 128) return fail(c, PASS_EINVAL, "tune.prefill_rows: a multiple of 128, 128 .. %d", cap);
    c->pws.rows = value;
    return PASS_OK;
  }
  if (!strcmp(name, "tune.prefill_tile")) {
    // query rows of an attention workgroup of the tiled prompt pass
    if (value != 0 && value != 16 && value != 32 && value != 128) return fail(c, PASS_EINVAL, "tune.prefill_tile: 0 (default), 16, 32 or 128");
    c->pws.attn_rows = value;
    return PASS_OK;
  }
  if (!strcmp(name, "tune.prefill_strips")) {
    if (value != 0 && value != 1 && value != 2 && value != 4) return fail(c, PASS_EINVAL, "tune.prefill_strips: 0 (by row count), 1, 2 or 4");
    c->pws.resid_strips_opt = value;
    return PASS_OK;
  }
  if (!strcmp(name, "tune.prefill_block")) {
    const int bn = value / 100, bm = value % 100;
    if (value < 0 || bn > 64 || bm > 64 || (bn == 0) != (bm == 0)) return fail(c, PASS_EINVAL, "tune.prefill_block: tiles along the features * 100 + tiles along the rows (1 .. 64 each), or 0");
    c->pws.blk_n = bn;
    c->pws.blk_m = bm;
    return PASS_OK;
  }
  if (!strcmp(name, "kernel_timing")) {
    c->opt_kernel_timing = value;
    c->kernel_ms = 0;
    c->kernel_launches = 0;
    return PASS_OK;
  }
  if (!strcmp(name, "attention")) {
    if (c->weights_loaded) return fail(c, PASS_ESTATE, "\"attention\" must be set before pass_load_weights");
    c->opt_attn = value;
    return PASS_OK;
  }
  if (!strcmp(name, "path")) {
    if (c->weights_loaded) return fail(c, PASS_ESTATE, "\"path\" must be set before pass_load_weights");
    c->opt_path = value;
    return PASS_OK;
  }
  return fail(c, PASS_EINVAL, "unknown option %s", name);
}

int pass_time_step(pass_ctx *c, const int32_t *slots, int n_slots, int warmup, int iters, double *out_ms) {
  if (!c) return PASS_EINVAL;
  int rc;
  if ((rc = check_slots(c, slots, n_slots, 1))) return rc;
  if (iters < 1 || warmup < 0 || !out_ms) return fail(c, PASS_EINVAL, "bad argument");
  const int k = c->cfg.k;
  for (int b = 0; b < n_slots; ++b) {
    if (c->slots[slots[b]].kv_len + 1 + k > c->cfg.max_seq_len) return fail(c, PASS_ECAPACITY, "slot %d is full", slots[b]);
    if ((rc = ensure_pages(c, slots[b], c->slots[slots[b]].kv_len + 1 + k))) return rc;
  }
  if ((rc = set_step_slots(c, slots, n_slots))) return rc;
  pass_sampling sp = {0.f, 0, 0};
  for (int i = 0; i < warmup + iters; ++i) {
    if (i == warmup) HIP_TRY(c, hipEventRecord(c->ev[0], c->stream));
    if ((rc = issue_draft(c, slots, n_slots, &sp, 0))) return rc;
  }
  HIP_TRY(c, hipEventRecord(c->ev[1], c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  float ms = 0;
  HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[0], c->ev[1]));
  *out_ms = (double)ms / iters;
  return PASS_OK;
}

const char *pass_last_error(pass_ctx *c) { return c ? c->err.c_str() : g_create_error.c_str(); }

void pass_destroy(pass_ctx *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (auto &ev : c->ev) (void)hipEventDestroy(ev);
  for (auto &set : c->ev2)
    for (auto &ev : set) (void)hipEventDestroy(ev);
  for (auto &ev : c->kev) (void)hipEventDestroy(ev);
  for (auto &g : c->graphs) (void)hipGraphExecDestroy(g.second);
  if (c->report_host) (void)hipHostFree(c->report_host);
  if (c->block_table_host) (void)hipHostFree(c->block_table_host);
  if (c->train_loss_host) (void)hipHostFree(c->train_loss_host);
  delete c;
}

}  // extern "C"
