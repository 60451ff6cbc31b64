/*
 * pass_oracle.c -- plain CPU oracle for the PaSS (parallel speculative sampling) decode path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * accelerated path must compute.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper with the HIP
 * library, and the HIP library never calls it.
 *
 * What it implements, and from where:
 *   - A LLaMA-style decoder-only transformer forward with a per-sequence K/V cache
 *     (paper, Experiments: the authors' own 7B LLaMA re-implementation; Baselines: the KV
 *     cache is updated after every model call; Training details: bfloat16 models).
 *   - Algorithm 1 (PaSS): draft call on (last token, [LA]_1..[LA]_L), validation call on
 *     (x_{n+1}, drafts), accept chain r < min(1, p/d), residual resampling from (p - d)_+,
 *     extra token when every draft is accepted.  Section 2.2 gives the two-phase structure,
 *     Section 2.2.1 the look-ahead embeddings appended after the sequence.
 *   - Algorithm 2 (appendix: speculative sampling with a separate drafting model): L sequential
 *     single-row calls of the drafter, then the same validation call and accept / reject chain.
 *
 * Arithmetic: double precision everywhere, except where a storage format fixes the value:
 * weights are read in their storage type (fp32 or bfloat16), the K/V cache of a bfloat16 model
 * holds bfloat16 values (round-to-nearest-even on write), logits are emitted as fp32.
 * The bfloat16 of the paper's Training details is read as a statement about storage: nothing
 * between two matrix products is stored, so nothing else is rounded.  With act_bf16 = 1 the
 * oracle additionally rounds the tensors an all-bfloat16 execution would round (normalised
 * activations, q, attention output, gated FFN activation); that variant exists to measure how
 * far such an execution sits from this one, it is not the reference.  The residual stream stays
 * in double either way.
 *
 * Every row of a call is computed by the same sequence of operations whatever other rows share
 * the call, so a (1+k)-row call equals k+1 single-row calls bit for bit.
 *
 * Readings of the paper taken here (all listed in the design notes of the repository):
 *   - positions in the accept loop are relative to n after the "n <- n+1" that follows the
 *     draft call; each accepted draft grows the sequence by one token;
 *   - the draft distribution d_t is conditioned on the sequence without x_{n+1} (they are
 *     sampled in the same call), the target distribution p_t is conditioned on it;
 *   - p and d are post-temperature softmax distributions;
 *   - look-ahead rows take consecutive RoPE positions after the last token and an ordinary
 *     causal mask;
 *   - "sample" = Gumbel-max over the counter-based Philox4x32-10 generator, which is exact in
 *     distribution and independent of summation order; ties go to the lowest index;
 *   - r is drawn from the open interval (0,1); the test is ln r + ln d(x) < ln p(x);
 *   - temperature 0 means greedy: every sample is an argmax (the one-hot limit of the rule);
 *   - the second baseline (Baselines: a fixed [UNK] token in place of the trained look-ahead
 *     embeddings) is the same algorithm with the embedding of one fixed token appended k times;
 *   - top-k sampling (Experimental setup: k = 10, and k = 25 for pass@10): the draft and the
 *     target distribution are each the softmax over the row's own k largest logits (ties at the
 *     boundary go to the lower index), zero elsewhere; the accept test and the residual use
 *     these filtered distributions.  top_k = 0 means no filter; greedy ignores it.
 *
 * parity status: the forward pass of large random models has no external reference value
 * (structure is pinned by closed forms, row independence and greedy equivalence; absolute
 * logits of 7B/13B-shaped random models are "parity unpinned" beyond that).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_ROWS 64
#define ORC_MAX_K 15

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_DRAFT = 0, ORC_ACCEPT = 1, ORC_RESIDUAL = 2, ORC_BONUS = 3 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ESTATE = -2, ORC_ECAPACITY = -3 };

typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;    /* ORC_F32 / ORC_BF16: storage type of every model tensor */
  int32_t k;        /* number of look-ahead embeddings, L in Algorithm 1 */
  int32_t act_bf16; /* also round activations between matrix products to bfloat16 (see header) */
  int32_t la_token; /* < 0: the drafting call appends the look-ahead embeddings (PaSS);
                       >= 0: it appends the embedding of this fixed token k times instead (the
                       paper's second baseline, Baselines: a fixed [UNK] token as look-ahead) */
} orc_config;

typedef struct {
  const void *tok_emb, *lm_head, *final_norm, *lookahead;
  const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
  const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} orc_weights;

typedef struct {
  float temperature; /* 0 = greedy */
  int32_t top_k;     /* 0 = off; K > 0: sample from the K largest logits of a row only */
  uint64_t seed;
} orc_sampling;

typedef struct orc_model {
  orc_config c;
  const void *tok_emb, *lm_head, *final_norm, *lookahead;
  const void **attn_norm, **wq, **wk, **wv, **wo, **ffn_norm, **w_gate, **w_up, **w_down;
} orc_model;

typedef struct orc_seq {
  const orc_model *m;
  int32_t max_len;
  int32_t kv_len;      /* number of cached positions = (#tokens of the sequence) - 1 */
  int32_t pending;     /* last token of the sequence; its K/V are not cached yet */
  int32_t state;       /* 0 empty, 1 ready for draft, 2 ready for verify */
  uint32_t seq_id;
  uint32_t iteration;  /* PaSS iterations completed */
  int64_t n_generated;
  double *kc, *vc;     /* [n_layers][max_len][n_heads*head_dim] */
  int32_t first;               /* x_{n+1} of the running iteration */
  int32_t drafts[ORC_MAX_K];   /* drafted tokens of the running iteration */
  float *draft_logits;         /* [(1+k)][vocab] logits of the draft call */
  float *verify_logits;        /* [(1+k)][vocab] logits of the validation call */
  /* decision record of the last draft / verify call, for margin-aware comparisons */
  int32_t draft_stable[ORC_MAX_K + 1];
  int32_t accept_stable[ORC_MAX_K + 1];
  int32_t final_stable;
  int32_t fallback_count;      /* residual numerically empty after a reject */
} orc_seq;

/* ------------------------------------------------------------------------------------------ */
/* storage formats                                                                             */
/* ------------------------------------------------------------------------------------------ */
static inline double load_elem(const void *base, int dtype, size_t i) {
  if (dtype == ORC_F32) return (double)((const float *)base)[i];
  uint32_t u = (uint32_t)((const uint16_t *)base)[i] << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* round a double to the nearest bfloat16 value (8 significant bits), ties to even */
double orc_bf16_round(double x) {
  if (x == 0.0 || !isfinite(x)) return x;
  int e;
  double m = frexp(x, &e);            /* x = m * 2^e, 0.5 <= |m| < 1 */
  double r = nearbyint(ldexp(m, 8));  /* default rounding mode: ties to even */
  return ldexp(r, e - 8);
}

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3")   */
/* ------------------------------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The uniform variate attached to (seed, sequence id, iteration, row, purpose, index j).
 * key = (seed low, seed high); counter = (j / 4, iteration, row | purpose << 8, sequence id);
 * word j % 4 of the block; the top 23 bits give u = (bits + 0.5) * 2^-23 in (0,1), a value
 * that fp32 holds exactly.
 */
double orc_uniform(uint64_t seed, uint32_t seq_id, uint32_t iteration, uint32_t row,
                   uint32_t purpose, uint32_t j) {
  uint32_t ctr[4] = {j >> 2, iteration, row | (purpose << 8), seq_id};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return ((double)(out[j & 3] >> 9) + 0.5) * (1.0 / 8388608.0);
}

/* out[i] = orc_uniform(.., first + i) for i < n: the same variates, many at a time, for tests. */
void orc_uniforms(uint64_t seed, uint32_t seq_id, uint32_t iteration, uint32_t row, uint32_t purpose,
                  uint32_t first, size_t n, double *out) {
  for (size_t i = 0; i < n; ++i) out[i] = orc_uniform(seed, seq_id, iteration, row, purpose, first + (uint32_t)i);
}

static inline double gumbel(double u) { return -log(-log(u)); }

/* ------------------------------------------------------------------------------------------ */
/* sampling primitives (Algorithm 1: "sample", accept test, residual)                          */
/* ------------------------------------------------------------------------------------------ */
typedef struct {
  uint64_t seed;
  uint32_t seq_id, iteration, row, purpose;
} orc_ctr;

/*
 * Top-k filter: keep[j] = 1 for the K largest logits of the row, found one maximum at a time
 * (ties: lower index first); K <= 0 or K >= V keeps every entry.  Returns 1 iff the kept set
 * cannot change when every score l_j * inv_temp moves by at most tau.
 */
static int topk_keep(const float *logits, int V, int K, double inv_temp, double tau,
                     unsigned char *keep) {
  if (K <= 0 || K >= V) { memset(keep, 1, (size_t)V); return 1; }
  memset(keep, 0, (size_t)V);
  double last = 0.0;
  for (int n = 0; n < K; ++n) {
    int best = -1;
    for (int j = 0; j < V; ++j)
      if (!keep[j] && (best < 0 || logits[j] > logits[best])) best = j;
    keep[best] = 1;
    last = (double)logits[best];
  }
  double next = -INFINITY;
  for (int j = 0; j < V; ++j)
    if (!keep[j] && (double)logits[j] > next) next = (double)logits[j];
  return (tau == 0.0) ? 1 : ((last - next) * inv_temp > 2.0 * tau);
}

/* ln sum_{j kept} exp(l_j * inv_temp) */
static double log_sum_exp(const float *logits, const unsigned char *keep, int V, double inv_temp) {
  double mx = -INFINITY;
  for (int j = 0; j < V; ++j) {
    if (!keep[j]) continue;
    double a = (double)logits[j] * inv_temp;
    if (a > mx) mx = a;
  }
  double s = 0.0;
  for (int j = 0; j < V; ++j)
    if (keep[j]) s += exp((double)logits[j] * inv_temp - mx);
  return mx + log(s);
}

/*
 * Draw from softmax(logits / temperature), restricted to the row's top_k logits when top_k > 0,
 * by Gumbel-max: argmax_j (l_j/T + G_j).  temperature == 0: plain argmax.  Ties go to the lowest
 * index.  *stable = 1 iff the winner (and the kept set) cannot change when every score moves by
 * at most tau.
 */
int orc_sample_softmax(const float *logits, int V, double temperature, int top_k, const orc_ctr *c,
                       double tau, int *stable) {
  unsigned char *keep = (unsigned char *)malloc((size_t)V);
  int set_ok = topk_keep(logits, V, temperature == 0.0 ? 0 : top_k,
                         temperature == 0.0 ? 1.0 : 1.0 / temperature, tau, keep);
  int best = 0;
  double sb = -INFINITY, s2 = -INFINITY;
  for (int j = 0; j < V; ++j) {
    if (!keep[j]) continue;
    double s;
    if (temperature == 0.0) {
      s = (double)logits[j];
    } else {
      double u = orc_uniform(c->seed, c->seq_id, c->iteration, c->row, c->purpose, (uint32_t)j);
      s = (double)logits[j] / temperature + gumbel(u);
    }
    if (s > sb) { s2 = sb; sb = s; best = j; }
    else if (s > s2) { s2 = s; }
  }
  free(keep);
  if (stable) *stable = (tau == 0.0) ? 1 : (set_ok && sb - s2 > 2.0 * tau);
  return best;
}

/*
 * Accept test of Algorithm 1 for one drafted token x:  r < min(1, p(x)/d(x)), written as
 * ln r + ln d(x) < ln p(x) with p, d the post-temperature (top-k filtered) softmax of the
 * verify / draft row; p(x) = 0 (x outside the target's top k) rejects.
 * Greedy: accept iff x is the argmax of the verify row (one-hot limit).
 */
int orc_accept(const float *p_logits, const float *d_logits, int V, int x, double temperature,
               int top_k, const orc_ctr *c, double tau, int *stable) {
  if (temperature == 0.0) {
    int st;
    int am = orc_sample_softmax(p_logits, V, 0.0, 0, c, tau, &st);
    if (stable) {
      if (am == x) *stable = st;
      else {
        /* rejected: stable iff x cannot overtake the maximum */
        *stable = (tau == 0.0) ? 1 : ((double)p_logits[am] - (double)p_logits[x] > 2.0 * tau);
      }
    }
    return am == x;
  }
  double it = 1.0 / temperature;
  unsigned char *kp = (unsigned char *)malloc((size_t)V), *kd = (unsigned char *)malloc((size_t)V);
  int set_ok = topk_keep(p_logits, V, top_k, it, tau, kp) & topk_keep(d_logits, V, top_k, it, tau, kd);
  int in_p = kp[x], in_d = kd[x];
  double lp = in_p ? (double)p_logits[x] * it - log_sum_exp(p_logits, kp, V, it) : -INFINITY;
  double ld = in_d ? (double)d_logits[x] * it - log_sum_exp(d_logits, kd, V, it) : -INFINITY;
  free(kp);
  free(kd);
  double r = orc_uniform(c->seed, c->seq_id, c->iteration, c->row, ORC_ACCEPT, 0);
  double lhs = log(r) + ld;
  if (stable) *stable = (tau == 0.0) ? 1 : (set_ok && (!in_p || fabs(lp - lhs) > 4.0 * tau));
  return lhs < lp;
}

/*
 * Draw from the normalised residual (p - d)_+ by Gumbel-max over ln max(0, p_j - d_j) + G_j
 * (the normaliser cancels in an argmax), p and d top-k filtered as above.  Greedy: argmax of the
 * verify row.  If the residual is empty (possible only through rounding), fall back to sampling
 * from p; *fallback = 1.
 * *stable: winner unchanged when ln p_j and ln d_j each move by at most tau (and the kept sets
 * cannot change).
 */
int orc_sample_residual(const float *p_logits, const float *d_logits, int V, double temperature,
                        int top_k, const orc_ctr *c, double tau, int *stable, int *fallback) {
  if (fallback) *fallback = 0;
  if (temperature == 0.0) return orc_sample_softmax(p_logits, V, 0.0, 0, c, tau, stable);
  double it = 1.0 / temperature;
  unsigned char *kp = (unsigned char *)malloc((size_t)V), *kd = (unsigned char *)malloc((size_t)V);
  int set_ok = topk_keep(p_logits, V, top_k, it, tau, kp) & topk_keep(d_logits, V, top_k, it, tau, kd);
  double zp = log_sum_exp(p_logits, kp, V, it), zd = log_sum_exp(d_logits, kd, V, it);
  int best = -1;
  double sb = -INFINITY;
  for (int j = 0; j < V; ++j) {
    double p = kp[j] ? exp((double)p_logits[j] * it - zp) : 0.0;
    double d = kd[j] ? exp((double)d_logits[j] * it - zd) : 0.0;
    double w = p - d;
    if (!(w > 0.0)) continue;
    double u = orc_uniform(c->seed, c->seq_id, c->iteration, c->row, c->purpose, (uint32_t)j);
    double s = log(w) + gumbel(u);
    if (s > sb) { sb = s; best = j; }
  }
  if (best < 0) {
    free(kp);
    free(kd);
    if (fallback) *fallback = 1;
    if (stable) *stable = 0;
    return orc_sample_softmax(p_logits, V, temperature, top_k, c, tau, NULL);
  }
  if (stable) {
    if (tau == 0.0) { *stable = 1; free(kp); free(kd); return best; }
    double up = exp(tau), dn = exp(-tau);
    double pb = kp[best] ? exp((double)p_logits[best] * it - zp) : 0.0;
    double db = kd[best] ? exp((double)d_logits[best] * it - zd) : 0.0;
    double wlo = pb * dn - db * up;
    int ok = set_ok && wlo > 0.0;
    double ub = orc_uniform(c->seed, c->seq_id, c->iteration, c->row, c->purpose, (uint32_t)best);
    double slo = ok ? log(wlo) + gumbel(ub) - tau : -INFINITY;
    for (int j = 0; ok && j < V; ++j) {
      if (j == best) continue;
      double p = kp[j] ? exp((double)p_logits[j] * it - zp) : 0.0;
      double d = kd[j] ? exp((double)d_logits[j] * it - zd) : 0.0;
      double whi = p * up - d * dn;
      if (!(whi > 0.0)) continue;
      double u = orc_uniform(c->seed, c->seq_id, c->iteration, c->row, c->purpose, (uint32_t)j);
      if (log(whi) + gumbel(u) + tau >= slo) ok = 0;
    }
    *stable = ok;
  }
  free(kp);
  free(kd);
  return best;
}

/* ------------------------------------------------------------------------------------------ */
/* model                                                                                       */
/* ------------------------------------------------------------------------------------------ */
static const void **dup_ptrs(const void *const *p, int n) {
  const void **q = (const void **)malloc(sizeof(void *) * (size_t)n);
  for (int i = 0; i < n; ++i) q[i] = p[i];
  return q;
}

/* The oracle borrows the weight buffers: the caller keeps them alive until orc_model_free. */
orc_model *orc_model_create(const orc_config *c, const orc_weights *w) {
  if (!c || !w || c->k < 0 || c->k > ORC_MAX_K || c->n_layers < 0 || (c->head_dim & 1)) return NULL;
  if (c->la_token >= c->vocab) return NULL;
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  m->c = *c;
  m->tok_emb = w->tok_emb; m->lm_head = w->lm_head;
  m->final_norm = w->final_norm; m->lookahead = w->lookahead;
  int L = c->n_layers;
  m->attn_norm = dup_ptrs(w->attn_norm, L); m->wq = dup_ptrs(w->wq, L);
  m->wk = dup_ptrs(w->wk, L); m->wv = dup_ptrs(w->wv, L); m->wo = dup_ptrs(w->wo, L);
  m->ffn_norm = dup_ptrs(w->ffn_norm, L); m->w_gate = dup_ptrs(w->w_gate, L);
  m->w_up = dup_ptrs(w->w_up, L); m->w_down = dup_ptrs(w->w_down, L);
  return m;
}

void orc_model_free(orc_model *m) {
  if (!m) return;
  free(m->attn_norm); free(m->wq); free(m->wk); free(m->wv); free(m->wo);
  free(m->ffn_norm); free(m->w_gate); free(m->w_up); free(m->w_down);
  free(m);
}

orc_seq *orc_seq_create(const orc_model *m, int max_len, uint32_t seq_id) {
  if (!m || max_len < 1) return NULL;
  orc_seq *s = (orc_seq *)calloc(1, sizeof(orc_seq));
  s->m = m; s->max_len = max_len; s->seq_id = seq_id;
  size_t hd = (size_t)m->c.n_heads * m->c.head_dim;
  size_t n = (size_t)m->c.n_layers * max_len * hd;
  s->kc = (double *)calloc(n ? n : 1, sizeof(double));
  s->vc = (double *)calloc(n ? n : 1, sizeof(double));
  size_t nl = (size_t)(1 + m->c.k) * m->c.vocab;
  s->draft_logits = (float *)calloc(nl, sizeof(float));
  s->verify_logits = (float *)calloc(nl, sizeof(float));
  return s;
}

void orc_seq_free(orc_seq *s) {
  if (!s) return;
  free(s->kc); free(s->vc); free(s->draft_logits); free(s->verify_logits); free(s);
}

/* y = x * rsqrt(mean(x^2) + eps) * g */
static void rmsnorm(const orc_model *m, const double *x, const void *g, double *y) {
  int d = m->c.d_model;
  double ss = 0.0;
  for (int i = 0; i < d; ++i) ss += x[i] * x[i];
  double inv = 1.0 / sqrt(ss / d + (double)m->c.rms_eps);
  for (int i = 0; i < d; ++i) {
    double v = x[i] * inv * load_elem(g, m->c.dtype, (size_t)i);
    y[i] = m->c.act_bf16 ? orc_bf16_round(v) : v;
  }
}

/* Y[r][n] = sum_k W[n][k] X[r][k];  W is [N][K] row-major in the model's storage type. */
static void matmul(const orc_model *m, const double *X, const void *W, int R, int K, int N,
                   double *Y) {
  int dtype = m->c.dtype;
  /* the rows side by side, Xt[k][r] = X[r][k]: the sums below then walk memory in order (same
   * products, same order of additions per output as with X itself) */
  double *Xt = (double *)malloc(sizeof(double) * (size_t)R * K);
  for (int r = 0; r < R; ++r)
    for (int k = 0; k < K; ++k) Xt[(size_t)k * R + r] = X[(size_t)r * K + k];
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    double acc[ORC_MAX_ROWS];
    for (int r = 0; r < R; ++r) acc[r] = 0.0;
    size_t base = (size_t)n * K;
    for (int k = 0; k < K; ++k) {
      double w = load_elem(W, dtype, base + k);
      const double *xk = Xt + (size_t)k * R;
      for (int r = 0; r < R; ++r) acc[r] += w * xk[r];
    }
    for (int r = 0; r < R; ++r) Y[(size_t)r * N + n] = acc[r];
  }
  free(Xt);
}

/* rotate interleaved pairs (2i, 2i+1) of every head by pos * base^(-2i/head_dim) */
static void rope(const orc_model *m, double *v, int pos) {
  int H = m->c.n_heads, hd = m->c.head_dim;
  for (int h = 0; h < H; ++h)
    for (int i = 0; i < hd / 2; ++i) {
      double theta = pow((double)m->c.rope_base, -2.0 * i / hd);
      double a = pos * theta, cs = cos(a), sn = sin(a);
      double *p = v + (size_t)h * hd + 2 * i;
      double x0 = p[0], x1 = p[1];
      p[0] = x0 * cs - x1 * sn;
      p[1] = x0 * sn + x1 * cs;
    }
}

static void round_vec(double *v, size_t n) {
  for (size_t i = 0; i < n; ++i) v[i] = orc_bf16_round(v[i]);
}

/*
 * One model call on R rows at consecutive positions pos0 .. pos0+R-1 of one sequence.
 * Row r is the token ids[r] (la[r] == 0) or look-ahead embedding number ids[r] (la[r] == 1,
 * ids[r] in 0..k-1).  K/V of the rows are written to the cache at their positions; row r
 * attends to cached positions 0 .. pos0+r (causal).  logits_out, if not NULL, receives
 * [R][vocab] fp32.  The cached length kv_len is NOT changed: the caller decides what to keep.
 */
int orc_forward(orc_seq *s, int R, const int32_t *ids, const int32_t *la, int pos0,
                float *logits_out) {
  const orc_model *m = s->m;
  const orc_config *c = &m->c;
  if (R < 1 || R > ORC_MAX_ROWS) return ORC_EINVAL;
  if (pos0 < 0 || pos0 + R > s->max_len) return ORC_ECAPACITY;
  int d = c->d_model, H = c->n_heads, hd = c->head_dim, F = c->d_ffn, V = c->vocab;
  int D = H * hd;
  for (int r = 0; r < R; ++r) {
    if (la[r]) { if (ids[r] < 0 || ids[r] >= c->k) return ORC_EINVAL; }
    else if (ids[r] < 0 || ids[r] >= V) return ORC_EINVAL;
  }
  size_t Rz = (size_t)R;
  double *h = (double *)malloc(sizeof(double) * Rz * d);
  double *xn = (double *)malloc(sizeof(double) * Rz * d);
  double *q = (double *)malloc(sizeof(double) * Rz * D);
  double *kk = (double *)malloc(sizeof(double) * Rz * D);
  double *vv = (double *)malloc(sizeof(double) * Rz * D);
  double *ao = (double *)malloc(sizeof(double) * Rz * D);
  double *t0 = (double *)malloc(sizeof(double) * Rz * d);
  double *g = (double *)malloc(sizeof(double) * Rz * F);
  double *u = (double *)malloc(sizeof(double) * Rz * F);
  double *sc_all = (double *)malloc(sizeof(double) * Rz * H * (size_t)(pos0 + R)); /* scores of each (row, head) */

  /* row assembly: token embedding or look-ahead embedding (Section 2.2.1) */
  for (int r = 0; r < R; ++r) {
    const void *src = la[r] ? m->lookahead : m->tok_emb;
    for (int i = 0; i < d; ++i) h[(size_t)r * d + i] = load_elem(src, c->dtype, (size_t)ids[r] * d + i);
  }

  for (int l = 0; l < c->n_layers; ++l) {
    for (int r = 0; r < R; ++r) rmsnorm(m, h + (size_t)r * d, m->attn_norm[l], xn + (size_t)r * d);
    matmul(m, xn, m->wq[l], R, d, D, q);
    matmul(m, xn, m->wk[l], R, d, D, kk);
    matmul(m, xn, m->wv[l], R, d, D, vv);
    for (int r = 0; r < R; ++r) {
      rope(m, q + (size_t)r * D, pos0 + r);
      rope(m, kk + (size_t)r * D, pos0 + r);
    }
    if (c->dtype == ORC_BF16) { round_vec(kk, Rz * D); round_vec(vv, Rz * D); } /* cache storage format */
    if (c->act_bf16) round_vec(q, Rz * D);
    double *kc = s->kc + (size_t)l * s->max_len * D, *vc = s->vc + (size_t)l * s->max_len * D;
    for (int r = 0; r < R; ++r) {
      memcpy(kc + (size_t)(pos0 + r) * D, kk + (size_t)r * D, sizeof(double) * D);
      memcpy(vc + (size_t)(pos0 + r) * D, vv + (size_t)r * D, sizeof(double) * D);
    }
    double scale = 1.0 / sqrt((double)hd);
    /* heads are independent: the threads share them out (as they share the output features of a
     * matrix product); every (row, head) runs the same operations in the same order on any thread */
#pragma omp parallel for schedule(static) collapse(2)
    for (int r = 0; r < R; ++r) {
      for (int hh = 0; hh < H; ++hh) {
        int nk = pos0 + r + 1; /* keys at positions 0 .. pos0+r */
        double *sc = sc_all + ((size_t)r * H + hh) * (size_t)(pos0 + R);
        const double *qv = q + (size_t)r * D + (size_t)hh * hd;
        double mx = -INFINITY;
        for (int j = 0; j < nk; ++j) {
          const double *kv = kc + (size_t)j * D + (size_t)hh * hd;
          double dot = 0.0;
          for (int i = 0; i < hd; ++i) dot += qv[i] * kv[i];
          sc[j] = dot * scale;
          if (sc[j] > mx) mx = sc[j];
        }
        double den = 0.0;
        for (int j = 0; j < nk; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
        double *o = ao + (size_t)r * D + (size_t)hh * hd;
        for (int i = 0; i < hd; ++i) o[i] = 0.0;
        for (int j = 0; j < nk; ++j) {
          const double *vj = vc + (size_t)j * D + (size_t)hh * hd;
          double pj = sc[j] / den;
          for (int i = 0; i < hd; ++i) o[i] += pj * vj[i];
        }
      }
    }
    if (c->act_bf16) round_vec(ao, Rz * D);
    matmul(m, ao, m->wo[l], R, D, d, t0);
    for (size_t i = 0; i < Rz * d; ++i) h[i] += t0[i];

    for (int r = 0; r < R; ++r) rmsnorm(m, h + (size_t)r * d, m->ffn_norm[l], xn + (size_t)r * d);
    matmul(m, xn, m->w_gate[l], R, d, F, g);
    matmul(m, xn, m->w_up[l], R, d, F, u);
    for (size_t i = 0; i < Rz * F; ++i) {
      double a = g[i] / (1.0 + exp(-g[i])) * u[i]; /* SwiGLU: silu(gate) * up */
      g[i] = c->act_bf16 ? orc_bf16_round(a) : a;
    }
    matmul(m, g, m->w_down[l], R, F, d, t0);
    for (size_t i = 0; i < Rz * d; ++i) h[i] += t0[i];
  }

  if (logits_out) {
    double *lg = (double *)malloc(sizeof(double) * Rz * V);
    for (int r = 0; r < R; ++r) rmsnorm(m, h + (size_t)r * d, m->final_norm, xn + (size_t)r * d);
    matmul(m, xn, m->lm_head, R, d, V, lg);
    for (size_t i = 0; i < Rz * V; ++i) logits_out[i] = (float)lg[i];
    free(lg);
  }
  free(h); free(xn); free(q); free(kk); free(vv); free(ao); free(t0); free(g); free(u); free(sc_all);
  return ORC_OK;
}

/* ------------------------------------------------------------------------------------------ */
/* PaSS loop (Algorithm 1)                                                                     */
/* ------------------------------------------------------------------------------------------ */

/* Optional observer of long prompt passes (tests print a progress line from it): called after
 * every chunk of rows with (rows done, rows in all).  No part of the computation. */
static void (*g_progress)(int, int) = NULL;
void orc_set_progress(void (*cb)(int, int)) { g_progress = cb; }

/* Cache K/V of prompt[0..n-2]; prompt[n-1] becomes the pending token.  The rows go through the
 * model 32 at a time (rows are independent of what shares their call: pinned bit for bit). */
int orc_prefill(orc_seq *s, const int32_t *prompt, int n) {
  if (!s || !prompt || n < 1) return ORC_EINVAL;
  if (n - 1 + 1 + s->m->c.k > s->max_len) return ORC_ECAPACITY;
  int32_t la[ORC_MAX_ROWS] = {0};
  int done = 0;
  while (done < n - 1) {
    int R = n - 1 - done;
    if (R > 32) R = 32;
    int rc = orc_forward(s, R, prompt + done, la, done, NULL);
    if (rc) return rc;
    done += R;
    if (g_progress) g_progress(done, n - 1);
  }
  s->kv_len = n - 1;
  s->pending = prompt[n - 1];
  s->state = 1;
  s->iteration = 0;
  s->n_generated = 0;
  return ORC_OK;
}

/*
 * Drafting phase: one call on (pending, [LA]_1 .. [LA]_k) at positions kv_len .. kv_len+k.
 * Row 0 gives x_{n+1} (an ordinary sample, not part of the draft); row t gives draft t.
 * Afterwards kv_len += 1 (only the real token's K/V are kept) and pending = x_{n+1}.
 */
int orc_draft(orc_seq *s, const orc_sampling *sp, double tau, int32_t *out_first,
              int32_t *out_drafts) {
  if (!s || !sp || sp->top_k < 0 || sp->temperature < 0) return ORC_EINVAL;
  if (s->state != 1) return ORC_ESTATE;
  const orc_config *c = &s->m->c;
  int k = c->k, V = c->vocab;
  if (s->kv_len + 1 + k > s->max_len) return ORC_ECAPACITY;
  int32_t ids[ORC_MAX_K + 1], la[ORC_MAX_K + 1];
  ids[0] = s->pending; la[0] = 0;
  for (int t = 1; t <= k; ++t) {
    if (c->la_token >= 0) { ids[t] = c->la_token; la[t] = 0; }
    else { ids[t] = t - 1; la[t] = 1; }
  }
  int rc = orc_forward(s, 1 + k, ids, la, s->kv_len, s->draft_logits);
  if (rc) return rc;
  for (int t = 0; t <= k; ++t) {
    orc_ctr ctr = {sp->seed, s->seq_id, s->iteration, (uint32_t)t, ORC_DRAFT};
    int tok = orc_sample_softmax(s->draft_logits + (size_t)t * V, V, sp->temperature, sp->top_k, &ctr,
                                 tau, &s->draft_stable[t]);
    if (t == 0) s->first = tok; else s->drafts[t - 1] = tok;
  }
  s->kv_len += 1;
  s->pending = s->first;
  s->n_generated += 1;
  s->state = 2;
  if (out_first) *out_first = s->first;
  if (out_drafts) for (int t = 0; t < k; ++t) out_drafts[t] = s->drafts[t];
  return ORC_OK;
}

/*
 * Validation phase: one call on (x_{n+1}, drafts) at positions kv_len .. kv_len+k.  Verify row
 * t-1 is the target distribution for draft t.  Accept drafts in order until the first reject;
 * a reject is replaced by a residual sample; if all k are accepted an extra token is sampled
 * from the last row.  out_tokens receives the a accepted drafts followed by that final token.
 * Afterwards kv_len += 1 + a and pending = the final token.
 */
int orc_verify(orc_seq *s, const orc_sampling *sp, double tau, int32_t *out_n_accepted,
               int32_t *out_tokens) {
  if (!s || !sp || sp->top_k < 0 || sp->temperature < 0) return ORC_EINVAL;
  if (s->state != 2) return ORC_ESTATE;
  const orc_config *c = &s->m->c;
  int k = c->k, V = c->vocab;
  if (s->kv_len + 1 + k > s->max_len) return ORC_ECAPACITY;
  int32_t ids[ORC_MAX_K + 1], la[ORC_MAX_K + 1];
  ids[0] = s->first; la[0] = 0;
  for (int t = 1; t <= k; ++t) { ids[t] = s->drafts[t - 1]; la[t] = 0; }
  int rc = orc_forward(s, 1 + k, ids, la, s->kv_len, s->verify_logits);
  if (rc) return rc;
  int a = 0, y = -1;
  for (int t = 0; t <= k; ++t) s->accept_stable[t] = 1;
  for (int t = 1; t <= k; ++t) {
    const float *p = s->verify_logits + (size_t)(t - 1) * V;
    const float *dl = s->draft_logits + (size_t)t * V;
    orc_ctr ctr = {sp->seed, s->seq_id, s->iteration, (uint32_t)t, ORC_ACCEPT};
    if (orc_accept(p, dl, V, s->drafts[t - 1], sp->temperature, sp->top_k, &ctr, tau,
                   &s->accept_stable[t])) {
      if (out_tokens) out_tokens[a] = s->drafts[t - 1];
      a += 1;
    } else {
      int fb = 0;
      ctr.purpose = ORC_RESIDUAL;
      y = orc_sample_residual(p, dl, V, sp->temperature, sp->top_k, &ctr, tau, &s->final_stable, &fb);
      s->fallback_count += fb;
      break;
    }
  }
  if (a == k) {
    orc_ctr ctr = {sp->seed, s->seq_id, s->iteration, (uint32_t)(k + 1), ORC_BONUS};
    y = orc_sample_softmax(s->verify_logits + (size_t)k * V, V, sp->temperature, sp->top_k, &ctr, tau,
                           &s->final_stable);
  }
  if (out_tokens) out_tokens[a] = y;
  if (out_n_accepted) *out_n_accepted = a;
  s->kv_len += 1 + a;
  s->pending = y;
  s->n_generated += 1 + a;
  s->iteration += 1;
  s->state = 1;
  return ORC_OK;
}

/*
 * Algorithm 1's while loop: iterate draft + verify until at least max_new tokens exist, return
 * the first max_new.  per_iter_accepted / per_iter_stable (may be NULL, capacity max_iters)
 * record the accepted count and whether every decision of the iteration was stable under tau.
 */
int orc_generate(orc_seq *s, int max_new, const orc_sampling *sp, double tau, int32_t *out_tokens,
                 int32_t *per_iter_accepted, int32_t *per_iter_stable, int max_iters,
                 int32_t *out_iters) {
  if (!s || max_new < 0) return ORC_EINVAL;
  int k = s->m->c.k, n = 0, it = 0;
  int32_t buf[ORC_MAX_K + 2];
  while (n < max_new) {
    int32_t first, a;
    int rc = orc_draft(s, sp, tau, &first, NULL);
    if (rc) return rc;
    rc = orc_verify(s, sp, tau, &a, buf + 1);
    if (rc) return rc;
    buf[0] = first;
    int got = a + 2; /* x_{n+1}, a accepted drafts, final token: between 2 and k+2 */
    for (int i = 0; i < got && n < max_new; ++i) out_tokens[n++] = buf[i];
    if (it < max_iters) {
      if (per_iter_accepted) per_iter_accepted[it] = a;
      if (per_iter_stable) {
        int st = s->final_stable;
        for (int t = 0; t <= k; ++t) st &= s->draft_stable[t];
        for (int t = 1; t <= a + 1 && t <= k; ++t) st &= s->accept_stable[t];
        per_iter_stable[it] = st;
      }
    }
    it += 1;
  }
  if (out_iters) *out_iters = it;
  return ORC_OK;
}

/*
 * Plain auto-regressive decoding with the KV cache (the paper's first baseline): one token per
 * single-row call.  Token number i (0-based) uses the counters PaSS with k = 0 would use:
 * even i -> (DRAFT, row 0, iteration i/2), odd i -> (BONUS, row 1, iteration i/2).
 */
int orc_generate_ar(orc_seq *s, int max_new, const orc_sampling *sp, int32_t *out_tokens) {
  if (!s || !sp || max_new < 0) return ORC_EINVAL;
  if (s->state != 1) return ORC_ESTATE;
  int V = s->m->c.vocab;
  float *lg = (float *)malloc(sizeof(float) * (size_t)V);
  int32_t la = 0;
  for (int i = 0; i < max_new; ++i) {
    int32_t id = s->pending;
    int rc = orc_forward(s, 1, &id, &la, s->kv_len, lg);
    if (rc) { free(lg); return rc; }
    orc_ctr ctr = {sp->seed, s->seq_id, (uint32_t)(i / 2), (uint32_t)(i & 1),
                   (i & 1) ? ORC_BONUS : ORC_DRAFT};
    int tok = orc_sample_softmax(lg, V, sp->temperature, sp->top_k, &ctr, 0.0, NULL);
    s->kv_len += 1;
    s->pending = tok;
    out_tokens[i] = tok;
  }
  free(lg);
  return ORC_OK;
}

/*
 * One iteration of Algorithm 2 (appendix: speculative sampling with an auto-regressive target and an
 * auto-regressive drafting model; the paper writes q for the target and p for the drafter there).
 * `target` and `drafter` hold the same tokens (same length, same pending token x_n); L is the
 * target model's k.
 *   for t = 1..L: one single-row call of the drafter on the last token of (x_1..x_n, d_1..d_{t-1});
 *                 draft d_t is sampled from its distribution (random stream: draft row t of the
 *                 target sequence's iteration);
 *   one call of the target on the rows (x_n, d_1..d_L): row t-1 is the target distribution for d_t;
 *   accept d_t iff r < min(1, target_t(d_t) / drafter_t(d_t)) in order; the first reject is replaced
 *   by a sample from the normalised (target_t - drafter_t)_+; if all L are accepted one more token is
 *   sampled from the last row.
 * That second half is Algorithm 1's validation phase on a draft that came from elsewhere, and it is
 * run by the same function (orc_verify), with x_n in the place of x_{n+1}.  An iteration adds
 * a + 1 tokens (1 .. L+1).  Afterwards both sequences again hold the same tokens: the drafter keeps
 * the cache rows of x_n, d_1..d_a (when all L were accepted the row of d_L does not exist yet: one
 * more single-row call makes it) and takes over the target's pending token.
 * out_tokens: the a accepted drafts followed by the final token.  drafter_logits (may be NULL)
 * receives the L rows of drafter logits, [L][vocab].
 */
int orc_sps_iteration(orc_seq *target, orc_seq *drafter, const orc_sampling *sp, double tau,
                      int32_t *out_n_accepted, int32_t *out_tokens, float *drafter_logits) {
  if (!target || !drafter || !sp || sp->top_k < 0 || sp->temperature < 0) return ORC_EINVAL;
  if (target->state != 1 || drafter->state != 1) return ORC_ESTATE;
  const int L = target->m->c.k, V = target->m->c.vocab;
  if (drafter->m->c.vocab != V) return ORC_EINVAL;
  if (drafter->kv_len != target->kv_len || drafter->pending != target->pending) return ORC_ESTATE;
  if (target->kv_len + 1 + L > target->max_len || drafter->kv_len + 1 + L > drafter->max_len) return ORC_ECAPACITY;
  const int n0 = drafter->kv_len;
  int32_t la = 0;
  /* drafting: L sequential single-row calls */
  for (int t = 1; t <= L; ++t) {
    int32_t id = drafter->pending;
    float *row = target->draft_logits + (size_t)t * V; /* the slot orc_verify reads draft row t from */
    int rc = orc_forward(drafter, 1, &id, &la, drafter->kv_len, row);
    if (rc) return rc;
    orc_ctr ctr = {sp->seed, target->seq_id, target->iteration, (uint32_t)t, ORC_DRAFT};
    int tok = orc_sample_softmax(row, V, sp->temperature, sp->top_k, &ctr, tau, &target->draft_stable[t]);
    target->drafts[t - 1] = tok;
    drafter->kv_len += 1;
    drafter->pending = tok;
    if (drafter_logits) memcpy(drafter_logits + (size_t)(t - 1) * V, row, sizeof(float) * (size_t)V);
  }
  target->draft_stable[0] = 1;
  /* validation: the target's one call on (x_n, drafts) and the accept / reject chain */
  target->first = target->pending;
  target->state = 2;
  int32_t a = 0;
  int32_t toks[ORC_MAX_K + 1];
  int rc = orc_verify(target, sp, tau, &a, toks);
  if (rc) return rc;
  /* the drafter follows: rows of rejected drafts are dropped, a missing row is made */
  if (a == L) {
    int32_t id = drafter->pending; /* d_L (x_n itself when L = 0) */
    rc = orc_forward(drafter, 1, &id, &la, drafter->kv_len, NULL);
    if (rc) return rc;
  }
  drafter->kv_len = n0 + 1 + a;
  drafter->pending = target->pending;
  drafter->iteration += 1;
  if (out_n_accepted) *out_n_accepted = a;
  if (out_tokens) for (int t = 0; t <= a; ++t) out_tokens[t] = toks[t];
  return ORC_OK;
}

/* Algorithm 2's while loop: iterate until at least max_new tokens exist, return the first max_new. */
int orc_generate_sps(orc_seq *target, orc_seq *drafter, int max_new, const orc_sampling *sp, double tau,
                     int32_t *out_tokens, int32_t *per_iter_accepted, int32_t *per_iter_stable, int max_iters,
                     int32_t *out_iters) {
  if (!target || !drafter || max_new < 0) return ORC_EINVAL;
  int L = target->m->c.k, n = 0, it = 0;
  int32_t buf[ORC_MAX_K + 1];
  while (n < max_new) {
    int32_t a;
    int rc = orc_sps_iteration(target, drafter, sp, tau, &a, buf, NULL);
    if (rc) return rc;
    for (int i = 0; i <= a && n < max_new; ++i) out_tokens[n++] = buf[i];
    if (it < max_iters) {
      if (per_iter_accepted) per_iter_accepted[it] = a;
      if (per_iter_stable) {
        int st = target->final_stable;
        for (int t = 1; t <= L; ++t) st &= target->draft_stable[t];
        for (int t = 1; t <= a + 1 && t <= L; ++t) st &= target->accept_stable[t];
        per_iter_stable[it] = st;
      }
    }
    it += 1;
  }
  if (out_iters) *out_iters = it;
  return ORC_OK;
}

/* accessors for the ctypes wrapper */
int orc_seq_kv_len(const orc_seq *s) { return s->kv_len; }
int orc_seq_pending(const orc_seq *s) { return s->pending; }
int64_t orc_seq_n_generated(const orc_seq *s) { return s->n_generated; }
int orc_seq_fallbacks(const orc_seq *s) { return s->fallback_count; }
const float *orc_seq_logits(const orc_seq *s, int which) { return which ? s->verify_logits : s->draft_logits; }
void orc_seq_decision_flags(const orc_seq *s, int32_t *draft_stable, int32_t *accept_stable,
                            int32_t *final_stable) {
  for (int t = 0; t <= s->m->c.k; ++t) { draft_stable[t] = s->draft_stable[t]; accept_stable[t] = s->accept_stable[t]; }
  *final_stable = s->final_stable;
}
/* K (which = 0) or V (which = 1) of one cached position of one layer, [n_heads*head_dim] */
void orc_seq_read_kv(const orc_seq *s, int which, int layer, int pos, double *out) {
  size_t D = (size_t)s->m->c.n_heads * s->m->c.head_dim;
  const double *src = (which ? s->vc : s->kc) + ((size_t)layer * s->max_len + pos) * D;
  memcpy(out, src, sizeof(double) * D);
}
/* overwrite the pending token and state: lets a test put a sequence in a chosen situation */
void orc_seq_set_pending(orc_seq *s, int32_t tok) { s->pending = tok; }

/* Start `dst` from the state `src` is in between iterations: cached K/V, length, pending token,
 * iteration and token counters (not the sequence id).  Both must belong to models of the same
 * layer shapes and weights (they may differ in the number of look-ahead embeddings, which the
 * prompt pass never touches): a sweep over the number of look-ahead rows prefills once. */
int orc_seq_copy_state(orc_seq *dst, const orc_seq *src) {
  if (!dst || !src || src->state != 1) return ORC_EINVAL;
  const orc_config *a = &dst->m->c, *b = &src->m->c;
  if (a->n_layers != b->n_layers || a->n_heads != b->n_heads || a->head_dim != b->head_dim ||
      a->d_model != b->d_model || a->dtype != b->dtype)
    return ORC_EINVAL;
  if (src->kv_len + 1 + a->k > dst->max_len) return ORC_ECAPACITY;
  size_t D = (size_t)a->n_heads * a->head_dim;
  for (int l = 0; l < a->n_layers; ++l) {
    memcpy(dst->kc + (size_t)l * dst->max_len * D, src->kc + (size_t)l * src->max_len * D, sizeof(double) * D * src->kv_len);
    memcpy(dst->vc + (size_t)l * dst->max_len * D, src->vc + (size_t)l * src->max_len * D, sizeof(double) * D * src->kv_len);
  }
  dst->kv_len = src->kv_len;
  dst->pending = src->pending;
  dst->state = 1;
  dst->iteration = src->iteration;
  dst->n_generated = src->n_generated;
  return ORC_OK;
}
/* overwrite the stored draft (tokens and logits) before a verify call: the verify half is then
 * the speculative-sampling rule of Algorithm 2 with an arbitrary draft distribution */
void orc_seq_set_draft(orc_seq *s, const int32_t *drafts, const float *draft_logits) {
  int k = s->m->c.k, V = s->m->c.vocab;
  for (int t = 0; t < k; ++t) s->drafts[t] = drafts[t];
  if (draft_logits) memcpy(s->draft_logits, draft_logits, sizeof(float) * (size_t)(1 + k) * V);
}
