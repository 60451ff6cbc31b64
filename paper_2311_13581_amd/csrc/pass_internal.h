// Internal declarations shared by the HIP translation units of libpass_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pass.h"

namespace pass {

enum StepMode { MODE_PREFILL = 0, MODE_DRAFT = 1, MODE_VERIFY = 2 };
enum Purpose { PURPOSE_DRAFT = 0, PURPOSE_ACCEPT = 1, PURPOSE_RESIDUAL = 2, PURPOSE_BONUS = 3 };

constexpr int kMaxK = PASS_MAX_K;
constexpr int kMaxRows = PASS_MAX_ROWS;
constexpr int kAttnRowsPerGroup = 8;  // queries one attention workgroup carries in registers
constexpr int kMaxSplits = 32;
constexpr int kPrefillRows = 2048;  // most prompt rows the tiled prompt pass takes through the weights at once
constexpr int kAttnResident = 768;  // matrix-core attention workgroups resident on the chip (256 CUs x 3)

// How the matrix-core attention kernel cuts a row group's keys into splits: a function of the
// sequence's own key count and of the model (number of heads) only, so that a sequence's
// arithmetic cannot depend on what else is batched.  A split is 128 keys (one step of a
// 4-wavefront workgroup) until splits x heads no longer fit the chip at once: then the steps per
// split grow, because a second round of workgroups costs more than a second step inside one.
__host__ __device__ inline void split_plan_mfma(int n_keys, int n_heads, int &n_splits, int &chunk) {
  const int steps = (n_keys + 127) / 128;
  int per = (steps + kMaxSplits - 1) / kMaxSplits;  // steps per split
  while (((steps + per - 1) / per) * n_heads > kAttnResident && per < steps) ++per;
  chunk = per * 128;
  n_splits = (n_keys + chunk - 1) / chunk;
}
// The plan is not monotone in the key count: when the steps per split grow, the split count drops
// (32 heads: 3072 keys give 24 splits, 3073 give 13).  A launch that serves row groups of several
// lengths, or whose host only knows an upper bound of the lengths, therefore sizes its grid for the
// largest split count any length up to that bound can have; surplus workgroups exit at once.
inline int max_splits_mfma(int max_keys, int n_heads) {
  int best = 1;
  for (int steps = 1; (steps - 1) * 128 < max_keys; ++steps) {  // within one step count the last key count has most splits
    int n_splits, chunk;
    split_plan_mfma(steps * 128 < max_keys ? steps * 128 : max_keys, n_heads, n_splits, chunk);
    if (n_splits > best) best = n_splits;
  }
  return best;
}

// bfloat16 storage type: raw bits, converted with shifts (round-to-nearest-even on store)
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round to nearest even; gfx950 has the conversion in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// two values into one register: `lo` in bits 0..15, `hi` in bits 16..31
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
// (hi, lo) split of two values, x = hi + lo with both halves bf16: the hi pair or the lo pair
__device__ __forceinline__ uint32_t split2_bf16(float a, float b, bool take_hi) {
  uint32_t ph = pack2_bf16(a, b);
  uint32_t pl = pack2_bf16(a - __uint_as_float(ph << 16), b - __uint_as_float(ph & 0xffff0000u));
  return take_hi ? ph : pl;
}
__device__ __forceinline__ float load_f(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f(const bf16_t *p, size_t i) { return bf16_to_f32(p[i].bits); }
__device__ __forceinline__ void store_f(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_f(bf16_t *p, size_t i, float v) { p[i].bits = f32_to_bf16(v); }

// Everything a kernel needs to find its way around the arena.  Passed by value.
struct Params {
  // shape
  int L, d, H, hd, D, F, V, k;
  int k_act;     // look-ahead rows per call right now (0 .. k; buffers keep their stride 1 + k)
  int la_token;  // < 0: drafting rows are the look-ahead embeddings; >= 0: this token's embedding, k_act times
  int max_slots, max_seq_len, page_size, page_shift, n_pages, pages_per_seq;
  int gen_cap;
  int v_transposed;  // V pages hold [head][dim][page_size] (matrix-core attention) instead of [head][page_size][dim]
  float eps, rope_base;
  // per-slot state (device), indexed by slot
  int32_t *kv_len, *pending, *first, *drafts /*[slot][kMaxK]*/, *n_gen, *n_acc, *frozen, *gen_limit;
  uint32_t *iter, *seq_id;
  int32_t *last_out;  // [slot][kMaxK+1]: accepted drafts then the final token of the last verify
  int32_t *gen;       // [slot][gen_cap]: every generated token since the prefill
  float *logz_d, *logz_p;  // [slot][kMaxK+1]: ln sum exp(logit/T) of each draft / verify row
  int32_t *argmax_p;       // [slot][kMaxK+1]
  uint32_t *flt_key_d, *flt_key_p;  // [slot][kMaxK+1]: top-k filter of each draft / verify row (threshold key,
  int32_t *flt_tie_d, *flt_tie_p;   //   highest index kept among the logits equal to the threshold)
  int32_t *fallbacks;      // [1]: residual numerically empty after a reject
  int32_t *block_table;    // [slot][pages_per_seq]
  float *draft_logits, *verify_logits;  // [slot][1+k][V]
  // per-step tables (device)
  int32_t *step_slots;   // [B]
  int32_t *prefill_ids;  // [R]
  int32_t *row_pos, *row_slot, *row_out;  // [M]
  float *rope_cos, *rope_sin;             // [M][hd/2]
  double *rope_theta;                     // [hd/2] base^(-2i/hd), filled at create
  // workspaces
  float *h;        // [M][d]   residual stream
  float *xn;       // [M][d]
  float *qkv;      // [M][3D]  q | k | v
  float *attn;     // [M][D]
  float *gu;       // [M][2F]  gate | up
  float *act;      // [M][F]
  // matrix-core path: activations as (hi, lo) bf16 pairs, x = hi + lo, laid out
  // [group of 8 rows][16 pseudo-rows: hi of rows 0..7, lo of rows 0..7][K]
  uint16_t *attn_x;  // K = D  attention output
  uint16_t *act_x;   // K = F  silu(gate) * up
  uint16_t *xg;      // K = d  h * gain of the next norm
  float *ssq;           // [d/16][kMaxRows] per-strip partial sums of h^2
  float *part_acc, *part_m, *part_l;  // attention partials [M][H][S][hd], [M][H][S]
  float *lse;  // [M][H], or null: where the attention combine also leaves ln sum exp of the row's scaled scores (training)
  // K/V pools: [layer][page][head][page_size][hd] in the model's storage type
  void *k_pool, *v_pool;
};

__device__ __forceinline__ size_t kv_offset(const Params &p, int layer, int slot, int pos, int head) {
  int page = p.block_table[(size_t)slot * p.pages_per_seq + (pos >> p.page_shift)];
  int off = pos & (p.page_size - 1);
  return ((((size_t)layer * p.n_pages + page) * p.H + head) * p.page_size + off) * (size_t)p.hd;
}

// A slot whose rows would lie beyond max_seq_len is dead for this call: pass_generate keeps a slot
// that has reached its token target stepping with the batch (its state is frozen, its outputs are
// dropped), and such a slot may sit within k positions of its capacity.  Its rows take part in the
// matrix products (rows are independent) but write no K/V, read no cache (their attention output is
// zero) and so never index the block table past the slot's own entries.  The host never lets a
// live slot get there (PASS_ECAPACITY first).
__device__ __forceinline__ bool row_is_dead(const Params &p, int mode, int slot, int R) {
  return mode != MODE_PREFILL && p.kv_len[slot] + R > p.max_seq_len;
}
// token ids read back from device state index the embedding table: keep them inside it whatever a
// dead row's sampler produced
__device__ __forceinline__ int clamp_token(const Params &p, int t) { return t < 0 ? 0 : (t >= p.V ? p.V - 1 : t); }

struct SampleArgs {
  float temperature;
  uint32_t seed_lo, seed_hi;
  int commit;  // 0: compute but leave the sequence state untouched (timing replays)
  int top_k;   // 0: no filter; K: sample from the K largest logits of a row only
  // Two-model speculative sampling (Algorithm 2 of the appendix) reuses the drafting epilogue:
  int row_base;    // added to the row number in the random streams: the drafting model's t-th single-row call draws
                   //   with the stream of draft row t
  int stats_only;  // 1: rows 1.. hold logits drafted elsewhere: only their filter and ln-sum-exp are computed,
                   //   no token is drawn and no state changes (row 0 is skipped)
};

// ---- launchers (each checks nothing but launches; shapes are validated by the caller) ----
// generic path (any storage type, fp32 activations)
void launch_assemble(const Params &p, int dtype, const void *tok_emb, const void *lookahead, int mode, int B,
                     int R, hipStream_t s);
void launch_rmsnorm(const Params &p, int dtype, const float *x, const void *gain, float *out, int M, hipStream_t s);
void launch_gemm_generic(int dtype, const float *X, const void *W, float *out, int M, int N, int K, int ldc,
                         const int32_t *rowmap, int accumulate, hipStream_t s);
void launch_rope_kv(const Params &p, int dtype, int layer, int M, hipStream_t s);
void launch_silu_mul(const Params &p, int M, hipStream_t s);
// attention (both paths).  out_split: 0 = fp32 into p.attn, 1 = (hi, lo) bf16 pairs into p.attn_x
void launch_attention(const Params &p, int dtype, int layer, int B, int R, int n_splits, int out_split,
                      hipStream_t s);
// sampling epilogues (both paths)
void launch_draft_epilogue(const Params &p, const SampleArgs &a, int B, int R, hipStream_t s);
void launch_verify_epilogue(const Params &p, const SampleArgs &a, int B, int R, hipStream_t s);
void launch_poke(int32_t *const *ptrs, const int32_t *vals, int n, hipStream_t s);
void launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t s);
void launch_plain_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t s);
void launch_rng_uniforms(float *out, uint32_t j0, int n, uint64_t seed, uint32_t seq_id, uint32_t iteration,
                         uint32_t row, uint32_t purpose, hipStream_t s);

// matrix-core path (bf16, 16x32 weight tiles)
void launch_pack_tiles(const uint16_t *src, uint16_t *dst, int N, int K, int strip_off, int strip_stride,
                       hipStream_t s);
void launch_assemble_mfma(const Params &p, const void *tok_emb, const void *lookahead, const void *gain0, int mode,
                          int B, int R, hipStream_t s);
// Launch shapes of the decode-sized matrix-core GEMMs, per context.  kind: 0 QKV, 1 Wo, 2 gate/up,
// 3 LM head, 4 down.  The "tune.gemm_cfg" option writes it (see pass_set_option in pass_api.hip).
struct GemmTuning {
  int waves[5], unroll[5];          // calls of up to 8 rows: wavefronts per workgroup (0 = by strip count), k-tiles per trip
  int big_waves[5], big_blocks[5];  // calls with more than 8 rows: wavefronts and output blocks per workgroup
  int split_ks;                     // K slices of the split residual GEMMs (0 = never split)
  GemmTuning();
  int set(int kind, int w, int u);            // wavefronts 4/8/16, k-tiles per trip 1/2/4; -1 = rejected
  int set_big(int kind, int w, int blocks);   // wavefronts 4/8/16, blocks 0..4
  int set_split(int ks);                      // 0..8
};
void launch_gemm_qkv(const Params &p, const GemmTuning &tn, const void *W, int layer, int M, hipStream_t s);
void launch_gemm_resid(const Params &p, const GemmTuning &tn, const void *W, const uint16_t *X, int K,
                       const void *gain_next, int M, hipStream_t s);
void launch_gemm_gateup(const Params &p, const GemmTuning &tn, const void *W, int M, hipStream_t s);
// (hi, lo) activation buffers of the matrix-core path, K features per row, tiled like the MFMA B
// operand: [m / 8][K / 32][64 lanes][8 features]; lane = (k / 8 % 4) * 16 + m % 8 for the hi half,
// 8 lanes further for the lo half.  Element index of the hi half of feature k of row m:
__device__ __forceinline__ size_t xs_index(int m, int K, int k) {
  return ((((size_t)(m >> 3) * (K >> 5) + (k >> 5)) * 64 + ((k >> 3) & 3) * 16 + (m & 7)) << 3) + (k & 7);
}
constexpr int kXsLoOffset = 64;  // elements from a hi half to its lo half
// (hi, lo) of four consecutive features k .. k+3 of row m: x = hi + lo up to 2^-17 relative
__device__ __forceinline__ void store_split4(uint16_t *xs, int m, int K, int k, const float (&v)[4]) {
  uint2 ph, pl;
  ph.x = pack2_bf16(v[0], v[1]);
  ph.y = pack2_bf16(v[2], v[3]);
  pl.x = pack2_bf16(v[0] - __uint_as_float(ph.x << 16), v[1] - __uint_as_float(ph.x & 0xffff0000u));
  pl.y = pack2_bf16(v[2] - __uint_as_float(ph.y << 16), v[3] - __uint_as_float(ph.y & 0xffff0000u));
  uint16_t *hp = xs + xs_index(m, K, k);
  *(uint2 *)hp = ph;
  *(uint2 *)(hp + kXsLoOffset) = pl;
}

// Tiled prompt pass (bf16 models on the matrix-core path with transposed V pages): up to `rows`
// prompt rows per pass over the weights.  The kernels take a Params copy whose h, xg, ssq,
// rope_cos, rope_sin, attn_x and act_x point at buffers of that many rows; the rest is here.
struct PrefillWs {
  int rows;       // capacity in rows (multiple of 128); also the row stride of the partial sums of h^2
  int np;         // partial sums of h^2 per row of this pass: one per resid_strips strips of 16 features
  int resid_strips;  // strips per wavefront of the residual projections in this pass (prefill_resid_strips)
  int resid_strips_opt;  // 1, 2 or 4: strips per wavefront of every GEMM fixed by the caller (gate/up: at least 2); 0 = by row count
  int blk_n, blk_m;  // tiles (along the features, along the rows) of the block one die works on at a time; 0 = default
  int attn_rows;  // query rows of an attention workgroup: 16, 32 or 128 (0 = 128 for passes of more than 512 rows, else 32)
  float *q;       // [rows][D] rotated queries
};
// Whose rows a tiled pass carries: the pass is cut into blocks of 128 rows, block i holds `rows[i]` prompt rows
// (0 .. 128, the rest of the block is padding) of sequence `slot[i]` starting at position `pos[i]`.  A prompt
// longer than a block fills consecutive blocks; several prompts share a pass, each starting on a block.
constexpr int kPrefillBlockRows = 128;
struct PrefillSegs {
  int n_blocks;
  int slot[kPrefillRows / kPrefillBlockRows], pos[kPrefillRows / kPrefillBlockRows], rows[kPrefillRows / kPrefillBlockRows];
};
// row assembly of a pass described by `segs` (p.prefill_ids: one token per row of the pass, padding rows any valid token)
void launch_assemble_prefill_segs(const Params &p, const void *tok_emb, const void *gain0, const PrefillSegs &segs, int M,
                                  int ssq_parts, int ssq_stride, hipStream_t s);
void launch_prefill_qkv(const Params &p, const PrefillWs &w, const void *W, int layer, const PrefillSegs &segs, int M,
                        hipStream_t s);
void launch_prefill_attention(const Params &p, const PrefillWs &w, int layer, int slot, int pos0, int R,
                              hipStream_t s);
void launch_prefill_resid(const Params &p, const PrefillWs &w, const void *W, const uint16_t *X, int K,
                          const void *gain_next, int M, hipStream_t s);
void launch_prefill_gateup(const Params &p, const PrefillWs &w, const void *W, int M, hipStream_t s);
int prefill_resid_strips(const Params &p, int M);

void launch_gemm_logits(const Params &p, const GemmTuning &tn, const void *W, float *logits, int M, hipStream_t s);

// ---- look-ahead embedding training: matrix-core pieces (kernels_mfma.hip) ----
void launch_gemm_gateup_save(const Params &p, const void *W, float *gu_save, int M, hipStream_t s);
int plain_gemm_slices(int N, int K);
int launch_gemm_plain(const Params &p, const void *W, const uint16_t *X, int M, int N, int K, float *part, hipStream_t s);
void launch_transpose_packed(const void *src, void *dst, int N, int K, hipStream_t s);
// ---- look-ahead embedding training (kernels_train.hip) ----
constexpr int kTrainSplits = 32;    // row slices of a transposed projection (partial sums: kTrainSplits x M x K floats)
constexpr int kTrainMaxKeys = 8192; // longest context a training step takes
constexpr int kTrainAttnChunk = 256; // keys per workgroup of the attention backward
constexpr int kTrainAttnSplits = kTrainMaxKeys / kTrainAttnChunk;  // its partial dq: [kTrainAttnSplits][kMaxRows][D] floats
void launch_assemble_train(const Params &p, int dtype, const void *tok_emb, const float *master, int B, int R, hipStream_t s);
void launch_assemble_train_mfma(const Params &p, const void *tok_emb, const float *master, const void *gain0, int B, int R,
                                hipStream_t s);
// x_out not null: the gradient leaves as (hi, lo) tiles of V features instead of in place
void launch_ce_grad(float *logits, const int32_t *targets, float scale, float *row_loss, int M, int V, uint16_t *x_out,
                    hipStream_t s);
void launch_gemm_t(int dtype, const float *dY, int ldy, const void *W, float *part, float *out, int ldo, int M, int N, int K,
                   hipStream_t s);
// gradients that come out of a matrix-core product arrive as KS slices, `slice_stride` floats apart, which the
// consumer adds in order (KS = 1: a plain array); *_x outputs: (hi, lo) tiles for the next matrix-core product
void launch_rmsnorm_bwd(const Params &p, int dtype, const float *x, const void *gain, const float *dy, int KS, size_t slice_stride,
                        float *dx_acc, int M, int accumulate, uint16_t *dx_x, hipStream_t s);
void launch_swiglu_bwd(const Params &p, const float *gu, const float *dact, float *dgu, int M, hipStream_t s);
void launch_swiglu_bwd_tiles(const Params &p, const float *gu, const float *dact, int KS, size_t slice_stride, uint16_t *dgu_x,
                             int M, hipStream_t s);
// q_saved [M][ldq] rotated queries; o / o_x: the forward pass's attention output as fp32 [M][D] or as (hi, lo) tiles
// (one of them null); lse [M][H]; dattn [M][D]; dq_part: workspace; result: dqkv [M][3D] fp32, or, with dqkv_x not
// null, (hi, lo) tiles of it (dqkv still serves as workspace)
void launch_attn_bwd(const Params &p, int dtype, int layer, int B, int R, int max_keys, const float *q_saved, int ldq,
                     const float *o, const uint16_t *o_x, const float *lse, const float *dattn, int KS, size_t slice_stride,
                     float *dq_part, float *dqkv, uint16_t *dqkv_x, hipStream_t s);
void launch_lookahead_adamw(int dtype, const float *dh, int B, int R, int d, float *grad, float *master, float *m1, float *m2,
                            void *model_la, float lr, float beta1, float beta2, float eps, float wd, float bc1, float bc2,
                            hipStream_t s);
void launch_lookahead_init(int dtype, const void *tok_emb, void *model_la, int token, int k, int d, float *master, float *m1,
                           float *m2, hipStream_t s);
void launch_lookahead_store(int dtype, const float *master, int k, int d, void *model_la, hipStream_t s);

}  // namespace pass
