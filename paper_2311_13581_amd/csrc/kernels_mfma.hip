// Matrix-core path of the (1+k)-row decode step for bf16 models on gfx950.
//
// The step is bound by streaming the weights once (Section 2.2 of the paper: a few extra rows
// cost about as much as one row because decoding is memory-bound).  Every weight matrix is
// repacked at load time into tiles of 16 output features x 32 input features, stored in the lane
// order of v_mfma_f32_16x16x32_bf16's A operand, so that one wavefront fetches a tile as 64
// adjacent 16-byte loads (1 KB, fully coalesced) and a strip of 16 output features is one
// contiguous run of K/32 KB.  The M <= 64 activation rows are the B operand (rows padded to 16
// per MFMA).  A workgroup of 4 to 16 wavefronts owns one strip (a gate and an up strip for
// gate/up; up to four strips for calls with more than 8 rows) and splits K among its wavefronts;
// the next trip's weight tiles are requested before the current trip computes; partial tiles are
// reduced through LDS in a fixed order (deterministic).  No workgroup shares weights with another,
// and the activation rows (tens of KB) sit in every XCD's L2, so the block-to-XCD mapping needs
// no special order.
//
// Activations keep fp32-like precision although the matrix core takes bf16: every activation x
// is carried as a pair (hi, lo) of bf16 values, hi = bf16(x), lo = bf16(x - hi).  Eight rows fill
// one 16-column MFMA: columns 0..7 take the hi halves, columns 8..15 the lo halves of the same
// rows, and the epilogue adds column j+8 to column j.  So a (1+k)-row call with k <= 7 costs one
// MFMA and one activation load per weight tile, and nothing but the weights and the K/V cache is
// ever rounded to 8 bits of mantissa (the paper's bfloat16 is read as the storage format of the
// model, Training details).  Activation buffers are laid out for that, in tiles like the weights:
// [group of 8 rows][K/32][64 lanes][8], lane (k/8 % 4) * 16 + c holds 8 consecutive features of
// pseudo-row c (c < 8: hi of row c, c >= 8: lo of row c - 8), so a wavefront fetches its B operand
// of a k-tile as 1 KB of whole cache lines.
//
// Fused epilogues:
//   QKV     : RMSNorm scale, rotary embedding, q (fp32) to the workspace, K/V rows (bf16) into
//             the paged cache
//   RESID   : residual add into h (fp32), (hi, lo) of h * gain of the next norm, per-strip
//             partial sums of h^2
//   GATEUP  : RMSNorm scale, silu(gate) * up as (hi, lo)
//   LOGITS  : RMSNorm scale, fp32 logits into the slot's logits rows
// RMSNorm has no kernel: the producer stores (hi, lo) of h * gain and partial sums of h^2; the
// consumer multiplies its accumulators by rsqrt(mean(h^2) + eps), which commutes with the GEMM.
#include <algorithm>

#include "pass_internal.h"

namespace pass {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


// ---------------------------------------------------------------------------------------------
// Weight repacking: plain [N][K] bf16 -> tiles [strip][K/32][64 lanes][8], lane l of a tile holds
// row (l % 16), columns (l / 16) * 8 .. + 8 of the tile.  Destination strip = off + stride * s.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_tiles_kernel(const uint4 *src, uint4 *dst, int N, int K,
                                                         int strip_off, int strip_stride) {
  const int KT = K / 32;
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // one 16-byte chunk each
  size_t total = (size_t)(N / 16) * KT * 64;
  if (idx >= total) return;
  int lane = (int)(idx & 63);
  size_t tile = idx >> 6;
  int kt = (int)(tile % KT);
  int s = (int)(tile / KT);
  int row = s * 16 + (lane & 15);
  int col = kt * 32 + (lane >> 4) * 8;
  size_t dstrip = (size_t)strip_off + (size_t)strip_stride * s;
  dst[(dstrip * KT + kt) * 64 + lane] = src[((size_t)row * K + col) / 8];
}

void launch_pack_tiles(const uint16_t *src, uint16_t *dst, int N, int K, int strip_off, int strip_stride,
                       hipStream_t s) {
  size_t total = (size_t)(N / 16) * (K / 32) * 64;
  pack_tiles_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint4 *)src, (uint4 *)dst, N, K,
                                                                      strip_off, strip_stride);
}

// ---------------------------------------------------------------------------------------------
// Row assembly for the matrix-core path: h (fp32), (hi, lo) of h * gain of the first norm,
// partial sums of h^2 (partial 0 carries the whole row, the others are zero), rotary table,
// row tables.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void assemble_mfma_kernel(Params p, const uint16_t *tok_emb,
                                                            const uint16_t *lookahead, const uint16_t *gain0,
                                                            int mode, int R, int ssq_parts, int ssq_stride,
                                                            int row_tables) {
  __shared__ float red[4];
  int m = blockIdx.x, b = m / R, r = m % R;
  int slot = p.step_slots[b];
  int pos = p.kv_len[slot] + r;
  const bool dead = row_is_dead(p, mode, slot, R);
  const uint16_t *src;
  if (mode == MODE_PREFILL) {
    src = tok_emb + (size_t)p.prefill_ids[r] * p.d;
  } else if (r == 0) {
    src = tok_emb + (size_t)clamp_token(p, p.pending[slot]) * p.d;
  } else if (mode == MODE_DRAFT) {
    // look-ahead embedding r (Section 2.2.1), or the fixed token of the paper's second baseline
    src = p.la_token >= 0 ? tok_emb + (size_t)p.la_token * p.d : lookahead + (size_t)(r - 1) * p.d;
  } else {
    src = tok_emb + (size_t)clamp_token(p, p.drafts[slot * kMaxK + (r - 1)]) * p.d;
  }
  // eight consecutive features per thread and trip: one 16-byte load of the embedding row and of
  // the gain, two 16-byte stores of h, one 16-byte store each of the hi and the lo tile slots
  float ss = 0.f;
  for (int c0 = threadIdx.x * 8; c0 < p.d; c0 += 256 * 8) {
    const uint4 sv = *(const uint4 *)(src + c0), gv = *(const uint4 *)(gain0 + c0);
    const uint32_t sw[4] = {sv.x, sv.y, sv.z, sv.w}, gw[4] = {gv.x, gv.y, gv.z, gv.w};
    float v[8], x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] = __uint_as_float(sw[e] << 16);
      v[2 * e + 1] = __uint_as_float(sw[e] & 0xffff0000u);
      x[2 * e] = v[2 * e] * __uint_as_float(gw[e] << 16);
      x[2 * e + 1] = v[2 * e + 1] * __uint_as_float(gw[e] & 0xffff0000u);
    }
    float4 *hp = (float4 *)(p.h + (size_t)m * p.d + c0);
    hp[0] = make_float4(v[0], v[1], v[2], v[3]);
    hp[1] = make_float4(v[4], v[5], v[6], v[7]);
    uint4 hi, lo;
    hi.x = split2_bf16(x[0], x[1], true); lo.x = split2_bf16(x[0], x[1], false);
    hi.y = split2_bf16(x[2], x[3], true); lo.y = split2_bf16(x[2], x[3], false);
    hi.z = split2_bf16(x[4], x[5], true); lo.z = split2_bf16(x[4], x[5], false);
    hi.w = split2_bf16(x[6], x[7], true); lo.w = split2_bf16(x[6], x[7], false);
    uint16_t *xh = p.xg + xs_index(m, p.d, c0);
    *(uint4 *)xh = hi;
    *(uint4 *)(xh + kXsLoOffset) = lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  for (int i = threadIdx.x; i < ssq_parts; i += 256)
    p.ssq[(size_t)i * ssq_stride + m] = (i == 0) ? (red[0] + red[1] + red[2] + red[3]) : 0.f;
  int half = p.hd / 2;
  for (int i = threadIdx.x; i < half; i += 256) {
    double sn, cs;
    sincos((double)pos * p.rope_theta[i], &sn, &cs);
    p.rope_cos[(size_t)m * half + i] = (float)cs;
    p.rope_sin[(size_t)m * half + i] = (float)sn;
  }
  if (threadIdx.x == 0 && row_tables) {
    p.row_pos[m] = dead ? 0 : pos;
    p.row_slot[m] = dead ? -1 : slot;
    p.row_out[m] = slot * (1 + p.k) + r;
  }
}

void launch_assemble_mfma(const Params &p, const void *tok_emb, const void *lookahead, const void *gain0, int mode,
                          int B, int R, hipStream_t s) {
  assemble_mfma_kernel<<<B * R, 256, 0, s>>>(p, (const uint16_t *)tok_emb, (const uint16_t *)lookahead,
                                             (const uint16_t *)gain0, mode, R, p.d / 16, kMaxRows, 1);
}

// ---------------------------------------------------------------------------------------------
// The streaming GEMM
// ---------------------------------------------------------------------------------------------
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_GATEUP = 2, EPI_LOGITS = 3, EPI_PARTIAL = 4, EPI_GATEUP_SAVE = 5 };

struct GemmArgs {
  const u32x4 *W;             // packed weight tiles
  const uint16_t *X;          // activation rows as (hi, lo) tiles [ceil(M/8)][K/32][64 lanes][8]
  int M, K;
  int layer;
  const uint16_t *gain_next;  // RESID: gain of the norm that follows
  float *logits;              // LOGITS: base of the [slot][1+k][V] logits
  int kt_split;               // PARTIAL: k-tiles per workgroup row (blockIdx.y picks the slice of K); else 0
  float *partial;             // PARTIAL: [gridDim.y][kMaxRows][N] sums over the slice of K
  int n_strips;               // strips of the matrix (NB = 3: the last workgroup may own fewer blocks)
  int ldy;                    // PARTIAL: features per row of `partial`
  float *gu_save;             // GATEUP_SAVE: [M][2F] gate | up before the activation (what its derivative needs)
};

// MT = number of 8-row groups (one MFMA column block each); NB = output blocks per workgroup (a
// block is one strip of 16 features, or the gate strip and the up strip of 16 FFN features).
// Every activation tile a wavefront loads is used for all NB blocks, so the activation traffic
// out of L2 per weight byte falls as 1/NB: that traffic, not HBM, bounds the calls with many rows.
template <int MT, int EPI, int WAVES, int U, int NB>
__global__ __launch_bounds__(WAVES * 64) void gemm_mfma_kernel(Params p, GemmArgs a) {
  constexpr int kGemmWaves = WAVES;
  constexpr bool GU = (EPI == EPI_GATEUP || EPI == EPI_GATEUP_SAVE);
  constexpr int PER = GU ? 2 : 1;  // strips per block
  constexpr int NS = NB * PER;
  constexpr bool NORM = (EPI != EPI_RESID && EPI != EPI_PARTIAL);
  static_assert(WAVES * NS <= 32 && NB <= WAVES, "reduction buffer must fit the static LDS limit");
  __shared__ floatx4 red[kGemmWaves][NS][64];  // one 8-row group at a time
  __shared__ float red_ss[kGemmWaves][MT][8];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ml = lane & 15, g = lane >> 4;  // ml: MFMA column = pseudo-row; g: k-group of 8
  const int KT = a.K >> 5;                                        // k-tiles of the whole K (strip stride)
  const int KTl = (EPI == EPI_PARTIAL) ? a.kt_split : KT;         // k-tiles this workgroup walks
  const int kbase = (EPI == EPI_PARTIAL) ? blockIdx.y * KTl : 0;  // first of them
  const int strip0 = blockIdx.x * NS;

  floatx4 acc[NS][MT];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[s][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Activation loads go through a buffer descriptor: a lane whose pseudo-row belongs to a row
  // >= M gets an out-of-range offset and the hardware returns zeros without touching memory.
  // All loads are unconditional instructions, so outstanding requests are counted exactly and a
  // trip can wait for its activations while the next trip's weight tiles stay in flight.
  const int n_groups = (a.M + 7) >> 3;
  const __amdgpu_buffer_rsrc_t xr =
      __builtin_amdgcn_make_buffer_rsrc((void *)a.X, 0, n_groups * 16 * a.K * 2, 0x00020000);
  int xoff[MT];  // byte offset of this lane's 16 bytes in k-tile 0
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int m = mt * 8 + (ml & 7);
    xoff[mt] = (m < a.M) ? ((mt * KT + kbase) * 64 + lane) * 16 : 0x40000000;
  }
  const u32x4 *wp = a.W + ((size_t)strip0 * KT + kbase) * 64 + lane;
  // strip s of this workgroup, relative to strip0.  NB = 3 does not divide every matrix: strips
  // past the end repeat the last one (in bounds; their results are dropped in the epilogue)
  int soff[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) soff[s] = (NB == 3) ? min(s, a.n_strips - 1 - strip0) : s;

  auto load_a = [&](u32x4 (&dst)[U][NS], int kt0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s = 0; s < NS; ++s)
        dst[u][s] = __builtin_nontemporal_load(wp + ((size_t)soff[s] * KT + kt0 + u * kGemmWaves) * 64);
  };
  auto load_b = [&](u32x4 (&dst)[U][MT], int kt0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        dst[u][mt] = __builtin_amdgcn_raw_buffer_load_b128(xr, xoff[mt] + (kt0 + u * kGemmWaves) * 1024, 0, 0);
  };
  auto mma = [&](const u32x4 (&av)[U][NS], const u32x4 (&bv)[U][MT]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[s][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[u][s]),
                                                               __builtin_bit_cast(bf16x8, bv[u][mt]), acc[s][mt], 0, 0, 0);
  };

  // full trips: k-tiles kt0 + u * WAVES, u < U, with kt0 = wave + trip * WAVES * U (interleaved
  // over the wavefronts, so the workgroup walks its strip front to back)
  const int trip_tiles = kGemmWaves * U;
  const int n_trips = KTl / trip_tiles;
  if (n_trips > 0) {
    // Both operands of trip t+1 are requested during trip t, activations first, so a trip only
    // ever waits for requests that have had a whole trip to complete.
    u32x4 a_cur[U][NS], a_nxt[U][NS], b_cur[U][MT], b_nxt[U][MT];
    load_b(b_cur, wave);
    load_a(a_cur, wave);
    for (int t = 0; t < n_trips - 1; ++t) {
      const int kt1 = wave + (t + 1) * trip_tiles;
      load_b(b_nxt, kt1);
      load_a(a_nxt, kt1);
      mma(a_cur, b_cur);
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int s = 0; s < NS; ++s) a_cur[u][s] = a_nxt[u][s];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b_cur[u][mt] = b_nxt[u][mt];
      }
    }
    mma(a_cur, b_cur);
  }
  // tail: the k-tiles that do not fill a trip, one per wavefront and step (wavefront-uniform bound)
  for (int kt = n_trips * trip_tiles + wave; kt < KTl; kt += kGemmWaves) {
    u32x4 bv[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) bv[mt] = __builtin_amdgcn_raw_buffer_load_b128(xr, xoff[mt] + kt * 1024, 0, 0);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4 av = __builtin_nontemporal_load(wp + ((size_t)soff[s] * KT + kt) * 64);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[s][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av),
                                                             __builtin_bit_cast(bf16x8, bv[mt]), acc[s][mt], 0, 0, 0);
    }
  }

  // partial sums of h^2 (written by the producer of X) -> this wavefront's share.
  // Lane (ml & 7) covers row mt*8 + (ml & 7); the two halves of the columns take alternate partials.
  if constexpr (NORM) {
    const int NP = p.d / 16;
    // requested in batches of 8 through a buffer descriptor (indices past the end read as zero):
    // one trip to L2 per batch instead of one per partial
    const __amdgpu_buffer_rsrc_t sr = __builtin_amdgcn_make_buffer_rsrc((void *)p.ssq, 0, NP * kMaxRows * 4, 0x00020000);
    for (int mt = 0; mt < MT; ++mt) {
      float ss = 0.f;
      for (int i0 = wave * 8 + g * 2 + (ml >> 3); i0 < NP; i0 += kGemmWaves * 64) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          v[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
              sr, ((i0 + u * kGemmWaves * 8) * kMaxRows + mt * 8 + (ml & 7)) * 4, 0, 0));
#pragma unroll
        for (int u = 0; u < 8; ++u) ss += v[u];
      }
      ss += __shfl_xor(ss, 8);
      ss += __shfl_xor(ss, 16);
      ss += __shfl_xor(ss, 32);
      if (lane < 8) red_ss[wave][mt][lane] = ss;
    }
  }
  // Per 8-row group: every wavefront posts its partial tiles, wavefront j < NB reduces those of
  // block j in a fixed order, adds the lo columns to the hi columns and runs the fused epilogue.
  // Lanes with ml < 8 hold Y[m = mt*8 + ml][n0 + 4g .. 4g+3].
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt > 0) __syncthreads();  // the previous group has been read
#pragma unroll
    for (int s = 0; s < NS; ++s) red[wave][s][lane] = acc[s][mt];
    __syncthreads();
    if (wave >= NB) continue;
    const int blk = wave;
    const int strip = strip0 + blk * PER;
    if (NB == 3 && strip >= a.n_strips) continue;  // this workgroup's last block does not exist
    floatx4 y[PER];
#pragma unroll
    for (int s = 0; s < PER; ++s) {
      y[s] = red[0][blk * PER + s][lane];
#pragma unroll
      for (int w = 1; w < kGemmWaves; ++w) y[s] += red[w][blk * PER + s][lane];
#pragma unroll
      for (int r = 0; r < 4; ++r) y[s][r] += __shfl_xor(y[s][r], 8);
    }
    const int m = mt * 8 + (ml & 7);
    float inv = 1.f;
    if constexpr (NORM) {
      float ss = 0.f;
#pragma unroll
      for (int w = 0; w < kGemmWaves; ++w) ss += red_ss[w][mt][ml & 7];
      inv = 1.0f / sqrtf(ss / (float)p.d + p.eps);
    }
    const bool live = m < a.M && ml < 8;

    if constexpr (EPI == EPI_LOGITS) {
      if (live) {
        float *o = a.logits + (size_t)p.row_out[m] * p.V + strip * 16 + 4 * g;
        *(floatx4 *)o = y[0] * inv;
      }
    } else if constexpr (GU) {
      if (live) {
        // strips 2b (gate) and 2b+1 (up) of the interleaved matrix both belong to features 16b..16b+15
        int f0 = (blockIdx.x * NB + blk) * 16 + 4 * g;
        float t[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float gt = y[0][r] * inv, up = y[1][r] * inv;
          t[r] = gt / (1.0f + __expf(-gt)) * up;
        }
        store_split4(p.act_x, m, p.F, f0, t);
        if constexpr (EPI == EPI_GATEUP_SAVE) {
          *(floatx4 *)(a.gu_save + (size_t)m * 2 * p.F + f0) = y[0] * inv;
          *(floatx4 *)(a.gu_save + (size_t)m * 2 * p.F + p.F + f0) = y[1] * inv;
        }
      }
    } else if constexpr (EPI == EPI_PARTIAL) {
      // sums over this workgroup's slice of K; the slices are added up by resid_reduce_kernel
      if (live)
        *(floatx4 *)(a.partial + ((size_t)blockIdx.y * kMaxRows + m) * a.ldy + strip * 16 + 4 * g) = y[0];
    } else if constexpr (EPI == EPI_RESID) {
      int n = strip * 16 + 4 * g;
      float ss = 0.f;
      if (live) {
        float *hp = p.h + (size_t)m * p.d + n;
        floatx4 hv = *(floatx4 *)hp + y[0];
        *(floatx4 *)hp = hv;
        float t[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          t[r] = hv[r] * bf16_to_f32(a.gain_next[n + r]);
          ss += hv[r] * hv[r];
        }
        store_split4(p.xg, m, p.d, n, t);
      }
      ss += __shfl_xor(ss, 16);
      ss += __shfl_xor(ss, 32);
      if (lane < 8) p.ssq[(size_t)strip * kMaxRows + m] = ss;  // rows >= M get 0
    } else {  // EPI_QKV
      if (live) {
        int n = strip * 16 + 4 * g;       // column in [0, 3D)
        int which = n / p.D;              // 0 q, 1 k, 2 v
        int c = n - which * p.D;          // column inside the projection
        int head = c / p.hd, dim = c - head * p.hd;
        floatx4 v = y[0] * inv;
        if (which < 2) {
          int half = p.hd / 2;
          const float *cs = p.rope_cos + (size_t)m * half + dim / 2;
          const float *sn = p.rope_sin + (size_t)m * half + dim / 2;
          float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
          v[0] = x0 * cs[0] - x1 * sn[0];
          v[1] = x0 * sn[0] + x1 * cs[0];
          v[2] = x2 * cs[1] - x3 * sn[1];
          v[3] = x2 * sn[1] + x3 * cs[1];
        }
        if (which == 0) {
          *(floatx4 *)(p.qkv + (size_t)m * 3 * p.D + c) = v;
        } else if (p.row_slot[m] >= 0) {  // a dead row (see row_is_dead) has no place in the cache
          // the cache is bf16 storage: the one place besides the weights where values are rounded
          uint16_t *pool = (uint16_t *)(which == 1 ? p.k_pool : p.v_pool);
          if (which == 2 && p.v_transposed) {
            // V page for the matrix-core attention: [head][dim][page_size]
            int pos = p.row_pos[m];
            int page = p.block_table[(size_t)p.row_slot[m] * p.pages_per_seq + (pos >> p.page_shift)];
            size_t base = ((((size_t)a.layer * p.n_pages + page) * p.H + head) * p.hd + dim) * p.page_size +
                          (pos & (p.page_size - 1));
#pragma unroll
            for (int r = 0; r < 4; ++r) pool[base + (size_t)r * p.page_size] = f32_to_bf16(v[r]);
          } else {
            size_t off = kv_offset(p, a.layer, p.row_slot[m], p.row_pos[m], head) + dim;
            uint2 pk;
            pk.x = pack2_bf16(v[0], v[1]);
            pk.y = pack2_bf16(v[2], v[3]);
            *(uint2 *)(pool + off) = pk;
          }
        }
      }
    }
  }
}

// Launch shape of the decode-sized GEMMs: GemmTuning (a member of the context, so two contexts
// never share a setting).  Defaults chosen by sweeping the benchmark on MI355X.
GemmTuning::GemmTuning()
    : waves{0, 0, 4, 16, 0},       // QKV, Wo, gate/up, LM head, down; 0 = by strip count (launch_gemm_epi)
      unroll{1, 1, 1, 2, 1},
      // Calls with more than 8 rows are bound by what one compute unit can pull through its vector
      // memory path, and every workgroup pulls all M activation rows whatever it owns of the
      // weights: best is one workgroup per compute unit with as many blocks as that leaves it
      // (QKV: 768 strips = 256 x 3; gate/up: 688 pairs = 230 x 3).
      big_waves{8, 16, 4, 8, 16},
      big_blocks{0, 1, 0, 4, 1},   // 0 = as many as leave one workgroup per compute unit
      split_ks(4) {}

int GemmTuning::set(int kind, int w, int u) {
  if (kind < 0 || kind > 4) return -1;
  if (w != 4 && w != 8 && w != 16) return -1;
  if (u != 1 && u != 2 && u != 4) return -1;
  waves[kind] = w;
  unroll[kind] = u;
  return 0;
}

int GemmTuning::set_big(int kind, int w, int blocks) {
  if (kind < 0 || kind > 4) return -1;
  if (w != 4 && w != 8 && w != 16) return -1;
  if (blocks < 0 || blocks > 4) return -1;
  big_waves[kind] = w;
  big_blocks[kind] = blocks;
  return 0;
}

int GemmTuning::set_split(int ks) {
  if (ks < 0 || ks > 8) return -1;
  split_ks = ks;
  return 0;
}

template <int EPI, int W, int U>
static void launch_one(const Params &p, const GemmArgs &a, int grid, hipStream_t s) {
  gemm_mfma_kernel<1, EPI, W, U, 1><<<grid, W * 64, 0, s>>>(p, a);
}

template <int EPI, int W, int NB>
static void launch_big(const Params &p, const GemmArgs &a, int n_blocks, int mt, hipStream_t s) {
  constexpr int PER = (EPI == EPI_GATEUP || EPI == EPI_GATEUP_SAVE) ? 2 : 1;
  if constexpr (W * NB * PER > 32) {
    launch_big<EPI, 8, 1>(p, a, n_blocks, mt, s);
  } else {
    const int grid = (n_blocks + NB - 1) / NB;
    constexpr int T = W * 64;
    constexpr int U2 = (NB == 1 && W == 16) ? 2 : 1;  // two k-tiles per trip while registers allow
    switch (mt) {
      case 2: gemm_mfma_kernel<2, EPI, W, U2, NB><<<grid, T, 0, s>>>(p, a); break;
      case 3: gemm_mfma_kernel<3, EPI, W, U2, NB><<<grid, T, 0, s>>>(p, a); break;
      case 4: gemm_mfma_kernel<4, EPI, W, U2, NB><<<grid, T, 0, s>>>(p, a); break;
      case 5: gemm_mfma_kernel<5, EPI, W, 1, NB><<<grid, T, 0, s>>>(p, a); break;
      case 6: gemm_mfma_kernel<6, EPI, W, 1, NB><<<grid, T, 0, s>>>(p, a); break;
      case 7: gemm_mfma_kernel<7, EPI, W, 1, NB><<<grid, T, 0, s>>>(p, a); break;
      default: gemm_mfma_kernel<8, EPI, W, 1, NB><<<grid, T, 0, s>>>(p, a); break;
    }
  }
}

template <int EPI>
static void launch_gemm_epi(const Params &p, const GemmTuning &tn, const GemmArgs &a, int n_strips, hipStream_t s,
                            int kind = EPI) {
  constexpr int PER = (EPI == EPI_GATEUP) ? 2 : 1;
  const int n_blocks = n_strips / PER;
  int mt = (a.M + 7) / 8;
  if (mt == 1) {
    const int grid = n_blocks;
    // QKV and the residual projections: when the strips fill the 256 compute units evenly
    // (d = 4096: 768 and 256 strips) coarse workgroups are best (8 and 16 wavefronts); otherwise
    // (d = 5120: 960 and 320 strips) finer ones, of which a unit holds several, balance better.
    const bool even = n_blocks % 256 == 0;
    const int w = tn.waves[kind] ? tn.waves[kind] : (kind == 0 ? (even ? 8 : 4) : (even ? 16 : 8));
    const int u = tn.unroll[kind];
    switch (w * 10 + u) {
      case 161: launch_one<EPI, 16, 1>(p, a, grid, s); break;
      case 162: launch_one<EPI, 16, 2>(p, a, grid, s); break;
      case 164: launch_one<EPI, 16, 4>(p, a, grid, s); break;
      case 81: launch_one<EPI, 8, 1>(p, a, grid, s); break;
      case 82: launch_one<EPI, 8, 2>(p, a, grid, s); break;
      case 84: launch_one<EPI, 8, 4>(p, a, grid, s); break;
      case 41: launch_one<EPI, 4, 1>(p, a, grid, s); break;
      case 42: launch_one<EPI, 4, 2>(p, a, grid, s); break;
      default: launch_one<EPI, 4, 4>(p, a, grid, s); break;
    }
    return;
  }
  int w = tn.big_waves[kind], nb = tn.big_blocks[kind];
  if (nb == 0) nb = std::min(PER == 2 ? 3 : 4, (n_blocks + 255) / 256);  // 7B: QKV 768 / 256 = 3, gate/up 688 pairs -> 3
  if (mt == 8 && nb == 4) nb = 2;                 // 64 rows x 4 blocks does not fit the register file
  if (nb == 3 && mt * PER > 10) nb = 2;           // nor do 3 blocks of more than 40 rows (gate/up) / 80
  while (nb != 3 && nb > 1 && n_blocks % nb != 0) nb >>= 1;  // a workgroup's blocks must all exist (3: the kernel copes)
  switch (w * 10 + nb) {
    case 161: launch_big<EPI, 16, 1>(p, a, n_blocks, mt, s); break;
    case 162: launch_big<EPI, 16, 2>(p, a, n_blocks, mt, s); break;
    case 81: launch_big<EPI, 8, 1>(p, a, n_blocks, mt, s); break;
    case 82: launch_big<EPI, 8, 2>(p, a, n_blocks, mt, s); break;
    case 84: launch_big<EPI, 8, 4>(p, a, n_blocks, mt, s); break;
    case 83: launch_big<EPI, 8, 3>(p, a, n_blocks, mt, s); break;
    case 43: launch_big<EPI, 4, 3>(p, a, n_blocks, mt, s); break;
    case 41: launch_big<EPI, 4, 1>(p, a, n_blocks, mt, s); break;
    case 42: launch_big<EPI, 4, 2>(p, a, n_blocks, mt, s); break;
    case 44: launch_big<EPI, 4, 4>(p, a, n_blocks, mt, s); break;
    default: launch_big<EPI, 16, 1>(p, a, n_blocks, mt, s); break;
  }
}

// ---------------------------------------------------------------------------------------------
// Residual projections (Wo, down) of calls with more than 8 rows.  N = d gives only d/16 strips,
// one per compute unit at best, and every workgroup would have to pull all M activation rows
// through its L1: that traffic, not HBM, bounds the kernel.  So K is cut into KS slices across
// workgroups that each own 4 strips (an activation tile fetched is used 4 times); the slices'
// sums go to a workspace and this kernel adds them in slice order (deterministic), then does what
// the fused epilogue does: residual add into h, (hi, lo) of h * gain of the next norm, per-strip
// partial sums of h^2.  One workgroup per strip of 16 features: thread = (row, 4 features).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void resid_reduce_kernel(Params p, const float *partial, int KS, int M,
                                                           const uint16_t *gain_next) {
  const int strip = blockIdx.x, m = threadIdx.x >> 2, n = strip * 16 + (threadIdx.x & 3) * 4;
  float ss = 0.f;
  if (m < M) {
    float *hp = p.h + (size_t)m * p.d + n;
    floatx4 hv = *(floatx4 *)hp;
    floatx4 part[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)  // all slices requested at once (index clamped, surplus dropped)
      part[ks] = *(const floatx4 *)(partial + ((size_t)min(ks, KS - 1) * kMaxRows + m) * p.d + n);
    floatx4 y = part[0];
#pragma unroll
    for (int ks = 1; ks < 8; ++ks)
      if (ks < KS) y += part[ks];
    hv += y;
    *(floatx4 *)hp = hv;
    float t[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      t[r] = hv[r] * bf16_to_f32(gain_next[n + r]);
      ss += hv[r] * hv[r];
    }
    store_split4(p.xg, m, p.d, n, t);
  }
  ss += __shfl_xor(ss, 1);
  ss += __shfl_xor(ss, 2);
  if ((threadIdx.x & 3) == 0) p.ssq[(size_t)strip * kMaxRows + m] = ss;  // rows >= M get 0
}

// wavefronts per workgroup and strips per workgroup of the split residual GEMM (K slices: GemmTuning)
constexpr int kSplitWaves = 8, kSplitBlocks = 4;

static bool launch_resid_split(const Params &p, const GemmTuning &tn, const GemmArgs &a0, int mt, hipStream_t s) {
  const int n_strips = p.d / 16, KT = a0.K >> 5, KS = tn.split_ks;
  if (KS < 2 || n_strips % kSplitBlocks != 0 || KT % KS != 0) return false;
  if ((size_t)KS * p.d > (size_t)2 * p.F) return false;  // the slices' sums borrow the generic path's gate/up workspace
  GemmArgs a = a0;
  a.kt_split = KT / KS;
  a.partial = p.gu;
  a.ldy = p.d;
  dim3 grid(n_strips / kSplitBlocks, KS);
  constexpr int T = kSplitWaves * 64;
  switch (mt) {
    case 2: gemm_mfma_kernel<2, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 3: gemm_mfma_kernel<3, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 4: gemm_mfma_kernel<4, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 5: gemm_mfma_kernel<5, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 6: gemm_mfma_kernel<6, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 7: gemm_mfma_kernel<7, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    default: gemm_mfma_kernel<8, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
  }
  resid_reduce_kernel<<<n_strips, 256, 0, s>>>(p, a.partial, KS, a.M, a.gain_next);
  return true;
}

void launch_gemm_qkv(const Params &p, const GemmTuning &tn, const void *W, int layer, int M, hipStream_t s) {
  GemmArgs a{(const u32x4 *)W, p.xg, M, p.d, layer, nullptr, nullptr, 0, nullptr, 3 * p.D / 16};
  launch_gemm_epi<EPI_QKV>(p, tn, a, 3 * p.D / 16, s);
}
void launch_gemm_resid(const Params &p, const GemmTuning &tn, const void *W, const uint16_t *X, int K,
                       const void *gain_next, int M, hipStream_t s) {
  GemmArgs a{(const u32x4 *)W, X, M, K, 0, (const uint16_t *)gain_next, nullptr, 0, nullptr, p.d / 16};
  if (M > 8 && launch_resid_split(p, tn, a, (M + 7) / 8, s)) return;
  launch_gemm_epi<EPI_RESID>(p, tn, a, p.d / 16, s, K == p.F ? 4 : 1);  // the down projection has its own shape
}
void launch_gemm_gateup(const Params &p, const GemmTuning &tn, const void *W, int M, hipStream_t s) {
  GemmArgs a{(const u32x4 *)W, p.xg, M, p.d, 0, nullptr, nullptr, 0, nullptr, 2 * p.F / 16};
  launch_gemm_epi<EPI_GATEUP>(p, tn, a, 2 * p.F / 16, s);
}
void launch_gemm_logits(const Params &p, const GemmTuning &tn, const void *W, float *logits, int M, hipStream_t s) {
  GemmArgs a{(const u32x4 *)W, p.xg, M, p.d, 0, nullptr, logits, 0, nullptr, p.V / 16};
  launch_gemm_epi<EPI_LOGITS>(p, tn, a, p.V / 16, s);
}


// ---------------------------------------------------------------------------------------------
// What the training of the look-ahead embeddings adds (kernels_train.hip has the rest).
// ---------------------------------------------------------------------------------------------
// The gate/up GEMM that also keeps gate | up before the activation, in the decode call's launch shapes.
void launch_gemm_gateup_save(const Params &p, const void *W, float *gu_save, int M, hipStream_t s) {
  GemmArgs a{(const u32x4 *)W, p.xg, M, p.d, 0, nullptr, nullptr, 0, nullptr, 2 * p.F / 16, 0, gu_save};
  const int n_blocks = p.F / 16, mt = (M + 7) / 8;
  if (mt == 1)
    launch_one<EPI_GATEUP_SAVE, 4, 1>(p, a, n_blocks, s);
  else if (mt <= 5)
    launch_big<EPI_GATEUP_SAVE, 4, 3>(p, a, n_blocks, mt, s);
  else if (n_blocks % 2 == 0)  // three blocks of more than 40 rows do not fit the register file
    launch_big<EPI_GATEUP_SAVE, 4, 2>(p, a, n_blocks, mt, s);
  else
    launch_big<EPI_GATEUP_SAVE, 4, 1>(p, a, n_blocks, mt, s);
}

// Plain product Y = X W^T on packed tiles: X as (hi, lo) tiles of K features, W packed [N][K], Y fp32.
// K is cut into KS slices across workgroups of 8 wavefronts that own 4 strips each; slice ks leaves its
// sums in part[ks][kMaxRows][N] and the consumer adds the slices in order.  Needs N % 64 == 0 and
// (K / 32) % KS == 0; returns the KS it used (plain_gemm_slices: what the consumer must add up).
int plain_gemm_slices(int N, int K) {
  const int KT = K / 32, wgs = N / 64;
  int best = 1;
  for (int ks = 1; ks <= 8; ks *= 2) {
    if (KT % ks != 0 || KT / ks < 8) break;
    best = ks;
    if (wgs * ks >= 256) break;  // one workgroup per compute unit: each pulls its slice of the rows once
  }
  return best;
}
int launch_gemm_plain(const Params &p, const void *W, const uint16_t *X, int M, int N, int K, float *part, hipStream_t s) {
  const int KS = plain_gemm_slices(N, K);
  GemmArgs a{(const u32x4 *)W, X, M, K, 0, nullptr, nullptr, (K / 32) / KS, part, N / 16, N, nullptr};
  dim3 grid(N / 64, KS);
  constexpr int T = kSplitWaves * 64;
  switch ((M + 7) / 8) {
    case 1: gemm_mfma_kernel<1, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 2: gemm_mfma_kernel<2, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 3: gemm_mfma_kernel<3, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 4: gemm_mfma_kernel<4, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 5: gemm_mfma_kernel<5, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 6: gemm_mfma_kernel<6, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    case 7: gemm_mfma_kernel<7, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
    default: gemm_mfma_kernel<8, EPI_PARTIAL, kSplitWaves, 1, kSplitBlocks><<<grid, T, 0, s>>>(p, a); break;
  }
  return KS;
}

// Packed tiles of W [N][K] -> packed tiles of its transpose [K][N] (the backward pass multiplies by
// W^T with the same kernels).  One 16-byte chunk of the destination per thread: row k of W^T, eight
// consecutive n.  Run once when training is set up.
__global__ __launch_bounds__(256) void transpose_packed_kernel(const uint16_t *src, uint16_t *dst, int N, int K) {
  const int KT = K / 32, NT = N / 32;  // k-tiles of the source, of the destination
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x, total = (size_t)(K / 16) * NT * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t tile = idx >> 6;
  const int nt = (int)(tile % NT), ks = (int)(tile / NT);  // destination k-tile (over n), strip (over k)
  const int k = ks * 16 + (lane & 15), n0 = nt * 32 + (lane >> 4) * 8;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int n = n0 + e;
    v[e] = src[((((size_t)(n >> 4) * KT + (k >> 5)) * 64 + ((k >> 3) & 3) * 16 + (n & 15)) << 3) + (k & 7)];
  }
  uint4 o;
  o.x = v[0] | (uint32_t)v[1] << 16; o.y = v[2] | (uint32_t)v[3] << 16;
  o.z = v[4] | (uint32_t)v[5] << 16; o.w = v[6] | (uint32_t)v[7] << 16;
  *(uint4 *)(dst + idx * 8) = o;
}
void launch_transpose_packed(const void *src, void *dst, int N, int K, hipStream_t s) {
  const size_t total = (size_t)(K / 16) * (N / 32) * 64;
  transpose_packed_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t *)src, (uint16_t *)dst, N, K);
}

}  // namespace pass
