// Prompt pass ("initial prompt sequence" of Algorithm 1) as a compute-bound problem.
//
// The decode kernels stream every weight once per call of at most 64 rows; a prompt of thousands
// of tokens pushed through them re-reads the model dozens of times and leaves the matrix cores
// idle.  Here up to 2048 prompt rows go through each layer in one pass:
//
//   gemm_tile_kernel   a workgroup of 4 wavefronts computes 256 (or 128, 64) output features x 64
//                      rows.  The activation tile of a k-step (rows x 32 features, as (hi, lo)
//                      pairs) is staged once in LDS and read by all wavefronts; every
//                      wavefront streams the weight tiles of its own strips straight into
//                      registers, three k-steps ahead.  Accumulators (128 registers per lane)
//                      stay in the register file for the whole K loop: no split of K, one fixed
//                      summation order.  Same operand formats and the same fused epilogues as the
//                      decode GEMM (RMSNorm scale, rotary embedding and K/V page writes, SiLU * up,
//                      residual add with (hi, lo) of the next norm's input).
//   attn_prefill_kernel causal attention of a block of 32 (or 16) query rows of one head over the
//                      paged cache, without a split of the keys across workgroups: the four
//                      wavefronts take alternate 32-key steps and merge once at the end.  K and V
//                      tiles are used for all row groups of the block.
//   attn_prefill_shared_kernel  the same for passes of more than 512 rows: 128 rows per workgroup,
//                      the K and V tiles of a step fetched once into LDS for all four wavefronts.
//
// Workgroup -> tile mapping: consecutive workgroup ids go to different dies (XCDs), each with its
// own L2.  The 64 workgroups a die holds at a time are given a block of 8 x 8 tiles, so a weight
// tile and an activation tile fetched into that L2 are each used by 8 workgroups.
#include "pass_internal.h"

namespace pass {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// value of the lane 8 columns further in the same row of 16 (row_ror 8): lo half <-> hi half
__device__ __forceinline__ float other_half(float v) { return dpp_mov<0x128>(v); }

template <int I> struct ic { static constexpr int value = I; };

enum { TILE_QKV = 0, TILE_RESID = 1, TILE_GATEUP = 2 };

struct TileArgs {
  const u32x4 *W;             // packed weight tiles [strip][K/32][64 lanes]
  const uint16_t *X;          // activation rows as (hi, lo) tiles [ceil(M/8)][K/32][64 lanes][8]
  int M, K, n_strips;
  int layer;
  const uint16_t *gain_next;  // RESID: gain of the norm that follows
  PrefillSegs segs;           // QKV: whose rows these are (K/V go to that sequence's pages)
  int tiles_m, tiles_n;
  int blk_n, blk_m, blocks_m, n_blocks;  // blocks of tiles, one per die at a time
};

constexpr int kTileStrips = 4;  // strips of 16 features per wavefront (fewer when the tiles would not fill the chip)

// MG = 8-row groups per workgroup tile (rows = 8 * MG).
// Two wavefronts per SIMD (256 registers each): above that budget the compiler moves the
// accumulators to AGPRs and, the MFMA then not being tied to its accumulator, permutes them
// every trip with hundreds of register copies.
// SW = strips of 16 features per wavefront: the tile is 64 * SW features x 8 * MG rows.
template <int EPI, int MG, int SW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_tile_kernel(Params p, PrefillWs w, TileArgs a) {
  constexpr int NT = 256;
  constexpr int ROWS = MG * 8;
  constexpr bool NORM = (EPI != TILE_RESID);
  constexpr int BL = MG / 4;  // 16-byte chunks of the activation tile each thread stages per k-step
  __shared__ u32x4 sB[2][MG][64];
  __shared__ float s_inv[ROWS];
  __shared__ float s_part[NT];

  // tile of this workgroup (see the note on dies at the top): the `per` workgroups that one die
  // holds at a time form a block of blk_n x blk_m tiles
  const int per = a.blk_n * a.blk_m;
  const int loc = blockIdx.x >> 3;
  const int block = (loc / per) * 8 + (blockIdx.x & 7), within = loc % per;
  if (block >= a.n_blocks) return;
  const int tn = (block / a.blocks_m) * a.blk_n + within / a.blk_m;
  const int tm = (block % a.blocks_m) * a.blk_m + within % a.blk_m;
  if (tn >= a.tiles_n || tm >= a.tiles_m) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ml = lane & 15, g4 = lane >> 4;
  const int KT = a.K >> 5;
  const int m0 = tm * ROWS;
  const int strip0 = (tn * 4 + wave) * SW;

  // 1 / rms of the tile's rows from the producer's partial sums of h^2
  if constexpr (NORM) {
    constexpr int TG = NT / ROWS;
    const int row = tid % ROWS, tg = tid / ROWS;
    float ss = 0.f;
    if (m0 + row < a.M) {
      // eight requests at a time (indices past the end repeat the last partial and are dropped)
      for (int i0 = tg; i0 < w.np; i0 += 8 * TG) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p.ssq[(size_t)min(i0 + u * TG, w.np - 1) * w.rows + m0 + row];
#pragma unroll
        for (int u = 0; u < 8; ++u) ss += (i0 + u * TG < w.np) ? v[u] : 0.f;
      }
    }
    s_part[tid] = ss;
    __syncthreads();
    if (tid < ROWS) {
      float tot = 0.f;
#pragma unroll
      for (int j = 0; j < TG; ++j) tot += s_part[j * ROWS + tid];
      s_inv[tid] = 1.0f / sqrtf(tot / (float)p.d + p.eps);
    }
    // published by the barriers of the main loop
  }

  floatx4 acc[SW][MG];
#pragma unroll
  for (int s = 0; s < SW; ++s)
#pragma unroll
    for (int g = 0; g < MG; ++g) acc[s][g] = floatx4{0.f, 0.f, 0.f, 0.f};

  // activation tile: thread (wave, lane) stages lane slot `lane` of groups j * 4 + wave.  Loads go
  // through a buffer descriptor; slots of rows >= M get an out-of-range offset and read as zero.
  const int n_groups = (a.M + 7) >> 3;
  const __amdgpu_buffer_rsrc_t xr =
      __builtin_amdgcn_make_buffer_rsrc((void *)a.X, 0, n_groups * 16 * a.K * 2, 0x00020000);
  int boff[BL];
#pragma unroll
  for (int j = 0; j < BL; ++j) {
    const int grp = tm * MG + j * 4 + wave;
    boff[j] = (grp * 8 + (lane & 7) < a.M) ? (grp * KT * 64 + lane) * 16 : 0x40000000;
  }
  // weight tiles of this wavefront's strips (strips past the end repeat the last one; their
  // results are dropped)
  const u32x4 *wp[SW];
#pragma unroll
  for (int s = 0; s < SW; ++s) wp[s] = a.W + (size_t)min(strip0 + s, a.n_strips - 1) * KT * 64 + lane;

  constexpr int AD = 3;  // k-steps both operands are requested ahead
  u32x4 aR[AD + 1][SW], bR[AD + 1][BL];
  auto load_a = [&](u32x4 (&dst)[SW], int kt) {
#pragma unroll
    for (int s = 0; s < SW; ++s) dst[s] = wp[s][(size_t)kt * 64];
  };
  auto load_b = [&](u32x4 (&dst)[BL], int kt) {
#pragma unroll
    for (int j = 0; j < BL; ++j) dst[j] = __builtin_amdgcn_raw_buffer_load_b128(xr, boff[j] + kt * 1024, 0, 0);
  };
  auto store_b = [&](int buf, const u32x4 (&src)[BL]) {
#pragma unroll
    for (int j = 0; j < BL; ++j) sB[buf][j * 4 + wave][lane] = src[j];
  };
  auto compute = [&](const u32x4 (&av)[SW], int buf) {
    // four activation fragments in flight: the fragment of group g + 4 is requested from LDS as
    // soon as group g has been issued
    u32x4 b[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) b[g] = sB[buf][g][lane];
#pragma unroll
    for (int g = 0; g < MG; ++g) {
#pragma unroll
      for (int s = 0; s < SW; ++s)
        acc[s][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[s]),
                                                            __builtin_bit_cast(bf16x8, b[g & 3]), acc[s][g], 0, 0, 0);
      if (g + 4 < MG) b[g & 3] = sB[buf][g + 4][lane];
    }
    // the order above is the order wanted: left alone, the scheduler moves every LDS read down to
    // its first use to save registers, and the wavefront then waits out the LDS latency once per
    // group.  (0x100 = LDS read, 0x008 = MFMA.)
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int g = 0; g < MG; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, SW, 0);
      if (g + 4 < MG) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  };
  // k-step kt: request both operands of step kt+3 (indices past the end repeat the last step: in
  // bounds, never used), hand the activation tile of step kt+1 (requested two steps ago) over to
  // LDS buffer (kt+1) & 1, compute from buffer kt & 1.  Loads return in order, so a wait for any
  // request also waits for everything requested before it: every wait here is for requests at
  // least two steps old, and a step costs its MFMAs, not a trip to memory.  One barrier per step:
  // a buffer is rewritten only after the barrier that follows its last reader, and read only
  // after the barrier that follows its writers.
  auto step = [&](auto I, int kt) {
    constexpr int i = decltype(I)::value;
    load_b(bR[(i + AD) % (AD + 1)], min(kt + AD, KT - 1));
    load_a(aR[(i + AD) % (AD + 1)], min(kt + AD, KT - 1));
    // the requests leave before the step computes (left alone, the instruction scheduler sinks
    // them to the point of use and the step pays their whole latency), and no instruction moves
    // from one step into the next
    __builtin_amdgcn_sched_barrier(0);
    store_b((kt + 1) & 1, bR[(i + 1) % (AD + 1)]);
    compute(aR[i], kt & 1);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };
#pragma unroll
  for (int j = 0; j < AD; ++j) load_b(bR[j], min(j, KT - 1));
#pragma unroll
  for (int j = 0; j < AD; ++j) load_a(aR[j], min(j, KT - 1));
  store_b(0, bR[0]);
  __syncthreads();
  int kt = 0;
  for (; kt + AD < KT; kt += AD + 1) {
    step(ic<0>{}, kt);
    step(ic<1>{}, kt + 1);
    step(ic<2>{}, kt + 2);
    if constexpr (AD == 3) step(ic<3>{}, kt + 3);
  }
  if (kt < KT) {
    step(ic<0>{}, kt);
    if (kt + 1 < KT) step(ic<1>{}, kt + 1);
    if (AD == 3 && kt + 2 < KT) step(ic<2>{}, kt + 2);
  }

  // Epilogue.  After adding the lo columns to the hi columns, lane (ml < 8, g4) holds
  // Y[m0 + 8g + ml][16 strip + 4 g4 .. + 3].
  float ss_row[MG];  // RESID: this wavefront's sum of h^2 per row
#pragma unroll
  for (int g = 0; g < MG; ++g) {
    const int m = m0 + g * 8 + (ml & 7);
    const bool row_live = m < a.M && ml < 8;
    float inv = 1.f;
    if constexpr (NORM) inv = s_inv[g * 8 + (ml & 7)];
    float ss = 0.f;
    if constexpr (EPI == TILE_GATEUP) {
#pragma unroll
      for (int s = 0; s < SW; s += 2) {
        floatx4 yg = acc[s][g], yu = acc[s + 1][g];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          yg[r] += other_half(yg[r]);
          yu[r] += other_half(yu[r]);
        }
        if (row_live && strip0 + s + 1 < a.n_strips) {
          const int f0 = ((strip0 + s) >> 1) * 16 + 4 * g4;
          float tv[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float gt = yg[r] * inv, up = yu[r] * inv;
            tv[r] = gt / (1.0f + __expf(-gt)) * up;
          }
          store_split4(p.act_x, m, p.F, f0, tv);
        }
      }
    } else {
#pragma unroll
      for (int s = 0; s < SW; ++s) {
        floatx4 y = acc[s][g];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] += other_half(y[r]);
        const int strip = strip0 + s;
        const bool live = row_live && strip < a.n_strips;
        const int n = strip * 16 + 4 * g4;
        if constexpr (EPI == TILE_RESID) {
          if (live) {
            float *hp = p.h + (size_t)m * p.d + n;
            floatx4 hv = *(floatx4 *)hp + y;
            *(floatx4 *)hp = hv;
            float tv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              tv[r] = hv[r] * bf16_to_f32(a.gain_next[n + r]);
              ss += hv[r] * hv[r];
            }
            store_split4(p.xg, m, p.d, n, tv);
          }
        } else {  // TILE_QKV
          if (live) {
            const int which = n / p.D;        // 0 q, 1 k, 2 v
            const int c = n - which * p.D;    // column inside the projection
            const int head = c / p.hd, dim = c - head * p.hd;
            floatx4 v = y * inv;
            if (which < 2) {
              const int half = p.hd / 2;
              const float *cs = p.rope_cos + (size_t)m * half + dim / 2;
              const float *sn = p.rope_sin + (size_t)m * half + dim / 2;
              const float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
              v[0] = x0 * cs[0] - x1 * sn[0];
              v[1] = x0 * sn[0] + x1 * cs[0];
              v[2] = x2 * cs[1] - x3 * sn[1];
              v[3] = x2 * sn[1] + x3 * cs[1];
            }
            if (which == 0) {
              *(floatx4 *)(w.q + (size_t)m * p.D + c) = v;
            } else {
              // K rows [page][head][pos][dim], V pages transposed [page][head][dim][pos]; bf16 storage
              // (the eight rows of a group share a block: the index is uniform over the wavefront)
              const int sb = __builtin_amdgcn_readfirstlane(m / kPrefillBlockRows), sr = m % kPrefillBlockRows;
              if (sr >= a.segs.rows[sb]) continue;  // a padding row: nothing to cache
              const int pos = a.segs.pos[sb] + sr;
              const int page = p.block_table[(size_t)a.segs.slot[sb] * p.pages_per_seq + (pos >> p.page_shift)];
              const size_t hbase = ((size_t)a.layer * p.n_pages + page) * p.H + head;
              const int off = pos & (p.page_size - 1);
              if (which == 1) {
                uint2 pk;
                pk.x = pack2_bf16(v[0], v[1]);
                pk.y = pack2_bf16(v[2], v[3]);
                *(uint2 *)((uint16_t *)p.k_pool + (hbase * p.page_size + off) * p.hd + dim) = pk;
              } else {
                uint16_t *vp = (uint16_t *)p.v_pool + (hbase * p.hd + dim) * p.page_size + off;
#pragma unroll
                for (int r = 0; r < 4; ++r) vp[(size_t)r * p.page_size] = f32_to_bf16(v[r]);
              }
            }
          }
        }
      }
    }
    ss_row[g] = ss;
  }
  if constexpr (EPI == TILE_RESID) {
    // partial sum of h^2 over this wavefront's 16 * SW features, one per row: partial index =
    // wavefront strip group, rows past M get 0
    const int part = tn * 4 + wave;
    if (part < w.np) {
#pragma unroll
      for (int g = 0; g < MG; ++g) {
        float ss = ss_row[g];
        ss += __shfl_xor(ss, 16);
        ss += __shfl_xor(ss, 32);
        if (lane < 8) p.ssq[(size_t)part * w.rows + m0 + g * 8 + lane] = ss;
      }
    }
  }
}

template <int EPI>
void launch_tile(const Params &p, const PrefillWs &w, TileArgs a, int sw, hipStream_t s) {
  a.tiles_n = (a.n_strips + 4 * sw - 1) / (4 * sw);
  a.tiles_m = (a.M + 63) / 64;
  // a die (32 compute units, two workgroups each) holds 64 workgroups: a block of 8 x 8 tiles
  // re-reads the least per multiply-add (2048 features and 512 rows per die at a time)
  a.blk_n = w.blk_n ? w.blk_n : 8;
  a.blk_m = w.blk_m ? w.blk_m : 8;
  a.blocks_m = (a.tiles_m + a.blk_m - 1) / a.blk_m;
  a.n_blocks = a.blocks_m * ((a.tiles_n + a.blk_n - 1) / a.blk_n);
  const int grid = ((a.n_blocks + 7) / 8) * 8 * a.blk_n * a.blk_m;
  if constexpr (EPI != TILE_GATEUP) {  // (a gate/up wavefront needs a gate strip and its up strip)
    if (sw == 1) { gemm_tile_kernel<EPI, 8, 1><<<grid, 256, 0, s>>>(p, w, a); return; }
  }
  if (sw == 2) { gemm_tile_kernel<EPI, 8, 2><<<grid, 256, 0, s>>>(p, w, a); return; }
  gemm_tile_kernel<EPI, 8, kTileStrips><<<grid, 256, 0, s>>>(p, w, a);
}

// Strips per wavefront for a GEMM of n_strips strips on M rows: halved (down to `least`) until
// there are at least 384 tiles for the chip's 512 workgroup slots (measured on 7B shapes: 384 wide
// tiles beat 768 narrow ones, 256 do not beat 512).  Narrow tiles pull more operand bytes per
// multiply-add, but a pass with few rows is bound by how many workgroups walk K side by side.
int tile_strips(int n_strips, int M, int least) {
  int sw = kTileStrips;
  const int tiles_m = (M + 63) / 64;
  while (sw > least && tiles_m * ((n_strips + 4 * sw - 1) / (4 * sw)) < 384) sw >>= 1;
  return sw;
}

// ---------------------------------------------------------------------------------------------
// Causal attention of RG * 16 consecutive prompt rows of one head (bf16 cache, head_dim 128, V pages
// transposed).  Scores S^T[key][row] = K[key][:] . Q[row][:] with K rows as the MFMA A operand (key
// order inside the two 16-key tiles chosen so that a lane ends up with 8 consecutive keys) and 16
// query rows as the columns of the B operand; the probabilities of 8 consecutive keys feed
// O^T[dim][row] += V^T[dim][key] P[key][row] with one 16-byte load of the transposed V page as A
// operand.  Queries and probabilities keep fp32-like precision as (hi, lo) bf16 pairs; unlike the
// decode kernel, which puts the two halves of 8 rows side by side in the 16 columns, the halves go
// into separate MFMAs here: S = K q_hi + K q_lo accumulate into one score tile, the softmax runs
// once per (row, key) (side by side it runs in the hi and in the lo column, and that vector
// arithmetic, not the matrix cores, bounds the kernel), and P_hi, P_lo are two B operands that
// accumulate into one output tile.  A wavefront walks 32-key steps base = 32 * wave, + 128, ...
// with online softmax; wavefronts 1..3 leave (max, sum, accumulator) in LDS and wavefront 0 merges
// the four in wavefront order, normalises and stores the rows as (hi, lo) pairs for the Wo GEMM.
// ---------------------------------------------------------------------------------------------
template <int RG>  // groups of 16 rows per workgroup
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_prefill_kernel(Params p, PrefillWs w, int layer, int slot, int pos0,
                                                                                                       int R) {
  constexpr int HD = 128, RQ = 16 * RG;
  __shared__ float s_m[3][RQ], s_l[3][RQ];
  __shared__ float s_acc[3][RQ][HD];

  const int blk = gridDim.x - 1 - blockIdx.x;  // blocks with the most keys first
  const int head = blockIdx.y;
  const int r0 = blk * RQ;
  const int nr = min(RQ, R - r0);
  const int k_hi = pos0 + r0 + nr;  // keys 0 .. k_hi - 1 are visible to the block's last row

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ml = lane & 15, g = lane >> 4;
  const uint16_t *kpool = (const uint16_t *)p.k_pool, *vpool = (const uint16_t *)p.v_pool;

  // query fragments: column ml = row rg * 16 + ml, scaled by 1/sqrt(hd), as separate hi and lo operands
  u32x4 qh[RG][4], ql[RG][4];
  {
    const float scale = rsqrtf((float)HD);
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      const int rr = rg * 16 + ml;
      const bool live = rr < nr;
      const float *qp = w.q + (size_t)(r0 + (live ? rr : 0)) * p.D + head * HD + g * 8;
      floatx4 raw[4][2];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        raw[j][0] = *(const floatx4 *)(qp + j * 32);
        raw[j][1] = *(const floatx4 *)(qp + j * 32 + 4);
      }
      const float sc_q = live ? scale : 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          qh[rg][j][2 * h] = split2_bf16(raw[j][h][0] * sc_q, raw[j][h][1] * sc_q, true);
          qh[rg][j][2 * h + 1] = split2_bf16(raw[j][h][2] * sc_q, raw[j][h][3] * sc_q, true);
          ql[rg][j][2 * h] = split2_bf16(raw[j][h][0] * sc_q, raw[j][h][1] * sc_q, false);
          ql[rg][j][2 * h + 1] = split2_bf16(raw[j][h][2] * sc_q, raw[j][h][3] * sc_q, false);
        }
    }
  }

  floatx4 o[RG][8];
  float m_run[RG], l_run[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    m_run[rg] = -INFINITY;
    l_run[rg] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[rg][db] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  for (int base = wave * 32; base < k_hi; base += 128) {
    // one page holds the 32 keys (page_size is a multiple of 32); the lookup is wavefront-uniform
    const int page = p.block_table[(size_t)slot * p.pages_per_seq + (base >> p.page_shift)];
    const int poff = base & (p.page_size - 1);
    const size_t hbase = ((size_t)layer * p.n_pages + page) * p.H + head;
    const uint16_t *kp = kpool + (hbase * p.page_size + poff) * HD;   // K[key][dim]
    const uint16_t *vp = vpool + hbase * HD * p.page_size + poff;     // Vt[dim][key]
    u32x4 kt[2][4], vt[8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = (ml >> 2) * 8 + t * 4 + (ml & 3);  // key slot ml of tile t
#pragma unroll
      for (int j = 0; j < 4; ++j) kt[t][j] = *(const u32x4 *)(kp + (size_t)key * HD + j * 32 + g * 8);
    }
#pragma unroll
    for (int db = 0; db < 8; ++db) vt[db] = *(const u32x4 *)(vp + (size_t)(db * 16 + ml) * p.page_size + g * 8);
    __builtin_amdgcn_sched_barrier(0);  // all sixteen requests leave before anything is computed

#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      // a row group whose last row comes before this step's first key sees none of the step
      if (base > pos0 + r0 + rg * 16 + 15) continue;
      floatx4 sc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kt[t][j]),
                                                          __builtin_bit_cast(bf16x8, qh[rg][j]), sc[t], 0, 0, 0);
          sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kt[t][j]),
                                                          __builtin_bit_cast(bf16x8, ql[rg][j]), sc[t], 0, 0, 0);
        }
      }
      // lane (column ml, g) holds the scores of row rg * 16 + ml for keys base + 8g + 4t + r
      const int rr = rg * 16 + ml;
      float sv[8];
      float m_blk = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = base + 8 * g + 4 * t + r;
          const bool ok = (rr < nr) && (key <= pos0 + r0 + rr);
          const float v = ok ? sc[t][r] : -INFINITY;
          sv[4 * t + r] = v;
          m_blk = fmaxf(m_blk, v);
        }
      m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 16));
      m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
      const float m_new = fmaxf(m_run[rg], m_blk);
      const float alpha = (m_run[rg] == -INFINITY) ? 0.f : __expf(m_run[rg] - m_new);
      float pv[8], psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pv[i] = (sv[i] == -INFINITY) ? 0.f : __expf(sv[i] - m_new);
        psum += pv[i];
      }
      l_run[rg] = l_run[rg] * alpha + psum;
      m_run[rg] = m_new;
      u32x4 ph, pl;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ph[i] = pack2_bf16(pv[2 * i], pv[2 * i + 1]);
        pl[i] = pack2_bf16(pv[2 * i] - __uint_as_float(ph[i] << 16), pv[2 * i + 1] - __uint_as_float(ph[i] & 0xffff0000u));
      }
      // once the running maxima have settled alpha is 1 in every lane: skip the rescaling then
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int db = 0; db < 8; ++db) o[rg][db] *= alpha;
      }
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        o[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[db]),
                                                            __builtin_bit_cast(bf16x8, ph), o[rg][db], 0, 0, 0);
        o[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[db]),
                                                            __builtin_bit_cast(bf16x8, pl), o[rg][db], 0, 0, 0);
      }
    }
  }

  // a row's sum of probabilities is spread over the four g groups; lane (ml, g) holds dims
  // db * 16 + 4g + r of row rg * 16 + ml
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    l_run[rg] += __shfl_xor(l_run[rg], 16);
    l_run[rg] += __shfl_xor(l_run[rg], 32);
  }
  if (wave > 0) {
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      const int rr = rg * 16 + ml;
      if (g == 0) { s_m[wave - 1][rr] = m_run[rg]; s_l[wave - 1][rr] = l_run[rg]; }
#pragma unroll
      for (int db = 0; db < 8; ++db) *(floatx4 *)&s_acc[wave - 1][rr][db * 16 + 4 * g] = o[rg][db];
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      const int rr = rg * 16 + ml;
      if (rr >= nr) continue;
      float m_n = m_run[rg];
#pragma unroll
      for (int j = 0; j < 3; ++j) m_n = fmaxf(m_n, s_m[j][rr]);
      // row rr always sees key 0, so m_n is finite
      float f0 = (m_run[rg] == -INFINITY) ? 0.f : __expf(m_run[rg] - m_n);
      float l_n = l_run[rg] * f0;
      floatx4 acc[8];
#pragma unroll
      for (int db = 0; db < 8; ++db) acc[db] = o[rg][db] * f0;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float mj = s_m[j][rr];
        const float f = (mj == -INFINITY) ? 0.f : __expf(mj - m_n);
        l_n += s_l[j][rr] * f;
#pragma unroll
        for (int db = 0; db < 8; ++db) acc[db] += *(const floatx4 *)&s_acc[j][rr][db * 16 + 4 * g] * f;
      }
      const float inv_l = 1.0f / l_n;
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        const float tv[4] = {acc[db][0] * inv_l, acc[db][1] * inv_l, acc[db][2] * inv_l, acc[db][3] * inv_l};
        store_split4(p.attn_x, r0 + rr, p.D, head * HD + db * 16 + 4 * g, tv);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Long prompts: the same attention with the K/V tiles shared by the workgroup.  In the kernel above
// every block of 32 rows pulls all earlier keys through its compute unit's L1 on its own, and at
// thousands of rows that traffic out of L2 bounds it.  Here a workgroup owns 128 rows, 32 per
// wavefront; all four wavefronts walk the same 32-key steps, the step's K and V tiles (16 KB) are
// fetched once, by all wavefronts together (each fetches 2 of the 8 K fragments and 2 of the 8 V
// fragments, exactly as it would load them for itself), and laid down in LDS in fragment order, so
// that every wavefront reads a fragment as 1 KB of consecutive 16-byte words.  Requests run two
// steps ahead of their use (register ring, LDS double buffer, one barrier per step, as in
// gemm_tile_kernel).  A wavefront skips the steps past its own last row but keeps fetching and
// meeting the barriers.  No merge at the end: every wavefront owns its rows.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_prefill_shared_kernel(Params p, PrefillWs w, int layer, int slot,
                                                                                                            int pos0, int R) {
  constexpr int HD = 128, RG = 2, RW = 16 * RG, RQ = 4 * RW;  // 32 rows per wavefront, 128 per workgroup
  __shared__ u32x4 sK[2][8][64], sV[2][8][64];

  const int blk = gridDim.x - 1 - blockIdx.x;  // blocks with the most keys first
  const int head = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ml = lane & 15, g = lane >> 4;
  const int r0w = blk * RQ + wave * RW;        // first row of this wavefront
  const int nr = max(0, min(RW, R - r0w));     // its rows (0: the prompt ends before them)
  const int k_all = pos0 + min(R, blk * RQ + RQ);  // keys visible to the workgroup's last row
  const int k_own = pos0 + r0w + nr;               // keys visible to this wavefront's last row
  const uint16_t *kpool = (const uint16_t *)p.k_pool, *vpool = (const uint16_t *)p.v_pool;

  u32x4 qh[RG][4], ql[RG][4];
  {
    const float scale = rsqrtf((float)HD);
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      const int rr = rg * 16 + ml;
      const bool live = rr < nr;
      const float *qp = w.q + (size_t)(live ? r0w + rr : 0) * p.D + head * HD + g * 8;
      floatx4 raw[4][2];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        raw[j][0] = *(const floatx4 *)(qp + j * 32);
        raw[j][1] = *(const floatx4 *)(qp + j * 32 + 4);
      }
      const float sc_q = live ? scale : 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          qh[rg][j][2 * h] = split2_bf16(raw[j][h][0] * sc_q, raw[j][h][1] * sc_q, true);
          qh[rg][j][2 * h + 1] = split2_bf16(raw[j][h][2] * sc_q, raw[j][h][3] * sc_q, true);
          ql[rg][j][2 * h] = split2_bf16(raw[j][h][0] * sc_q, raw[j][h][1] * sc_q, false);
          ql[rg][j][2 * h + 1] = split2_bf16(raw[j][h][2] * sc_q, raw[j][h][3] * sc_q, false);
        }
    }
  }

  floatx4 o[RG][8];
  float m_run[RG], l_run[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    m_run[rg] = -INFINITY;
    l_run[rg] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) o[rg][db] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  const int n_steps = (k_all + 31) >> 5;
  // this wavefront's share of a step's tiles: K fragments 2 * wave, 2 * wave + 1 (fragment t * 4 + j:
  // 16 keys of tile t x dims j * 32 ..), V fragments of dim blocks 2 * wave, 2 * wave + 1
  u32x4 rK[3][2], rV[3][2];
  auto fetch = [&](u32x4 (&dk)[2], u32x4 (&dv)[2], int step) __attribute__((always_inline)) {
    const int base = step << 5;
    const int page = p.block_table[(size_t)slot * p.pages_per_seq + (base >> p.page_shift)];
    const int poff = base & (p.page_size - 1);
    const size_t hbase = ((size_t)layer * p.n_pages + page) * p.H + head;
    const uint16_t *kp = kpool + (hbase * p.page_size + poff) * HD;   // K[key][dim]
    const uint16_t *vp = vpool + hbase * HD * p.page_size + poff;     // Vt[dim][key]
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int f = wave * 2 + i, t = f >> 2, j = f & 3;
      const int key = (ml >> 2) * 8 + t * 4 + (ml & 3);  // key slot ml of tile t
      dk[i] = *(const u32x4 *)(kp + (size_t)key * HD + j * 32 + g * 8);
      dv[i] = *(const u32x4 *)(vp + (size_t)(f * 16 + ml) * p.page_size + g * 8);
    }
  };
  auto put = [&](int buf, const u32x4 (&dk)[2], const u32x4 (&dv)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      sK[buf][wave * 2 + i][lane] = dk[i];
      sV[buf][wave * 2 + i][lane] = dv[i];
    }
  };
  auto compute = [&](int buf, int base) __attribute__((always_inline)) {
    if (base >= k_own) return;  // past this wavefront's last row
    floatx4 sc[RG][2];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg)
#pragma unroll
      for (int t = 0; t < 2; ++t) sc[rg][t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32x4 kf = sK[buf][t * 4 + j][lane];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
          sc[rg][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf),
                                                              __builtin_bit_cast(bf16x8, qh[rg][j]), sc[rg][t], 0, 0, 0);
          sc[rg][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf),
                                                              __builtin_bit_cast(bf16x8, ql[rg][j]), sc[rg][t], 0, 0, 0);
        }
      }
    u32x4 ph[RG], pl[RG];
    float alpha[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      const int rr = rg * 16 + ml;
      float sv[8];
      float m_blk = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = base + 8 * g + 4 * t + r;
          const bool ok = (rr < nr) && (key <= pos0 + r0w + rr);
          const float v = ok ? sc[rg][t][r] : -INFINITY;
          sv[4 * t + r] = v;
          m_blk = fmaxf(m_blk, v);
        }
      m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 16));
      m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
      const float m_new = fmaxf(m_run[rg], m_blk);
      alpha[rg] = (m_run[rg] == -INFINITY) ? 0.f : __expf(m_run[rg] - m_new);
      float pv[8], psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pv[i] = (sv[i] == -INFINITY) ? 0.f : __expf(sv[i] - m_new);
        psum += pv[i];
      }
      l_run[rg] = l_run[rg] * alpha[rg] + psum;
      m_run[rg] = m_new;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ph[rg][i] = pack2_bf16(pv[2 * i], pv[2 * i + 1]);
        pl[rg][i] = pack2_bf16(pv[2 * i] - __uint_as_float(ph[rg][i] << 16),
                               pv[2 * i + 1] - __uint_as_float(ph[rg][i] & 0xffff0000u));
      }
      // once the running maxima have settled alpha is 1 in every lane: skip the rescaling then
      if (__builtin_amdgcn_ballot_w64(alpha[rg] != 1.0f) != 0) {
#pragma unroll
        for (int db = 0; db < 8; ++db) o[rg][db] *= alpha[rg];
      }
    }
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const u32x4 vf = sV[buf][db][lane];
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) {
        o[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                            __builtin_bit_cast(bf16x8, ph[rg]), o[rg][db], 0, 0, 0);
        o[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                            __builtin_bit_cast(bf16x8, pl[rg]), o[rg][db], 0, 0, 0);
      }
    }
  };
  // step s: request the tiles of step s+2 (past the end: the last step again, in bounds, unused),
  // lay the tiles of step s+1 (requested a step ago) down in LDS buffer (s+1) & 1, compute from
  // buffer s & 1.  A buffer is rewritten only after the barrier that follows its last reader.
  auto step = [&](auto I, int st) __attribute__((always_inline)) {
    constexpr int i = decltype(I)::value;
    fetch(rK[(i + 2) % 3], rV[(i + 2) % 3], min(st + 2, n_steps - 1));
    __builtin_amdgcn_sched_barrier(0);
    put((st + 1) & 1, rK[(i + 1) % 3], rV[(i + 1) % 3]);
    compute(st & 1, st << 5);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };
  fetch(rK[0], rV[0], 0);
  fetch(rK[1], rV[1], min(1, n_steps - 1));
  put(0, rK[0], rV[0]);
  __syncthreads();
  int st = 0;
  for (; st + 2 < n_steps; st += 3) {
    step(ic<0>{}, st);
    step(ic<1>{}, st + 1);
    step(ic<2>{}, st + 2);
  }
  if (st < n_steps) {
    step(ic<0>{}, st);
    if (st + 1 < n_steps) step(ic<1>{}, st + 1);
  }

  // lane (ml, g) holds dims db * 16 + 4g + r of row rg * 16 + ml; a row's sum of probabilities is
  // spread over the four g groups
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    const int rr = rg * 16 + ml;
    float l = l_run[rg];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (rr >= nr) continue;
    const float inv_l = 1.0f / l;  // every live row sees key 0
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const float tv[4] = {o[rg][db][0] * inv_l, o[rg][db][1] * inv_l, o[rg][db][2] * inv_l, o[rg][db][3] * inv_l};
      store_split4(p.attn_x, r0w + rr, p.D, head * HD + db * 16 + 4 * g, tv);
    }
  }
}

}  // namespace

// Strips per wavefront of the residual projections for a pass of M rows.  Fixes the number of
// partial sums of h^2 per row (one per wavefront strip group), which the producer of the rows
// must know.
int prefill_resid_strips(const Params &p, int M) { return tile_strips(p.d / 16, M, 1); }

void launch_prefill_qkv(const Params &p, const PrefillWs &w, const void *W, int layer, const PrefillSegs &segs, int M,
                        hipStream_t s) {
  TileArgs a{(const u32x4 *)W, p.xg, M, p.d, 3 * p.D / 16, layer, nullptr, segs, 0, 0, 0, 0, 0, 0};
  launch_tile<TILE_QKV>(p, w, a, w.resid_strips_opt ? w.resid_strips_opt : tile_strips(a.n_strips, M, 1), s);
}
void launch_prefill_resid(const Params &p, const PrefillWs &w, const void *W, const uint16_t *X, int K,
                          const void *gain_next, int M, hipStream_t s) {
  TileArgs a{(const u32x4 *)W, X, M, K, p.d / 16, 0, (const uint16_t *)gain_next, PrefillSegs{}, 0, 0, 0, 0, 0, 0};
  launch_tile<TILE_RESID>(p, w, a, w.resid_strips, s);
}
void launch_prefill_gateup(const Params &p, const PrefillWs &w, const void *W, int M, hipStream_t s) {
  TileArgs a{(const u32x4 *)W, p.xg, M, p.d, 2 * p.F / 16, 0, nullptr, PrefillSegs{}, 0, 0, 0, 0, 0, 0};
  launch_tile<TILE_GATEUP>(p, w, a, w.resid_strips_opt > 1 ? w.resid_strips_opt : tile_strips(a.n_strips, M, 2), s);
}
void launch_prefill_attention(const Params &p, const PrefillWs &w, int layer, int slot, int pos0, int R,
                              hipStream_t s) {
  // 128 rows per workgroup with shared K/V tiles once a pass is long enough for the traffic out of
  // L2 to matter (measured: equal at 512 rows, -4 % of the pass at 2048, -7 % at 4096)
  if (w.attn_rows == 128 || (w.attn_rows == 0 && R > 512)) {
    dim3 grid((R + 127) / 128, p.H);
    attn_prefill_shared_kernel<<<grid, 256, 0, s>>>(p, w, layer, slot, pos0, R);
  } else if (w.attn_rows == 16) {
    dim3 grid((R + 15) / 16, p.H);
    attn_prefill_kernel<1><<<grid, 256, 0, s>>>(p, w, layer, slot, pos0, R);
  } else {
    dim3 grid((R + 31) / 32, p.H);
    attn_prefill_kernel<2><<<grid, 256, 0, s>>>(p, w, layer, slot, pos0, R);
  }
}

// Row assembly of a tiled pass that carries rows of several sequences (see PrefillSegs): h (fp32), (hi, lo) of
// h * gain of the first norm, partial sums of h^2 (partial 0 carries the whole row), rotary table at the row's
// own position.  Padding rows are assembled like any other (their token is whatever `p.prefill_ids` holds for
// them, position 0): rows are independent, and nothing of a padding row is ever cached or read.
__global__ __launch_bounds__(256) void assemble_prefill_segs_kernel(Params p, const uint16_t *tok_emb, const uint16_t *gain0,
                                                                    PrefillSegs segs, int ssq_parts, int ssq_stride) {
  __shared__ float red[4];
  const int m = blockIdx.x, sb = m / kPrefillBlockRows, sr = m % kPrefillBlockRows;
  const int pos = sr < segs.rows[sb] ? segs.pos[sb] + sr : 0;
  const uint16_t *src = tok_emb + (size_t)clamp_token(p, p.prefill_ids[m]) * p.d;
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
    const float x0[4] = {x[0], x[1], x[2], x[3]}, x1[4] = {x[4], x[5], x[6], x[7]};
    store_split4(p.xg, m, p.d, c0, x0);
    store_split4(p.xg, m, p.d, c0 + 4, x1);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  for (int i = threadIdx.x; i < ssq_parts; i += 256)
    p.ssq[(size_t)i * ssq_stride + m] = (i == 0) ? (red[0] + red[1] + red[2] + red[3]) : 0.f;
  const int half = p.hd / 2;
  for (int i = threadIdx.x; i < half; i += 256) {
    double sn, cs;
    sincos((double)pos * p.rope_theta[i], &sn, &cs);
    p.rope_cos[(size_t)m * half + i] = (float)cs;
    p.rope_sin[(size_t)m * half + i] = (float)sn;
  }
}

void launch_assemble_prefill_segs(const Params &p, const void *tok_emb, const void *gain0, const PrefillSegs &segs, int M,
                                  int ssq_parts, int ssq_stride, hipStream_t s) {
  assemble_prefill_segs_kernel<<<M, 256, 0, s>>>(p, (const uint16_t *)tok_emb, (const uint16_t *)gain0, segs, ssq_parts, ssq_stride);
}

}  // namespace pass
