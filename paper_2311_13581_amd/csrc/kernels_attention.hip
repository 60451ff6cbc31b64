// Split-KV decode attention for the (1+k)-row block over the paged K/V cache.
//
// A call carries R rows per slot at consecutive positions; row r attends to cached positions
// 0 .. pos0 + r, which includes the K/V its own call wrote (causal inside the new block).  Every
// K/V byte is read once for all rows of a group: that is the premise of the method (Section 2.2:
// a few extra tokens cost about as much as one because decoding is bound by memory traffic).
//
// Two split kernels, one merge kernel.  The matrix-core kernel (bf16 cache, head_dim 128, V pages
// transposed; described at its definition) carries the benchmarked configurations; the
// lane-per-key kernel below carries fp32 caches, head_dim 64 and odd page sizes.
//
// Grid: (split, head, group).  A group is up to 8 consecutive rows of one slot.  Within the
// workgroup (4 wavefronts) of the lane-per-key kernel 16 lanes share one key: each lane holds hd/16 dimensions, so a key or
// value row is fetched as 16 adjacent 16-byte loads.  An iteration covers 64 keys: every 16-lane
// group requests the K and V chunks of 4 keys before it computes on any of them.  The 16-lane dot
// product is reduced with DPP row operations (no LDS traffic).  The 16 lane groups merge their
// (max, sum, accumulator) triples through LDS; the workgroup writes its split's triple to a
// workspace and a second, tiny kernel merges the splits.
#include "pass_internal.h"

namespace pass {

// How a row group's keys are cut into splits.  A function of the group's own key count only, so
// that a sequence's arithmetic (and therefore its tokens) cannot depend on what else is batched.
__device__ __forceinline__ void split_plan(int n_keys, int &n_splits, int &chunk) {
  n_splits = min(kMaxSplits, (n_keys + 63) / 64);
  chunk = ((n_keys + n_splits - 1) / n_splits + 15) & ~15;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a DPP row; every lane of the row ends with the total
__device__ __forceinline__ float row_sum16(float v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror
  v += dpp_move<0x140>(v);  // row_mirror
  return v;
}

template <int DPL>
__device__ __forceinline__ void unpack_chunk(const float4 (&raw)[DPL / 4], float (&o)[DPL], const float *) {
#pragma unroll
  for (int i = 0; i < DPL / 4; ++i) { o[4 * i] = raw[i].x; o[4 * i + 1] = raw[i].y; o[4 * i + 2] = raw[i].z; o[4 * i + 3] = raw[i].w; }
}
template <int DPL>
__device__ __forceinline__ void unpack_chunk(const uint32_t (&raw)[DPL / 2], float (&o)[DPL], const bf16_t *) {
#pragma unroll
  for (int i = 0; i < DPL / 2; ++i) { o[2 * i] = __uint_as_float(raw[i] << 16); o[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u); }
}
template <int DPL>
__device__ __forceinline__ void load_raw(const float *p, float4 (&raw)[DPL / 4]) {
#pragma unroll
  for (int i = 0; i < DPL / 4; ++i) raw[i] = *(const float4 *)(p + 4 * i);
}
template <int DPL>
__device__ __forceinline__ void load_raw(const bf16_t *p, uint32_t (&raw)[DPL / 2]) {
  if constexpr (DPL == 8) {
    uint4 v = *(const uint4 *)p;
    raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
  } else {
    uint2 v = *(const uint2 *)p;
    raw[0] = v.x; raw[1] = v.y;
  }
}
template <typename T, int DPL> struct RawChunk;
template <int DPL> struct RawChunk<float, DPL> { float4 v[DPL / 4]; };
template <int DPL> struct RawChunk<bf16_t, DPL> { uint32_t v[DPL / 2]; };

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_split_kernel(Params p, int layer, int R) {
  constexpr int DPL = HD / 16;
  constexpr int RQ = kAttnRowsPerGroup;
  constexpr int KU = 4;    // keys per 16-lane group and iteration
  constexpr int NG = 16;   // 16-lane groups per workgroup
  __shared__ float s_m[NG][RQ], s_l[NG][RQ];
  __shared__ float s_acc[NG][RQ][HD];

  const int split = blockIdx.x, head = blockIdx.y, g = blockIdx.z;
  const int groups_per_slot = (R + RQ - 1) / RQ;
  const int b = g / groups_per_slot;
  const int r0 = (g % groups_per_slot) * RQ;
  const int nr = min(RQ, R - r0);
  const int slot = p.row_slot[b * R + r0];
  if (slot < 0) return;  // dead rows (beyond the slot's capacity): the merge kernel writes zeros
  const int pos0 = p.row_pos[b * R + r0];  // position of the group's first row
  const int n_keys = pos0 + nr;
  int n_splits, chunk;
  split_plan(n_keys, n_splits, chunk);
  if (split >= n_splits) return;
  const int k_lo = split * chunk;
  const int k_hi = min(n_keys, k_lo + chunk);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane >> 4, dl = lane & 15;
  const int grp = wave * 4 + sub;
  const T *kpool = (const T *)p.k_pool, *vpool = (const T *)p.v_pool;
  const float scale = rsqrtf((float)HD);

  float q[RQ][DPL], acc[RQ][DPL], mx[RQ], ls[RQ];
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    mx[r] = -INFINITY;
    ls[r] = 0.f;
#pragma unroll
    for (int i = 0; i < DPL; ++i) {
      acc[r][i] = 0.f;
      q[r][i] = 0.f;
    }
    if (r < nr) {
      const float *qp = p.qkv + (size_t)(b * R + r0 + r) * 3 * p.D + head * HD + dl * DPL;
#pragma unroll
      for (int i = 0; i < DPL; ++i) q[r][i] = qp[i] * scale;
    }
  }

  for (int base = k_lo; base < k_hi; base += NG * KU) {
    // request everything this iteration needs; keys past the range re-read the range's first key
    RawChunk<T, DPL> kraw[KU], vraw[KU];
    int key[KU];
#pragma unroll
    for (int j = 0; j < KU; ++j) {
      key[j] = base + j * NG + grp;
      const int kk = key[j] < k_hi ? key[j] : k_lo;
      const size_t off = kv_offset(p, layer, slot, kk, head) + dl * DPL;
      load_raw<DPL>(kpool + off, kraw[j].v);
      load_raw<DPL>(vpool + off, vraw[j].v);
    }
#pragma unroll
    for (int j = 0; j < KU; ++j) {
      const bool valid = key[j] < k_hi;
      float kf[DPL], vf[DPL];
      unpack_chunk<DPL>(kraw[j].v, kf, (const T *)nullptr);
      unpack_chunk<DPL>(vraw[j].v, vf, (const T *)nullptr);
#pragma unroll
      for (int r = 0; r < RQ; ++r) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < DPL; ++i) s = fmaf(q[r][i], kf[i], s);
        s = row_sum16(s);
        const bool ok = valid && (r < nr) && (key[j] <= pos0 + r);
        if (ok) {
          float m_new = fmaxf(mx[r], s);
          float alpha = (mx[r] == -INFINITY) ? 0.f : __expf(mx[r] - m_new);
          float pw = __expf(s - m_new);
          ls[r] = ls[r] * alpha + pw;
#pragma unroll
          for (int i = 0; i < DPL; ++i) acc[r][i] = acc[r][i] * alpha + pw * vf[i];
          mx[r] = m_new;
        }
      }
    }
  }

  // merge the 16 lane groups through LDS
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    if (dl == 0) { s_m[grp][r] = mx[r]; s_l[grp][r] = ls[r]; }
#pragma unroll
    for (int i = 0; i < DPL; ++i) s_acc[grp][r][dl * DPL + i] = acc[r][i];
  }
  __syncthreads();
  const size_t pbase = ((size_t)(b * R + r0) * p.H + head) * kMaxSplits;  // row r: + r * H * kMaxSplits
  for (int e = threadIdx.x; e < nr * HD; e += 256) {
    int r = e / HD, dim = e % HD;
    float m_n = -INFINITY;
#pragma unroll
    for (int w = 0; w < NG; ++w) m_n = fmaxf(m_n, s_m[w][r]);
    float l_n = 0.f, v = 0.f;
#pragma unroll
    for (int w = 0; w < NG; ++w) {
      float f = (s_m[w][r] == -INFINITY) ? 0.f : __expf(s_m[w][r] - m_n);
      l_n += s_l[w][r] * f;
      v += s_acc[w][r][dim] * f;
    }
    size_t pi = pbase + (size_t)r * p.H * kMaxSplits + split;
    p.part_acc[pi * HD + dim] = v;
    if (dim == 0) { p.part_m[pi] = m_n; p.part_l[pi] = l_n; }
  }
}

// ---------------------------------------------------------------------------------------------
// Matrix-core variant for bf16 caches with head_dim 128 and V stored transposed
// ([page][head][dim][page_size], page_size a multiple of 32).
//
// A wavefront owns 32 consecutive keys per step.  Scores: S^T[key][col] = K[key][:] . Q[col][:]
// with the K rows as the MFMA A operand (two 16-key tiles x four 32-dim blocks) and the queries as
// B operand; columns 0..7 carry the hi halves of the (scaled) query rows, columns 8..15 the lo
// halves (q = hi + lo, both bf16), so the sum of the two column halves is the fp32-accurate score.
// The key order inside the two tiles is chosen so that a lane ends up with the scores of 8
// consecutive keys -- exactly the 8 key slots it feeds, as probabilities (again hi / lo halves by
// column), into the second MFMA O^T[dim][col] += V^T[dim][key] P[key][col], whose A operand is
// eight consecutive keys of one dimension: one 16-byte load from the transposed V page.
// Online softmax keeps one running maximum per query row, shared by the lanes of a wavefront.
// ---------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void attn_split_mfma_kernel(Params p, int layer, int R) {
  constexpr int HD = 128, RQ = kAttnRowsPerGroup;
  __shared__ float s_m[4][RQ], s_l[4][RQ];
  __shared__ float s_acc[4][RQ][HD];

  const int split = blockIdx.x, head = blockIdx.y, grp_id = blockIdx.z;
  const int groups_per_slot = (R + RQ - 1) / RQ;
  const int b = grp_id / groups_per_slot;
  const int r0 = (grp_id % groups_per_slot) * RQ;
  const int nr = min(RQ, R - r0);
  const int m0 = b * R + r0;
  // Requests that depend on each other come in three rounds and no more: (slot, position), then
  // (page of the first step, query rows), then the first step's K and V.  The slot takes part in the
  // first branch only so that the compiler requests it together with the position instead of after
  // that branch.
  const int slot = p.row_slot[m0];
  const int pos0 = p.row_pos[m0];
  const int n_keys = pos0 + nr;
  int n_splits, chunk;
  split_plan_mfma(n_keys, p.H, n_splits, chunk);
  if (slot < 0 || split >= n_splits) return;
  const int k_lo = split * chunk;
  const int k_hi = min(n_keys, k_lo + chunk);

  // the wavefront index as a scalar: the page lookup below then is a scalar load
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ml = lane & 15, g = lane >> 4;
  const int row = ml & 7;  // query row of this lane's column (both column halves)
  const uint16_t *kpool = (const uint16_t *)p.k_pool, *vpool = (const uint16_t *)p.v_pool;

  u32x4_t kt[2][4], vt[8];
  // requests the K tiles and V rows of the 32 keys from `at` on (one page holds them: page_size is a
  // multiple of 32; the lookup is wavefront-uniform)
  auto request = [&](int at) __attribute__((always_inline)) {
    const int page = p.block_table[(size_t)slot * p.pages_per_seq + (at >> p.page_shift)];
    const int poff = at & (p.page_size - 1);
    const size_t hbase = ((size_t)layer * p.n_pages + page) * p.H + head;
    const uint16_t *kp = kpool + (hbase * p.page_size + poff) * HD;   // K[key][dim]
    const uint16_t *vp = vpool + hbase * HD * p.page_size + poff;     // Vt[dim][key]
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = (ml >> 2) * 8 + t * 4 + (ml & 3);  // key slot ml of tile t
#pragma unroll
      for (int j = 0; j < 4; ++j) kt[t][j] = *(const u32x4_t *)(kp + (size_t)key * HD + j * 32 + g * 8);
    }
#pragma unroll
    for (int db = 0; db < 8; ++db) vt[db] = *(const u32x4_t *)(vp + (size_t)(db * 16 + ml) * p.page_size + g * 8);
  };

  // query fragment: column ml = hi (ml < 8) or lo (ml >= 8) half of row (ml & 7), scaled by 1/sqrt(hd)
  u32x4_t qf[4];
  int base = k_lo + wave * 32;
  {
    const float scale = rsqrtf((float)HD);
    const bool live = row < nr;
    const float *qp = p.qkv + (size_t)(m0 + (live ? row : 0)) * 3 * p.D + head * HD + g * 8;
    // all eight 16-byte loads are issued before any is used (rows that do not exist read row 0
    // and are zeroed afterwards: a load under a condition would be waited for on the spot)
    f32x4_t raw[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      raw[j][0] = *(const f32x4_t *)(qp + j * 32);
      raw[j][1] = *(const f32x4_t *)(qp + j * 32 + 4);
    }
    // the first step's K and V leave before the query rows are waited for (a wavefront without keys
    // in this split asks for the split's first keys, which exist, and skips the loop)
    request(base < k_hi ? base : k_lo);
    __builtin_amdgcn_sched_barrier(0);
    const float sc_q = live ? scale : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        qf[j][2 * h] = split2_bf16(raw[j][h][0] * sc_q, raw[j][h][1] * sc_q, ml < 8);
        qf[j][2 * h + 1] = split2_bf16(raw[j][h][2] * sc_q, raw[j][h][3] * sc_q, ml < 8);
      }
  }

  f32x4_t o[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  for (; base < k_hi; base += 128) {
    // (the step's sixteen requests are in flight: those of the first step since before the loop,
    // those of a later step since the end of the step before it)
    f32x4_t sc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      sc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kt[t][j]),
                                                        __builtin_bit_cast(bf16x8_t, qf[j]), sc[t], 0, 0, 0);
    }
    // lane (column ml, g) now holds the scores of keys base + 8g + 4t + r; add the lo-half column
    float s[8];
    float m_blk = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = sc[t][r];
        v += dpp_move<0x128>(v);  // row_ror 8: column ml <-> ml + 8
        const int key = base + 8 * g + 4 * t + r;
        const bool ok = (row < nr) && (key < k_hi) && (key <= pos0 + row);
        v = ok ? v : -INFINITY;
        s[4 * t + r] = v;
        m_blk = fmaxf(m_blk, v);
      }
    m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 16));
    m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
    const float m_new = fmaxf(m_run, m_blk);
    const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
    float pv[8], psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = (s[i] == -INFINITY) ? 0.f : __expf(s[i] - m_new);
      psum += pv[i];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    const u32x4_t pf = {split2_bf16(pv[0], pv[1], ml < 8), split2_bf16(pv[2], pv[3], ml < 8),
                        split2_bf16(pv[4], pv[5], ml < 8), split2_bf16(pv[6], pv[7], ml < 8)};
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      o[db] *= alpha;
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vt[db]),
                                                      __builtin_bit_cast(bf16x8_t, pf), o[db], 0, 0, 0);
    }
    if (base + 128 < k_hi) {
      request(base + 128);
      // all sixteen requests leave before anything is computed: left alone, the instruction
      // scheduler moves the V requests behind the score MFMAs to save registers, and the step
      // pays two trips to memory in a row
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // a row's sum of probabilities is spread over the four g groups
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  // hi + lo column halves; lane (ml < 8, g) then holds dims db*16 + 4g + r of row ml
#pragma unroll
  for (int db = 0; db < 8; ++db)
#pragma unroll
    for (int r = 0; r < 4; ++r) o[db][r] += dpp_move<0x128>(o[db][r]);
  if (ml < 8) {
    if (g == 0) { s_m[wave][ml] = m_run; s_l[wave][ml] = l_run; }
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int r = 0; r < 4; ++r) s_acc[wave][ml][db * 16 + 4 * g + r] = o[db][r];
  }
  __syncthreads();
  const size_t pbase = ((size_t)m0 * p.H + head) * kMaxSplits;
  for (int e = threadIdx.x; e < nr * HD; e += 256) {
    int r = e / HD, dim = e % HD;
    float m_n = fmaxf(fmaxf(s_m[0][r], s_m[1][r]), fmaxf(s_m[2][r], s_m[3][r]));
    float l_n = 0.f, v = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float f = (s_m[w][r] == -INFINITY) ? 0.f : __expf(s_m[w][r] - m_n);
      l_n += s_l[w][r] * f;
      v += s_acc[w][r][dim] * f;
    }
    size_t pi = pbase + (size_t)r * p.H * kMaxSplits + split;
    p.part_acc[pi * HD + dim] = v;
    if (dim == 0) { p.part_m[pi] = m_n; p.part_l[pi] = l_n; }
  }
}

// Merge the split partials of one (row, head): out = sum_s acc_s e^{m_s - m} / sum_s l_s e^{m_s - m}.
// A kernel of its own: handing partials between workgroups inside one kernel needs device-scope
// fences, which on this multi-die part write back and invalidate the per-die L2s and cost far more
// than a launch.
// Q = 1: HD threads, one per dimension, walk all splits.  Q = 4 (more than 8 splits): 4 * HD
// threads, quarter q takes splits 8q .. 8q+7 (one batch of requests each), the quarters' triples
// are merged through LDS in quarter order.  Both give the same bits for up to 8 splits.
template <int HD, int OUT, int Q>
__global__ __launch_bounds__(HD * Q) void attn_combine_kernel(Params p, int R, int mfma_plan) {
  __shared__ float sm[Q], sl[Q], sv[Q][HD];
  const int m = blockIdx.x, head = blockIdx.y, dim = threadIdx.x % HD, q = threadIdx.x / HD;
  // One batch of eight splits per thread, requested before the plan is known so that the lookup of the
  // row's position and the partials share one round trip to memory: slots 0 .. kMaxSplits - 1 of a
  // (row, head) always exist, those beyond the plan hold stale values that are never used.
  static_assert(Q * 8 <= kMaxSplits, "a quarter's eight slots must exist");
  constexpr int RQ = kAttnRowsPerGroup;
  const int b = m / R, r = m % R, r0 = (r / RQ) * RQ;
  const int pos0 = p.row_pos[b * R + r0];  // position of the group's first row
  const bool dead = p.row_slot[m] < 0;     // no split kernel ran for this row: its output is zero
  const size_t pi = ((size_t)m * p.H + head) * kMaxSplits;
  const int s_begin = (Q == 1) ? 0 : q * 8;
  float pm[8], pl[8], pa[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    pm[u] = p.part_m[pi + s_begin + u];
    pl[u] = p.part_l[pi + s_begin + u];
    pa[u] = p.part_acc[(pi + s_begin + u) * HD + dim];
  }
  // the split plan of the row's group, recomputed exactly as the split kernel did
  const int n_keys = pos0 + min(RQ, R - r0);
  int n_splits, chunk;
  if (mfma_plan)
    split_plan_mfma(n_keys, p.H, n_splits, chunk);
  else
    split_plan(n_keys, n_splits, chunk);
  const int s_end = min(n_splits, s_begin + 8);
  // merged in split order
  float m_n = -INFINITY, l_n = 0.f, v = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (s_begin + u < s_end) m_n = fmaxf(m_n, pm[u]);
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (s_begin + u < s_end) {
      const float f = (pm[u] == -INFINITY) ? 0.f : __expf(pm[u] - m_n);
      l_n += pl[u] * f;
      v += pa[u] * f;
    }
  if constexpr (Q > 1) {
    if (dim == 0) { sm[q] = m_n; sl[q] = l_n; }
    sv[q][dim] = v;
    __syncthreads();
    if (q != 0) return;
    float m_all = sm[0];
#pragma unroll
    for (int i = 1; i < Q; ++i) m_all = fmaxf(m_all, sm[i]);
    l_n = 0.f;
    v = 0.f;
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const float f = (sm[i] == -INFINITY) ? 0.f : __expf(sm[i] - m_all);
      l_n += sl[i] * f;
      v += sv[i][dim] * f;
    }
    m_n = m_all;
  }
  if (p.lse != nullptr && dim == 0) p.lse[(size_t)m * p.H + head] = dead ? 0.f : m_n + logf(l_n);
  float o = dead ? 0.f : v / l_n;
  if (OUT == 1) {
    // (hi, lo) pair in the tiled activation layout of the matrix-core GEMMs
    uint16_t hi = f32_to_bf16(o);
    size_t xi = xs_index(m, p.D, head * HD + dim);
    p.attn_x[xi] = hi;
    p.attn_x[xi + kXsLoOffset] = f32_to_bf16(o - bf16_to_f32(hi));
  } else {
    p.attn[(size_t)m * p.D + head * HD + dim] = o;
  }
}

template <int HD>
static void launch_combine(const Params &p, dim3 cgrid, int R, int n_splits, int out_split, int mfma_plan,
                           hipStream_t s) {
  if (n_splits > 8) {
    if (out_split)
      attn_combine_kernel<HD, 1, 4><<<cgrid, HD * 4, 0, s>>>(p, R, mfma_plan);
    else
      attn_combine_kernel<HD, 0, 4><<<cgrid, HD * 4, 0, s>>>(p, R, mfma_plan);
  } else {
    if (out_split)
      attn_combine_kernel<HD, 1, 1><<<cgrid, HD, 0, s>>>(p, R, mfma_plan);
    else
      attn_combine_kernel<HD, 0, 1><<<cgrid, HD, 0, s>>>(p, R, mfma_plan);
  }
}

void launch_attention(const Params &p, int dtype, int layer, int B, int R, int n_splits, int out_split,
                      hipStream_t s) {
  int groups = B * ((R + kAttnRowsPerGroup - 1) / kAttnRowsPerGroup);
  dim3 grid(n_splits, p.H, groups), cgrid(B * R, p.H);
  if (p.v_transposed) {  // bf16, head_dim 128, page_size % 32 == 0: matrix-core kernel
    attn_split_mfma_kernel<<<grid, 256, 0, s>>>(p, layer, R);
    launch_combine<128>(p, cgrid, R, n_splits, out_split, 1, s);
    return;
  }
  if (p.hd == 128) {
    if (dtype == PASS_F32)
      attn_split_kernel<float, 128><<<grid, 256, 0, s>>>(p, layer, R);
    else
      attn_split_kernel<bf16_t, 128><<<grid, 256, 0, s>>>(p, layer, R);
    launch_combine<128>(p, cgrid, R, n_splits, out_split, 0, s);
  } else {
    if (dtype == PASS_F32)
      attn_split_kernel<float, 64><<<grid, 256, 0, s>>>(p, layer, R);
    else
      attn_split_kernel<bf16_t, 64><<<grid, 256, 0, s>>>(p, layer, R);
    launch_combine<64>(p, cgrid, R, n_splits, out_split, 0, s);
  }
}

}  // namespace pass
