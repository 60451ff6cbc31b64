// Sampling epilogues of the two model calls of Algorithm 1, on fp32 logits.
//
// Drafting call: row 0 gives x_{n+1} (an ordinary sample, not part of the draft), row t gives
// draft t; the rows' ln-sum-exp is kept so that the validation call can evaluate d_t(x).
// Validation call: accept draft t iff  ln r_t + ln d_t(x) < ln p_t(x)  (r < min(1, p/d)), in
// order; the first reject is replaced by a draw from the normalised (p_t - d_t)_+; if all k are
// accepted one more token is drawn from the last row.  Then kv_len += 1 + a: rows of rejected
// drafts stay in the cache as dead entries.
//
// Every "draw" is a Gumbel-max: argmax_j (score_j - ln(-ln u_j)), u_j from Philox4x32-10 with
// key = seed and counter = (j/4, iteration, row | purpose << 8, sequence id); an argmax is
// independent of reduction order, so wavefront reductions give the same winner as a serial loop.
// Ties go to the lowest index.  temperature == 0 is greedy (argmax of the logits).
//
// Top-k sampling (the paper's sampler, Experimental setup: k = 10, and 25 for pass@10): the draft
// and the target distribution are each the softmax over the row's own K largest logits, zero
// elsewhere; ties at the boundary keep the lower indices.  A row's filter is two numbers found by
// a radix select over order-preserving integer keys: the key of the K-th largest logit and the
// highest index that may still be kept among the logits equal to it.  Entries outside the filter
// are skipped by every scan (ln-sum-exp, draws, residual) and have probability zero in the accept
// test.  K = 0 is no filter (key 0, every index allowed).
#include "pass_internal.h"

namespace pass {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    // one 32 x 32 -> 64 bit multiply per product (v_mad_u64_u32) instead of a high and a low one
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// top 23 bits -> (bits + 0.5) * 2^-23, in (0,1), exact in fp32
__device__ __forceinline__ float u01(uint32_t x) { return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f); }
// The per-element transcendentals use the hardware exp2 / log2 (absolute error around 1e-6 on
// the scores in play), inside the fp32 margin the decision comparison allows; the ln-sum-exp
// totals, the accept test and the merges of partial sums, a handful of values per row, stay precise.
__device__ __forceinline__ float gumbel(float u) { return -__logf(-__logf(u)); }

struct Best {
  float s;
  int idx;
};
__device__ __forceinline__ Best better(Best a, Best b) {
  // larger score wins; equal scores: lower index; idx < 0 means "no candidate"
  if (b.idx < 0) return a;
  if (a.idx < 0) return b;
  if (b.s > a.s || (b.s == a.s && b.idx < a.idx)) return b;
  return a;
}
__device__ __forceinline__ Best wave_best(Best v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Best t;
    t.s = __shfl_xor(v.s, o);
    t.idx = __shfl_xor(v.idx, o);
    v = better(v, t);
  }
  return v;
}

struct MaxSum {
  float m, s;  // running max and sum of exp(a - m)
};
__device__ __forceinline__ MaxSum ms_merge(MaxSum a, MaxSum b) {
  if (b.m == -INFINITY) return a;
  if (a.m == -INFINITY) return b;
  MaxSum r;
  r.m = fmaxf(a.m, b.m);
  r.s = a.s * expf(a.m - r.m) + b.s * expf(b.m - r.m);
  return r;
}
__device__ __forceinline__ MaxSum wave_ms(MaxSum v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    MaxSum t;
    t.m = __shfl_xor(v.m, o);
    t.s = __shfl_xor(v.s, o);
    v = ms_merge(v, t);
  }
  return v;
}

constexpr int kEpiThreads = 1024;
constexpr int kEpiWaves = kEpiThreads / 64;

__device__ Best block_best(Best v, Best *sh) {
  v = wave_best(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  Best r = sh[0];
  for (int w = 1; w < kEpiWaves; ++w) r = better(r, sh[w]);
  return r;
}
__device__ MaxSum block_ms(MaxSum v, MaxSum *sh) {
  v = wave_ms(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  MaxSum r = sh[0];
  for (int w = 1; w < kEpiWaves; ++w) r = ms_merge(r, sh[w]);
  return r;
}

// Walk NR logits rows of V entries in groups of four consecutive entries ("quads", the unit one
// Philox call covers): f(quad index, values[NR][4], number of valid entries).  A thread takes
// quads threadIdx.x, + kEpiThreads, ... in ascending order.  When V is a multiple of 4 a quad is
// one 16-byte load and the loads of four quads are issued before the first is used (indices
// clamped, results of quads that do not exist dropped): a load under a condition would be
// waited for on the spot, and a row is only V / (4 * kEpiThreads) quads deep per thread.
template <int NR, typename F>
__device__ __forceinline__ void scan_rows(const float *const (&rows)[NR], int V, F &&f) {
  if ((V & 3) == 0) {
    constexpr int U = 4;
    const int V4 = V >> 2;
    for (int q0 = threadIdx.x; q0 < V4; q0 += U * kEpiThreads) {
      float4 v[U][NR];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < NR; ++r) v[u][r] = ((const float4 *)rows[r])[min(q0 + u * kEpiThreads, V4 - 1)];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = q0 + u * kEpiThreads;
        if (q < V4) {
          float x[NR][4];
#pragma unroll
          for (int r = 0; r < NR; ++r) { x[r][0] = v[u][r].x; x[r][1] = v[u][r].y; x[r][2] = v[u][r].z; x[r][3] = v[u][r].w; }
          f(q, x, 4);
        }
      }
    }
  } else {
    for (int q = threadIdx.x; q * 4 < V; q += kEpiThreads) {
      const int n = min(4, V - q * 4);
      float x[NR][4];
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[r][e] = rows[r][q * 4 + min(e, n - 1)];
      f(q, x, n);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// top-k filter
// ---------------------------------------------------------------------------------------------
// order-preserving key of a logit: a > b  <=>  key(a) > key(b); -0 and +0 share a key
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
struct RowFilter {
  uint32_t key;  // key of the K-th largest logit (0: keep everything)
  int tie_max;   // highest index kept among the logits whose key equals `key`
};
__device__ __forceinline__ bool kept(const RowFilter &f, float l, int j) {
  uint32_t k = order_key(l);
  return k > f.key || (k == f.key && j <= f.tie_max);
}

constexpr int kSelBins = 2048;  // 11 + 11 + 10 bits
struct SelectShared {
  int hist[kSelBins];
  int wave_tot[kEpiWaves];
  int bin, rank;
};

// Exclusive prefix sum over the threads of the workgroup, in thread order.
__device__ int block_exclusive_scan(int v, int *wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int off = 0;
  for (int w = 0; w < wave; ++w) off += wave_tot[w];
  return off + inc - v;
}

// The histogram holds counts per digit; find the digit that contains the rank-th largest element
// (rank >= 1, counted from the top digit down) and the rank inside that digit.
__device__ void find_digit(SelectShared &sh, int n_bins, int rank, int &digit, int &rank_in) {
  const int bpt = n_bins / kEpiThreads;           // bins per thread (n_bins is a multiple of 512)
  const int hi = n_bins - threadIdx.x * bpt - 1;  // thread 0 owns the top bins
  int local = 0;
  for (int i = 0; i < bpt; ++i) local += sh.hist[hi - i];
  const int above = block_exclusive_scan(local, sh.wave_tot);
  if (above < rank && rank <= above + local) {
    int acc = above;
    for (int i = 0; i < bpt; ++i) {
      int c = sh.hist[hi - i];
      if (rank <= acc + c) { sh.bin = hi - i; sh.rank = rank - acc; break; }
      acc += c;
    }
  }
  __syncthreads();
  digit = sh.bin;
  rank_in = sh.rank;
  __syncthreads();
}

// Filter of one row for top-K sampling, by the whole workgroup: three counting passes over the
// row (it sits in L2: the LM head has just written it).  K <= 0 or K >= V: no filter.
__device__ RowFilter select_top_k(const float *row, int V, int K, SelectShared &sh) {
  RowFilter f;
  f.key = 0;
  f.tie_max = V;
  if (K <= 0 || K >= V) return f;
  const float *const rows[1] = {row};
  uint32_t prefix = 0, mask = 0;
  int rank = K;
  const int shifts[3] = {21, 10, 0}, bits[3] = {11, 11, 10};
  for (int pass = 0; pass < 3; ++pass) {
    const int n_bins = 1 << bits[pass];
    for (int i = threadIdx.x; i < kSelBins; i += kEpiThreads) sh.hist[i] = 0;
    __syncthreads();
    const int shift = shifts[pass];
    scan_rows<1>(rows, V, [&](int q4, const float (&x)[1][4], int n) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (e < n) {
          uint32_t k = order_key(x[0][e]);
          if ((k & mask) == prefix) atomicAdd(&sh.hist[(k >> shift) & (n_bins - 1)], 1);
        }
      }
    });
    __syncthreads();
    int digit, rank_in;
    find_digit(sh, n_bins < kEpiThreads ? kEpiThreads : n_bins, rank, digit, rank_in);
    prefix |= (uint32_t)digit << shift;
    mask |= (uint32_t)(n_bins - 1) << shift;
    if (pass == 2) {
      // `rank_in` of the sh.hist[digit] logits equal to the threshold are kept: the lowest indices
      const int n_equal = sh.hist[digit];
      f.key = prefix;
      if (rank_in < n_equal) {
        // rare (exactly equal logits across the boundary): one thread walks the row in index order
        if (threadIdx.x == 0) {
          int seen = 0, j = 0;
          for (; j < V; ++j)
            if (order_key(row[j]) == prefix && ++seen == rank_in) break;
          sh.bin = j;
        }
        __syncthreads();
        f.tie_max = sh.bin;
        __syncthreads();
      }
    }
    rank = rank_in;
  }
  return f;
}

// Gumbel-max over softmax(logits * inv_t) (or plain argmax when greedy) fused with ln-sum-exp.
__device__ void sample_row(const float *logits, int V, bool greedy, float inv_t, uint32_t k0, uint32_t k1,
                           uint32_t c1, uint32_t c2, uint32_t c3, const RowFilter &flt, Best &best, MaxSum &ms) {
  best.s = -INFINITY;
  best.idx = -1;
  ms.m = -INFINITY;
  ms.s = 0.f;
  const float *const rows[1] = {logits};
  scan_rows<1>(rows, V, [&](int q4, const float (&x)[1][4], int n) {
    uint32_t rnd[4] = {0, 0, 0, 0};
    if (!greedy) philox4x32_10((uint32_t)q4, c1, c2, c3, k0, k1, rnd);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (e < n && kept(flt, x[0][e], q4 * 4 + e)) {
        float l = x[0][e];
        float a = l * inv_t;
        if (a > ms.m) {
          ms.s = (ms.m == -INFINITY) ? 1.f : ms.s * __expf(ms.m - a) + 1.f;
          ms.m = a;
        } else {
          ms.s += __expf(a - ms.m);
        }
        Best c;
        c.s = greedy ? l : a + gumbel(u01(rnd[e]));
        c.idx = q4 * 4 + e;
        best = better(best, c);
      }
    }
  });
}

__global__ __launch_bounds__(kEpiThreads) void draft_epilogue_kernel(Params p, SampleArgs a, int R) {
  __shared__ Best sh_b[kEpiWaves];
  __shared__ MaxSum sh_m[kEpiWaves];
  __shared__ SelectShared sh_sel;
  int m = blockIdx.x, b = m / R, r = m % R;
  int slot = p.step_slots[b];
  if (a.stats_only && r == 0) return;  // row 0 of an externally drafted block is the last token, not a draft
  const float *logits = p.draft_logits + ((size_t)slot * (1 + p.k) + r) * p.V;
  bool greedy = a.temperature == 0.f;
  float inv_t = greedy ? 1.f : 1.f / a.temperature;
  const RowFilter flt = select_top_k(logits, p.V, greedy ? 0 : a.top_k, sh_sel);
  if (threadIdx.x == 0) {  // the validation call evaluates d_t through the same filter
    p.flt_key_d[slot * (kMaxK + 1) + r] = flt.key;
    p.flt_tie_d[slot * (kMaxK + 1) + r] = flt.tie_max;
  }
  Best best;
  MaxSum ms;
  sample_row(logits, p.V, greedy, inv_t, a.seed_lo, a.seed_hi, p.iter[slot], (uint32_t)(r + a.row_base) | (PURPOSE_DRAFT << 8),
             p.seq_id[slot], flt, best, ms);
  best = block_best(best, sh_b);
  ms = block_ms(ms, sh_m);
  if (threadIdx.x == 0) {
    p.logz_d[slot * (kMaxK + 1) + r] = ms.m + logf(ms.s);
    if (a.stats_only) {
      // the tokens were drafted elsewhere
    } else if (r > 0) {
      p.drafts[slot * kMaxK + (r - 1)] = best.idx;
    } else {
      p.first[slot] = best.idx;
      int ng = p.n_gen[slot];
      int frozen = ng >= p.gen_limit[slot];
      p.frozen[slot] = frozen;
      if (a.commit && !frozen) {
        // x_{n+1} is accepted unconditionally: it joins the sequence, its predecessor's K/V stay
        p.kv_len[slot] += 1;
        p.pending[slot] = best.idx;
        if (ng < p.gen_cap) p.gen[(size_t)slot * p.gen_cap + ng] = best.idx;
        p.n_gen[slot] = ng + 1;
      }
    }
  }
}

// ln-sum-exp (over the row's filter) and argmax of every validation row
__global__ __launch_bounds__(kEpiThreads) void verify_stats_kernel(Params p, SampleArgs a, int R) {
  __shared__ Best sh_b[kEpiWaves];
  __shared__ MaxSum sh_m[kEpiWaves];
  int m = blockIdx.x, b = m / R, r = m % R;
  int slot = p.step_slots[b];
  const float *logits = p.verify_logits + ((size_t)slot * (1 + p.k) + r) * p.V;
  __shared__ SelectShared sh_sel;
  bool greedy = a.temperature == 0.f;
  float inv_t = greedy ? 1.f : 1.f / a.temperature;
  const RowFilter flt = select_top_k(logits, p.V, greedy ? 0 : a.top_k, sh_sel);
  if (threadIdx.x == 0) {
    p.flt_key_p[slot * (kMaxK + 1) + r] = flt.key;
    p.flt_tie_p[slot * (kMaxK + 1) + r] = flt.tie_max;
  }
  Best best;
  MaxSum ms;
  sample_row(logits, p.V, true, inv_t, 0, 0, 0, 0, 0, flt, best, ms);
  best = block_best(best, sh_b);
  ms = block_ms(ms, sh_m);
  if (threadIdx.x == 0) {
    p.logz_p[slot * (kMaxK + 1) + r] = ms.m + logf(ms.s);
    p.argmax_p[slot * (kMaxK + 1) + r] = best.idx;
  }
}

__global__ __launch_bounds__(kEpiThreads) void verify_decide_kernel(Params p, SampleArgs a) {
  __shared__ Best sh_b[kEpiWaves];
  __shared__ int sh_a;
  const int slot = p.step_slots[blockIdx.x];
  const int k = p.k_act, V = p.V;  // rows of this call; the logits buffers keep the stride 1 + p.k
  const bool greedy = a.temperature == 0.f;
  const float inv_t = greedy ? 1.f : 1.f / a.temperature;
  const float *P = p.verify_logits + (size_t)slot * (1 + p.k) * V;
  const float *Dl = p.draft_logits + (size_t)slot * (1 + p.k) * V;
  const float *zp = p.logz_p + slot * (kMaxK + 1), *zd = p.logz_d + slot * (kMaxK + 1);
  const int32_t *drafts = p.drafts + slot * kMaxK;
  const uint32_t it = p.iter[slot], sid = p.seq_id[slot];
  // row filters (top-k) found by the two statistics kernels; greedy never filters
  auto filter_p = [&](int row) {
    RowFilter f;
    f.key = greedy ? 0u : p.flt_key_p[slot * (kMaxK + 1) + row];
    f.tie_max = greedy ? V : p.flt_tie_p[slot * (kMaxK + 1) + row];
    return f;
  };
  auto filter_d = [&](int row) {
    RowFilter f;
    f.key = greedy ? 0u : p.flt_key_d[slot * (kMaxK + 1) + row];
    f.tie_max = greedy ? V : p.flt_tie_d[slot * (kMaxK + 1) + row];
    return f;
  };

  if (threadIdx.x == 0) {
    int acc = 0;
    for (int t = 1; t <= k; ++t) {
      int x = drafts[t - 1];
      bool ok;
      if (greedy) {
        ok = x == p.argmax_p[slot * (kMaxK + 1) + (t - 1)];
      } else {
        // a token outside a row's filter has probability zero there
        const float pl = P[(size_t)(t - 1) * V + x], dl = Dl[(size_t)t * V + x];
        float lp = kept(filter_p(t - 1), pl, x) ? pl * inv_t - zp[t - 1] : -INFINITY;
        float ld = kept(filter_d(t), dl, x) ? dl * inv_t - zd[t] : -INFINITY;
        uint32_t rnd[4];
        philox4x32_10(0u, it, (uint32_t)t | (PURPOSE_ACCEPT << 8), sid, a.seed_lo, a.seed_hi, rnd);
        ok = logf(u01(rnd[0])) + ld < lp;
      }
      if (!ok) break;
      acc += 1;
    }
    sh_a = acc;
  }
  __syncthreads();
  const int acc = sh_a;
  int y;
  if (greedy) {
    y = p.argmax_p[slot * (kMaxK + 1) + acc];
  } else if (acc == k) {
    Best best;
    MaxSum ms;
    sample_row(P + (size_t)k * V, V, false, inv_t, a.seed_lo, a.seed_hi, it, (uint32_t)(k + 1) | (PURPOSE_BONUS << 8),
               sid, filter_p(k), best, ms);
    y = block_best(best, sh_b).idx;
  } else {
    const float *pr = P + (size_t)acc * V, *dr = Dl + (size_t)(acc + 1) * V;
    const float z_p = zp[acc], z_d = zd[acc + 1];
    const uint32_t c2 = (uint32_t)(acc + 1) | (PURPOSE_RESIDUAL << 8);
    const RowFilter fp = filter_p(acc), fd = filter_d(acc + 1);
    Best best;
    best.s = -INFINITY;
    best.idx = -1;
    const float *const rows[2] = {pr, dr};
    scan_rows<2>(rows, V, [&](int q4, const float (&x)[2][4], int n) {
      uint32_t rnd[4];
      philox4x32_10((uint32_t)q4, it, c2, sid, a.seed_lo, a.seed_hi, rnd);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (e < n) {
          const int j = q4 * 4 + e;
          float w = (kept(fp, x[0][e], j) ? __expf(x[0][e] * inv_t - z_p) : 0.f) -
                    (kept(fd, x[1][e], j) ? __expf(x[1][e] * inv_t - z_d) : 0.f);
          if (w > 0.f) {
            Best c;
            c.s = __logf(w) + gumbel(u01(rnd[e]));
            c.idx = q4 * 4 + e;
            best = better(best, c);
          }
        }
      }
    });
    best = block_best(best, sh_b);
    if (best.idx < 0) {
      // residual empty through rounding: draw from p_t with the same counters
      MaxSum ms;
      sample_row(pr, V, false, inv_t, a.seed_lo, a.seed_hi, it, c2, sid, fp, best, ms);
      best = block_best(best, sh_b);
      if (threadIdx.x == 0) atomicAdd(p.fallbacks, 1);
    }
    y = best.idx;
  }
  if (threadIdx.x == 0) {
    int32_t *lo = p.last_out + slot * (kMaxK + 1);
    for (int t = 0; t < acc; ++t) lo[t] = drafts[t];
    lo[acc] = y;
    p.n_acc[slot] = acc;
    if (a.commit && !p.frozen[slot]) {
      int ng = p.n_gen[slot];
      for (int t = 0; t <= acc; ++t)
        if (ng + t < p.gen_cap) p.gen[(size_t)slot * p.gen_cap + ng + t] = lo[t];
      p.n_gen[slot] = ng + acc + 1;
      p.kv_len[slot] += 1 + acc;  // K/V of x_{n+1} and of the accepted drafts are kept
      p.pending[slot] = y;
      p.iter[slot] = it + 1;
    }
  }
}

void launch_draft_epilogue(const Params &p, const SampleArgs &a, int B, int R, hipStream_t s) {
  draft_epilogue_kernel<<<B * R, kEpiThreads, 0, s>>>(p, a, R);
}

void launch_verify_epilogue(const Params &p, const SampleArgs &a, int B, int R, hipStream_t s) {
  verify_stats_kernel<<<B * R, kEpiThreads, 0, s>>>(p, a, R);
  verify_decide_kernel<<<B, kEpiThreads, 0, s>>>(p, a);
}

// The uniforms the epilogues attach to indices j0 .. j0 + n of one (sequence, iteration, row,
// purpose): the same generator and the same bits-to-float step as the draws above use.
__global__ void rng_uniforms_kernel(float *out, uint32_t j0, int n, uint32_t k0, uint32_t k1, uint32_t c1, uint32_t c2,
                                    uint32_t c3) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;  // quad of indices within the chunk; j0 % 4 == 0
  if (q * 4 >= n) return;
  uint32_t rnd[4];
  philox4x32_10(j0 / 4 + (uint32_t)q, c1, c2, c3, k0, k1, rnd);
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (q * 4 + e < n) out[q * 4 + e] = u01(rnd[e]);
}

void launch_rng_uniforms(float *out, uint32_t j0, int n, uint64_t seed, uint32_t seq_id, uint32_t iteration,
                         uint32_t row, uint32_t purpose, hipStream_t s) {
  const int quads = (n + 3) / 4;
  rng_uniforms_kernel<<<(quads + 255) / 256, 256, 0, s>>>(out, j0, n, (uint32_t)seed, (uint32_t)(seed >> 32), iteration,
                                                         row | (purpose << 8), seq_id);
}

}  // namespace pass
