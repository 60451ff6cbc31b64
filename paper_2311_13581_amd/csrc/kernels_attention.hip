// Split-KV decode attention for the (1+k)-row block over the paged K/V cache.
//
// A call carries R rows per slot at consecutive positions; row r attends to cached positions
// 0 .. pos0 + r, which includes the K/V its own call wrote (causal inside the new block).  Every
// K/V byte is read once for all rows of a group: that is the premise of the method (Section 2.2:
// a few extra tokens cost about as much as one because decoding is bound by memory traffic).
//
// Grid: (split, head, group).  A group is up to 8 consecutive rows of one slot.  Within the
// workgroup (4 wavefronts) 16 lanes share one key: each lane holds hd/16 dimensions, so a key or
// value row is fetched as 16 adjacent 16-byte loads; a wavefront covers 4 keys per iteration and
// the workgroup 16.  Partial (max, sum, accumulator) triples go to a workspace and a second
// kernel merges the splits.
#include "pass_internal.h"

namespace pass {

template <int DPL>
__device__ __forceinline__ void load_chunk(const float *p, float (&o)[DPL]) {
  static_assert(DPL == 4 || DPL == 8, "head_dim 64 or 128");
#pragma unroll
  for (int i = 0; i < DPL; i += 4) {
    float4 a = *(const float4 *)(p + i);
    o[i] = a.x; o[i + 1] = a.y; o[i + 2] = a.z; o[i + 3] = a.w;
  }
}
template <int DPL>
__device__ __forceinline__ void load_chunk(const bf16_t *p, float (&o)[DPL]) {
  if constexpr (DPL == 8) {
    uint4 v = *(const uint4 *)p;
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  } else {
    uint2 v = *(const uint2 *)p;
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  }
}

// How a row group's keys are cut into splits.  A function of the group's own key count only, so
// that a sequence's arithmetic (and therefore its tokens) cannot depend on what else is batched.
__device__ __forceinline__ void split_plan(int n_keys, int &n_splits, int &chunk) {
  n_splits = min(kMaxSplits, (n_keys + 63) / 64);
  chunk = ((n_keys + n_splits - 1) / n_splits + 15) & ~15;
}

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_split_kernel(Params p, int layer, int R) {
  constexpr int DPL = HD / 16;
  constexpr int RQ = kAttnRowsPerGroup;
  __shared__ float s_m[4][RQ], s_l[4][RQ];
  __shared__ float s_acc[4][RQ][HD];

  const int split = blockIdx.x, head = blockIdx.y, g = blockIdx.z;
  const int groups_per_slot = (R + RQ - 1) / RQ;
  const int b = g / groups_per_slot;
  const int r0 = (g % groups_per_slot) * RQ;
  const int nr = min(RQ, R - r0);
  const int slot = p.step_slots[b];
  const int pos0 = p.kv_len[slot] + r0;  // position of the group's first row
  const int n_keys = pos0 + nr;
  int n_splits, chunk;
  split_plan(n_keys, n_splits, chunk);
  if (split >= n_splits) return;
  const int k_lo = split * chunk;
  const int k_hi = min(n_keys, k_lo + chunk);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane >> 4, dl = lane & 15;
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

  for (int base = k_lo; base < k_hi; base += 16) {
    const int key = base + wave * 4 + sub;
    const bool valid = key < k_hi;
    float kf[DPL], vf[DPL];
    size_t off = 0;
    if (valid) {
      off = kv_offset(p, layer, slot, key, head) + dl * DPL;
      load_chunk<DPL>(kpool + off, kf);
      load_chunk<DPL>(vpool + off, vf);
    } else {
#pragma unroll
      for (int i = 0; i < DPL; ++i) { kf[i] = 0.f; vf[i] = 0.f; }
    }
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < DPL; ++i) s = fmaf(q[r][i], kf[i], s);
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      s += __shfl_xor(s, 8);
      const bool ok = valid && (r < nr) && (key <= pos0 + r);
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

  // merge the 4 key sub-groups of the wavefront (lanes differing in bits 4 and 5)
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
      float m_o = __shfl_xor(mx[r], o), l_o = __shfl_xor(ls[r], o);
      float m_n = fmaxf(mx[r], m_o);
      float fa = (mx[r] == -INFINITY) ? 0.f : __expf(mx[r] - m_n);
      float fb = (m_o == -INFINITY) ? 0.f : __expf(m_o - m_n);
      ls[r] = ls[r] * fa + l_o * fb;
#pragma unroll
      for (int i = 0; i < DPL; ++i) {
        float a_o = __shfl_xor(acc[r][i], o);
        acc[r][i] = acc[r][i] * fa + a_o * fb;
      }
      mx[r] = m_n;
    }
  }
  if (sub == 0) {
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
      if (dl == 0) { s_m[wave][r] = mx[r]; s_l[wave][r] = ls[r]; }
#pragma unroll
      for (int i = 0; i < DPL; ++i) s_acc[wave][r][dl * DPL + i] = acc[r][i];
    }
  }
  __syncthreads();
  // merge the 4 wavefronts and write the partial of this split
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
    size_t pi = ((size_t)(b * R + r0 + r) * p.H + head) * kMaxSplits + split;
    p.part_acc[pi * HD + dim] = v;
    if (dim == 0) { p.part_m[pi] = m_n; p.part_l[pi] = l_n; }
  }
}

// Merge the split partials of one (row, head): out = sum_s acc_s e^{m_s - m} / sum_s l_s e^{m_s - m}
template <int HD, int OUT>
__global__ __launch_bounds__(HD) void attn_combine_kernel(Params p, int R) {
  int m = blockIdx.x, head = blockIdx.y, dim = threadIdx.x;
  // the row's group and its split plan, recomputed exactly as the split kernel did
  constexpr int RQ = kAttnRowsPerGroup;
  int b = m / R, r = m % R, r0 = (r / RQ) * RQ;
  int n_keys = p.kv_len[p.step_slots[b]] + r0 + min(RQ, R - r0);
  int n_splits, chunk;
  split_plan(n_keys, n_splits, chunk);
  size_t pi = ((size_t)m * p.H + head) * kMaxSplits;
  float m_n = -INFINITY;
  for (int s = 0; s < n_splits; ++s) m_n = fmaxf(m_n, p.part_m[pi + s]);
  float l_n = 0.f, v = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    float ms = p.part_m[pi + s];
    float f = (ms == -INFINITY) ? 0.f : __expf(ms - m_n);
    l_n += p.part_l[pi + s] * f;
    v += p.part_acc[(pi + s) * HD + dim] * f;
  }
  float o = v / l_n;
  size_t oi = (size_t)m * p.D + head * HD + dim;
  if (OUT == 1) {
    // (hi, lo) pair in the matrix-core activation layout: [m / 8][16 pseudo-rows][D]
    uint16_t hi = f32_to_bf16(o);
    size_t xi = (size_t)((m >> 3) * 16 + (m & 7)) * p.D + head * HD + dim;
    p.attn_x[xi] = hi;
    p.attn_x[xi + (size_t)8 * p.D] = f32_to_bf16(o - bf16_to_f32(hi));
  } else {
    p.attn[oi] = o;
  }
}

void launch_attention(const Params &p, int dtype, int layer, int B, int R, int n_splits, int out_bf16,
                      hipStream_t s) {
  int groups = B * ((R + kAttnRowsPerGroup - 1) / kAttnRowsPerGroup);
  dim3 grid(n_splits, p.H, groups);
  if (p.hd == 128) {
    if (dtype == PASS_F32)
      attn_split_kernel<float, 128><<<grid, 256, 0, s>>>(p, layer, R);
    else
      attn_split_kernel<bf16_t, 128><<<grid, 256, 0, s>>>(p, layer, R);
    if (out_bf16 == 1)
      attn_combine_kernel<128, 1><<<dim3(B * R, p.H), 128, 0, s>>>(p, R);
    else
      attn_combine_kernel<128, 0><<<dim3(B * R, p.H), 128, 0, s>>>(p, R);
  } else {
    if (dtype == PASS_F32)
      attn_split_kernel<float, 64><<<grid, 256, 0, s>>>(p, layer, R);
    else
      attn_split_kernel<bf16_t, 64><<<grid, 256, 0, s>>>(p, layer, R);
    if (out_bf16 == 1)
      attn_combine_kernel<64, 1><<<dim3(B * R, p.H), 64, 0, s>>>(p, R);
    else
      attn_combine_kernel<64, 0><<<dim3(B * R, p.H), 64, 0, s>>>(p, R);
  }
}

}  // namespace pass
