// Generic kernels of the (1+k)-row decode step: any storage type, fp32 activations.
// They carry the fp32 configuration and any shape the matrix-core path does not take.
#include "pass_internal.h"

namespace pass {

// ---------------------------------------------------------------------------------------------
// Row assembly (Section 2.2.1: the look-ahead embeddings are appended after the sequence;
// Algorithm 1: drafting call on (x_n, [LA]_1..[LA]_k), validation call on (x_{n+1}, drafts)).
// Row m = b*R + r belongs to slot step_slots[b] at position kv_len[slot] + r.
// Also fills the rotary table of the step (angles in double: pos * base^(-2i/hd), the
// frequencies from the table made at create).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void assemble_kernel(Params p, const T *tok_emb, const T *lookahead, int mode,
                                                       int R) {
  int m = blockIdx.x, b = m / R, r = m % R;
  int slot = p.step_slots[b];
  int pos = p.kv_len[slot] + r;
  const bool dead = row_is_dead(p, mode, slot, R);
  const T *src;
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
  float *dst = p.h + (size_t)m * p.d;
  for (int i = threadIdx.x; i < p.d; i += blockDim.x) dst[i] = load_f(src, i);
  int half = p.hd / 2;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    double sn, cs;
    sincos((double)pos * p.rope_theta[i], &sn, &cs);
    p.rope_cos[(size_t)m * half + i] = (float)cs;
    p.rope_sin[(size_t)m * half + i] = (float)sn;
  }
  if (threadIdx.x == 0) {
    p.row_pos[m] = dead ? 0 : pos;
    p.row_slot[m] = dead ? -1 : slot;
    p.row_out[m] = slot * (1 + p.k) + r;
  }
}

void launch_assemble(const Params &p, int dtype, const void *tok_emb, const void *lookahead, int mode, int B,
                     int R, hipStream_t s) {
  if (dtype == PASS_F32)
    assemble_kernel<float><<<B * R, 256, 0, s>>>(p, (const float *)tok_emb, (const float *)lookahead, mode, R);
  else
    assemble_kernel<bf16_t><<<B * R, 256, 0, s>>>(p, (const bf16_t *)tok_emb, (const bf16_t *)lookahead, mode, R);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: out = x * rsqrt(mean(x^2) + eps) * gain
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *x, const T *gain, float *out, int d, float eps) {
  __shared__ float red[4];
  const float *xr = x + (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = red[0] + red[1] + red[2] + red[3];
  float inv = 1.0f / sqrtf(tot / (float)d + eps);
  float *o = out + (size_t)blockIdx.x * d;
  for (int i = threadIdx.x; i < d; i += 256) o[i] = xr[i] * inv * load_f(gain, i);
}

void launch_rmsnorm(const Params &p, int dtype, const float *x, const void *gain, float *out, int M, hipStream_t s) {
  if (dtype == PASS_F32)
    rmsnorm_kernel<float><<<M, 256, 0, s>>>(x, (const float *)gain, out, p.d, p.eps);
  else
    rmsnorm_kernel<bf16_t><<<M, 256, 0, s>>>(x, (const bf16_t *)gain, out, p.d, p.eps);
}

// ---------------------------------------------------------------------------------------------
// Skinny GEMM, generic: out[m][n] (+)= sum_k X[m][k] W[n][k].  One wavefront per output column,
// lanes stride over K in chunks of 8 elements (K % 8 == 0), rows in blocks of 8.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void load8(const float *w, float (&o)[8]) {
  float4 a = *(const float4 *)w, b = *(const float4 *)(w + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *w, float (&o)[8]) {
  uint4 v = *(const uint4 *)w;
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
  o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const float *X, const T *W, float *out, int M, int N,
                                                           int K, int ldc, const int32_t *rowmap, int accumulate) {
  constexpr int MB = 8;
  int lane = threadIdx.x & 63;
  int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  int n_waves = gridDim.x * 4;
  for (int n = wave; n < N; n += n_waves) {
    const T *wr = W + (size_t)n * K;
    for (int m0 = 0; m0 < M; m0 += MB) {
      int mr = min(MB, M - m0);
      float acc[MB];
#pragma unroll
      for (int i = 0; i < MB; ++i) acc[i] = 0.f;
      for (int k0 = lane * 8; k0 < K; k0 += 64 * 8) {
        float w[8];
        load8(wr + k0, w);
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          if (i < mr) {
            float x[8];
            load8(X + (size_t)(m0 + i) * K + k0, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[i] = fmaf(w[e], x[e], acc[i]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < MB; ++i) acc[i] = wave_sum(acc[i]);
      if (lane == 0) {
        for (int i = 0; i < mr; ++i) {
          int row = rowmap ? rowmap[m0 + i] : (m0 + i);
          float *o = out + (size_t)row * ldc + n;
          *o = accumulate ? (*o + acc[i]) : acc[i];
        }
      }
    }
  }
}

void launch_gemm_generic(int dtype, const float *X, const void *W, float *out, int M, int N, int K, int ldc,
                         const int32_t *rowmap, int accumulate, hipStream_t s) {
  int blocks = (N + 3) / 4;
  if (blocks > 4096) blocks = 4096;
  if (dtype == PASS_F32)
    gemm_generic_kernel<float><<<blocks, 256, 0, s>>>(X, (const float *)W, out, M, N, K, ldc, rowmap, accumulate);
  else
    gemm_generic_kernel<bf16_t><<<blocks, 256, 0, s>>>(X, (const bf16_t *)W, out, M, N, K, ldc, rowmap, accumulate);
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding on q and k (interleaved pairs), K/V rows written to the paged cache at the
// row's position.  q is rotated in place in the qkv workspace.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(Params p, int layer) {
  int m = blockIdx.x;
  int slot = p.row_slot[m], pos = p.row_pos[m];
  int half = p.hd / 2;
  float *q = p.qkv + (size_t)m * 3 * p.D;
  float *kk = q + p.D;
  float *vv = q + 2 * p.D;
  T *kpool = (T *)p.k_pool, *vpool = (T *)p.v_pool;
  for (int idx = threadIdx.x; idx < p.H * half; idx += blockDim.x) {
    int h = idx / half, i = idx % half;
    float cs = p.rope_cos[(size_t)m * half + i], sn = p.rope_sin[(size_t)m * half + i];
    int e = h * p.hd + 2 * i;
    float q0 = q[e], q1 = q[e + 1];
    q[e] = q0 * cs - q1 * sn;
    q[e + 1] = q0 * sn + q1 * cs;
    if (slot < 0) continue;  // a dead row (see row_is_dead) has no place in the cache
    float k0 = kk[e], k1 = kk[e + 1];
    size_t off = kv_offset(p, layer, slot, pos, h) + 2 * i;
    store_f(kpool, off, k0 * cs - k1 * sn);
    store_f(kpool, off + 1, k0 * sn + k1 * cs);
    store_f(vpool, off, vv[e]);
    store_f(vpool, off + 1, vv[e + 1]);
  }
}

void launch_rope_kv(const Params &p, int dtype, int layer, int M, hipStream_t s) {
  if (dtype == PASS_F32)
    rope_kv_kernel<float><<<M, 256, 0, s>>>(p, layer);
  else
    rope_kv_kernel<bf16_t><<<M, 256, 0, s>>>(p, layer);
}

// act = silu(gate) * up
__global__ __launch_bounds__(256) void silu_mul_kernel(const float *gu, float *act, int F) {
  int m = blockIdx.y;
  int f = blockIdx.x * 256 + threadIdx.x;
  if (f < F) {
    float g = gu[(size_t)m * 2 * F + f], u = gu[(size_t)m * 2 * F + F + f];
    float v = g / (1.0f + __expf(-g)) * u;
    act[(size_t)m * F + f] = v;
  }
}

void launch_silu_mul(const Params &p, int M, hipStream_t s) {
  dim3 grid((p.F + 255) / 256, M);
  silu_mul_kernel<<<grid, 256, 0, s>>>(p.gu, p.act, p.F);
}

// ---------------------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------------------
struct PokeArgs {
  int32_t *ptr[16];
  int32_t val[16];
  int n;
};
__global__ void poke_kernel(PokeArgs a) {
  int i = threadIdx.x;
  if (i < a.n) *a.ptr[i] = a.val[i];
}
void launch_poke(int32_t *const *ptrs, const int32_t *vals, int n, hipStream_t s) {
  PokeArgs a;
  a.n = n;
  for (int i = 0; i < n; ++i) { a.ptr[i] = ptrs[i]; a.val[i] = vals[i]; }
  poke_kernel<<<1, 16, 0, s>>>(a);
}

__global__ void fill_i32_kernel(int32_t *p, int32_t v, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}
// Reads n16 16-byte words and drops them: the yardstick of pass_plain_read.  Every workgroup owns
// a contiguous segment (the pattern that reads fastest on this device), 8 requests per thread in
// flight.  `never` is 0: the store only keeps the loads alive.
typedef uint32_t rd_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void plain_read_kernel(const rd_u32x4 *src, size_t n16, int never, uint32_t *sink) {
  constexpr int U = 8;
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = min(n16, lo + per);
  uint32_t acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + (U - 1) * 256 < hi; i += U * 256) {
    rd_u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u][u & 3];
  }
  for (; i < hi; i += 256) acc ^= __builtin_nontemporal_load(src + i)[0];
  if (never && acc == 0x9e3779b9u) *sink = acc;
}

void launch_plain_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t s) {
  plain_read_kernel<<<2048, 256, 0, s>>>((const rd_u32x4 *)src, bytes / 16, 0, sink);
}

void launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t s) {
  if (n == 0) return;
  // chunks of 2^30 elements keep the grid size inside 32 bits
  for (size_t done = 0; done < n; done += (size_t)1 << 30) {
    size_t m = n - done < ((size_t)1 << 30) ? n - done : (size_t)1 << 30;
    fill_i32_kernel<<<(unsigned)((m + 255) / 256), 256, 0, s>>>(p + done, v, m);
  }
}

}  // namespace pass
