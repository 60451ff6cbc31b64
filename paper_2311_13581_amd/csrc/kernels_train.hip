// Training of the look-ahead embeddings (Training details of the paper; Section 2.2.1): the model is
// frozen, only the L x d_model look-ahead embeddings learn, and the loss is taken on the outputs of
// the look-ahead rows of the block (w_T, [LA]_1 .. [LA]_L): row [LA]_i predicts token w_{T+1+i}.
//
// The forward pass of a training step is the drafting call with the look-ahead rows taken from fp32
// master values, each layer working in an area of its own so that what the backward pass needs stays
// behind: the residual stream before each norm, the rotated queries, the attention output and the
// ln-sum-exp of its rows, the gate / up pre-activations.  Nothing here needs a weight gradient, so
// those are the only activations kept (norms, softmax, SwiGLU); a projection y = W x is
// differentiated as dx = W^T dy.
//   matrix-core path (bf16 models): the forward kernels are the decode step's; dx = W^T dy is the same
//     streaming GEMM on a packed transpose of W (built once), its input dy travels as (hi, lo) tiles
//     written by the kernel that produces it, its output as slices over the contraction that the
//     consumer adds in order.  This file holds the elementwise backward kernels in that form.
//   generic path (fp32 models, or "path" = 1): fp32 arrays throughout, dx = W^T dy by gemm_t_*, which
//     streams the plain weights once more, row by row.
// Attention backward (both paths) is split over chunks of the keys like the forward pass.
#include "pass_internal.h"

namespace pass {

__device__ __forceinline__ float block_sum_256(float v, float *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max_256(float v, float *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// ---------------------------------------------------------------------------------------------
// Row assembly of a training step: row 0 of a slot is its pending token w_T, row i >= 1 the i-th
// look-ahead embedding, taken from the fp32 master values.  Row and rotary tables as in the
// decode path's assembly.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void assemble_train_kernel(Params p, const T *tok_emb, const float *master, int R) {
  const int m = blockIdx.x, b = m / R, r = m % R;
  const int slot = p.step_slots[b];
  const int pos = p.kv_len[slot] + r;
  float *dst = p.h + (size_t)m * p.d;
  if (r == 0) {
    const T *src = tok_emb + (size_t)clamp_token(p, p.pending[slot]) * p.d;
    for (int i = threadIdx.x; i < p.d; i += 256) dst[i] = load_f(src, i);
  } else {
    const float *src = master + (size_t)(r - 1) * p.d;
    for (int i = threadIdx.x; i < p.d; i += 256) dst[i] = src[i];
  }
  const int half = p.hd / 2;
  for (int i = threadIdx.x; i < half; i += 256) {
    double sn, cs;
    sincos((double)pos * p.rope_theta[i], &sn, &cs);
    p.rope_cos[(size_t)m * half + i] = (float)cs;
    p.rope_sin[(size_t)m * half + i] = (float)sn;
  }
  if (threadIdx.x == 0) {
    p.row_pos[m] = pos;
    p.row_slot[m] = slot;
    p.row_out[m] = m;
  }
}

void launch_assemble_train(const Params &p, int dtype, const void *tok_emb, const float *master, int B, int R, hipStream_t s) {
  if (dtype == PASS_F32)
    assemble_train_kernel<float><<<B * R, 256, 0, s>>>(p, (const float *)tok_emb, master, R);
  else
    assemble_train_kernel<bf16_t><<<B * R, 256, 0, s>>>(p, (const bf16_t *)tok_emb, master, R);
}

// The same rows for the matrix-core path (bf16 models): besides h, the (hi, lo) tiles of h * gain of the
// first norm and the partial sums of h^2 its consumer expects (partial 0 carries the whole row).
__global__ __launch_bounds__(256) void assemble_train_mfma_kernel(Params p, const bf16_t *tok_emb, const float *master,
                                                                  const bf16_t *gain0, int R) {
  __shared__ float red[4];
  const int m = blockIdx.x, b = m / R, r = m % R;
  const int slot = p.step_slots[b];
  const int pos = p.kv_len[slot] + r;
  const bf16_t *tok = tok_emb + (size_t)clamp_token(p, p.pending[slot]) * p.d;
  const float *la = master + (size_t)(r > 0 ? r - 1 : 0) * p.d;
  float ss = 0.f;
  for (int c0 = threadIdx.x * 4; c0 < p.d; c0 += 1024) {
    float v[4], x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = r == 0 ? load_f(tok, c0 + e) : la[c0 + e];
      x[e] = v[e] * load_f(gain0, c0 + e);
      ss += v[e] * v[e];
    }
    *(float4 *)(p.h + (size_t)m * p.d + c0) = make_float4(v[0], v[1], v[2], v[3]);
    store_split4(p.xg, m, p.d, c0, x);
  }
  ss = block_sum_256(ss, red);
  for (int i = threadIdx.x; i < p.d / 16; i += 256) p.ssq[(size_t)i * kMaxRows + m] = (i == 0) ? ss : 0.f;
  const int half = p.hd / 2;
  for (int i = threadIdx.x; i < half; i += 256) {
    double sn, cs;
    sincos((double)pos * p.rope_theta[i], &sn, &cs);
    p.rope_cos[(size_t)m * half + i] = (float)cs;
    p.rope_sin[(size_t)m * half + i] = (float)sn;
  }
  if (threadIdx.x == 0) {
    p.row_pos[m] = pos;
    p.row_slot[m] = slot;
    p.row_out[m] = m;
  }
}

void launch_assemble_train_mfma(const Params &p, const void *tok_emb, const float *master, const void *gain0, int B, int R,
                                hipStream_t s) {
  assemble_train_mfma_kernel<<<B * R, 256, 0, s>>>(p, (const bf16_t *)tok_emb, master, (const bf16_t *)gain0, R);
}

// ---------------------------------------------------------------------------------------------
// Cross-entropy of the look-ahead rows: loss of a row = ln sum exp(logits) - logit[target];
// logits are overwritten by d loss / d logits = (softmax - onehot) * scale (rows without a target,
// i.e. each slot's row 0, get zeros).  One workgroup per row.  With x_out not null the gradient goes there as
// (hi, lo) tiles of V features instead (input of the matrix-core product with the LM head's transpose).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ce_grad_kernel(float *logits, const int32_t *targets, float scale, float *row_loss, int V,
                                                      uint16_t *x_out) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  float *lg = logits + (size_t)m * V;
  const int tg = targets[m];
  if (tg < 0) {
    const float z[4] = {0.f, 0.f, 0.f, 0.f};
    if (x_out)
      for (int j = threadIdx.x * 4; j < V; j += 1024) store_split4(x_out, m, V, j, z);
    else
      for (int j = threadIdx.x; j < V; j += 256) lg[j] = 0.f;
    if (threadIdx.x == 0) row_loss[m] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < V; j += 256) mx = fmaxf(mx, lg[j]);
  mx = block_max_256(mx, red);
  float se = 0.f;
  for (int j = threadIdx.x; j < V; j += 256) se += expf(lg[j] - mx);
  se = block_sum_256(se, red);
  const float lse = mx + logf(se), inv = 1.f / se;
  if (threadIdx.x == 0) row_loss[m] = lse - lg[tg];
  __syncthreads();
  if (x_out) {
    for (int j = threadIdx.x * 4; j < V; j += 1024) {
      float t[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] = (expf(lg[j + e] - mx) * inv - (j + e == tg ? 1.f : 0.f)) * scale;
      store_split4(x_out, m, V, j, t);
    }
  } else {
    for (int j = threadIdx.x; j < V; j += 256) lg[j] = (expf(lg[j] - mx) * inv - (j == tg ? 1.f : 0.f)) * scale;
  }
}

void launch_ce_grad(float *logits, const int32_t *targets, float scale, float *row_loss, int M, int V, uint16_t *x_out,
                    hipStream_t s) {
  ce_grad_kernel<<<M, 256, 0, s>>>(logits, targets, scale, row_loss, V, x_out);
}

// ---------------------------------------------------------------------------------------------
// dX[m][k] = sum_n dY[m][n] W[n][k]: the transpose of a projection.  A workgroup owns 512 columns
// k (two per thread) and a slice of the rows n of W, which it streams once; the dY values of 64
// rows n at a time are staged in LDS and broadcast.  The slices' sums go to `part` and a second
// kernel adds them in slice order (deterministic).
// ---------------------------------------------------------------------------------------------
template <typename T, int MR>
__global__ __launch_bounds__(256) void gemm_t_partial_kernel(const float *dY, int ldy, const T *W, float *part, int M, int N,
                                                             int K, int n_per_split) {
  __shared__ float dy_s[MR][64];
  const int c = (blockIdx.x * 256 + threadIdx.x) * 2;
  const int n_lo = blockIdx.y * n_per_split, n_hi = min(N, n_lo + n_per_split);
  float acc[MR][2];
#pragma unroll
  for (int m = 0; m < MR; ++m) acc[m][0] = acc[m][1] = 0.f;
  for (int n0 = n_lo; n0 < n_hi; n0 += 64) {
    const int nn = min(64, n_hi - n0);
    __syncthreads();
    for (int e = threadIdx.x; e < MR * 64; e += 256) {
      const int m = e >> 6, j = e & 63;
      dy_s[m][j] = (m < M && j < nn) ? dY[(size_t)m * ldy + n0 + j] : 0.f;
    }
    __syncthreads();
    if (c < K) {
      for (int j = 0; j < nn; ++j) {
        const size_t wi = (size_t)(n0 + j) * K + c;
        const float w0 = load_f(W, wi), w1 = load_f(W, wi + 1);
#pragma unroll
        for (int m = 0; m < MR; ++m) {
          const float y = dy_s[m][j];
          acc[m][0] = fmaf(y, w0, acc[m][0]);
          acc[m][1] = fmaf(y, w1, acc[m][1]);
        }
      }
    }
  }
  if (c < K) {
#pragma unroll
    for (int m = 0; m < MR; ++m)
      if (m < M) {
        float *o = part + ((size_t)blockIdx.y * M + m) * K + c;
        o[0] = acc[m][0];
        o[1] = acc[m][1];
      }
  }
}

__global__ __launch_bounds__(256) void gemm_t_reduce_kernel(const float *part, int S, int M, int K, float *out, int ldo) {
  const int k = blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
  if (k >= K) return;
  float v = 0.f;
  for (int s = 0; s < S; ++s) v += part[((size_t)s * M + m) * K + k];
  out[(size_t)m * ldo + k] = v;
}

template <typename T>
static void gemm_t_dispatch(const float *dY, int ldy, const T *W, float *part, int M, int N, int K, int S, int nps, hipStream_t s) {
  dim3 grid((K + 511) / 512, S);
  switch ((M + 7) / 8) {
    case 1: gemm_t_partial_kernel<T, 8><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 2: gemm_t_partial_kernel<T, 16><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 3: gemm_t_partial_kernel<T, 24><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 4: gemm_t_partial_kernel<T, 32><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 5: gemm_t_partial_kernel<T, 40><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 6: gemm_t_partial_kernel<T, 48><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    case 7: gemm_t_partial_kernel<T, 56><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
    default: gemm_t_partial_kernel<T, 64><<<grid, 256, 0, s>>>(dY, ldy, W, part, M, N, K, nps); break;
  }
}

// part must hold kTrainSplits * M * K floats
void launch_gemm_t(int dtype, const float *dY, int ldy, const void *W, float *part, float *out, int ldo, int M, int N, int K,
                   hipStream_t s) {
  int nps = (N + kTrainSplits - 1) / kTrainSplits;
  nps = (nps + 63) / 64 * 64;  // whole stages of 64 rows
  const int S = (N + nps - 1) / nps;
  if (dtype == PASS_F32)
    gemm_t_dispatch<float>(dY, ldy, (const float *)W, part, M, N, K, S, nps, s);
  else
    gemm_t_dispatch<bf16_t>(dY, ldy, (const bf16_t *)W, part, M, N, K, S, nps, s);
  gemm_t_reduce_kernel<<<dim3((K + 255) / 256, M), 256, 0, s>>>(part, S, M, K, out, ldo);
}

// ---------------------------------------------------------------------------------------------
// y = x * rsqrt(mean(x^2) + eps) * g  ==>  dx = g dy r - x r^3 (sum_i g_i dy_i x_i) / d,  r = rsqrt(..)
// dx is added to `dx_acc` (the gradient of the residual stream).  One workgroup per row.
// ---------------------------------------------------------------------------------------------
// dy may come as KS slices (sums over slices of the contraction, `slice_stride` floats apart), added in
// order; with dx_x not null the updated gradient row also goes there as (hi, lo) tiles.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const float *x, const T *gain, const float *dy, int KS, size_t slice_stride,
                                                          float *dx_acc, int d, float eps, int accumulate, uint16_t *dx_x) {
  __shared__ float red[4];
  constexpr int CH = 8;  // chunks of four features a thread keeps in registers (rows of up to 8192 features)
  const int m = blockIdx.x;
  const size_t base = (size_t)m * d;
  float4 xv[CH], gy[CH];  // x, and gain * dy with the slices added up
  float ss = 0.f, c = 0.f;
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int i0 = (ch * 256 + threadIdx.x) * 4;
    xv[ch] = gy[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i0 < d) {
      xv[ch] = *(const float4 *)(x + base + i0);
      float4 sl[8];  // up to eight slices, requested together (index clamped, surplus dropped), added in order
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) sl[ks] = *(const float4 *)(dy + (size_t)min(ks, KS - 1) * slice_stride + base + i0);
      float4 dv = sl[0];
#pragma unroll
      for (int ks = 1; ks < 8; ++ks)
        if (ks < KS) { dv.x += sl[ks].x; dv.y += sl[ks].y; dv.z += sl[ks].z; dv.w += sl[ks].w; }
      gy[ch] = make_float4(load_f(gain, i0) * dv.x, load_f(gain, i0 + 1) * dv.y, load_f(gain, i0 + 2) * dv.z, load_f(gain, i0 + 3) * dv.w);
      ss += xv[ch].x * xv[ch].x + xv[ch].y * xv[ch].y + xv[ch].z * xv[ch].z + xv[ch].w * xv[ch].w;
      c += gy[ch].x * xv[ch].x + gy[ch].y * xv[ch].y + gy[ch].z * xv[ch].z + gy[ch].w * xv[ch].w;
    }
  }
  ss = block_sum_256(ss, red);
  c = block_sum_256(c, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  const float k3 = r * r * r * c / (float)d;
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int i0 = (ch * 256 + threadIdx.x) * 4;
    if (i0 < d) {
      float t[4] = {gy[ch].x * r - xv[ch].x * k3, gy[ch].y * r - xv[ch].y * k3, gy[ch].z * r - xv[ch].z * k3, gy[ch].w * r - xv[ch].w * k3};
      if (accumulate) {
        const float4 a = *(const float4 *)(dx_acc + base + i0);
        t[0] += a.x; t[1] += a.y; t[2] += a.z; t[3] += a.w;
      }
      *(float4 *)(dx_acc + base + i0) = make_float4(t[0], t[1], t[2], t[3]);
      if (dx_x) store_split4(dx_x, m, d, i0, t);
    }
  }
}

void launch_rmsnorm_bwd(const Params &p, int dtype, const float *x, const void *gain, const float *dy, int KS, size_t slice_stride,
                        float *dx_acc, int M, int accumulate, uint16_t *dx_x, hipStream_t s) {
  if (dtype == PASS_F32)
    rmsnorm_bwd_kernel<float><<<M, 256, 0, s>>>(x, (const float *)gain, dy, KS, slice_stride, dx_acc, p.d, p.eps, accumulate, dx_x);
  else
    rmsnorm_bwd_kernel<bf16_t><<<M, 256, 0, s>>>(x, (const bf16_t *)gain, dy, KS, slice_stride, dx_acc, p.d, p.eps, accumulate, dx_x);
}

// act = silu(gate) * up:  dgate = dact up s (1 + gate (1 - s)),  dup = dact gate s,  s = sigmoid(gate)
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const float *gu, const float *dact, float *dgu, int F) {
  const int m = blockIdx.y, f = blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const float g = gu[(size_t)m * 2 * F + f], u = gu[(size_t)m * 2 * F + F + f], da = dact[(size_t)m * F + f];
  const float sg = 1.0f / (1.0f + expf(-g));
  dgu[(size_t)m * 2 * F + f] = da * u * sg * (1.0f + g * (1.0f - sg));
  dgu[(size_t)m * 2 * F + F + f] = da * g * sg;
}
// The same for the matrix-core path: dact comes as KS slices; dgate and dup leave as (hi, lo) tiles of 2F
// features in the row order of the packed gate/up matrix (strips of 16 gate rows and 16 up rows alternate),
// which is the order its transpose contracts over.  Four consecutive features per thread.
__global__ __launch_bounds__(256) void swiglu_bwd_tiles_kernel(const float *gu, const float *dact, int KS, size_t slice_stride,
                                                               uint16_t *dgu_x, int F) {
  const int m = blockIdx.y, f = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (f >= F) return;
  float dg[4], du[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float g = gu[(size_t)m * 2 * F + f + e], u = gu[(size_t)m * 2 * F + F + f + e];
    float da = dact[(size_t)m * F + f + e];
    for (int ks = 1; ks < KS; ++ks) da += dact[ks * slice_stride + (size_t)m * F + f + e];
    const float sg = 1.0f / (1.0f + expf(-g));
    dg[e] = da * u * sg * (1.0f + g * (1.0f - sg));
    du[e] = da * g * sg;
  }
  const int row = (f >> 4) * 32 + (f & 15);  // packed row of gate feature f; its up row is 16 further
  store_split4(dgu_x, m, 2 * F, row, dg);
  store_split4(dgu_x, m, 2 * F, row + 16, du);
}

void launch_swiglu_bwd(const Params &p, const float *gu, const float *dact, float *dgu, int M, hipStream_t s) {
  swiglu_bwd_kernel<<<dim3((p.F + 255) / 256, M), 256, 0, s>>>(gu, dact, dgu, p.F);
}
void launch_swiglu_bwd_tiles(const Params &p, const float *gu, const float *dact, int KS, size_t slice_stride, uint16_t *dgu_x,
                             int M, hipStream_t s) {
  swiglu_bwd_tiles_kernel<<<dim3((p.F / 4 + 255) / 256, M), 256, 0, s>>>(gu, dact, KS, slice_stride, dgu_x, p.F);
}

// ---------------------------------------------------------------------------------------------
// Attention backward for the R rows of one slot, one head and one chunk of kTrainAttnChunk keys.
// Row r attends to keys 0 .. pos0 + r.  With the forward pass's ln-sum-exp of the row (lse) and its
// output O, a chunk of keys needs nothing from the others:
//   P_j = exp(scale q.K_j - lse),  dP_j = dO.V_j,  D = dO.O (= sum_j P_j dP_j),  dS_j = P_j (dP_j - D),
//   dq = scale sum_j dS_j K_j (summed over the chunks afterwards, in chunk order),
// and for the keys that are rows of this very block (positions >= pos0; each lies in one chunk):
//   dK_j = scale sum_r dS_rj q_r,  dV_j = sum_r P_rj dO_r.
// Keys before pos0 are the prompt's: nothing upstream of them is trained.  K and V come from the
// cache in its storage type (a bfloat16 cache holds rounded values: the gradient passes through
// the rounding), in tiles of 32 keys staged in LDS as fp32, whichever way the V pages are laid out.
// q is the rotated query kept by the forward pass; dq / dK / dV are still rotated here:
// attn_bwd_finish_kernel adds up the chunks and turns them back.
// ---------------------------------------------------------------------------------------------
// eight consecutive cache values as loaded, untouched until they are needed (so that the loads stay in flight)
template <typename T>
struct Raw8;
template <>
struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float *p, size_t off, bool in) {
    a = b = make_float4(0.f, 0.f, 0.f, 0.f);
    if (in) {
      a = *(const float4 *)(p + off);
      b = *(const float4 *)(p + off + 4);
    }
  }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <>
struct Raw8<bf16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const bf16_t *p, size_t off, bool in) {
    a = make_uint4(0u, 0u, 0u, 0u);
    if (in) a = *(const uint4 *)(p + off);
  }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] = __uint_as_float(w[e] << 16);
      v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
};

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// sum over each aligned group of 8 lanes; every lane of the group ends with the total
__device__ __forceinline__ float group_sum8(float v) {
  v += dpp_move<0x141>(v);  // row_half_mirror: lane i <-> 7 - i
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  return v;
}

// RB: compile-time bound of the rows (R <= RB; the rows beyond R are carried as zeros), so that the loops over the
// rows unroll and their LDS reads are requested together instead of one round trip after the other.
template <typename T, int HD, int RB>
__global__ __launch_bounds__(256) void attn_bwd_split_kernel(Params p, int layer, int R, const float *q_saved, int ldq,
                                                             const float *o_f32, const uint16_t *o_x, const float *lse,
                                                             const float *dattn, int KS, size_t slice_stride, float *dq_part,
                                                             float *dqkv) {
  constexpr int TK = 32, LD = HD + 4, RMAX = RB, PARTS = 256 / HD;
  __shared__ __align__(16) float tiles[2][TK][LD];  // K tile, V tile; at the end the parts' dq
  __shared__ __align__(16) float qs[RB][HD], dos[RB][HD];   // the rows' q and dO
  __shared__ __align__(16) float ds_s[RB][TK], p_s[RB][TK];  // dS and P of the tile in hand
  __shared__ float lse_s[RMAX], D_s[RMAX];
  __shared__ int pages_s[kTrainAttnChunk / 16 + 1];  // pages hold at least 16 positions
  static_assert(PARTS * RMAX * HD <= 2 * TK * LD, "the parts' dq must fit the tiles");
  const int split = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int m0 = b * R;
  const int slot = p.row_slot[m0], pos0 = p.row_pos[m0];
  const int n_keys = pos0 + R;
  const int k_lo = split * kTrainAttnChunk;
  if (slot < 0 || k_lo >= n_keys) return;  // uniform over the workgroup
  const int k_hi = min(n_keys, k_lo + kTrainAttnChunk);
  const T *kpool = (const T *)p.k_pool, *vpool = (const T *)p.v_pool;
  const float scale = rsqrtf((float)HD);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  for (int idx = tid; idx < RB * HD; idx += 256) {
    const int r = idx / HD, dm = idx % HD;
    float qv = 0.f, dv = 0.f;
    if (r < R) {
      qv = q_saved[(size_t)(m0 + r) * ldq + head * HD + dm];
      dv = dattn[(size_t)(m0 + r) * p.D + head * HD + dm];
      for (int ks = 1; ks < KS; ++ks) dv += dattn[ks * slice_stride + (size_t)(m0 + r) * p.D + head * HD + dm];  // slices, in order
    }
    qs[r][dm] = qv;
    dos[r][dm] = dv;
  }
  __syncthreads();
  for (int r = wave; r < R; r += 4) {  // D of row r: one wavefront, lanes over the dimensions
    float acc = 0.f;
    for (int dm = lane; dm < HD; dm += 64) {
      float o;
      if (o_f32) {
        o = o_f32[(size_t)(m0 + r) * p.D + head * HD + dm];
      } else {
        const uint16_t *x = o_x + xs_index(m0 + r, p.D, head * HD + dm);
        o = bf16_to_f32(x[0]) + bf16_to_f32(x[kXsLoOffset]);
      }
      acc = fmaf(dos[r][dm], o, acc);
    }
#pragma unroll
    for (int o2 = 32; o2 > 0; o2 >>= 1) acc += __shfl_xor(acc, o2);
    if (lane == 0) {
      D_s[r] = acc;
      lse_s[r] = lse[(size_t)(m0 + r) * p.H + head];
    }
  }
  if (tid >= R && tid < RB) D_s[tid] = lse_s[tid] = 0.f;

  // the chunk's pages, looked up once
  const int page_lo = k_lo >> p.page_shift;
  for (int i = tid; i <= ((k_hi - 1) >> p.page_shift) - page_lo; i += 256)
    pages_s[i] = p.block_table[(size_t)slot * p.pages_per_seq + page_lo + i];
  __syncthreads();  // pages_s, D_s and lse_s are in place

  const int dim = tid % HD, part = tid / HD;
  float dq[RMAX];
#pragma unroll
  for (int r = 0; r < RMAX; ++r) dq[r] = 0.f;

  // The next tile's K and V travel from memory into registers while the tile in hand is worked on; a thread
  // carries NCH chunks of eight values of each.  K: chunk = (key, eight dimensions).  V: the same when its pages
  // hold [position][dim]; when they hold [dim][position] (matrix-core attention), chunk = (dimension, eight
  // consecutive keys: a tile starts at a multiple of 32 keys and a page holds a multiple of 32, so they share a page).
  constexpr int NCH = TK * HD / 8 / 256;
  Raw8<T> kraw[NCH], vraw[NCH];
  auto fetch = [&](int t0) {
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int c = u * 256 + tid;
      {
        const int key = c / (HD / 8), d0 = (c % (HD / 8)) * 8, j = t0 + key;
        const bool in = j < k_hi;
        const size_t off =
            in ? ((((size_t)layer * p.n_pages + pages_s[(j >> p.page_shift) - page_lo]) * p.H + head) * p.page_size + (j & (p.page_size - 1))) * HD + d0 : 0;
        kraw[u].load(kpool, off, in);
        if (!p.v_transposed) vraw[u].load(vpool, off, in);
      }
      if (p.v_transposed) {
        const int dv = c / (TK / 8), j0 = t0 + (c % (TK / 8)) * 8;
        const bool in = j0 < k_hi;
        const size_t off =
            in ? ((((size_t)layer * p.n_pages + pages_s[(j0 >> p.page_shift) - page_lo]) * p.H + head) * HD + dv) * p.page_size + (j0 & (p.page_size - 1)) : 0;
        vraw[u].load(vpool, off, in);
      }
    }
  };
  auto stash = [&](int t0) {
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int c = u * 256 + tid;
      float kv[8], vv[8];
      kraw[u].get(kv);
      vraw[u].get(vv);
      const int key = c / (HD / 8), d0 = (c % (HD / 8)) * 8;
      *(float4 *)&tiles[0][key][d0] = make_float4(kv[0], kv[1], kv[2], kv[3]);
      *(float4 *)&tiles[0][key][d0 + 4] = make_float4(kv[4], kv[5], kv[6], kv[7]);
      if (!p.v_transposed) {
        *(float4 *)&tiles[1][key][d0] = make_float4(vv[0], vv[1], vv[2], vv[3]);
        *(float4 *)&tiles[1][key][d0 + 4] = make_float4(vv[4], vv[5], vv[6], vv[7]);
      } else {
        const int dv = c / (TK / 8), key0 = (c % (TK / 8)) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) tiles[1][key0 + e][dv] = (t0 + key0 + e < k_hi) ? vv[e] : 0.f;  // unwritten positions hold anything
      }
    }
  };
  fetch(k_lo);
  for (int t0 = k_lo; t0 < k_hi; t0 += TK) {
    __syncthreads();  // the previous tile has been consumed
    stash(t0);
    __syncthreads();
    if (t0 + TK < k_hi) fetch(t0 + TK);
    {  // scores, probabilities, dS: eight adjacent lanes share a key, each with an eighth of the dimensions in
       // registers for all rows (every K and V value leaves LDS once); the eighths meet through lane exchanges
      constexpr int DPT = HD / 8;
      const int key = tid >> 3, part8 = tid & 7, j = t0 + key;
      float kk[DPT], vv[DPT];
#pragma unroll
      for (int i4 = 0; i4 < DPT; i4 += 4) {
        const float4 kq = *(const float4 *)&tiles[0][key][part8 * DPT + i4], vq = *(const float4 *)&tiles[1][key][part8 * DPT + i4];
        kk[i4] = kq.x; kk[i4 + 1] = kq.y; kk[i4 + 2] = kq.z; kk[i4 + 3] = kq.w;
        vv[i4] = vq.x; vv[i4 + 1] = vq.y; vv[i4 + 2] = vq.z; vv[i4 + 3] = vq.w;
      }
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int i4 = 0; i4 < DPT; i4 += 4) {
          const float4 qq = *(const float4 *)&qs[r][part8 * DPT + i4], dd = *(const float4 *)&dos[r][part8 * DPT + i4];
          sc = fmaf(qq.x, kk[i4], sc); sc = fmaf(qq.y, kk[i4 + 1], sc); sc = fmaf(qq.z, kk[i4 + 2], sc); sc = fmaf(qq.w, kk[i4 + 3], sc);
          dp = fmaf(dd.x, vv[i4], dp); dp = fmaf(dd.y, vv[i4 + 1], dp); dp = fmaf(dd.z, vv[i4 + 2], dp); dp = fmaf(dd.w, vv[i4 + 3], dp);
        }
        sc = group_sum8(sc);
        dp = group_sum8(dp);
        if (part8 == 0) {
          const bool ok = r < R && j < k_hi && j <= pos0 + r;
          const float pj = ok ? expf(sc * scale - lse_s[r]) : 0.f;
          p_s[r][key] = pj;
          ds_s[r][key] = ok ? pj * (dp - D_s[r]) : 0.f;
        }
      }
    }
    __syncthreads();
    // dq: thread (part, dim) takes a run of TK / PARTS keys, four at a time
    {
      constexpr int KPP = TK / PARTS;
      const int key0 = part * KPP;
#pragma unroll
      for (int kb = 0; kb < KPP; kb += 4) {
        const float k0 = tiles[0][key0 + kb][dim], k1 = tiles[0][key0 + kb + 1][dim], k2 = tiles[0][key0 + kb + 2][dim],
                    k3 = tiles[0][key0 + kb + 3][dim];
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {  // rows beyond R carry dS = 0
          const float4 d4 = *(const float4 *)&ds_s[r][key0 + kb];
          dq[r] = fmaf(d4.x, k0, dq[r]); dq[r] = fmaf(d4.y, k1, dq[r]); dq[r] = fmaf(d4.z, k2, dq[r]); dq[r] = fmaf(d4.w, k3, dq[r]);
        }
      }
    }
    // the block's own keys in this tile
    for (int j = max(t0, pos0) + part; j < min(t0 + TK, k_hi); j += PARTS) {
      const int key = j - t0, jj = j - pos0;
      float dk = 0.f, dvv = 0.f;
      for (int r = jj; r < R; ++r) {
        dk = fmaf(ds_s[r][key], qs[r][dim], dk);
        dvv = fmaf(p_s[r][key], dos[r][dim], dvv);
      }
      dqkv[(size_t)(m0 + jj) * 3 * p.D + p.D + head * HD + dim] = dk * scale;
      dqkv[(size_t)(m0 + jj) * 3 * p.D + 2 * p.D + head * HD + dim] = dvv;
    }
  }
  __syncthreads();
  float *comb = &tiles[0][0][0];  // [PARTS][RMAX][HD]
#pragma unroll
  for (int r = 0; r < RMAX; ++r) comb[(part * RMAX + r) * HD + dim] = dq[r];
  __syncthreads();
  if (part == 0) {
    for (int r = 0; r < R; ++r) {
      float t = comb[r * HD + dim];
#pragma unroll
      for (int q2 = 1; q2 < PARTS; ++q2) t += comb[(q2 * RMAX + r) * HD + dim];
      dq_part[((size_t)split * kMaxRows + m0 + r) * p.D + head * HD + dim] = t * scale;
    }
  }
}

// The same for bfloat16 caches and up to eight rows per slot, with the two contractions over the head
// dimension on the matrix core: the K and V tiles stay in LDS as cached ([key][dim] bf16, whichever way the V
// pages are laid out), and are the A operand of v_mfma_f32_16x16x32_bf16; q (scaled) and dO are the B operand as
// (hi, lo) column pairs like every activation of the matrix-core path (columns 0..7 the hi halves of the rows,
// 8..15 the lo halves, added afterwards), so nothing but the cache is rounded.  Wavefront w takes the scores
// (w < 2) or dP (w >= 2) of 16 of the tile's 32 keys; probabilities and dS are then formed by one thread per
// (row, key), and dq, dK, dV as in the kernel above.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int HD, int RB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void attn_bwd_mfma_kernel(Params p, int layer, int R, const float *q_saved, int ldq,
                                                            const float *o_f32, const uint16_t *o_x, const float *lse,
                                                            const float *dattn, int KS, size_t slice_stride, float *dq_part,
                                                            float *dqkv) {
  constexpr int TK = 32, LDK = HD + 8, PARTS = 256 / HD, KT = HD / 32, RQ = 8;
  static_assert(RB <= RQ, "one (hi, lo) column group");
  __shared__ __align__(16) uint16_t kv_s[2][TK][LDK];        // K tile, V tile: [key][dim] bf16
  __shared__ __align__(16) float qs[RQ][HD], dos[RQ][HD];    // the rows' q and dO (rows beyond R: zeros)
  __shared__ __align__(16) float sp_s[RQ][TK], dd_s[RQ][TK];  // scores, then P; dP, then dS
  __shared__ __align__(16) float comb[PARTS][RB][HD];
  __shared__ float lse_s[RQ], D_s[RQ];
  __shared__ int pages_s[kTrainAttnChunk / 16 + 1];
  const int split = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int m0 = b * R;
  const int slot = p.row_slot[m0], pos0 = p.row_pos[m0];
  const int n_keys = pos0 + R;
  const int k_lo = split * kTrainAttnChunk;
  if (slot < 0 || k_lo >= n_keys) return;  // uniform over the workgroup
  const int k_hi = min(n_keys, k_lo + kTrainAttnChunk);
  const bf16_t *kpool = (const bf16_t *)p.k_pool, *vpool = (const bf16_t *)p.v_pool;
  const float scale = rsqrtf((float)HD);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  for (int idx = tid; idx < RQ * HD; idx += 256) {
    const int r = idx / HD, dm = idx % HD;
    float qv = 0.f, dv = 0.f;
    if (r < R) {
      qv = q_saved[(size_t)(m0 + r) * ldq + head * HD + dm];
      dv = dattn[(size_t)(m0 + r) * p.D + head * HD + dm];
      for (int ks = 1; ks < KS; ++ks) dv += dattn[ks * slice_stride + (size_t)(m0 + r) * p.D + head * HD + dm];  // slices, in order
    }
    qs[r][dm] = qv;
    dos[r][dm] = dv;
  }
  __syncthreads();
  for (int r = wave; r < R; r += 4) {  // D of row r: one wavefront, lanes over the dimensions
    float acc = 0.f;
    for (int dm = lane; dm < HD; dm += 64) {
      float o;
      if (o_f32) {
        o = o_f32[(size_t)(m0 + r) * p.D + head * HD + dm];
      } else {
        const uint16_t *x = o_x + xs_index(m0 + r, p.D, head * HD + dm);
        o = bf16_to_f32(x[0]) + bf16_to_f32(x[kXsLoOffset]);
      }
      acc = fmaf(dos[r][dm], o, acc);
    }
#pragma unroll
    for (int o2 = 32; o2 > 0; o2 >>= 1) acc += __shfl_xor(acc, o2);
    if (lane == 0) {
      D_s[r] = acc;
      lse_s[r] = lse[(size_t)(m0 + r) * p.H + head];
    }
  }
  if (tid >= R && tid < RQ) D_s[tid] = lse_s[tid] = 0.f;
  const int page_lo = k_lo >> p.page_shift;
  for (int i = tid; i <= ((k_hi - 1) >> p.page_shift) - page_lo; i += 256)
    pages_s[i] = p.block_table[(size_t)slot * p.pages_per_seq + page_lo + i];

  // this wavefront's B operand: q * scale (scores) or dO (dP), column c = hi (c < 8) or lo half of row c & 7
  const int c = lane & 15, g = lane >> 4;
  const int which = wave >> 1, kb = wave & 1;
  u32x4_t frag[KT];
  {
    const float(*src)[HD] = which ? dos : qs;
    const float f = which ? 1.f : scale;
    const bool hi = c < 8;
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      const float4 x0 = *(const float4 *)&src[c & 7][j * 32 + g * 8], x1 = *(const float4 *)&src[c & 7][j * 32 + g * 8 + 4];
      frag[j][0] = split2_bf16(x0.x * f, x0.y * f, hi);
      frag[j][1] = split2_bf16(x0.z * f, x0.w * f, hi);
      frag[j][2] = split2_bf16(x1.x * f, x1.y * f, hi);
      frag[j][3] = split2_bf16(x1.z * f, x1.w * f, hi);
    }
  }
  __syncthreads();  // pages_s, D_s and lse_s are in place

  const int dim = tid % HD, part = tid / HD;
  float dq[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) dq[r] = 0.f;

  // next tile's K and V in flight while the tile in hand is worked on (chunks as in the kernel above)
  constexpr int NCH = TK * HD / 8 / 256;
  Raw8<bf16_t> kraw[NCH], vraw[NCH];
  auto fetch = [&](int t0) {
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int ch = u * 256 + tid;
      {
        const int key = ch / (HD / 8), d0 = (ch % (HD / 8)) * 8, j = t0 + key;
        const bool in = j < k_hi;
        const size_t off =
            in ? ((((size_t)layer * p.n_pages + pages_s[(j >> p.page_shift) - page_lo]) * p.H + head) * p.page_size + (j & (p.page_size - 1))) * HD + d0 : 0;
        kraw[u].load(kpool, off, in);
        if (!p.v_transposed) vraw[u].load(vpool, off, in);
      }
      if (p.v_transposed) {
        const int dv = ch / (TK / 8), j0 = t0 + (ch % (TK / 8)) * 8;
        const bool in = j0 < k_hi;
        const size_t off =
            in ? ((((size_t)layer * p.n_pages + pages_s[(j0 >> p.page_shift) - page_lo]) * p.H + head) * HD + dv) * p.page_size + (j0 & (p.page_size - 1)) : 0;
        vraw[u].load(vpool, off, in);
      }
    }
  };
  auto stash = [&](int t0) {
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int ch = u * 256 + tid;
      const int key = ch / (HD / 8), d0 = (ch % (HD / 8)) * 8;
      *(uint4 *)&kv_s[0][key][d0] = kraw[u].a;
      if (!p.v_transposed) {
        *(uint4 *)&kv_s[1][key][d0] = vraw[u].a;
      } else {
        const int dv = ch / (TK / 8), key0 = (ch % (TK / 8)) * 8;
        const uint32_t w[4] = {vraw[u].a.x, vraw[u].a.y, vraw[u].a.z, vraw[u].a.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)  // unwritten positions hold anything
          kv_s[1][key0 + e][dv] = (t0 + key0 + e < k_hi) ? (uint16_t)(w[e >> 1] >> ((e & 1) * 16)) : (uint16_t)0;
      }
    }
  };
  fetch(k_lo);
  for (int t0 = k_lo; t0 < k_hi; t0 += TK) {
    __syncthreads();  // the previous tile has been consumed
    stash(t0);
    __syncthreads();
    if (t0 + TK < k_hi) fetch(t0 + TK);
    {  // scores or dP of this wavefront's 16 keys x 8 rows
      floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
      const uint16_t *row = &kv_s[which][kb * 16 + c][g * 8];
#pragma unroll
      for (int j = 0; j < KT; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8_t *)(row + j * 32), __builtin_bit_cast(bf16x8_t, frag[j]), acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] += dpp_move<0x128>(acc[r]);  // row_ror 8: the lo column onto its hi column
      if (c < 8) *(floatx4_t *)&(which ? dd_s : sp_s)[c][kb * 16 + 4 * g] = acc;  // lane (c, g): keys 4g .. 4g+3 of row c
    }
    __syncthreads();
    {  // probabilities and dS: one thread per (row, key)
      const int key = tid & 31, r = tid >> 5, j = t0 + key;
      const bool ok = r < R && j < k_hi && j <= pos0 + r;
      const float pj = ok ? expf(sp_s[r][key] - lse_s[r]) : 0.f;
      const float dsj = ok ? pj * (dd_s[r][key] - D_s[r]) : 0.f;
      sp_s[r][key] = pj;
      dd_s[r][key] = dsj;
    }
    __syncthreads();
    {  // dq: thread (part, dim) takes a run of TK / PARTS keys, four at a time
      constexpr int KPP = TK / PARTS;
      const int key0 = part * KPP;
#pragma unroll 2
      for (int kq = 0; kq < KPP; kq += 4) {
        const float k0 = bf16_to_f32(kv_s[0][key0 + kq][dim]), k1 = bf16_to_f32(kv_s[0][key0 + kq + 1][dim]),
                    k2 = bf16_to_f32(kv_s[0][key0 + kq + 2][dim]), k3 = bf16_to_f32(kv_s[0][key0 + kq + 3][dim]);
#pragma unroll
        for (int r = 0; r < RB; ++r) {  // rows beyond R carry dS = 0
          const float4 d4 = *(const float4 *)&dd_s[r][key0 + kq];
          dq[r] = fmaf(d4.x, k0, dq[r]); dq[r] = fmaf(d4.y, k1, dq[r]); dq[r] = fmaf(d4.z, k2, dq[r]); dq[r] = fmaf(d4.w, k3, dq[r]);
        }
      }
    }
    // the block's own keys in this tile
    for (int j = max(t0, pos0) + part; j < min(t0 + TK, k_hi); j += PARTS) {
      const int key = j - t0, jj = j - pos0;
      float dk = 0.f, dvv = 0.f;
      for (int r = jj; r < R; ++r) {
        dk = fmaf(dd_s[r][key], qs[r][dim], dk);
        dvv = fmaf(sp_s[r][key], dos[r][dim], dvv);
      }
      dqkv[(size_t)(m0 + jj) * 3 * p.D + p.D + head * HD + dim] = dk * scale;
      dqkv[(size_t)(m0 + jj) * 3 * p.D + 2 * p.D + head * HD + dim] = dvv;
    }
  }
#pragma unroll
  for (int r = 0; r < RB; ++r) comb[part][r][dim] = dq[r];
  __syncthreads();
  if (part == 0) {
    for (int r = 0; r < R; ++r) {
      float t = comb[0][r][dim];
#pragma unroll
      for (int q2 = 1; q2 < PARTS; ++q2) t += comb[q2][r][dim];
      dq_part[((size_t)split * kMaxRows + m0 + r) * p.D + head * HD + dim] = t * scale;
    }
  }
}

// The chunks' dq added in chunk order; dq and dK back through the rotary embedding (the transpose of a
// rotation is the opposite rotation); the row of dqkv as fp32 in place or as (hi, lo) tiles for the
// matrix-core projection that follows.  Four consecutive features (two rotary pairs) per thread.
__global__ __launch_bounds__(256) void attn_bwd_finish_kernel(Params p, int R, const float *dq_part, float *dqkv,
                                                              uint16_t *dqkv_x) {
  const int m = blockIdx.x, which = blockIdx.y, half = p.hd / 2;  // which: 0 q, 1 k, 2 v
  if (p.row_slot[m] < 0) return;
  const int n_splits = (p.row_pos[(m / R) * R] + R + kTrainAttnChunk - 1) / kTrainAttnChunk;
  for (int c = threadIdx.x * 4; c < p.D; c += 1024) {
    const int col = which * p.D + c;
    float t[4];
    if (which == 0) {
      t[0] = t[1] = t[2] = t[3] = 0.f;
      for (int s = 0; s < n_splits; ++s) {
        const float4 v = *(const float4 *)(dq_part + ((size_t)s * kMaxRows + m) * p.D + c);
        t[0] += v.x; t[1] += v.y; t[2] += v.z; t[3] += v.w;
      }
    } else {
      const float4 v = *(const float4 *)(dqkv + (size_t)m * 3 * p.D + col);
      t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
    }
    if (which < 2) {
      const int i = (c % p.hd) / 2;
      const float *cs = p.rope_cos + (size_t)m * half + i, *sn = p.rope_sin + (size_t)m * half + i;
      const float a0 = t[0], b0 = t[1], a1 = t[2], b1 = t[3];
      t[0] = a0 * cs[0] + b0 * sn[0];
      t[1] = -a0 * sn[0] + b0 * cs[0];
      t[2] = a1 * cs[1] + b1 * sn[1];
      t[3] = -a1 * sn[1] + b1 * cs[1];
    }
    if (dqkv_x)
      store_split4(dqkv_x, m, 3 * p.D, col, t);
    else
      *(float4 *)(dqkv + (size_t)m * 3 * p.D + col) = make_float4(t[0], t[1], t[2], t[3]);
  }
}

template <typename T, int HD>
static void attn_bwd_dispatch(const Params &p, dim3 grid, int layer, int R, const float *q_saved, int ldq, const float *o,
                              const uint16_t *o_x, const float *lse, const float *dattn, int KS, size_t slice_stride, float *dq_part,
                              float *dqkv, hipStream_t s) {
  if constexpr (sizeof(T) == 2) {  // bfloat16 cache, one column group of rows: the matrix-core kernel
#define PASS_ATTN_BWD_MFMA(RB) \
  attn_bwd_mfma_kernel<HD, RB><<<grid, 256, 0, s>>>(p, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv)
    if (R <= 8) {
      if (R <= 2) PASS_ATTN_BWD_MFMA(2);
      else if (R <= 3) PASS_ATTN_BWD_MFMA(3);
      else if (R <= 4) PASS_ATTN_BWD_MFMA(4);
      else if (R <= 5) PASS_ATTN_BWD_MFMA(5);
      else if (R <= 6) PASS_ATTN_BWD_MFMA(6);
      else PASS_ATTN_BWD_MFMA(8);
      return;
    }
#undef PASS_ATTN_BWD_MFMA
  }
#define PASS_ATTN_BWD(RB) \
  attn_bwd_split_kernel<T, HD, RB><<<grid, 256, 0, s>>>(p, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv)
  if (R <= 2) PASS_ATTN_BWD(2);
  else if (R <= 3) PASS_ATTN_BWD(3);
  else if (R <= 4) PASS_ATTN_BWD(4);
  else if (R <= 5) PASS_ATTN_BWD(5);
  else if (R <= 6) PASS_ATTN_BWD(6);
  else if (R <= 8) PASS_ATTN_BWD(8);
  else PASS_ATTN_BWD(kMaxK + 1);
#undef PASS_ATTN_BWD
}

void launch_attn_bwd(const Params &p, int dtype, int layer, int B, int R, int max_keys, const float *q_saved, int ldq,
                     const float *o, const uint16_t *o_x, const float *lse, const float *dattn, int KS, size_t slice_stride,
                     float *dq_part, float *dqkv, uint16_t *dqkv_x, hipStream_t s) {
  dim3 grid((max_keys + kTrainAttnChunk - 1) / kTrainAttnChunk, p.H, B);
  if (p.hd == 128) {
    if (dtype == PASS_F32)
      attn_bwd_dispatch<float, 128>(p, grid, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv, s);
    else
      attn_bwd_dispatch<bf16_t, 128>(p, grid, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv, s);
  } else {
    if (dtype == PASS_F32)
      attn_bwd_dispatch<float, 64>(p, grid, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv, s);
    else
      attn_bwd_dispatch<bf16_t, 64>(p, grid, layer, R, q_saved, ldq, o, o_x, lse, dattn, KS, slice_stride, dq_part, dqkv, s);
  }
  attn_bwd_finish_kernel<<<dim3(B * R, 3), 256, 0, s>>>(p, R, dq_part, dqkv, dqkv_x);
}

// ---------------------------------------------------------------------------------------------
// Gradient of the look-ahead embeddings (sum over the slots of the gradient of their rows), AdamW
// (decoupled weight decay) on the fp32 master values, and the model's own look-ahead tensor
// refreshed in its storage type so that the next drafting call uses what was learned.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void lookahead_adamw_kernel(const float *dh, int B, int R, int d, float *grad, float *master,
                                                              float *m1, float *m2, T *model_la, float lr, float beta1,
                                                              float beta2, float eps, float wd, float bc1, float bc2) {
  const int idx = blockIdx.x * 256 + threadIdx.x;  // over (R - 1) * d
  if (idx >= (R - 1) * d) return;
  const int i = idx / d, c = idx % d;
  float g = 0.f;
  for (int b = 0; b < B; ++b) g += dh[(size_t)(b * R + 1 + i) * d + c];
  grad[idx] = g;
  const float m = beta1 * m1[idx] + (1.f - beta1) * g;
  const float v = beta2 * m2[idx] + (1.f - beta2) * g * g;
  m1[idx] = m;
  m2[idx] = v;
  const float th = master[idx];
  const float nt = th - lr * ((m / bc1) / (sqrtf(v / bc2) + eps) + wd * th);
  master[idx] = nt;
  store_f(model_la, idx, nt);
}

void launch_lookahead_adamw(int dtype, const float *dh, int B, int R, int d, float *grad, float *master, float *m1, float *m2,
                            void *model_la, float lr, float beta1, float beta2, float eps, float wd, float bc1, float bc2,
                            hipStream_t s) {
  const int n = (R - 1) * d;
  if (n <= 0) return;
  if (dtype == PASS_F32)
    lookahead_adamw_kernel<float><<<(n + 255) / 256, 256, 0, s>>>(dh, B, R, d, grad, master, m1, m2, (float *)model_la, lr, beta1,
                                                                 beta2, eps, wd, bc1, bc2);
  else
    lookahead_adamw_kernel<bf16_t><<<(n + 255) / 256, 256, 0, s>>>(dh, B, R, d, grad, master, m1, m2, (bf16_t *)model_la, lr,
                                                                  beta1, beta2, eps, wd, bc1, bc2);
}

// master values from the embedding of one token (the paper starts from [UNK]) or from the model's own
// look-ahead tensor (token < 0); moments to zero
template <typename T>
__global__ __launch_bounds__(256) void lookahead_init_kernel(const T *tok_emb, const T *model_la, int token, int k, int d,
                                                             float *master, float *m1, float *m2, T *model_la_out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= k * d) return;
  const float v = token >= 0 ? load_f(tok_emb, (size_t)token * d + idx % d) : load_f(model_la, idx);
  master[idx] = v;
  m1[idx] = 0.f;
  m2[idx] = 0.f;
  store_f(model_la_out, idx, v);
}

void launch_lookahead_init(int dtype, const void *tok_emb, void *model_la, int token, int k, int d, float *master, float *m1,
                           float *m2, hipStream_t s) {
  const int n = k * d;
  if (n <= 0) return;
  if (dtype == PASS_F32)
    lookahead_init_kernel<float><<<(n + 255) / 256, 256, 0, s>>>((const float *)tok_emb, (const float *)model_la, token, k, d, master,
                                                                m1, m2, (float *)model_la);
  else
    lookahead_init_kernel<bf16_t><<<(n + 255) / 256, 256, 0, s>>>((const bf16_t *)tok_emb, (const bf16_t *)model_la, token, k, d,
                                                                 master, m1, m2, (bf16_t *)model_la);
}

// the model's own look-ahead tensor, in its storage type, from the fp32 master values
template <typename T>
__global__ __launch_bounds__(256) void lookahead_store_kernel(const float *master, int n, T *model_la) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx < n) store_f(model_la, idx, master[idx]);
}

void launch_lookahead_store(int dtype, const float *master, int k, int d, void *model_la, hipStream_t s) {
  const int n = k * d;
  if (n <= 0) return;
  if (dtype == PASS_F32)
    lookahead_store_kernel<float><<<(n + 255) / 256, 256, 0, s>>>(master, n, (float *)model_la);
  else
    lookahead_store_kernel<bf16_t><<<(n + 255) / 256, 256, 0, s>>>(master, n, (bf16_t *)model_la);
}

}  // namespace pass
