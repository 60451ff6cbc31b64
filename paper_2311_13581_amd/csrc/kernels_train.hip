// Training of the look-ahead embeddings (Training details of the paper; Section 2.2.1): the model is
// frozen, only the L x d_model look-ahead embeddings learn, and the loss is taken on the outputs of
// the look-ahead rows of the block (w_T, [LA]_1 .. [LA]_L): row [LA]_i predicts token w_{T+1+i}.
//
// The forward pass of a training step is the drafting call on the generic kernels (fp32
// activations, plain weight layout) with the look-ahead rows taken from fp32 master values; the
// host keeps a copy of what the backward pass needs of every layer (the residual stream before
// each norm, the rotated queries, the gate / up pre-activations).  This file holds what is new:
// the backward kernels for M <= 64 rows, and AdamW.
//
// Nothing here needs a weight gradient, so the only activations kept are those a non-linearity
// needs (norms, softmax, SwiGLU); a projection y = W x is differentiated as dx = W^T dy by
// gemm_t_*: the weights are streamed once more, row by row.
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

// ---------------------------------------------------------------------------------------------
// Cross-entropy of the look-ahead rows: loss of a row = ln sum exp(logits) - logit[target];
// logits are overwritten by d loss / d logits = (softmax - onehot) * scale (rows without a target,
// i.e. each slot's row 0, get zeros).  One workgroup per row.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ce_grad_kernel(float *logits, const int32_t *targets, float scale, float *row_loss, int V) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  float *lg = logits + (size_t)m * V;
  const int tg = targets[m];
  if (tg < 0) {
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
  for (int j = threadIdx.x; j < V; j += 256) lg[j] = (expf(lg[j] - mx) * inv - (j == tg ? 1.f : 0.f)) * scale;
}

void launch_ce_grad(float *logits, const int32_t *targets, float scale, float *row_loss, int M, int V, hipStream_t s) {
  ce_grad_kernel<<<M, 256, 0, s>>>(logits, targets, scale, row_loss, V);
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
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const float *x, const T *gain, const float *dy, float *dx_acc, int d,
                                                          float eps, int accumulate) {
  __shared__ float red[4];
  const size_t base = (size_t)blockIdx.x * d;
  float ss = 0.f, c = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float xv = x[base + i];
    ss += xv * xv;
    c += load_f(gain, i) * dy[base + i] * xv;
  }
  ss = block_sum_256(ss, red);
  c = block_sum_256(c, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  const float k3 = r * r * r * c / (float)d;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = load_f(gain, i) * dy[base + i] * r - x[base + i] * k3;
    dx_acc[base + i] = accumulate ? dx_acc[base + i] + v : v;
  }
}

void launch_rmsnorm_bwd(const Params &p, int dtype, const float *x, const void *gain, const float *dy, float *dx_acc, int M,
                        int accumulate, hipStream_t s) {
  if (dtype == PASS_F32)
    rmsnorm_bwd_kernel<float><<<M, 256, 0, s>>>(x, (const float *)gain, dy, dx_acc, p.d, p.eps, accumulate);
  else
    rmsnorm_bwd_kernel<bf16_t><<<M, 256, 0, s>>>(x, (const bf16_t *)gain, dy, dx_acc, p.d, p.eps, accumulate);
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

void launch_swiglu_bwd(const Params &p, const float *gu, const float *dact, float *dgu, int M, hipStream_t s) {
  swiglu_bwd_kernel<<<dim3((p.F + 255) / 256, M), 256, 0, s>>>(gu, dact, dgu, p.F);
}

// ---------------------------------------------------------------------------------------------
// Attention backward for the R rows of one slot and one head.  Row r attends to keys 0 .. pos0 + r:
//   P = softmax(scale q K^T),  O = P V,  dP_j = dO . V_j,  dS_j = P_j (dP_j - sum_i P_i dP_i),
//   dq = scale sum_j dS_j K_j,  and for the keys that are rows of this very block (positions >= pos0)
//   dK_j += scale dS_j q,  dV_j += P_j dO.
// Keys before pos0 are the prompt's: nothing upstream of them is trained.  The rows are walked in
// order, the block keys' sums kept in registers (one dimension per thread), so the result does not
// depend on scheduling.  Scores live in LDS (`max_keys` floats, dynamic).
// q is the rotated query kept by the forward pass; dq / dK / dV go to dqkv [M][3D] (still rotated:
// rope_bwd_kernel turns them back).  K/V come from the cache in its storage type (a bfloat16 cache
// holds rounded values: the gradient passes through the rounding).
// ---------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_bwd_kernel(Params p, int layer, int R, const float *q_saved, const float *dattn,
                                                       float *dqkv) {
  extern __shared__ float sc[];  // scores -> exponentials -> dS of the row in hand
  __shared__ float red[4];
  __shared__ float pblk[kMaxK + 1];
  constexpr int PARTS = 256 / HD;
  __shared__ float comb[PARTS][HD];
  const int head = blockIdx.x, b = blockIdx.y;
  const int m0 = b * R;
  const int slot = p.row_slot[m0], pos0 = p.row_pos[m0];
  const T *kpool = (const T *)p.k_pool, *vpool = (const T *)p.v_pool;
  const float scale = rsqrtf((float)HD);
  const int dim = threadIdx.x % HD, part = threadIdx.x / HD;
  float dk_acc[kMaxK + 1], dv_acc[kMaxK + 1];
#pragma unroll
  for (int j = 0; j <= kMaxK; ++j) dk_acc[j] = dv_acc[j] = 0.f;

  for (int r = 0; r < R; ++r) {
    const int n_keys = pos0 + r + 1;
    const float *qr = q_saved + (size_t)(m0 + r) * p.D + head * HD;
    const float *dor = dattn + (size_t)(m0 + r) * p.D + head * HD;
    __syncthreads();  // the previous row's scores have been consumed
    // scores
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < n_keys; j += 256) {
      const size_t off = kv_offset(p, layer, slot, j, head);
      float s = 0.f;
      for (int i = 0; i < HD; ++i) s = fmaf(qr[i], load_f(kpool, off + i), s);
      s *= scale;
      sc[j] = s;
      mx = fmaxf(mx, s);
    }
    mx = block_max_256(mx, red);
    float se = 0.f;
    for (int j = threadIdx.x; j < n_keys; j += 256) {
      const float e = expf(sc[j] - mx);
      sc[j] = e;
      se += e;
    }
    se = block_sum_256(se, red);
    const float inv = 1.f / se;
    // D = sum_j P_j (dO . V_j)
    float dsum = 0.f;
    for (int j = threadIdx.x; j < n_keys; j += 256) {
      const size_t off = kv_offset(p, layer, slot, j, head);
      float dp = 0.f;
      for (int i = 0; i < HD; ++i) dp = fmaf(dor[i], load_f(vpool, off + i), dp);
      dsum += sc[j] * inv * dp;
    }
    dsum = block_sum_256(dsum, red);
    // dS_j in place; P of the block's own keys kept aside
    for (int j = threadIdx.x; j < n_keys; j += 256) {
      const size_t off = kv_offset(p, layer, slot, j, head);
      float dp = 0.f;
      for (int i = 0; i < HD; ++i) dp = fmaf(dor[i], load_f(vpool, off + i), dp);
      const float pj = sc[j] * inv;
      if (j >= pos0) pblk[j - pos0] = pj;
      sc[j] = pj * (dp - dsum);
    }
    __syncthreads();
    // dq: thread (part, dim) sums the keys j = part, part + PARTS, ...; the parts are added in order
    float dq = 0.f;
    for (int j = part; j < n_keys; j += PARTS) dq = fmaf(sc[j], load_f(kpool, kv_offset(p, layer, slot, j, head) + dim), dq);
    comb[part][dim] = dq;
    __syncthreads();
    if (part == 0) {
      float t = comb[0][dim];
#pragma unroll
      for (int q2 = 1; q2 < PARTS; ++q2) t += comb[q2][dim];
      dqkv[(size_t)(m0 + r) * 3 * p.D + head * HD + dim] = t * scale;
      const float qd = qr[dim], dod = dor[dim];
#pragma unroll
      for (int jj = 0; jj <= kMaxK; ++jj)
        if (jj <= r) {
          dk_acc[jj] = fmaf(sc[pos0 + jj] * scale, qd, dk_acc[jj]);
          dv_acc[jj] = fmaf(pblk[jj], dod, dv_acc[jj]);
        }
    }
  }
  if (part == 0) {
#pragma unroll
    for (int jj = 0; jj <= kMaxK; ++jj)
      if (jj < R) {
        dqkv[(size_t)(m0 + jj) * 3 * p.D + p.D + head * HD + dim] = dk_acc[jj];
        dqkv[(size_t)(m0 + jj) * 3 * p.D + 2 * p.D + head * HD + dim] = dv_acc[jj];
      }
  }
}

// dq and dk back through the rotary embedding: the transpose of a rotation is the opposite rotation
__global__ __launch_bounds__(256) void rope_bwd_kernel(Params p, float *dqkv) {
  const int m = blockIdx.x, half = p.hd / 2;
  for (int idx = threadIdx.x; idx < 2 * p.H * half; idx += 256) {
    const int which = idx / (p.H * half), rem = idx % (p.H * half);
    const int h = rem / half, i = rem % half;
    const float cs = p.rope_cos[(size_t)m * half + i], sn = p.rope_sin[(size_t)m * half + i];
    float *v = dqkv + (size_t)m * 3 * p.D + (size_t)which * p.D + h * p.hd + 2 * i;
    const float a = v[0], b2 = v[1];
    v[0] = a * cs + b2 * sn;
    v[1] = -a * sn + b2 * cs;
  }
}

void launch_attn_bwd(const Params &p, int dtype, int layer, int B, int R, int max_keys, const float *q_saved, const float *dattn,
                     float *dqkv, hipStream_t s) {
  dim3 grid(p.H, B);
  const size_t lds = (size_t)max_keys * sizeof(float);
  if (p.hd == 128) {
    if (dtype == PASS_F32)
      attn_bwd_kernel<float, 128><<<grid, 256, lds, s>>>(p, layer, R, q_saved, dattn, dqkv);
    else
      attn_bwd_kernel<bf16_t, 128><<<grid, 256, lds, s>>>(p, layer, R, q_saved, dattn, dqkv);
  } else {
    if (dtype == PASS_F32)
      attn_bwd_kernel<float, 64><<<grid, 256, lds, s>>>(p, layer, R, q_saved, dattn, dqkv);
    else
      attn_bwd_kernel<bf16_t, 64><<<grid, 256, lds, s>>>(p, layer, R, q_saved, dattn, dqkv);
  }
  rope_bwd_kernel<<<B * R, 256, 0, s>>>(p, dqkv);
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
