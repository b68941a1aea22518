// The fp32 test build of the decode step (pl_model_cfg.dtype = PL_F32): weights, KV cache and every
// activation in fp32, plain kernels without matrix instructions, one accumulation order per output.
// It exists so that the engine around the kernels (slot table, paging, positions, rotary pairing, head
// mapping, residual stream, update protocol, sampler keying) can be checked against the oracle at a
// tolerance of 1e-4, where an indexing mistake cannot hide behind bf16 rounding.  Nothing here is tuned.
//
// Layouts of this build: every weight matrix row-major [out_features, in_features] (w_qkv = rows of q,
// then k, then v; w_gu = all gate rows, then all up rows); KV pool per layer
// [page][kv head][K | V][token in page][hd].
#include "pl_common.h"

namespace pl {
namespace {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ inline float block_sum_256(float v, float *red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// h[row] = E[token] (or h[row] += y[row] when y is given); a[row] = h[row] * g / sqrt(mean(h^2) + eps)
__global__ __launch_bounds__(256) void f32_norm_kernel(const float *embed, const int32_t *input_tok, int vocab,
                                                       const float *y, const float *g, float *h, float *a, int d, float eps) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  float *hr = h + (int64_t)row * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v;
    if (embed) v = embed[(int64_t)min(max(input_tok[row], 0), vocab - 1) * d + i];
    else v = hr[i] + y[(int64_t)row * d + i];
    hr[i] = v;
    ss += v * v;
  }
  ss = block_sum_256(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) a[(int64_t)row * d + i] = hr[i] * g[i] * r;
}

// y[m, n] = sum_k x[m, k] w[n, k]: one wavefront per output column n and group of 8 rows; lanes stride
// over k, shuffle reduction.
__global__ __launch_bounds__(64) void f32_gemm_kernel(const float *x, const float *w, float *y, int M, int N, int K) {
  const int n = blockIdx.x, m0 = blockIdx.y * 8, lane = threadIdx.x;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float *wr = w + (int64_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = wr[k];
#pragma unroll
    for (int r = 0; r < 8; ++r)
      if (m0 + r < M) acc[r] += x[(int64_t)(m0 + r) * K + k] * wv;
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float v = wave_sum(acc[r]);
    if (lane == 0 && m0 + r < M) y[(int64_t)(m0 + r) * N + n] = v;
  }
}

// mid[m, j] = silu(gu[m, j]) * gu[m, F + j]
__global__ void f32_swiglu_kernel(const float *gu, float *mid, int M, int F) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)M * F) return;
  const int m = (int)(idx / F), j = (int)(idx % F);
  const float g = gu[(int64_t)m * 2 * F + j], u = gu[(int64_t)m * 2 * F + F + j];
  mid[idx] = g / (1.f + expf(-g)) * u;
}

// rotate q and k of each row at its position, store q, append k and v to the row's page
__global__ void f32_rope_append_kernel(const float *qkv, const float *cs, const int32_t *pos, const int32_t *row_slot,
                                       const int32_t *page_table, float *q_out, float *kv_layer, int Hq, int Hkv, int hd,
                                       int page_tokens, int pages_per_seq) {
  const int row = blockIdx.y, hh = blockIdx.x, i = threadIdx.x, half = hd / 2;
  const float *src = qkv + (int64_t)row * (Hq + 2 * Hkv) * hd + (int64_t)hh * hd;
  const float x1 = src[i], x2 = src[half + i];
  const float c = cs[(int64_t)row * hd + i], sn = cs[(int64_t)row * hd + half + i];
  if (hh < Hq) {
    float *q = q_out + ((int64_t)row * Hq + hh) * hd;
    q[i] = x1 * c - x2 * sn;
    q[half + i] = x2 * c + x1 * sn;
    return;
  }
  const int p = pos[row];
  const int page = page_table[(int64_t)row_slot[row] * pages_per_seq + p / page_tokens], t = p % page_tokens;
  const bool is_k = hh < Hq + Hkv;
  const int g = is_k ? hh - Hq : hh - Hq - Hkv;
  float *dst = kv_layer + (((int64_t)page * Hkv + g) * 2 + (is_k ? 0 : 1)) * page_tokens * hd + (int64_t)t * hd;
  if (is_k) {
    dst[i] = x1 * c - x2 * sn;
    dst[half + i] = x2 * c + x1 * sn;
  } else {
    dst[i] = x1;
    dst[half + i] = x2;
  }
}

// One wavefront per (row, query head): the tokens of the row's history one after the other, lanes over the
// head dimension (two elements per lane for hd = 128), running soft-max.
__global__ __launch_bounds__(64) void f32_attention_kernel(const float *q, const float *kv_layer, const int32_t *page_table,
                                                           const int32_t *pos, const int32_t *row_slot, float *out, int Hq,
                                                           int Hkv, int hd, int page_tokens, int pages_per_seq) {
  const int row = blockIdx.y, h = blockIdx.x, lane = threadIdx.x;
  const int g = h / (Hq / Hkv), ctx = pos[row] + 1;
  const float *qr = q + ((int64_t)row * Hq + h) * hd;
  const float q0 = lane < hd ? qr[lane] : 0.f, q1 = lane + 64 < hd ? qr[lane + 64] : 0.f;
  const int32_t *pt = page_table + (int64_t)row_slot[row] * pages_per_seq;
  const float scale = 1.0f / sqrtf((float)hd);
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int j = 0; j < ctx; ++j) {
    const float *kb = kv_layer + ((int64_t)pt[j / page_tokens] * Hkv + g) * 2 * page_tokens * hd + (int64_t)(j % page_tokens) * hd;
    const float *vb = kb + (int64_t)page_tokens * hd;
    float s = (lane < hd ? q0 * kb[lane] : 0.f) + (lane + 64 < hd ? q1 * kb[lane + 64] : 0.f);
    s = wave_sum(s) * scale;
    const float mn = fmaxf(m, s), alpha = expf(m - mn), pj = expf(s - mn);
    l = l * alpha + pj;
    o0 = o0 * alpha + (lane < hd ? pj * vb[lane] : 0.f);
    o1 = o1 * alpha + (lane + 64 < hd ? pj * vb[lane + 64] : 0.f);
    m = mn;
  }
  float *orow = out + ((int64_t)row * Hq + h) * hd;
  if (lane < hd) orow[lane] = o0 / l;
  if (lane + 64 < hd) orow[lane + 64] = o1 / l;
}

}  // namespace

static inline int ok() { return hipGetLastError() == hipSuccess ? 0 : -7; }

int f32_launch_norm(const float *embed, const int32_t *input_tok, int vocab, const float *y, const float *g, float *h,
                    float *a, int n, int d, float eps, hipStream_t s) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(f32_norm_kernel, dim3(n), dim3(256), 0, s, embed, input_tok, vocab, y, g, h, a, d, eps);
  return ok();
}

int f32_launch_gemm(const float *x, const float *w, float *y, int M, int N, int K, hipStream_t s) {
  if (M <= 0) return 0;
  hipLaunchKernelGGL(f32_gemm_kernel, dim3(N, (M + 7) / 8), dim3(64), 0, s, x, w, y, M, N, K);
  return ok();
}

int f32_launch_swiglu(const float *gu, float *mid, int M, int F, hipStream_t s) {
  if (M <= 0) return 0;
  const int64_t total = (int64_t)M * F;
  hipLaunchKernelGGL(f32_swiglu_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, gu, mid, M, F);
  return ok();
}

int f32_launch_rope_append(const float *qkv, const float *cs, const int32_t *pos, const int32_t *row_slot,
                           const int32_t *page_table, float *q_out, float *kv_layer, int n, int Hq, int Hkv, int hd,
                           int page_tokens, int pages_per_seq, hipStream_t s) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(f32_rope_append_kernel, dim3(Hq + 2 * Hkv, n), dim3(hd / 2), 0, s, qkv, cs, pos, row_slot, page_table,
                     q_out, kv_layer, Hq, Hkv, hd, page_tokens, pages_per_seq);
  return ok();
}

int f32_launch_attention(const float *q, const float *kv_layer, const int32_t *page_table, const int32_t *pos,
                         const int32_t *row_slot, float *out, int n, int Hq, int Hkv, int hd, int page_tokens,
                         int pages_per_seq, hipStream_t s) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(f32_attention_kernel, dim3(Hq, n), dim3(64), 0, s, q, kv_layer, page_table, pos, row_slot, out, Hq, Hkv,
                     hd, page_tokens, pages_per_seq);
  return ok();
}

}  // namespace pl
