// Small row-wise kernels of the decode step: token select + embedding gather + RMSNorm, residual
// add (summing split-K partials) + RMSNorm, rotary tables, rotary + KV-cache append.
#include "pl_common.h"

namespace pl {
namespace {

__device__ inline float block_sum_256(float v) {
  __shared__ float red[4];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// h[row] = E[token]; a[row] = rmsnorm(h[row]) * g.  token = input_tok[row] if >= 0, else the token
// the previous step produced for this row's slot.
__global__ __launch_bounds__(256) void embed_rmsnorm_kernel(const bf16_t *embed, const bf16_t *g,
                                                            const int32_t *input_tok, const int32_t *last_tok,
                                                            const int32_t *row_slot, float *h, bf16_t *a,
                                                            int d, int vocab, float eps) {
  const int row = blockIdx.x;
  int tok = input_tok[row];
  if (tok < 0 && last_tok) tok = last_tok[row_slot[row]];
  tok = min(max(tok, 0), vocab - 1);
  const bf16_t *e = embed + (int64_t)tok * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = (float)e[i];
    h[(int64_t)row * d + i] = v;
    ss += v * v;
  }
  ss = block_sum_256(ss);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256)
    a[(int64_t)row * d + i] = (__bf16)(h[(int64_t)row * d + i] * r * (float)g[i]);
}

template <int NW>
__device__ inline float block_sum(float v) {
  __shared__ float red[NW];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += red[w];
  return t;
}

// h[row] += sum_s parts[s][row]; a[row] = rmsnorm(h[row]) * g.  Partials are added in slice order.
// One workgroup of NT threads per row, NV 16-byte pieces per thread (NT * NV * 4 >= d); the row stays in
// registers between the two passes.
template <int NT, int NV>
__global__ __launch_bounds__(NT) void resid_rmsnorm_kernel(float *h, const float *parts, int splits,
                                                           const bf16_t *g, bf16_t *a, int n, int d, float eps) {
  const int row = blockIdx.x, d4 = d >> 2;
  float4 *h4 = (float4 *)(h + (int64_t)row * d);
  float4 v[NV];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int idx = threadIdx.x + it * NT;
    if (idx < d4) {
      float4 x = h4[idx];
      // loads of up to 8 slices are issued together, the adds stay in slice order
      for (int s0 = 0; s0 < splits; s0 += 8) {
        float4 p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (s0 + u < splits) p[u] = ((const float4 *)(parts + ((int64_t)(s0 + u) * n + row) * d))[idx];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (s0 + u < splits) { x.x += p[u].x; x.y += p[u].y; x.z += p[u].z; x.w += p[u].w; }
      }
      h4[idx] = x;
      v[it] = x;
      ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
  }
  ss = block_sum<NT / 64>(ss);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int idx = threadIdx.x + it * NT;
    if (idx < d4) {
      const bf16x4 gg = ((const bf16x4 *)g)[idx];
      bf16x4 o;
      o[0] = (__bf16)(v[it].x * r * (float)gg[0]);
      o[1] = (__bf16)(v[it].y * r * (float)gg[1]);
      o[2] = (__bf16)(v[it].z * r * (float)gg[2]);
      o[3] = (__bf16)(v[it].w * r * (float)gg[3]);
      ((bf16x4 *)(a + (int64_t)row * d))[idx] = o;
    }
  }
}

// cos/sin of pos * theta^(-2i/hd), evaluated in double so long positions lose nothing; also the
// attention length of the step (pos + 1).
__global__ void rope_tables_kernel(const int32_t *pos, float *cs, int32_t *ctx_len, int n, int hd, float theta) {
  const int half = hd / 2;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * half) return;
  const int row = idx / half, i = idx % half;
  const double inv_freq = pow((double)theta, -2.0 * (double)i / (double)hd);
  const double ang = (double)pos[row] * inv_freq;
  cs[(int64_t)row * hd + i] = (float)cos(ang);
  cs[(int64_t)row * hd + half + i] = (float)sin(ang);
  if (i == 0) ctx_len[row] = pos[row] + 1;
}

// qkv (fp32, split-K partials) -> rotated q (bf16), rotated k and v into the row's cache page.
// One thread per four consecutive rotated pairs (i .. i + 3 with their partners half + i ..), 16-byte
// loads; a workgroup of 256 threads covers 1024 consecutive pairs of one row, i.e. several heads of q|k|v.
__global__ __launch_bounds__(256) void rope_append_kernel(const float *qkv, int splits, const float *cs, const int32_t *pos,
                                                          const int32_t *row_slot, const int32_t *page_table, bf16_t *q_out,
                                                          bf16_t *kv_layer, int n, int Hq, int Hkv, int hd, int page_tokens,
                                                          int pages_per_seq) {
  const int half = hd / 2, quads = half / 4;
  const int quad = blockIdx.x * 256 + threadIdx.x;
  if (quad >= (Hq + 2 * Hkv) * quads) return;
  const int row = blockIdx.y, hh = quad / quads, i = (quad % quads) * 4;
  const int width = (Hq + 2 * Hkv) * hd;
  f32x4 x1 = {0.f, 0.f, 0.f, 0.f}, x2 = {0.f, 0.f, 0.f, 0.f};
  // loads of up to 8 slices are issued together, the adds stay in slice order
  for (int s0 = 0; s0 < splits; s0 += 8) {
    f32x4 p1[8], p2[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < splits) {
        const float *src = qkv + ((int64_t)(s0 + u) * n + row) * width + hh * hd;
        p1[u] = *(const f32x4 *)(src + i);
        p2[u] = *(const f32x4 *)(src + half + i);
      }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < splits) { x1 += p1[u]; x2 += p2[u]; }
  }
  bf16x4 lo, hi;   // elements i .. i + 3 and half + i .. half + i + 3 of the head
  if (hh < Hq + Hkv) {
    const f32x4 c = *(const f32x4 *)(cs + (int64_t)row * hd + i), sn = *(const f32x4 *)(cs + (int64_t)row * hd + half + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      lo[e] = (__bf16)(x1[e] * c[e] - x2[e] * sn[e]);
      hi[e] = (__bf16)(x2[e] * c[e] + x1[e] * sn[e]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) { lo[e] = (__bf16)x1[e]; hi[e] = (__bf16)x2[e]; }
  }
  if (hh < Hq) {
    bf16_t *q = q_out + ((int64_t)row * Hq + hh) * hd;
    *(bf16x4 *)(q + i) = lo;
    *(bf16x4 *)(q + half + i) = hi;
    return;
  }
  const int p = pos[row];
  const int page = page_table[(int64_t)row_slot[row] * pages_per_seq + p / page_tokens];
  const int t = p % page_tokens;
  const int64_t page_elems = (int64_t)2 * page_tokens * hd;
  if (hh < Hq + Hkv) {
    // four consecutive dims of a token (i is a multiple of 4) are contiguous in the K block
    bf16_t *kb = kv_layer + ((int64_t)page * Hkv + (hh - Hq)) * page_elems;
    *(bf16x4 *)(kb + k_elem_offset(t, i, hd)) = lo;
    *(bf16x4 *)(kb + k_elem_offset(t, half + i, hd)) = hi;
  } else {
    bf16_t *vb = kv_layer + ((int64_t)page * Hkv + (hh - Hq - Hkv)) * page_elems + (int64_t)page_tokens * hd;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vb[v_elem_offset(t, i + e, hd)] = lo[e];
      vb[v_elem_offset(t, half + i + e, hd)] = hi[e];
    }
  }
}

// Read-only stream over a buffer (16-byte loads, 8 independent loads in flight per lane): measures
// what HBM delivers to a kernel that does nothing but read.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ p, uint32_t *sink, int64_t n_per_wg) {
  const u32x4 *base = p + (int64_t)blockIdx.x * n_per_wg;
  u32x4 acc = {0, 0, 0, 0};
  for (int64_t i = threadIdx.x; i < n_per_wg; i += 256 * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = NT ? __builtin_nontemporal_load(&base[i + u * 256]) : base[i + u * 256];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && sink) sink[0] = 1;   // keeps the loads alive
}

// LM head tied to the embedding table: dst = the [vocab, d] row-major table in the layout the LM-head
// GEMM streams (bf16: MFMA operand order, 16-byte pieces of 8 consecutive columns; fp32 build: a plain copy).
__global__ void tie_lm_head_kernel(const bf16x8 *__restrict__ embed, bf16x8 *__restrict__ dst, int vocab, int d) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 8-column piece
  const int d8 = d >> 3;
  if (idx >= (int64_t)vocab * d8) return;
  const int r = (int)(idx / d8), c = (int)(idx % d8) * 8;
  const int64_t o = ((int64_t)(c / 64) * (vocab / 32) + r / 32) * 2048 + ((c % 32) / 8) * 512 + ((c % 64) / 32) * 256 + (r % 32) * 8;
  dst[o >> 3] = embed[idx];
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

}  // namespace

static inline int ok() { return hipGetLastError() == hipSuccess ? 0 : -7; }

int launch_embed_rmsnorm(const bf16_t *embed, const bf16_t *g, const int32_t *input_tok,
                         const int32_t *last_tok, const int32_t *row_slot, float *h, bf16_t *a, int n,
                         int d, int vocab, float eps, hipStream_t s) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(embed_rmsnorm_kernel, dim3(n), dim3(256), 0, s, embed, g, input_tok, last_tok, row_slot,
                     h, a, d, vocab, eps);
  return ok();
}

int launch_resid_rmsnorm(float *h, const float *parts, int splits, const bf16_t *g, bf16_t *a, int n, int d,
                         float eps, hipStream_t s) {
  if (n <= 0) return 0;
  // rows of up to 4096 floats: 1024 threads, one 16-byte piece each (all loads of a row in flight at
  // once); wider rows: 1024 threads x 2 pieces (d <= 8192)
  if (d <= 4096)
    hipLaunchKernelGGL((resid_rmsnorm_kernel<1024, 1>), dim3(n), dim3(1024), 0, s, h, parts, splits, g, a, n, d, eps);
  else
    hipLaunchKernelGGL((resid_rmsnorm_kernel<1024, 2>), dim3(n), dim3(1024), 0, s, h, parts, splits, g, a, n, d, eps);
  return ok();
}

int launch_rope_tables(const int32_t *pos, float *cs, int32_t *ctx_len, int n, int hd, float theta,
                       hipStream_t s) {
  if (n <= 0) return 0;
  int total = n * (hd / 2);
  hipLaunchKernelGGL(rope_tables_kernel, dim3((total + 255) / 256), dim3(256), 0, s, pos, cs, ctx_len, n, hd,
                     theta);
  return ok();
}

int launch_rope_append(const float *qkv, int splits, const float *cs, const int32_t *pos,
                       const int32_t *row_slot, const int32_t *page_table, bf16_t *q_out, bf16_t *kv_layer,
                       int n, int Hq, int Hkv, int hd, int page_tokens, int pages_per_seq, hipStream_t s) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(rope_append_kernel, dim3(((Hq + 2 * Hkv) * (hd / 8) + 255) / 256, n), dim3(256), 0, s, qkv, splits, cs, pos, row_slot,
                     page_table, q_out, kv_layer, n, Hq, Hkv, hd, page_tokens, pages_per_seq);
  return ok();
}

int64_t launch_stream_read(const void *p, int64_t nbytes, uint32_t *sink, bool nontemporal, hipStream_t s) {
  const int wgs = 8192;
  int64_t n_per_wg = nbytes / 16 / wgs / 2048 * 2048;
  if (n_per_wg <= 0) return 0;
  if (nontemporal)
    hipLaunchKernelGGL(stream_read_kernel<true>, dim3(wgs), dim3(256), 0, s, (const u32x4 *)p, sink, n_per_wg);
  else
    hipLaunchKernelGGL(stream_read_kernel<false>, dim3(wgs), dim3(256), 0, s, (const u32x4 *)p, sink, n_per_wg);
  return hipGetLastError() == hipSuccess ? n_per_wg * 16 * wgs : -7;
}

int launch_tie_lm_head(const void *embed, void *lm_head, int vocab, int d, bool f32, hipStream_t s) {
  if (f32) return hipMemcpyAsync(lm_head, embed, (size_t)vocab * d * 4, hipMemcpyDeviceToDevice, s) == hipSuccess ? 0 : -7;
  const int64_t pieces = (int64_t)vocab * (d / 8);
  hipLaunchKernelGGL(tie_lm_head_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, (const bf16x8 *)embed,
                     (bf16x8 *)lm_head, vocab, d);
  return ok();
}

int launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t s) {
  if (n <= 0) return 0;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, v, n);
  return ok();
}

}  // namespace pl
