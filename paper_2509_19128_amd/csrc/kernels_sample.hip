// Fused log-softmax + Gumbel-max sampler over fp32 logits.
//
// Each step draws y ~ softmax(logits / T) (Sec. 2.1 eq. 1 of the paper) and records
// log softmax(logits / T)[y], the behaviour log-prob the trainer's truncated importance weights
// divide by.  The draw is argmax_i (z_i + g_i) with g_i = -log(-log u_i) and u_i from
// Philox4x32-10 keyed by (seed; vocabulary index / 4, position, sequence id).  The decision is made
// in fp32 with a fixed operation order (plain multiplies and adds, no fused multiply-add: this file
// is compiled with floating-point contraction off), so it can be reproduced exactly elsewhere:
//   u = (2 (bits >> 9) + 1) 2^-24;  z = logit * inv_T;  y = z + -LOG(-LOG(u));  lowest index wins ties
//   LOG(x): e = exponent - 127, m = mantissa in [1,2); if bits(m) > 0x3FB504F3 { m *= 0.5; e += 1 }
//           f = m - 1; p = C8; p = p f + Cj (j = 7..0); f2 = f f; r = (f2 f) p; r += -0.5 f2;
//           r += e LN2_LO; r += f; LOG = e LN2_HI + r
// One pass over the logits: every workgroup scans a slice of one row keeping (max z, sum exp,
// best y, its index); a second small kernel merges the slices of a row in slice order.
#include "pl_common.h"

#include <mutex>
#pragma clang fp contract(off)

namespace pl {
namespace {

constexpr int SLICE = 8192;   // vocabulary entries per workgroup

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                     uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline float spec_log(float x) {
#pragma clang fp contract(off)
  const uint32_t bits = __float_as_uint(x);
  int e = (int)(bits >> 23) - 127;
  uint32_t mb = (bits & 0x007FFFFFu) | 0x3F800000u;
  float m = __uint_as_float(mb);
  if (mb > 0x3FB504F3u) { m = m * 0.5f; e += 1; }
  const float f = m - 1.0f;
  const float C[9] = {__uint_as_float(0x3EAAAAAAu), __uint_as_float(0xBE7FFFFEu), __uint_as_float(0x3E4CCEADu),
                      __uint_as_float(0xBE2AADA5u), __uint_as_float(0x3E11E90Du), __uint_as_float(0xBDFE7A63u),
                      __uint_as_float(0x3DEF5141u), __uint_as_float(0xBDEB1ADEu), __uint_as_float(0x3D8EC753u)};
  float p = C[8];
#pragma unroll
  for (int j = 7; j >= 0; --j) {
    p = __fmul_rn(p, f);
    p = __fadd_rn(p, C[j]);
  }
  const float f2 = __fmul_rn(f, f);
  float r = __fmul_rn(__fmul_rn(f2, f), p);
  r = __fadd_rn(r, __fmul_rn(-0.5f, f2));
  const float ef = (float)e;
  r = __fadd_rn(r, __fmul_rn(ef, __uint_as_float(0x35BFBE8Eu)));
  r = __fadd_rn(r, f);
  return __fadd_rn(__fmul_rn(ef, __uint_as_float(0x3F317200u)), r);
}

__device__ inline float gumbel(uint32_t bits) {
  const float k = (float)(bits >> 9);
  const float u = __fmul_rn(__fadd_rn(__fmul_rn(k, 2.0f), 1.0f), 5.9604644775390625e-08f);
  return -spec_log(-spec_log(u));
}

struct Part { float mx, sum, besty; int32_t besti; };

__device__ inline void merge_best(float &by, int &bi, float y, int i) {
  if (y > by || (y == by && i < bi)) { by = y; bi = i; }
}

__global__ __launch_bounds__(256) void sample_slice_kernel(SampleParams p, int nslice) {
  const int row = blockIdx.y, sl = blockIdx.x;
  const float *lg = p.logits + (int64_t)row * p.vocab;
  const float inv_t = p.inv_t[row];
  const uint64_t sid = p.seq_id[row];
  const uint32_t pos = (uint32_t)p.position[row];
  const uint32_t k0 = (uint32_t)p.seed, k1 = (uint32_t)(p.seed >> 32);
  const int beg = sl * SLICE, end = min(p.vocab, beg + SLICE);
  float mx = -INFINITY, sum = 0.f, by = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int i4 = beg / 4 + threadIdx.x; i4 * 4 < end; i4 += 256) {
    uint32_t rnd[4];
    philox4x32_10((uint32_t)i4, pos, (uint32_t)sid, (uint32_t)(sid >> 32), k0, k1, rnd);
    float zv[4];
    if (i4 * 4 + 3 < end) {
      const float4 v = *(const float4 *)(lg + i4 * 4);
      zv[0] = v.x; zv[1] = v.y; zv[2] = v.z; zv[3] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) zv[e] = (i4 * 4 + e < end) ? lg[i4 * 4 + e] : -INFINITY;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = i4 * 4 + e;
      if (i >= end) continue;
      const float z = __fmul_rn(zv[e], inv_t);
      const float y = __fadd_rn(z, gumbel(rnd[e]));
      merge_best(by, bi, y, i);
      if (z > mx) { sum = sum * __expf(mx - z) + 1.f; mx = z; }
      else sum += __expf(z - mx);
    }
  }
  // workgroup reduction
  __shared__ Part sm[256];
  sm[threadIdx.x] = Part{mx, sum, by, bi};
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      Part a = sm[threadIdx.x], b = sm[threadIdx.x + o];
      const float M = fmaxf(a.mx, b.mx);
      float s = 0.f;
      if (a.mx > -INFINITY) s += a.sum * __expf(a.mx - M);
      if (b.mx > -INFINITY) s += b.sum * __expf(b.mx - M);
      int ai = a.besti; float ay = a.besty;
      merge_best(ay, ai, b.besty, b.besti);
      sm[threadIdx.x] = Part{M, s, ay, ai};
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) ((Part *)p.workspace)[(int64_t)row * nslice + sl] = sm[0];
}

__global__ void sample_merge_kernel(SampleParams p, int nslice) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= p.n) return;
  const Part *pp = (const Part *)p.workspace + (int64_t)row * nslice;
  float M = -INFINITY;
  for (int s = 0; s < nslice; ++s) M = fmaxf(M, pp[s].mx);
  float sum = 0.f, by = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int s = 0; s < nslice; ++s) {
    if (pp[s].mx > -INFINITY) sum += pp[s].sum * __expf(pp[s].mx - M);
    merge_best(by, bi, pp[s].besty, pp[s].besti);
  }
  int tok = p.forced ? p.forced[row] : -1;
  if (tok < 0) tok = bi;
  tok = min(max(tok, 0), p.vocab - 1);
  const float z = __fmul_rn(p.logits[(int64_t)row * p.vocab + tok], p.inv_t[row]);
  p.token[row] = tok;
  p.logprob[row] = (z - M) - logf(sum);
  if (p.last_tok) p.last_tok[p.row_slot[row]] = tok;
}

}  // namespace

// ---- slice partials kept in the library's own device memory, for callers that cannot allocate ------
namespace {
constexpr int STATIC_MAX_ROWS = 512, STATIC_MAX_VOCAB = 262144;
constexpr int64_t STATIC_SCRATCH_BYTES = (int64_t)STATIC_MAX_ROWS * (STATIC_MAX_VOCAB / SLICE) * (int64_t)sizeof(Part);   // 256 KiB
// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress: the address kernels use is looked up once per device below.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mu;
}  // namespace

// Device address of the current device's scratch array (looked up on the first call on that device)
// and the largest launch it serves.  Returns 0, -1 if the shape does not fit, -7 on a HIP error.
int sample_static_workspace(int n, int vocab, void **ptr) {
  if (n < 1 || n > STATIC_MAX_ROWS || vocab < 1 || vocab > STATIC_MAX_VOCAB ||
      sample_workspace_bytes(n, vocab) > STATIC_SCRATCH_BYTES)
    return -1;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return -7;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return -7;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return 0;
}
void sample_static_limits(int *max_rows, int *max_vocab) { *max_rows = STATIC_MAX_ROWS; *max_vocab = STATIC_MAX_VOCAB; }

int64_t sample_workspace_bytes(int n, int vocab) {
  return (int64_t)n * ((vocab + SLICE - 1) / SLICE) * (int64_t)sizeof(Part);
}

int launch_sample(const SampleParams &p, hipStream_t s) {
  if (p.n <= 0) return 0;
  if (p.vocab % 4) return -1;
  const int nslice = (p.vocab + SLICE - 1) / SLICE;
  hipLaunchKernelGGL(sample_slice_kernel, dim3(nslice, p.n), dim3(256), 0, s, p, nslice);
  hipLaunchKernelGGL(sample_merge_kernel, dim3((p.n + 63) / 64), dim3(64), 0, s, p, nslice);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace pl
