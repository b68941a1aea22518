// Trainer-side consumer of the recorded behaviour log-probs (Sec. 2.1 of the paper): truncated
// token-level importance weights w = min(c, pi / mu) and the normalised effective sample size
// (sum w)^2 / (N sum w^2), per packed sequence and over the whole batch.  A stream of 8 bytes in and
// 4 bytes out per token; all arithmetic in fp64, reductions in a fixed order (no atomics), so the
// result does not depend on scheduling.
#include "pl_common.h"

namespace pl {
namespace {

template <int NW>
__device__ inline void block_sum2(double &a, double &b, double *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_xor(a, o, 64);
    b += __shfl_xor(b, o, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[2 * wave] = a; red[2 * wave + 1] = b; }
  __syncthreads();
  a = 0.0; b = 0.0;
  for (int w = 0; w < NW; ++w) { a += red[2 * w]; b += red[2 * w + 1]; }
}

// one workgroup per sequence: tokens [offsets[s], offsets[s + 1])
__global__ __launch_bounds__(256) void is_seq_kernel(const float *__restrict__ lp_pi, const float *__restrict__ lp_mu,
                                                     const int64_t *__restrict__ offsets, double c,
                                                     float *__restrict__ w_out, double *__restrict__ seq_sums,
                                                     double *__restrict__ ess_seq) {
  __shared__ double red[8];
  const int s = blockIdx.x;
  const int64_t a = offsets[s], b = offsets[s + 1];
  double s1 = 0.0, s2 = 0.0;
  for (int64_t i0 = a + threadIdx.x; i0 < b; i0 += 4 * 256) {
    float p[4], m[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + u * 256;
      if (i < b) { p[u] = lp_pi[i]; m[u] = lp_mu[i]; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + u * 256;
      if (i < b) {
        const double w = fmin(c, exp((double)p[u] - (double)m[u]));
        if (w_out) w_out[i] = (float)w;
        s1 += w;
        s2 += w * w;
      }
    }
  }
  block_sum2<4>(s1, s2, red);
  if (threadIdx.x == 0) {
    seq_sums[2 * s] = s1;
    seq_sums[2 * s + 1] = s2;
    ess_seq[s] = b > a ? s1 * s1 / ((double)(b - a) * s2) : __longlong_as_double(0x7FF8000000000000LL);
  }
}

// totals[0..2] = sum w, sum w^2, normalised ESS over all tokens; one workgroup, fixed order
__global__ __launch_bounds__(1024) void is_total_kernel(const double *__restrict__ seq_sums,
                                                        const int64_t *__restrict__ offsets, int n_seq,
                                                        double *__restrict__ totals) {
  __shared__ double red[32];
  double s1 = 0.0, s2 = 0.0;
  for (int s = threadIdx.x; s < n_seq; s += 1024) { s1 += seq_sums[2 * s]; s2 += seq_sums[2 * s + 1]; }
  block_sum2<16>(s1, s2, red);
  if (threadIdx.x == 0) {
    const int64_t n = offsets[n_seq] - offsets[0];
    totals[0] = s1;
    totals[1] = s2;
    totals[2] = n > 0 ? s1 * s1 / ((double)n * s2) : __longlong_as_double(0x7FF8000000000000LL);
  }
}

}  // namespace

int launch_is_ess(const float *lp_pi, const float *lp_mu, const int64_t *offsets, int n_seq, double c, float *w_out,
                  double *seq_sums, double *ess_seq, double *totals, hipStream_t s) {
  if (n_seq < 1) return -1;
  hipLaunchKernelGGL(is_seq_kernel, dim3(n_seq), dim3(256), 0, s, lp_pi, lp_mu, offsets, c, w_out, seq_sums, ess_seq);
  hipLaunchKernelGGL(is_total_kernel, dim3(1), dim3(1024), 0, s, seq_sums, offsets, n_seq, totals);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace pl
