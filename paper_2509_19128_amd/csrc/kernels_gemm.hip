// Skinny-M bf16 GEMM y = x W^T for the decode projections (QKV, O, gate/up + SwiGLU, down, LM head).
//
// With M = batch <= 256 rows these products are bound by streaming W once from HBM; W is never
// reused across workgroups, so it bypasses LDS: every wavefront loads the W rows it owns straight
// into MFMA B-operand registers (each lane reads 64 contiguous bytes of one row per 64-wide k
// step).  The small activation tile x is what all workgroups share; it is staged through LDS
// (padded rows, conflict-free 16-byte reads) and feeds the A operand.  32x32x16 bf16 MFMAs
// accumulate in fp32.  K can be split across workgroups (partials summed by the consumer in a
// fixed order) so that narrow outputs still occupy every compute unit.
#include "pl_common.h"

namespace pl {
namespace {

constexpr int BK = 64;          // k elements per main-loop step
constexpr int LDS_ROW = 72;     // padded row length (elements) of the x tile in LDS

// Workgroup = 4 wavefronts arranged WM x WN; each owns (AT*32) x (BT*32) outputs.
template <int WM, int WN, int AT, int BT, int MODE>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W,
                                                   void *__restrict__ Yv, int M, int N, int K, int ksteps) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  constexpr int XCH = BM * (BK / 8) / 256;       // 16-byte chunks of the x tile per thread
  static_assert(WM * WN == 4 && XCH >= 1, "tile");
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][BM * LDS_ROW];

  const int tid = threadIdx.x, wave = tid >> 6, l = tid & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int n0 = blockIdx.x * BN + wn * BT * 32;
  const int m0 = blockIdx.z * BM;
  const int split = blockIdx.y;
  const int kbeg = split * ksteps * BK;
  const int lrow = l & 31, half = l >> 5;

  const bf16_t *wp[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) {
    int n = min(n0 + bt * 32 + lrow, N - 1);
    wp[bt] = W + (int64_t)n * K + kbeg + half * 32;
  }
  const bf16_t *xp[XCH];
  int xoff[XCH];
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    int ch = tid + i * 256, row = ch >> 3, col = (ch & 7) * 8;
    xp[i] = X + (int64_t)min(m0 + row, M - 1) * K + kbeg + col;
    xoff[i] = row * LDS_ROW + col;
  }

  f32x16 acc[AT][BT];
#pragma unroll
  for (int a = 0; a < AT; ++a)
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  bf16x8 wf[BT][4], xr[XCH];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt)
#pragma unroll
    for (int j = 0; j < 4; ++j) wf[bt][j] = *(const bf16x8 *)(wp[bt] + j * 8);
#pragma unroll
  for (int i = 0; i < XCH; ++i) xr[i] = *(const bf16x8 *)xp[i];
#pragma unroll
  for (int i = 0; i < XCH; ++i) *(bf16x8 *)(&xs[0][xoff[i]]) = xr[i];
  __syncthreads();

  const int a_off = (wm * AT * 32 + lrow) * LDS_ROW + half * 32;
  for (int ks = 0; ks < ksteps; ++ks) {
    const int cur = ks & 1;
    bf16x8 wc[BT][4];
#pragma unroll
    for (int bt = 0; bt < BT; ++bt)
#pragma unroll
      for (int j = 0; j < 4; ++j) wc[bt][j] = wf[bt][j];
    const bool more = ks + 1 < ksteps;
    if (more) {
      const int ko = (ks + 1) * BK;
#pragma unroll
      for (int bt = 0; bt < BT; ++bt)
#pragma unroll
        for (int j = 0; j < 4; ++j) wf[bt][j] = *(const bf16x8 *)(wp[bt] + ko + j * 8);
#pragma unroll
      for (int i = 0; i < XCH; ++i) xr[i] = *(const bf16x8 *)(xp[i] + ko);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int a = 0; a < AT; ++a) {
        bf16x8 af = *(const bf16x8 *)(&xs[cur][a_off + a * 32 * LDS_ROW + j * 8]);
#pragma unroll
        for (int b = 0; b < BT; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, wc[b][j], acc[a][b], 0, 0, 0);
      }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < XCH; ++i) *(bf16x8 *)(&xs[cur ^ 1][xoff[i]]) = xr[i];
    }
    __syncthreads();
  }

  // epilogue: accumulator register i of lane l is row (i/4)*8 + (l/32)*4 + i%4, column l%32
#pragma unroll
  for (int a = 0; a < AT; ++a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0 + wm * AT * 32 + a * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
      if (m >= M) continue;
      if (MODE == 0) {
        float *Y = (float *)Yv + ((int64_t)split * M + m) * N;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          int n = n0 + b * 32 + lrow;
          if (n < N) Y[n] = acc[a][b][i];
        }
      } else {
        // SwiGLU: the two column tiles of a wavefront are the gate and the up half of a 64-row block
        bf16_t *Y = (bf16_t *)Yv + (int64_t)m * (N / 2);
        int n = n0 + lrow;
        if (n < N) {
          float gte = acc[a][0][i], up = acc[a][BT - 1][i];
          float sv = gte / (1.f + __expf(-gte));
          Y[(n0 >> 1) + lrow] = (__bf16)(sv * up);
        }
      }
    }
  }
}

template <int WM, int WN, int AT, int BT>
int launch_cfg(const bf16_t *x, const bf16_t *w, void *y, int M, int N, int K, int mode, int splits,
               hipStream_t s) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  dim3 grid((N + BN - 1) / BN, splits, (M + BM - 1) / BM);
  int ksteps = K / BK / splits;
  if (mode == 0)
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, BT, 0>), grid, dim3(256), 0, s, x, w, y, M, N, K, ksteps);
  else
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, BT, 1>), grid, dim3(256), 0, s, x, w, y, M, N, K, ksteps);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace

int gemm_pick_splits(int M, int N, int K) {
  // Enough workgroups for every compute unit (about two per unit), never fewer than 4 k-steps each.
  int bn = M > 128 ? 128 : 256;
  int tiles = ((N + bn - 1) / bn) * ((M + 255) / 256);
  int ksteps = K / BK, best = 1;
  for (int s = 1; s <= 32 && s <= ksteps; ++s) {
    if (ksteps % s) continue;
    if (ksteps / s < 4 && s > 1) break;
    best = s;
    if (tiles * s >= 480) break;
  }
  return best;
}

int launch_gemm(const bf16_t *x, const bf16_t *w, void *y, int M, int N, int K, int mode, int splits,
                hipStream_t s) {
  if (M < 1 || M > 512 || K % BK || N % 32 || splits < 1 || (K / BK) % splits) return -1;
  if (mode == 1 && (splits != 1 || N % 64)) return -1;
  if (mode != 0 && mode != 1) return -1;
  if (M <= 32) return launch_cfg<1, 4, 1, 2>(x, w, y, M, N, K, mode, splits, s);
  if (M <= 64) return launch_cfg<1, 4, 2, 2>(x, w, y, M, N, K, mode, splits, s);
  if (M <= 128) return launch_cfg<1, 4, 4, 2>(x, w, y, M, N, K, mode, splits, s);
  return launch_cfg<2, 2, 4, 2>(x, w, y, M, N, K, mode, splits, s);
}

}  // namespace pl
