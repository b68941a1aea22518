// Skinny-M bf16 GEMM y = x W^T for the decode projections (QKV, O, gate/up + SwiGLU, down, LM head).
//
// With M = batch <= 256 rows these products are bound by streaming W once from HBM; W is never
// reused across workgroups, so it bypasses LDS: every wavefront loads the W rows it owns straight
// into MFMA B-operand registers.  W is stored in operand order (blocks of 32 rows x 64 k, see
// pl_weight_layout in pl.h), so each of those loads is one contiguous KiB per wavefront.  The small activation tile x is what all workgroups share; it is staged through LDS
// (padded rows, conflict-free 16-byte reads) and feeds the A operand.  32x32x16 bf16 MFMAs
// accumulate in fp32.  K can be split across workgroups (partials summed by the consumer in a
// fixed order) so that narrow outputs still occupy every compute unit.
#include "pl_common.h"

#include <type_traits>

namespace pl {
namespace {

constexpr int BK = 64;          // k elements per main-loop step
constexpr int LDS_ROW = 72;     // padded row length (elements) of the x tile in LDS

// Workgroup = 4 wavefronts arranged WM x WN; each owns (AT*32) x (BT*32) outputs.
// Software pipeline: W fragments live in a 4-deep register ring (loads run three k-steps ahead of
// the MFMAs that consume them, which is what hides HBM latency with one wavefront per SIMD); the x
// tile runs two k-steps ahead through a 2-deep register stage and a double-buffered LDS tile.
// Within a k-step the x loads are issued before the W loads, so waiting for an x tile (in-order
// completion) never waits for the younger W loads.
template <int WM, int WN, int AT, int BT, int MODE>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W,
                                                   void *__restrict__ Yv, int M, int N, int K, int ksteps,
                                                   int n_base, int n_end, int nrow) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  constexpr int XCH = BM * (BK / 8) / 256;       // 16-byte chunks of the x tile per thread
  static_assert(WM * WN == 4 && XCH >= 1, "tile");
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][BM * LDS_ROW];

  const int tid = threadIdx.x, l = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps W offsets in scalar registers
  const int wm = wave / WN, wn = wave % WN;
  // Tile of this workgroup.  nrow = 0: (column tile, row tile) = (blockIdx.x, blockIdx.z).  nrow > 0:
  // a flat grid in which the row tiles of one column tile sit 8 workgroup ids apart, so the hardware's
  // round-robin deal of consecutive ids to the 8 XCDs puts them on the same XCD at the same moment
  // and the second reader of a W tile finds it in that XCD's L2.
  int ctile = blockIdx.x, rtile = blockIdx.z;
  if (nrow > 0) {
    rtile = (blockIdx.x >> 3) % nrow;
    ctile = (blockIdx.x / (8 * nrow)) * 8 + (blockIdx.x & 7);
    if (n_base + ctile * BN >= n_end) return;   // padding of the flat grid (uniform for the workgroup)
  }
  const int n0 = n_base + ctile * BN + wn * BT * 32;
  const int m0 = rtile * BM;
  const int split = blockIdx.y;
  const int kbeg = split * ksteps * BK;
  const int nks = min(ksteps, K / BK - split * ksteps);
  const int lrow = l & 31, half = l >> 5;

  // Buffer addressing: one resource per operand, a per-lane byte offset in a VGPR, everything that
  // is uniform across the wavefront in scalar registers; rows of x at or beyond M read as zeros.
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((int64_t)N * K * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)X, 0, (int)((int64_t)M * K * 2), 0x00020000);
  // operand-ordered W: block (k-step, n / 32) is 4096 bytes: [j][lane][16 B], lane = half * 32 + row.
  // Blocks are k-step-major: workgroups walk K in step, so at any moment the whole chip reads one
  // contiguous plane of W and the traffic spreads over every HBM channel (with row-block-major
  // order all streams sit a multiple of 8 blocks apart and camp on a fraction of the channels).
  const int w_lane = l * 16;
  const uint32_t w_plane = (uint32_t)(N >> 5) * 4096u;
  uint32_t w_blk[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt)
    w_blk[bt] = (uint32_t)(split * ksteps) * w_plane + (uint32_t)min((n0 >> 5) + bt, (N >> 5) - 1) * 4096u;
  // x tile: 16-byte chunk ch = tid + 256 i is row ch / 8, k columns (ch % 8) * 8
  const int x_lane = ((m0 + (tid >> 3)) * K + kbeg + (tid & 7) * 8) * 2;
  const int x_lds = (tid >> 3) * LDS_ROW + (tid & 7) * 8;

  f32x16 acc[AT][BT];
#pragma unroll
  for (int a = 0; a < AT; ++a)
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  bf16x8 wf[4][BT][4], xr[2][XCH];
  auto load_w = [&](int stage, int ks) {
#pragma unroll
    for (int bt = 0; bt < BT; ++bt)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        wf[stage][bt][j] = __builtin_bit_cast(
            bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rw, w_lane + j * 1024, (int)(w_blk[bt] + (uint32_t)ks * w_plane), 0));
  };
  auto load_x = [&](int stage, int ks) {
#pragma unroll
    for (int i = 0; i < XCH; ++i)
      xr[stage][i] = __builtin_bit_cast(
          bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rx, x_lane, ks * (BK * 2) + i * 64 * K, 0));
  };
  auto store_x = [&](int stage, int buf) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) *(bf16x8 *)(&xs[buf][x_lds + i * 32 * LDS_ROW]) = xr[stage][i];
  };

  // nks is a multiple of 4 and at least 4 (the host splits K in units of 4 k-steps)
  load_x(0, 0);
  load_w(0, 0);
  load_x(1, 1);
  load_w(1, 1);
  load_w(2, 2);
  store_x(0, 0);
  __syncthreads();

  const int a_off = (wm * AT * 32 + lrow) * LDS_ROW + half * 32;
  // one k-step: u = k-step index mod 4 (compile time), LX/LW/SX say which transfers are still needed
  // Scheduling-group fences: the loads and LDS stores of a k-step are issued one at a time between
  // MFMAs instead of in a burst, so the memory pipeline fills while the matrix pipeline stays busy.
#define PL_SG_MFMA 0x008
#define PL_SG_VMEM_READ 0x020
#define PL_SG_DS_WRITE 0x200
  auto kstep = [&](auto U, auto LX, auto LW, auto SX, int ks) {
    constexpr int u = decltype(U)::value;
    // A fragments are read from LDS two 16-wide k-slices ahead of the MFMAs that use them (a
    // 2-deep register ring); the fences pin that order.
    bf16x8 af[2][AT];
    auto read_a = [&](int j) {
#pragma unroll
      for (int a = 0; a < AT; ++a) af[j & 1][a] = *(const bf16x8 *)(&xs[u & 1][a_off + a * 32 * LDS_ROW + j * 8]);
    };
    auto mma = [&](int j) {
#pragma unroll
      for (int a = 0; a < AT; ++a)
#pragma unroll
        for (int b = 0; b < BT; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[j & 1][a], wf[u][b][j], acc[a][b], 0, 0, 0);
    };
    read_a(0);
    read_a(1);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(LX)::value) load_x(u & 1, ks + 2);     // x before W: waiting for x never waits for W
    mma(0);
    if constexpr (decltype(LX)::value) {
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        __builtin_amdgcn_sched_group_barrier(PL_SG_MFMA, (AT * BT) / XCH > 0 ? (AT * BT) / XCH : 1, 0);
        __builtin_amdgcn_sched_group_barrier(PL_SG_VMEM_READ, 1, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    read_a(2);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(LW)::value) load_w((u + 3) & 3, ks + 3);
    mma(1);
    if constexpr (decltype(LW)::value) {
#pragma unroll
      for (int i = 0; i < BT * 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(PL_SG_MFMA, (AT * BT) / (BT * 4) > 0 ? (AT * BT) / (BT * 4) : 1, 0);
        __builtin_amdgcn_sched_group_barrier(PL_SG_VMEM_READ, 1, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    read_a(3);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(SX)::value) store_x((u + 1) & 1, (u + 1) & 1);
    mma(2);
    mma(3);
    if constexpr (decltype(SX)::value) {
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        __builtin_amdgcn_sched_group_barrier(PL_SG_MFMA, (2 * AT * BT) / XCH > 0 ? (2 * AT * BT) / XCH : 1, 0);
        __builtin_amdgcn_sched_group_barrier(PL_SG_DS_WRITE, 1, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  };
  using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
  using Y = std::true_type; using No = std::false_type;
  int ks = 0;
  for (; ks < nks - 4; ks += 4) {
    kstep(I0{}, Y{}, Y{}, Y{}, ks);
    kstep(I1{}, Y{}, Y{}, Y{}, ks + 1);
    kstep(I2{}, Y{}, Y{}, Y{}, ks + 2);
    kstep(I3{}, Y{}, Y{}, Y{}, ks + 3);
  }
  kstep(I0{}, Y{}, Y{}, Y{}, ks);
  kstep(I1{}, Y{}, No{}, Y{}, ks + 1);
  kstep(I2{}, No{}, No{}, Y{}, ks + 2);
  kstep(I3{}, No{}, No{}, No{}, ks + 3);

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

// Launch over output columns [n_begin, n_end) (multiples of the tile width, except the matrix edge).
template <int WM, int WN, int AT, int BT>
int launch_cfg(const bf16_t *x, const bf16_t *w, void *y, int M, int N, int K, int mode, int splits,
               int n_begin, int n_end, hipStream_t s, bool paired = false) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  if (n_end <= n_begin) return 0;
  dim3 grid((n_end - n_begin + BN - 1) / BN, splits, (M + BM - 1) / BM);
  int nrow = 0;
  if (paired) {   // flat grid, column tiles padded to a multiple of 8 (see the kernel)
    nrow = grid.z;
    grid.x = ((grid.x + 7) / 8) * 8 * nrow;
    grid.z = 1;
  }
  int ksteps = 4 * ((K / (4 * BK) + splits - 1) / splits);
  if (mode == 0)
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, BT, 0>), grid, dim3(256), 0, s, x, w, y, M, N, K, ksteps, n_begin,
                       n_end, nrow);
  else
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, BT, 1>), grid, dim3(256), 0, s, x, w, y, M, N, K, ksteps, n_begin,
                       n_end, nrow);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace

int gemm_pick_splits(int M, int N, int K) {
  // One workgroup fits on a compute unit: split K so that the output tiles times the number of
  // slices comes close to, but not above, the 256 units, with at least 4 k-steps per slice.
  int total = K / (4 * BK), best = 1;   // slices are made of groups of 4 k-steps
  // Short K at 129..256 rows: 128 x 128 tiles, two workgroups per unit, four slices (measured best
  // for the QKV and O projections of the 7B shape: fewer partial sums to write and to add up).
  if (M > 128 && M <= 256 && K <= 4096 && total >= 4 && 3 * ((total + 3) / 4) < total) return 4;
  int bn = M > 128 ? 128 : 256;
  int tiles = ((N + bn - 1) / bn) * ((M + 255) / 256);
  for (int s = 2; s <= 32 && tiles * s <= 256; ++s) {
    int c = (total + s - 1) / s;
    if ((s - 1) * c >= total) continue;   // slices must be non-empty
    best = s;
  }
  return best;
}

int launch_gemm(const bf16_t *x, const bf16_t *w, void *y, int M, int N, int K, int mode, int splits,
                hipStream_t s) {
  if (M < 1 || M > 512 || K % (4 * BK) || N % 32 || splits < 1 || splits > K / (4 * BK)) return -1;
  if ((splits - 1) * ((K / (4 * BK) + splits - 1) / splits) >= K / (4 * BK)) return -1;   // an empty slice
  if (mode == 1 && (splits != 1 || N % 64)) return -1;
  if (mode != 0 && mode != 1) return -1;
  // beyond this the descriptor's size field and the 32-bit offsets wrap and loads read zeros
  if ((int64_t)N * K * 2 >= GEMM_MAX_OPERAND_BYTES || (int64_t)M * K * 2 >= GEMM_MAX_OPERAND_BYTES) return -1;
  if (M <= 32) return launch_cfg<1, 4, 1, 2>(x, w, y, M, N, K, mode, splits, 0, N, s);
  if (M <= 64) return launch_cfg<1, 4, 2, 2>(x, w, y, M, N, K, mode, splits, 0, N, s);
  if (M <= 128) return launch_cfg<1, 4, 4, 2>(x, w, y, M, N, K, mode, splits, 0, N, s);
  if (M <= 256 && splits == 1 && N >= 128 * 256) {
    // Wide matrices without a K split: 128 x 256 tiles in XCD-local pairs.  Each wavefront owns its
    // own 64 columns of W (no fragment is loaded twice by one workgroup) and the x tile is half as
    // tall, which cuts the vector-memory and LDS-store traffic per MFMA; the second row tile reads W
    // from L2.  When the tile count is a little over a multiple of 256 the last round would run on a
    // few units at full length: those columns go to a second launch of 64 x 128 tiles instead.
    const int ctiles = (N + 255) / 256, tiles = 2 * ctiles, rem = tiles % 256;
    if (tiles > 256 && rem > 0 && rem <= 64) {
      const int n_main = ((tiles - rem) / 2) * 256;
      int rc = launch_cfg<1, 4, 4, 2>(x, w, y, M, N, K, mode, splits, 0, n_main, s, true);
      return rc ? rc : launch_cfg<2, 2, 1, 2>(x, w, y, M, N, K, mode, splits, n_main, N, s);
    }
    return launch_cfg<1, 4, 4, 2>(x, w, y, M, N, K, mode, splits, 0, N, s, true);
  }
  if (M <= 256 && splits > 1 && K <= 4096) return launch_cfg<2, 2, 2, 2>(x, w, y, M, N, K, mode, splits, 0, N, s);
  // otherwise 256 x 128 tiles, one per compute unit and round
  return launch_cfg<2, 2, 4, 2>(x, w, y, M, N, K, mode, splits, 0, N, s);
}

}  // namespace pl
