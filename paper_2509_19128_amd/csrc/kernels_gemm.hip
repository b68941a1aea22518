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

#include <algorithm>
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
//
// gemm_tile computes one tile (column tile at n_tile0, rows from m0, K slice `split`) with the whole
// workgroup; the kernels below are thin wrappers that pick the tile(s) of a workgroup.
template <int WM, int WN, int AT, int BT, int MODE>
__device__ __forceinline__ void gemm_tile(bf16_t (*xs)[WM * AT * 32 * LDS_ROW], const bf16_t *__restrict__ X,
                                          const bf16_t *__restrict__ W, void *__restrict__ Yv, int M, int N, int K,
                                          int ksteps, int n_tile0, int m0, int split, int n_end, int ldy, int y_col0) {
  constexpr int BM = WM * AT * 32;
  constexpr int XCH = BM * (BK / 8) / 256;       // 16-byte chunks of the x tile per thread
  static_assert(WM * WN == 4 && XCH >= 1, "tile");
  const int tid = threadIdx.x, l = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps W offsets in scalar registers
  const int wm = wave / WN, wn = wave % WN;
  const int n0 = n_tile0 + wn * BT * 32;
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
        // partial sums of slice `split`: row stride ldy, columns counted from y_col0
        float *Y = (float *)Yv + ((int64_t)split * M + m) * ldy - y_col0;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          int n = n0 + b * 32 + lrow;
          if (n < n_end) Y[n] = acc[a][b][i];
        }
      } else {
        // SwiGLU: the two column tiles of a wavefront are the gate and the up half of a 64-row block
        bf16_t *Y = (bf16_t *)Yv + (int64_t)m * (N / 2);
        int n = n0 + lrow;
        if (n < n_end) {
          float gte = acc[a][0][i], up = acc[a][BT - 1][i];
          float sv = gte / (1.f + __expf(-gte));
          Y[(n0 >> 1) + lrow] = (__bf16)(sv * up);
        }
      }
    }
  }
}

// Two tiles back to back in one workgroup without draining the pipeline between them: tile A (all of
// K, SwiGLU epilogue into mid, columns below n_main) and then K slice `split` of tile B (fp32 partial
// sums into ws, as gemm_tile<MODE 0> writes them).  The last k-steps of A, which have nothing of their
// own left to load, issue the first loads of B into the ring slots they free, so B starts with its
// operands already on the way while A's epilogue runs.  Same k order per output element as gemm_tile.
// K / BK and B's k-step count are multiples of 4 and at least 4.
template <int WM, int WN, int AT, int BT>
__device__ __forceinline__ void gemm_tile2(bf16_t (*xs)[WM * AT * 32 * LDS_ROW], const bf16_t *__restrict__ X,
                                           const bf16_t *__restrict__ W, bf16_t *__restrict__ mid, float *__restrict__ ws,
                                           int M, int N, int K, int n_tileA, int m0A, int n_main, int n_tileB, int m0B,
                                           int split, int kstepsB) {
  constexpr int BM = WM * AT * 32;
  constexpr int XCH = BM * (BK / 8) / 256;
  static_assert(WM * WN == 4 && XCH >= 1 && BT == 2, "tile");
  const int tid = threadIdx.x, l = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int n0A = n_tileA + wn * BT * 32, n0B = n_tileB + wn * BT * 32;
  const int nksA = K / BK;
  const int nksB = min(kstepsB, K / BK - split * kstepsB);
  const int lrow = l & 31, half = l >> 5;
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((int64_t)N * K * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)X, 0, (int)((int64_t)M * K * 2), 0x00020000);
  const int w_lane = l * 16;
  const uint32_t w_plane = (uint32_t)(N >> 5) * 4096u;
  uint32_t w_blkA[BT], w_blkB[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) {
    w_blkA[bt] = (uint32_t)min((n0A >> 5) + bt, (N >> 5) - 1) * 4096u;
    w_blkB[bt] = (uint32_t)(split * kstepsB) * w_plane + (uint32_t)min((n0B >> 5) + bt, (N >> 5) - 1) * 4096u;
  }
  const int x_laneA = ((m0A + (tid >> 3)) * K + (tid & 7) * 8) * 2;
  const int x_laneB = ((m0B + (tid >> 3)) * K + split * kstepsB * BK + (tid & 7) * 8) * 2;
  const int x_lds = (tid >> 3) * LDS_ROW + (tid & 7) * 8;

  f32x16 acc[AT][BT];
  auto zero_acc = [&]() {
#pragma unroll
    for (int a = 0; a < AT; ++a)
#pragma unroll
      for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  };
  zero_acc();

  bf16x8 wf[4][BT][4], xr[2][XCH];
  // SEG: 1 = tile A, 2 = tile B
  auto load_w = [&](auto SEG, int stage, int ks) {
#pragma unroll
    for (int bt = 0; bt < BT; ++bt)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        wf[stage][bt][j] = __builtin_bit_cast(
            bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                        rw, w_lane + j * 1024, (int)((decltype(SEG)::value == 1 ? w_blkA[bt] : w_blkB[bt]) + (uint32_t)ks * w_plane), 0));
  };
  auto load_x = [&](auto SEG, int stage, int ks) {
#pragma unroll
    for (int i = 0; i < XCH; ++i)
      xr[stage][i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                                                    rx, decltype(SEG)::value == 1 ? x_laneA : x_laneB, ks * (BK * 2) + i * 64 * K, 0));
  };
  auto store_x = [&](int stage, int buf) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) *(bf16x8 *)(&xs[buf][x_lds + i * 32 * LDS_ROW]) = xr[stage][i];
  };
  using S0 = std::integral_constant<int, 0>; using S1 = std::integral_constant<int, 1>; using S2 = std::integral_constant<int, 2>;
  using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
  using Y = std::true_type; using No = std::false_type;

  load_x(S1{}, 0, 0);
  load_w(S1{}, 0, 0);
  load_x(S1{}, 1, 1);
  load_w(S1{}, 1, 1);
  load_w(S1{}, 2, 2);
  store_x(0, 0);
  __syncthreads();

  const int a_off = (wm * AT * 32 + lrow) * LDS_ROW + half * 32;
  // one k-step in ring slot u; LX / LW: segment whose x tile (k-step ksx) / W tiles (k-step ksw) are
  // loaded meanwhile (S0: none); SX: whether the x tile loaded one step earlier goes to LDS
  auto kstep = [&](auto U, auto LX, auto LW, auto SX, int ksx, int ksw) {
    constexpr int u = decltype(U)::value;
    constexpr bool lx = decltype(LX)::value != 0, lw = decltype(LW)::value != 0;
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
    if constexpr (lx) load_x(LX, u & 1, ksx);
    mma(0);
    if constexpr (lx) {
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        __builtin_amdgcn_sched_group_barrier(PL_SG_MFMA, (AT * BT) / XCH > 0 ? (AT * BT) / XCH : 1, 0);
        __builtin_amdgcn_sched_group_barrier(PL_SG_VMEM_READ, 1, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    read_a(2);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (lw) load_w(LW, (u + 3) & 3, ksw);
    mma(1);
    if constexpr (lw) {
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

  // tile A; its last three k-steps load the first operands of tile B
  int ks = 0;
  for (; ks < nksA - 4; ks += 4) {
    kstep(I0{}, S1{}, S1{}, Y{}, ks + 2, ks + 3);
    kstep(I1{}, S1{}, S1{}, Y{}, ks + 3, ks + 4);
    kstep(I2{}, S1{}, S1{}, Y{}, ks + 4, ks + 5);
    kstep(I3{}, S1{}, S1{}, Y{}, ks + 5, ks + 6);
  }
  kstep(I0{}, S1{}, S1{}, Y{}, ks + 2, ks + 3);
  kstep(I1{}, S1{}, S2{}, Y{}, ks + 3, 0);
  kstep(I2{}, S2{}, S2{}, Y{}, 0, 1);
  kstep(I3{}, S2{}, S2{}, Y{}, 1, 2);

  // epilogue of A (SwiGLU): accumulator register i of lane l is row (i/4)*8 + (l/32)*4 + i%4, column l%32
#pragma unroll
  for (int a = 0; a < AT; ++a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0A + wm * AT * 32 + a * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
      if (m >= M) continue;
      bf16_t *Y_ = mid + (int64_t)m * (N / 2);
      if (n0A + lrow < n_main) {
        const float gte = acc[a][0][i], up = acc[a][BT - 1][i];
        const float sv = gte / (1.f + __expf(-gte));
        Y_[(n0A >> 1) + lrow] = (__bf16)(sv * up);
      }
    }
  }
  zero_acc();

  // K slice of tile B: its first two x tiles and three W tiles are already loaded or on the way
  for (ks = 0; ks < nksB - 4; ks += 4) {
    kstep(I0{}, S2{}, S2{}, Y{}, ks + 2, ks + 3);
    kstep(I1{}, S2{}, S2{}, Y{}, ks + 3, ks + 4);
    kstep(I2{}, S2{}, S2{}, Y{}, ks + 4, ks + 5);
    kstep(I3{}, S2{}, S2{}, Y{}, ks + 5, ks + 6);
  }
  kstep(I0{}, S2{}, S2{}, Y{}, ks + 2, ks + 3);
  kstep(I1{}, S2{}, S0{}, Y{}, ks + 3, 0);
  kstep(I2{}, S0{}, S0{}, Y{}, 0, 0);
  kstep(I3{}, S0{}, S0{}, No{}, 0, 0);

  const int ldy = N - n_main;
#pragma unroll
  for (int a = 0; a < AT; ++a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0B + wm * AT * 32 + a * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
      if (m >= M) continue;
      float *Y_ = ws + ((int64_t)split * M + m) * ldy - n_main;
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        const int n = n0B + b * 32 + lrow;
        if (n < N) Y_[n] = acc[a][b][i];
      }
    }
  }
}

template <int WM, int WN, int AT, int BT, int MODE>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W,
                                                   void *__restrict__ Yv, int M, int N, int K, int ksteps,
                                                   int n_base, int n_end, int nrow, int ldy, int y_col0) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][BM * LDS_ROW];
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
  gemm_tile<WM, WN, AT, BT, MODE>(xs, X, W, Yv, M, N, K, ksteps, n_base + ctile * BN, rtile * BM, blockIdx.y, n_end, ldy, y_col0);
}

// The SwiGLU product of a 129..256-row batch in ONE launch of one workgroup per compute unit.  Workgroup i
// computes main tile i (128 x 256, row tiles paired on an XCD as above) with the SwiGLU epilogue.  The
// columns left over beyond the last full round of tiles, [n_main, N), are cut into 128 x 256 tiles and
// those along K into `rem_splits` slices; workgroup i also takes slice i % rem_splits of tile
// i / rem_splits and writes its fp32 partial sums to ws, as a launch of the plain kernel with that K
// split would (same slices, same k order); swiglu_reduce_kernel finishes them.  A workgroup that has
// both runs them back to back through gemm_tile2, the slice's first loads issued under the main tile's
// last k-steps.  Every unit thus works 56 + 12 k-steps at the 7B shape instead of 256 units 56 and then
// 160 units 56 more on quarter-size tiles.
template <int WM, int WN, int AT, int BT>
__global__ __launch_bounds__(256) void gemm_gu_fused_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W,
                                                            bf16_t *__restrict__ mid, float *__restrict__ ws, int M, int N,
                                                            int K, int n_main, int rem_splits, int rem_ksteps) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][BM * LDS_ROW];
  const int nrow = (M + BM - 1) / BM;
  const int rtileA = (blockIdx.x >> 3) % nrow, ctileA = (blockIdx.x / (8 * nrow)) * 8 + (blockIdx.x & 7);
  const bool hasA = ctileA * BN < n_main;
  const int item = blockIdx.x / rem_splits, split = blockIdx.x % rem_splits;
  const int rem_ctiles = (N - n_main + BN - 1) / BN;
  const bool hasB = item < rem_ctiles * nrow;
  const int ctileB = item / nrow, rtileB = item % nrow;
  if (hasA && hasB)   // uniform for the workgroup
    gemm_tile2<WM, WN, AT, BT>(xs, X, W, mid, ws, M, N, K, ctileA * BN, rtileA * BM, n_main, n_main + ctileB * BN,
                               rtileB * BM, split, rem_ksteps);
  else if (hasA)
    gemm_tile<WM, WN, AT, BT, 1>(xs, X, W, mid, M, N, K, K / BK, ctileA * BN, rtileA * BM, 0, n_main, 0, 0);
  else if (hasB)
    gemm_tile<WM, WN, AT, BT, 0>(xs, X, W, ws, M, N, K, rem_ksteps, n_main + ctileB * BN, rtileB * BM, split, N, N - n_main, n_main);
}

// SwiGLU over K-split partial sums: parts [splits][M][ld] holds columns [col0, col0 + ld) of the
// interleaved gate/up product (blocks of 64 columns: 32 gate, then the 32 matching up columns);
// mid[m][(col0 + c) / 2 ...] = silu(sum_s gate) * (sum_s up), slices added in order.
__global__ __launch_bounds__(256) void swiglu_reduce_kernel(const float *__restrict__ parts, int splits, int M, int ld,
                                                            int col0, bf16_t *__restrict__ mid, int F) {
  const int quads = ld >> 3;   // four outputs per thread (ld is a multiple of 64)
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)M * quads) return;
  const int m = (int)(idx / quads), j = (int)(idx % quads) * 4;
  const int c = (j >> 5) * 64 + (j & 31);
  f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
  for (int sl = 0; sl < splits; ++sl) {
    const float *row = parts + ((int64_t)sl * M + m) * ld;
    g += *(const f32x4 *)(row + c);
    u += *(const f32x4 *)(row + c + 32);
  }
  bf16x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (__bf16)(g[i] / (1.f + __expf(-g[i])) * u[i]);
  *(bf16x4 *)(mid + (int64_t)m * F + (col0 >> 1) + j) = o;
}

struct Launch {
  const bf16_t *x, *w;
  void *y;
  int M, N, K, mode, splits, n_begin, n_end, ldy, y_col0;
  bool paired;
  hipStream_t s;
};

// Launch over output columns [n_begin, n_end) (multiples of the tile width, except the matrix edge).
template <int WM, int WN, int AT, int BT>
int launch_cfg(const Launch &L) {
  constexpr int BM = WM * AT * 32, BN = WN * BT * 32;
  if (L.n_end <= L.n_begin) return 0;
  if (BT == 1 && L.mode == 1) return -1;   // the SwiGLU epilogue needs a gate and an up tile per wavefront
  dim3 grid((L.n_end - L.n_begin + BN - 1) / BN, L.splits, (L.M + BM - 1) / BM);
  int nrow = 0;
  if (L.paired) {   // flat grid, column tiles padded to a multiple of 8 (see the kernel)
    nrow = grid.z;
    grid.x = ((grid.x + 7) / 8) * 8 * nrow;
    grid.z = 1;
  }
  int ksteps = 4 * ((L.K / (4 * BK) + L.splits - 1) / L.splits);
  if (L.mode == 0)
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, BT, 0>), grid, dim3(256), 0, L.s, L.x, L.w, L.y, L.M, L.N, L.K, ksteps,
                       L.n_begin, L.n_end, nrow, L.ldy, L.y_col0);
  else
    hipLaunchKernelGGL((gemm_kernel<WM, WN, AT, (BT > 1 ? BT : 2), 1>), grid, dim3(256), 0, L.s, L.x, L.w, L.y, L.M, L.N,
                       L.K, ksteps, L.n_begin, L.n_end, nrow, L.ldy, L.y_col0);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

int launch_by_id(int cfg, const Launch &L) {
  switch (cfg) {
    case GEMM_32x256: return launch_cfg<1, 4, 1, 2>(L);
    case GEMM_64x256: return launch_cfg<1, 4, 2, 2>(L);
    case GEMM_128x256: return launch_cfg<1, 4, 4, 2>(L);
    case GEMM_64x128: return launch_cfg<2, 2, 1, 2>(L);
    case GEMM_128x128: return launch_cfg<2, 2, 2, 2>(L);
    case GEMM_256x128: return launch_cfg<2, 2, 4, 2>(L);
    case GEMM_64x64: return launch_cfg<2, 2, 1, 1>(L);
    case GEMM_128x64: return launch_cfg<2, 2, 2, 1>(L);
    case GEMM_32x128: return launch_cfg<1, 4, 1, 1>(L);
    case GEMM_128x64P: return launch_cfg<4, 1, 1, 2>(L);
    case GEMM_256x64P: return launch_cfg<4, 1, 2, 2>(L);
    default: return -1;
  }
}

bool splits_valid(int K, int splits) {
  const int total = K / (4 * BK);
  return splits >= 1 && splits <= total && (splits - 1) * ((total + splits - 1) / splits) < total;   // no empty slice
}

int swiglu_reduce(const float *parts, int splits, int M, int ld, int col0, bf16_t *mid, int F, hipStream_t s) {
  const int64_t total = (int64_t)M * (ld / 8);
  hipLaunchKernelGGL(swiglu_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, parts, splits, M, ld, col0, mid, F);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace

int gemm_tile_rows(int cfg) {
  static const int rows[GEMM_N_CFGS] = {32, 64, 128, 64, 128, 256, 64, 128, 32, 128, 256};
  return cfg >= 0 && cfg < GEMM_N_CFGS ? rows[cfg] : 0;
}

// One launch of one tile configuration over a column range (tuning and tests).  mode 1 with
// splits > 1 writes fp32 partials to ws and finishes with the SwiGLU reduction.
int launch_gemm_cfg(int cfg, const bf16_t *x, const bf16_t *w, void *y, float *ws, int M, int N, int K, int mode,
                    int splits, int n_begin, int n_end, bool paired, hipStream_t s) {
  if (M < 1 || M > 512 || K % (4 * BK) || N % 32 || !splits_valid(K, splits)) return -1;
  if (mode != 0 && mode != 1) return -1;
  if (mode == 1 && (N % 64 || n_begin % 64 || n_end % 64)) return -1;
  if (n_begin < 0 || n_end > N || n_begin % 32 || n_end % 32) return -1;
  if ((int64_t)N * K * 2 >= GEMM_MAX_OPERAND_BYTES || (int64_t)M * K * 2 >= GEMM_MAX_OPERAND_BYTES) return -1;
  if (paired && splits != 1) return -1;
  Launch L{x, w, y, M, N, K, mode, splits, n_begin, n_end, N, 0, paired, s};
  if (mode == 1 && splits > 1) {
    if (!ws) return -1;
    L.mode = 0; L.y = ws; L.ldy = n_end - n_begin; L.y_col0 = n_begin;
    int rc = launch_by_id(cfg, L);
    return rc ? rc : swiglu_reduce(ws, splits, M, n_end - n_begin, n_begin, (bf16_t *)y, N / 2, s);
  }
  return launch_by_id(cfg, L);
}

// K split of a mode-0 product for calls of up to M rows.  The tile shapes named here are the ones
// launch_gemm uses for such calls; the counts come from sweeps over tile shape and split count at the
// benchmark's shapes (weights cold, launches back to back): a launch costs a fixed 3-9 us (first
// loads, drain, partial sums written) plus its weight bytes at 3.5-4.5 TB/s, so narrow outputs want
// about one workgroup per compute unit and as few slices as that allows.
int gemm_pick_splits(int M, int N, int K) {
  auto largest = [&](int tiles, int cap) {
    int best = 1;
    for (int sp = 2; sp <= 32 && tiles * sp <= cap; ++sp)
      if (splits_valid(K, sp)) best = sp;
    return best;
  };
  if (M <= 32 && N < 16384) return largest((N + 127) / 128, 256);               // 32 x 128 tiles
  if (M <= 64 && N < 16384) return largest((N + 63) / 64, 256);                 // 64 x 64 tiles
  if (M <= 128) return largest((N + 255) / 256, 256);                           // 128 x 256 tiles
  // 129..256 rows: at these rows two, three or four slices of the short-K products (QKV, O) and eight or
  // nine of the long one (down) take the same time within a microsecond; the larger counts are kept
  // because an engine sized for 256 rows also runs steps of a few rows (a batch that is not refilled
  // decays), and with few rows the bytes in flight, hence the weight bandwidth, grow with the slices.
  if (M <= 256 && K <= 4096 && splits_valid(K, 4)) return 4;                    // 128 x 128 tiles
  return largest(((N + 127) / 128) * ((M + 255) / 256), 256);                   // 256 x 128 tiles
}

// How K is split for a product, as a function of the LARGEST row count the caller will ever pass
// (so that every pass, whatever its row count, adds up each output element in the same order).
// mode 0: one split count for all columns (the caller's output holds that many slices).
// mode 1: columns [0, n_main) with `splits` slices, columns [n_main, N) with `rem_splits`; wherever a
// count exceeds 1 the partial sums go through the workspace and the SwiGLU is applied by a reduction.
// Launched on their own, no SwiGLU product gained from a K split in the sweeps (64 x 128 tiles fill the
// chip for narrow batches).  The one split chosen is the column remainder of a wide product at 129..256
// rows, whose slices ride in the launch of the main tiles (gemm_gu_fused_kernel): 1.2 % of the 7B step.
GemmSplit gemm_pick_split(int M_max, int N, int K, int mode) {
  GemmSplit ks{1, N, 1};
  if (mode == 0) {
    ks.splits = gemm_pick_splits(M_max, N, K);
    return ks;
  }
  if (M_max > 128 && M_max <= 256 && N >= 128 * 256) {
    // 128 x 256 tiles, two row tiles: what is left over a multiple of 256 tiles is split along K so that
    // every compute unit gets one slice on top of its main tile (gemm_gu_fused_kernel)
    const int ctiles = (N + 255) / 256, tiles = 2 * ctiles, rem = tiles % 256;
    if (tiles > 256 && rem > 0 && rem <= 96) {
      int best = 1;
      for (int sp = 2; sp <= 16 && rem * sp <= 256; ++sp)
        if (splits_valid(K, sp)) best = sp;
      if (best > 1) {
        ks.n_main = ((tiles - rem) / 2) * 256;
        ks.rem_splits = best;
      }
    }
  }
  return ks;
}

// fp32 elements of workspace a mode-1 product of up to M_max rows needs (0 if K is not split)
int64_t gemm_workspace_elems(int M_max, int N, const GemmSplit &ks) {
  int64_t need = 0;
  if (ks.splits > 1) need = (int64_t)ks.splits * M_max * ks.n_main;
  if (ks.n_main < N && ks.rem_splits > 1) need = std::max<int64_t>(need, (int64_t)ks.rem_splits * M_max * (N - ks.n_main));
  return need;
}

int launch_gemm(const bf16_t *x, const bf16_t *w, void *y, float *ws, int M, int N, int K, int mode,
                const GemmSplit &ks, hipStream_t s) {
  if (M < 1 || M > 512 || K % (4 * BK) || N % 32 || !splits_valid(K, ks.splits)) return -1;
  if (mode != 0 && mode != 1) return -1;
  if (mode == 1 && (N % 64 || ks.n_main % 64 || !splits_valid(K, ks.rem_splits))) return -1;
  if (mode == 0 && ks.n_main != N) return -1;
  if (ks.n_main < 0 || ks.n_main > N) return -1;
  // tile shape from the rows of this call
  int cfg;
  bool paired = false;
  if (mode == 1) {
    if (M <= 32) cfg = GEMM_32x256;
    else if (M <= 64) cfg = GEMM_64x128;
    else if (M <= 128) cfg = GEMM_128x256;
    else if (M <= 256 && N >= 128 * 256) { cfg = GEMM_128x256; paired = ks.splits == 1; }
    else cfg = GEMM_256x128;
  } else {
    if (M <= 32) cfg = N >= 16384 ? GEMM_32x256 : GEMM_32x128;   // all four wavefronts stream their own columns
    else if (M <= 64 && N < 16384) cfg = GEMM_64x64;
    else if (M <= 64) cfg = GEMM_64x256;
    else if (M <= 128) cfg = GEMM_128x256;
    else if (M <= 256 && ks.splits == 1 && N >= 128 * 256) { cfg = GEMM_128x256; paired = true; }
    else if (M <= 256 && K <= 4096) cfg = ks.splits <= 2 ? GEMM_128x64 : GEMM_128x128;
    else cfg = GEMM_256x128;
  }
  int n_main = ks.n_main;
  if (paired && n_main == N) {
    // Wide matrices without a K split: 128 x 256 tiles in XCD-local pairs.  When the tile count is a
    // little over a multiple of 256 the last round would run on a few units at full length: those
    // columns go to a second launch of 64 x 128 tiles instead.
    const int ctiles = (N + 255) / 256, tiles = 2 * ctiles, rem = tiles % 256;
    if (tiles > 256 && rem > 0 && rem <= 64) n_main = ((tiles - rem) / 2) * 256;
  }
  if (mode == 1 && paired && n_main < N && ks.rem_splits > 1 && ks.splits == 1 && ws) {
    // main tiles and K slices of the remainder in one launch, then the SwiGLU over the slices
    if ((int64_t)N * K * 2 >= GEMM_MAX_OPERAND_BYTES || (int64_t)M * K * 2 >= GEMM_MAX_OPERAND_BYTES) return -1;
    const int nrow = (M + 127) / 128, rem_ctiles = (N - n_main + 255) / 256;
    const int wgs = std::max(((n_main / 256 + 7) / 8) * 8 * nrow, rem_ctiles * nrow * ks.rem_splits);
    const int rem_ksteps = 4 * ((K / (4 * BK) + ks.rem_splits - 1) / ks.rem_splits);
    hipLaunchKernelGGL((gemm_gu_fused_kernel<1, 4, 4, 2>), dim3(wgs), dim3(256), 0, s, x, w, (bf16_t *)y, ws, M, N, K, n_main,
                       ks.rem_splits, rem_ksteps);
    if (hipGetLastError() != hipSuccess) return -7;
    return swiglu_reduce(ws, ks.rem_splits, M, N - n_main, n_main, (bf16_t *)y, N / 2, s);
  }
  int rc = launch_gemm_cfg(cfg, x, w, y, ws, M, N, K, mode, ks.splits, 0, n_main, paired, s);
  if (rc || n_main == N) return rc;
  return launch_gemm_cfg(GEMM_64x128, x, w, y, ws, M, N, K, mode, mode == 1 ? ks.rem_splits : ks.splits, n_main, N,
                         false, s);
}

}  // namespace pl
