// Ragged grouped-query decode attention over the paged bf16 KV cache (gfx950).
//
// One decode step of "generate next tokens" (Alg. 2 of the paper) attends one new query per
// sequence over that sequence's whole cached history; the work is a stream of K and V bytes at a
// few flops per byte, so the kernel is built around HBM reads: every load instruction of a
// wavefront fetches one contiguous KiB that is already in MFMA operand order (the page layout is
// chosen for that), the query heads that share a kv head ride along as the 16 columns of one
// 16x16x32 MFMA so each K/V byte is read once for the whole group, and soft-max statistics are
// reduced with cross-lane shuffles.  Work is split over (sequence, kv head, chunk of tokens);
// chunks of one sequence are merged by a second kernel in a fixed order.
#include "pl_common.h"

#ifndef PL_ATTN_NS
#define PL_ATTN_NS 2   // register stages of K/V runs per wavefront
#endif
#ifndef PL_ATTN_CHUNK
#define PL_ATTN_CHUNK 8192   // largest number of tokens one workgroup handles
#endif

namespace pl {
namespace {

__device__ inline float shfl_xor(float v, int mask) { return __shfl_xor(v, mask, 64); }

template <int HD, int NS>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnParams p) {
  constexpr int NJ = HD / 32;   // QK MFMAs per 16-token tile
  constexpr int NV = HD / 16;   // PV MFMAs per 32-token run
  // Work items come from a compact list built on the device for this step: every launched workgroup
  // up to the list's length has work (full chunks first, then the last chunks, longest first), so
  // consecutive workgroup ids, which the hardware deals round-robin to the 8 XCDs, load all XCDs
  // evenly whatever the mix of context lengths.  An item is one 32-byte record (sequence, chunk,
  // context length, slot, and the first four page ids of the chunk), so that the first K/V loads of
  // a workgroup are one dependent scalar load away (its record; records beyond the list's end say so
  // themselves) instead of five: with the memory system saturated each such load takes about a
  // microsecond during which the workgroup has nothing in flight.
  const int item = blockIdx.x / p.Hkv, g = blockIdx.x % p.Hkv;
  const int4 *rec = (const int4 *)(p.work + 8 + 8 * (int64_t)item);
  const int4 r0 = rec[0], r1 = rec[1];
  const int b = r0.x, c = r0.y, ctx = r0.z, slot = r0.w;
  if (ctx <= 0) return;   // beyond the end of the list (the list kernel clears the records up to the buffer's end)
  const int t0 = c * p.chunk;
  const int t1 = min(ctx, t0 + p.chunk);
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int head = l & 15, qg = l >> 4;
  const int G = p.Hq / p.Hkv;
  const int32_t *pt = p.page_table + (int64_t)slot * p.pages_per_seq;
  const int page_first = t0 / p.page_tokens;   // r1 holds the ids of pages page_first .. page_first + 3
  const float scale = 1.4426950408889634f / sqrtf((float)HD);   // log2(e) / sqrt(hd)

  // Query operand: column = head of the group (zero for the padding columns), k = head-dim slice.
  bf16x8 qf[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (head < G) {
      qf[j] = *(const bf16x8 *)(p.q + ((int64_t)b * p.Hq + g * G + head) * HD + j * 32 + qg * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[j][e] = (__bf16)0.0f;
    }
  }

  f32x4 o[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, lsum = 0.f;

  const int nblk = (t1 - t0 + 31) >> 5;
  const int64_t page_elems = (int64_t)2 * p.page_tokens * HD;   // K block + V block of one kv head
  // page id of a run, and the address of its K fragments given that id: the id of the run a stage will
  // hold next is fetched one refill ahead, so that no K/V load waits for a page-table load
  auto page_of = [&](int blk) -> int {
    const int t = t0 + blk * 32;
    const int rel = t / p.page_tokens - page_first;
    return rel == 0 ? r1.x : rel == 1 ? r1.y : rel == 2 ? r1.z : rel == 3 ? r1.w : pt[t / p.page_tokens];
  };
  auto run_base = [&](int blk, int page) -> const bf16_t * {
    const int r = ((t0 + blk * 32) % p.page_tokens) >> 5;
    return p.kv + ((int64_t)page * p.Hkv + g) * page_elems + (int64_t)r * 32 * HD + l * 8;
  };

  // NS register stages per wavefront: stage s holds the K and V fragments of run (it * NS + s) * 4 +
  // wave.  As soon as a stage's K fragments have gone through the QK MFMAs they are reloaded for the
  // run NS rounds later, likewise the V fragments after the PV MFMAs, so about NS runs (16 KiB each)
  // per wavefront are always in flight.
  // K and V are read once per step and never again before they are evicted: non-temporal loads keep
  // them from displacing each other in L2 on the way (measured +6 to 10 % bandwidth).
  bf16x8 kf[NS][2][NJ], vf[NS][NV];
  auto load_k = [&](int st, const bf16_t *kb) {
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int j = 0; j < NJ; ++j) kf[st][T][j] = __builtin_nontemporal_load((const bf16x8 *)(kb + (T * NJ + j) * 512));
  };
  auto load_v = [&](int st, const bf16_t *kb) {
    const bf16_t *vb = kb + (int64_t)p.page_tokens * HD;
#pragma unroll
    for (int i = 0; i < NV; ++i) vf[st][i] = __builtin_nontemporal_load((const bf16x8 *)(vb + i * 512));
  };
  int page_next[NS];   // page of the run stage st takes after the one it holds
#pragma unroll
  for (int st = 0; st < NS; ++st) {
    const int b0 = wave + 4 * st;
    if (b0 < nblk) { const bf16_t *kb = run_base(b0, page_of(b0)); load_k(st, kb); load_v(st, kb); }
    page_next[st] = b0 + 4 * NS < nblk ? page_of(b0 + 4 * NS) : 0;
  }
  for (int base = wave; base < nblk; base += 4 * NS) {
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      const int blk = base + 4 * st;
      if (blk < nblk) {
        // scores of the 32 tokens of this run: two 16-token tiles
        f32x4 s4[2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
          s4[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            s4[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[st][T][j], qf[j], s4[T], 0, 0, 0);
        }
        const int nxt = blk + 4 * NS;
        const bf16_t *nb = nullptr;
        if (nxt < nblk) {
          nb = run_base(nxt, page_next[st]);
          load_k(st, nb);
          page_next[st] = nxt + 4 * NS < nblk ? page_of(nxt + 4 * NS) : 0;
        }
        const int tbase = t0 + blk * 32 + qg * 8;
        float s[8];
        float mb = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float v = s4[e >> 2][e & 3] * scale;
          v = (tbase + e < t1) ? v : -INFINITY;
          s[e] = v;
          mb = fmaxf(mb, v);
        }
        mb = fmaxf(mb, shfl_xor(mb, 16));
        mb = fmaxf(mb, shfl_xor(mb, 32));
        const float m_new = fmaxf(m, mb);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float psum = 0.f;
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float pe = __builtin_amdgcn_exp2f(s[e] - m_new);
          psum += pe;
          pf[e] = (__bf16)pe;
        }
        lsum = lsum * alpha + psum;
        m = m_new;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          o[i] *= alpha;
          o[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[st][i], pf, o[i], 0, 0, 0);
        }
        if (nb) load_v(st, nb);
      }
    }
  }
  lsum += shfl_xor(lsum, 16);
  lsum += shfl_xor(lsum, 32);

  // merge the four wavefronts of the workgroup
  __shared__ float sm_o[4][16][HD];
  __shared__ float sm_m[4][16], sm_l[4][16];
  if (head < G) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) sm_o[wave][head][i * 16 + qg * 4 + e] = o[i][e];
    if (qg == 0) { sm_m[wave][head] = m; sm_l[wave][head] = lsum; }
  }
  __syncthreads();
  const bool single = ctx <= p.chunk;
  const int64_t pidx = ((int64_t)b * p.Hkv + g) * p.max_chunks + c;
  for (int idx = threadIdx.x; idx < G * HD; idx += 256) {
    int h = idx / HD, d = idx % HD;
    float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float f = __builtin_amdgcn_exp2f(sm_m[w][h] - M);
      L += sm_l[w][h] * f;
      O += sm_o[w][h][d] * f;
    }
    if (single) {
      p.out[((int64_t)b * p.Hq + g * G + h) * HD + d] = (__bf16)(O / L);
    } else {
      p.part_o[(pidx * G + h) * HD + d] = O;
      if (d == 0) { p.part_ml[(pidx * G + h) * 2] = M; p.part_ml[(pidx * G + h) * 2 + 1] = L; }
    }
  }
}

// Inclusive prefix sum over the 1024 threads of the workgroup (wave shuffles, then the 16 wave totals).
__device__ inline int block_scan_1024(int v, int *wsum, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(v, o, 64);
    if (lane >= o) v += t;
  }
  __syncthreads();   // wsum may still be read from a previous call
  if (lane == 63) wsum[wave] = v;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int x = wsum[w];
    all += x;
    if (w < wave) before += x;
  }
  *total = all;
  return v + before;
}

// work[0] = number of items, work[1] = number of sequences longer than one chunk (listed in `multi` as
// row | chunks << 12, the rest of the list -1);
// the items are 8-int records from work[8] on: {sequence, chunk, context length, slot, ids of the
// chunk's first four pages}.  All full chunks come first, then each
// sequence's last (partial or full) chunk, longest first, so that the workgroups still running when
// the grid drains are the short ones.  One workgroup; n_seq <= 1024.
__global__ __launch_bounds__(1024) void attn_worklist_kernel(const int32_t *ctx_len, const int32_t *row_slot,
                                                             const int32_t *page_table, int32_t *work, int32_t *multi,
                                                             int n_seq, int chunk, int page_tokens, int pages_per_seq) {
  __shared__ int wsum[16];
  __shared__ __attribute__((aligned(16))) int tail[1024];
  const int b = threadIdx.x;
  const int ctx = b < n_seq ? ctx_len[b] : 0;
  const int slot = b < n_seq ? (row_slot ? row_slot[b] : b) : 0;
  const int n = (ctx + chunk - 1) / chunk;
  const int full = n > 0 ? n - 1 : 0;
  const int32_t *pt = page_table + (int64_t)slot * pages_per_seq;
  const int last_page = ctx > 0 ? (ctx - 1) / page_tokens : 0;
  auto put = [&](int i, int c) {
    int4 *rec = (int4 *)(work + 8 + 8 * (int64_t)i);
    const int p0 = c * chunk / page_tokens;
    rec[0] = make_int4(b, c, ctx, slot);
    rec[1] = make_int4(pt[min(p0, last_page)], pt[min(p0 + 1, last_page)], pt[min(p0 + 2, last_page)],
                       pt[min(p0 + 3, last_page)]);
  };
  int total_full, n_last;
  const int at = block_scan_1024(full, wsum, &total_full) - full;
  for (int c = 0; c < full; ++c) put(at + c, c);
  const int rem = n > 0 ? ctx - (n - 1) * chunk : 0;
  tail[b] = rem;   // 0 for empty rows and for threads at or beyond n_seq
  (void)block_scan_1024(n > 0, wsum, &n_last);   // also orders the writes to tail before the reads below
  if (n > 0) {   // rank among the last chunks: longer first, lower sequence index first among equals
    int rank = 0;
    const int4 *t4 = (const int4 *)tail;
    for (int o4 = 0; o4 < (n_seq + 3) / 4; ++o4) {
      const int4 t = t4[o4];
      const int o = o4 * 4;
      rank += (t.x > rem) || (t.x == rem && o < b);
      rank += (t.y > rem) || (t.y == rem && o + 1 < b);
      rank += (t.z > rem) || (t.z == rem && o + 2 < b);
      rank += (t.w > rem) || (t.w == rem && o + 3 < b);
    }
    put(total_full + rank, n - 1);
  }
  // rows that span several chunks, in row order: what the merge kernel walks
  int n_multi;
  const int mi = block_scan_1024(n > 1, wsum, &n_multi) - (n > 1);
  if (n > 1) multi[mi] = b | (n << 12);   // row and its number of chunks in one word (n_seq <= 1024)
  for (int i = n_multi + b; i < n_seq; i += 1024) multi[i] = -1;   // beyond the list's end
  if (b == 0) { work[0] = total_full + n_last; work[1] = n_multi; }
  // records beyond the list's end, up to the end of the record area (the multi list starts there), say
  // "no item": a workgroup of the decode kernel learns that from its own record, without a second
  // dependent load of the list's length
  const int cap = (int)((multi - (work + 8)) / 8);
  for (int i = total_full + n_last + b; i < cap; i += 1024) ((int4 *)(work + 8 + 8 * (int64_t)i))[0] = make_int4(0, 0, 0, 0);
}

// Merge of the chunks of multi-chunk sequences, in chunk order.  One workgroup of HD threads per
// (listed sequence, query head); the list is the work-list kernel's, the grid is sized by the
// caller's bound on its length.  The kernel is latency bound (a few KiB per workgroup), so every load
// that does not depend on another is issued at once: thread c fetches the statistics of chunk c, the
// weights go through LDS, and each thread then sums its output element over the chunks, eight loads
// at a time, in chunk order.
template <int HD>
__global__ __launch_bounds__(HD < 64 ? 64 : HD) void attn_combine_kernel(AttnParams p) {
  constexpr int NT = HD < 64 ? 64 : HD;   // threads: whole wavefronts; thread d < HD owns output element d
  // one list entry = row | number of chunks << 12, negative beyond the list's end: the chunk statistics
  // are one dependent load away
  const int entry = p.multi[blockIdx.y];
  if (entry < 0) return;
  const int b = entry & 0xFFF, nchunk = entry >> 12, hq = blockIdx.x;
  const int G = p.Hq / p.Hkv, g = hq / G, h = hq % G;
  const int64_t base = ((int64_t)b * p.Hkv + g) * p.max_chunks;
  const float *ml = p.part_ml + (base * G + h) * 2;                   // chunk c at ml[c * G * 2]
  const float *po = p.part_o + (base * G + h) * HD + (threadIdx.x < HD ? threadIdx.x : 0);   // chunk c at po[c * G * HD]
  __shared__ float sw[NT];      // weight of chunk c (NT chunks at a time)
  __shared__ float red[2][NT / 64];
  const int d = threadIdx.x, lane = d & 63, wave = d >> 6;
  float O = 0.f, L = 0.f;
  // the running maximum over all chunks first (chunks beyond HD are walked in rounds of HD)
  float M = -INFINITY;
  for (int c0 = 0; c0 < nchunk; c0 += NT) {
    float m = c0 + d < nchunk ? ml[(int64_t)(c0 + d) * G * 2] : -INFINITY;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if (lane == 0) red[0][wave] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) M = fmaxf(M, red[0][w]);
    __syncthreads();
  }
  for (int c0 = 0; c0 < nchunk; c0 += NT) {
    const int nc = min(NT, nchunk - c0);
    float wgt = 0.f, lw = 0.f;
    if (d < nc) {
      const float2 v = *(const float2 *)(ml + (int64_t)(c0 + d) * G * 2);
      wgt = __builtin_amdgcn_exp2f(v.x - M);
      lw = v.y * wgt;
    }
    sw[d] = wgt;
    // L: sum of l_c w_c in a fixed order (lanes by shuffle tree, then the waves in order)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o, 64);
    if (lane == 0) red[1][wave] = lw;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) L += red[1][w];
    for (int c = 0; c < nc; c += 8) {
      float o8[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) o8[u] = c + u < nc ? po[(int64_t)(c0 + c + u) * G * HD] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (c + u < nc) O += o8[u] * sw[c + u];
    }
    __syncthreads();
  }
  if (d < HD) p.out[((int64_t)b * p.Hq + hq) * HD + d] = (__bf16)(O / L);
}

}  // namespace

int attention_chunk_tokens(int n_seq, int Hkv, int max_ctx) {
  // Tokens per workgroup: large enough that the merge is a small fraction of the bytes, small
  // enough that a few hundred compute units all get work.  A function of the launch shape only,
  // never of the contexts, so a sequence's result does not depend on its neighbours' lengths.
  int chunk = PL_ATTN_CHUNK;
  while (chunk > 128 && (int64_t)n_seq * Hkv * ((max_ctx + chunk - 1) / chunk) < 2048) chunk >>= 1;
  return chunk;
}

// ints of the work buffer (which must be 32-byte aligned): a header of 8, one 8-int record per item,
// then the list of multi-chunk sequences
int64_t attention_worklist_ints(int n_seq, int max_chunks) { return 8 + 8 * (int64_t)n_seq * max_chunks + n_seq; }
const int32_t *attention_multi_list(const int32_t *work, int n_seq, int max_chunks) {
  return work + 8 + 8 * (int64_t)n_seq * max_chunks;
}

int launch_attention_worklist(const int32_t *ctx_len, const int32_t *row_slot, const int32_t *page_table, int32_t *work,
                              int n_seq, int max_chunks, int chunk, int page_tokens, int pages_per_seq, hipStream_t s) {
  if (n_seq <= 0 || n_seq > 1024 || ((uintptr_t)work & 31)) return -1;
  hipLaunchKernelGGL(attn_worklist_kernel, dim3(1), dim3(1024), 0, s, ctx_len, row_slot, page_table, work,
                     (int32_t *)attention_multi_list(work, n_seq, max_chunks), n_seq, chunk, page_tokens, pages_per_seq);
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

// part: 0 = the decode kernel and, where a row spans several chunks, the merge kernel; 1 = the decode
// kernel alone; 2 = the merge kernel alone (so that a caller can time the two separately)
int launch_attention(const AttnParams &p, hipStream_t s, int part) {
  if (p.n_seq <= 0) return 0;
  // max_items and max_multi bound the two lists (a host that knows the step's contexts passes the
  // exact lengths; otherwise n_seq * max_chunks and n_seq)
  dim3 grid(p.max_items * p.Hkv), cgrid(p.Hq, p.max_multi > 0 ? p.max_multi : 1);
  const bool decode = part != 2, merge = p.max_multi > 0 && part != 1;
  switch (p.hd) {
    case 128:
      if (decode) hipLaunchKernelGGL((attn_decode_kernel<128, PL_ATTN_NS>), grid, dim3(256), 0, s, p);
      if (merge) hipLaunchKernelGGL(attn_combine_kernel<128>, cgrid, dim3(128), 0, s, p);
      break;
    case 64:
      if (decode) hipLaunchKernelGGL((attn_decode_kernel<64, PL_ATTN_NS>), grid, dim3(256), 0, s, p);
      if (merge) hipLaunchKernelGGL(attn_combine_kernel<64>, cgrid, dim3(64), 0, s, p);
      break;
    case 32:
      if (decode) hipLaunchKernelGGL((attn_decode_kernel<32, PL_ATTN_NS>), grid, dim3(256), 0, s, p);
      if (merge) hipLaunchKernelGGL(attn_combine_kernel<32>, cgrid, dim3(64), 0, s, p);
      break;
    default:
      return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // namespace pl
