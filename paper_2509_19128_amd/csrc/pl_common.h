// Internal declarations shared by the engine's host code and its kernels (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace pl {

// ---- KV page geometry (one layer, one page, one kv head: K block then V block) ---------------
// Tokens of a page are grouped in runs of 32 (t = 32 r + u).  Both blocks are laid out so that the
// 64 lanes of a wavefront read one MFMA operand with a single fully contiguous 1 KiB load.
__host__ __device__ inline int64_t k_elem_offset(int t, int d, int hd) {
  int r = t >> 5, u = t & 31;
  int T = (u >> 2) & 1, R = ((u >> 3) << 2) | (u & 3);
  return ((int64_t)((r * 2 + T) * (hd / 8) + d / 8)) * 128 + R * 8 + (d & 7);
}
__host__ __device__ inline int64_t v_elem_offset(int t, int d, int hd) {
  int r = t >> 5, u = t & 31;
  return ((int64_t)((r * (hd / 16) + d / 16) * 4 + (u >> 3))) * 128 + (d & 15) * 8 + (u & 7);
}

struct AttnParams {
  const bf16_t *q;          // [n_seq, Hq, hd]
  const bf16_t *kv;         // page pool of one layer
  const int32_t *page_table;// [n_slots, pages_per_seq], row = slot_of_row[row] (or row if null)
  const int32_t *ctx_len;   // [n_seq]
  const int32_t *row_slot;  // [n_seq] or null
  const int32_t *work;      // work list built by launch_attention_worklist for these ctx_len, row_slot and page_table
  const int32_t *multi;     // attention_multi_list(work, ...): rows longer than one chunk
  int32_t max_items;        // upper bound on the list length (sizes the grid)
  int32_t max_multi;        // upper bound on the number of rows longer than one chunk; 0 = none, no merge launch
  bf16_t *out;              // [n_seq, Hq, hd]
  float *part_o;            // [n_seq, Hkv, max_chunks, G, hd]
  float *part_ml;           // [n_seq, Hkv, max_chunks, G, 2]
  int32_t n_seq, Hq, Hkv, hd, page_tokens, pages_per_seq, chunk, max_chunks;
};
int launch_attention(const AttnParams &p, hipStream_t s, int part = 0);
int64_t attention_worklist_ints(int n_seq, int max_chunks);
const int32_t *attention_multi_list(const int32_t *work, int n_seq, int max_chunks);
int launch_attention_worklist(const int32_t *ctx_len, const int32_t *row_slot, const int32_t *page_table, int32_t *work,
                              int n_seq, int max_chunks, int chunk, int page_tokens, int pages_per_seq, hipStream_t s);
int attention_chunk_tokens(int n_seq, int Hkv, int max_ctx);

// x and W are each addressed through one buffer descriptor with 32-bit byte offsets kept in signed
// registers: an operand must stay below 2 GiB (launch_gemm returns -1 beyond that).
constexpr int64_t GEMM_MAX_OPERAND_BYTES = (int64_t)1 << 31;
// tile configurations of the GEMM kernel: rows x columns of a workgroup's tile ("P": the four wavefronts
// stacked along the rows, each holding a gate and an up tile)
enum { GEMM_32x256, GEMM_64x256, GEMM_128x256, GEMM_64x128, GEMM_128x128, GEMM_256x128, GEMM_64x64, GEMM_128x64,
       GEMM_32x128, GEMM_128x64P, GEMM_256x64P, GEMM_N_CFGS };
// How K is split: columns [0, n_main) in `splits` slices, columns [n_main, N) in `rem_splits` (mode 1
// only; mode 0 has n_main = N).  Chosen once per product from the largest row count (gemm_pick_split),
// so that every call adds up an output element in the same order whatever its row count.
struct GemmSplit { int splits, n_main, rem_splits; };
GemmSplit gemm_pick_split(int M_max, int N, int K, int mode);
int64_t gemm_workspace_elems(int M_max, int N, const GemmSplit &ks);
// ws: fp32 workspace of gemm_workspace_elems (mode 1 with split K), else may be null
int launch_gemm(const bf16_t *x, const bf16_t *w, void *y, float *ws, int M, int N, int K, int mode,
                const GemmSplit &ks, hipStream_t s);
int launch_gemm_cfg(int cfg, const bf16_t *x, const bf16_t *w, void *y, float *ws, int M, int N, int K, int mode,
                    int splits, int n_begin, int n_end, bool paired, hipStream_t s);
int gemm_tile_rows(int cfg);
int gemm_pick_splits(int M, int N, int K);

struct SampleParams {
  const float *logits; int32_t n, vocab;
  const uint64_t *seq_id; const int32_t *position; const float *inv_t; const int32_t *forced;
  uint64_t seed; int32_t *token; float *logprob; void *workspace;
  int32_t *last_tok; const int32_t *row_slot;   // optional: last_tok[row_slot[row]] = token
};
int64_t sample_workspace_bytes(int n, int vocab);
int launch_sample(const SampleParams &p, hipStream_t s);
int sample_static_workspace(int n, int vocab, void **ptr);
void sample_static_limits(int *max_rows, int *max_vocab);

// per-step metadata, one row per occupied slot (device copies of host arrays)
struct StepMeta {
  const int32_t *row_slot, *pos, *input_tok, *forced;
  const float *inv_t; const uint64_t *seq_id;
};
int launch_embed_rmsnorm(const bf16_t *embed, const bf16_t *g, const int32_t *input_tok,
                         const int32_t *last_tok, const int32_t *row_slot, float *h, bf16_t *a,
                         int n, int d, int vocab, float eps, hipStream_t s);
int launch_resid_rmsnorm(float *h, const float *parts, int splits, const bf16_t *g, bf16_t *a, int n,
                         int d, float eps, hipStream_t s);
int launch_rope_tables(const int32_t *pos, float *cs, int32_t *ctx_len, int n, int hd, float theta,
                       hipStream_t s);
int launch_rope_append(const float *qkv, int splits, const float *cs, const int32_t *pos,
                       const int32_t *row_slot, const int32_t *page_table, bf16_t *q_out, bf16_t *kv_layer,
                       int n, int Hq, int Hkv, int hd, int page_tokens, int pages_per_seq, hipStream_t s);
// fp32 test build (kernels_f32.hip)
int f32_launch_norm(const float *embed, const int32_t *input_tok, int vocab, const float *y, const float *g, float *h,
                    float *a, int n, int d, float eps, hipStream_t s);
int f32_launch_gemm(const float *x, const float *w, float *y, int M, int N, int K, hipStream_t s);
int f32_launch_swiglu(const float *gu, float *mid, int M, int F, hipStream_t s);
int f32_launch_rope_append(const float *qkv, const float *cs, const int32_t *pos, const int32_t *row_slot,
                           const int32_t *page_table, float *q_out, float *kv_layer, int n, int Hq, int Hkv, int hd,
                           int page_tokens, int pages_per_seq, hipStream_t s);
int f32_launch_attention(const float *q, const float *kv_layer, const int32_t *page_table, const int32_t *pos,
                         const int32_t *row_slot, float *out, int n, int Hq, int Hkv, int hd, int page_tokens,
                         int pages_per_seq, hipStream_t s);
int64_t launch_stream_read(const void *p, int64_t nbytes, uint32_t *sink, bool nontemporal, hipStream_t s);
int launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t s);
int launch_tie_lm_head(const void *embed, void *lm_head, int vocab, int d, bool f32, hipStream_t s);
int launch_is_ess(const float *lp_pi, const float *lp_mu, const int64_t *offsets, int n_seq, double c, float *w_out,
                  double *seq_sums, double *ess_seq, double *totals, hipStream_t s);

}  // namespace pl
