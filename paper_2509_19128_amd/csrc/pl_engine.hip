// Host side of the decode engine: slot table, KV page allocator, weight-buffer manager, step driver,
// and the extern "C" boundary declared in include/pl.h.
//
// The engine is the generation half of the Actor loop (Alg. 2 of the paper): a constant batch of
// slots, one token per occupied slot per step, refill through add/retire, and weight updates that
// are staged on a side stream and become active only between two steps while every sequence keeps
// its key/value pages (Sec. 5.1).
#include "../../include/pl.h"
#include "pl_common.h"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t _e = (expr);                                                                 \
    if (_e != hipSuccess) return fail(PL_E_HIP, "%s: %s", #expr, hipGetErrorString(_e));    \
  } while (0)

inline uint16_t f32_to_bf16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float bf16_bits_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

struct Tensor {
  std::string name;
  int64_t offset, rows, cols;
};

struct Seq {
  bool active = false;
  uint64_t seq_id = 0;
  std::vector<int32_t> prompt;
  std::vector<int32_t> hist;   // tokens read at positions [0, pos) (what a cache recomputation replays)
  bool hist_known = true;      // false for sequences admitted mid-life without their history
  bool reading = false;        // its prompt is being read in the background; not part of decode steps yet
  int32_t n_prompt = 0, max_new = 0, pos = 0, n_emitted = 0, next_input = -1;
  float inv_t = 1.f;
  std::vector<int32_t> pages;
};

struct LayerW {
  const bf16_t *g1, *w_qkv, *w_o, *g2, *w_gu, *w_d;
};

}  // namespace

struct pl_engine {
  pl_model_cfg cfg{};
  bool dry = false;
  int G = 1, page_tokens = 64, pages_per_seq = 0;
  int rows_cap = 0;   // rows the work buffers hold: max(max_batch, 256), so cache-only passes can take 256 rows
  int64_t n_pages = 0, layer_stride = 0, page_stride = 0;   // elements
  // weights
  std::vector<Tensor> layout;
  int64_t blob_elems = 0;        // elements of a device weight buffer (always with an LM head)
  int64_t host_blob_elems = 0;   // elements of the caller's blob: without the LM head when it is tied to the embedding
  bool tied = false;
  bool f32 = false;   // the fp32 test build
  int esz = 2;        // bytes per stored element (weights, KV, activations)
  char *wbuf[2] = {nullptr, nullptr};
  int active_buf = 0;
  uint32_t version = 0;
  bool loaded = false;
  bool staged = false, staged_wait = false, staged_recompute = false;
  uint32_t staged_version = 0;
  hipEvent_t ev_staged = nullptr, ev_copy0 = nullptr;
  // kv
  char *kv_pool = nullptr;   // bf16 pages in operand order, or fp32 pages of the test build
  std::vector<int32_t> free_pages;
  int32_t *pt_h = nullptr;   // host page table (pinned): the truth; each work set keeps a device copy of its own
  bool pt_dirty = false;
  std::vector<Seq> seqs;
  // Activation buffers and per-pass metadata come in two sets, each with its own stream: set 0 is the
  // decode step's, set 1 belongs to the cache-only passes (prompt reading, cache recomputation), so
  // that a prompt can be read in the background while decode steps go on.
  struct Work {
    hipStream_t stream = nullptr;
    int rows_cap = 0;
    char *meta_h = nullptr, *meta_d = nullptr;   // per-pass metadata: host (pinned) and device images, same layout
    float *h = nullptr, *parts = nullptr, *cs = nullptr, *attn_po = nullptr, *attn_pml = nullptr;
    bf16_t *a = nullptr, *q_rot = nullptr, *attn_out = nullptr, *mid = nullptr;
    int32_t *ctx_len = nullptr, *attn_work = nullptr;
    int32_t *pt = nullptr;   // device copy of the page table, written on this set's stream only
    int attn_items = 0;   // bound on this pass's attention work items
    int attn_multi = 0;   // rows of this pass that span more than one attention chunk
    // the 8-byte ids come first, so every array is aligned for its type whatever rows_cap is
    uint64_t *m_seq_id(bool dev) { return (uint64_t *)(dev ? meta_d : meta_h); }
    int32_t *m_row_slot(bool dev) { return (int32_t *)(m_seq_id(dev) + rows_cap); }
    int32_t *m_pos(bool dev) { return m_row_slot(dev) + rows_cap; }
    int32_t *m_input(bool dev) { return m_pos(dev) + rows_cap; }
    int32_t *m_forced(bool dev) { return m_input(dev) + rows_cap; }
    float *m_inv_t(bool dev) { return (float *)(m_forced(dev) + rows_cap); }
  };
  Work wk[2];
  int64_t meta_bytes = 0;
  // Host images of the cache-only passes in flight: a pass's image must stay intact until its copy to
  // the device has run, so the passes take images from a ring; each entry carries the events that
  // time its pass.
  struct PassImage {
    char *meta_h = nullptr;
    hipEvent_t ev_begin = nullptr, ev_end = nullptr;
    bool pending = false;
    double *ms_into = nullptr;
  };
  std::vector<PassImage> ring;
  size_t ring_next = 0;
  std::vector<hipEvent_t> ev_slot;   // per slot: end of its background prompt reading
  hipEvent_t ev_pre_last = nullptr;  // end of the last cache-only pass enqueued
  bool pre_pending = false;          // a cache-only pass may still be running
  // per weight buffer: end of the last cache-only pass that was enqueued while that buffer was active
  // (what a copy into the buffer, or a fill of it, has to wait for)
  hipEvent_t ev_pre_buf[2] = {nullptr, nullptr};
  bool pre_buf_pending[2] = {false, false};
  float *logits = nullptr;
  int32_t *tok_d = nullptr;
  float *lp_d = nullptr;
  void *samp_ws = nullptr;
  int32_t *tok_h = nullptr;
  float *lp_h = nullptr;
  int attn_chunk = 1024, attn_max_chunks = 1;
  pl::GemmSplit ks_qkv{1, 0, 1}, ks_o{1, 0, 1}, ks_gu{1, 0, 1}, ks_d{1, 0, 1}, ks_lm{1, 0, 1};
  hipStream_t s_dec = nullptr, s_copy = nullptr;
  hipEvent_t ev_a = nullptr, ev_b = nullptr, ev_c = nullptr;
  // The kernel sequence of a decode step, captured once per launch shape and replayed: what fixes a
  // shape is the number of rows, the weight buffer, and the (rounded-up) grid bounds of the two
  // attention kernels; everything that changes from step to step is read from device buffers.
  struct StepGraph {
    int n = 0, buf = 0, items = 0, multi = 0, set = 0;   // set: 0 decode step, 1 cache-only pass
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    uint64_t last_use = 0;
  };
  std::vector<StepGraph> graphs;
  uint64_t graph_clock = 0;
  bool use_graphs = true;
  // optional per-kernel-group timing: events[i] closes a segment of category cats[i]
  bool poison_inactive = false;   // debugging aid: after a flip, fill the buffer that went inactive with NaN
  int profile = 0;   // 0 off, 1 events around the attention launches only, 2 around every kernel group
  std::vector<hipEvent_t> prof_ev;
  std::vector<int> prof_cat;
  size_t prof_n = 0;
  double step_kv_tokens = 0;
  // last step
  int last_n = 0;
  pl_stats st{};
  int64_t streamed_weight_bytes = 0;

};

namespace {

void build_layout(pl_engine *e) {
  const pl_model_cfg &c = e->cfg;
  int64_t off = 0;
  auto add = [&](const std::string &n, int64_t r, int64_t cc) {
    e->layout.push_back(Tensor{n, off, r, cc});
    off += r * cc;
  };
  const int64_t d = c.d_model, qd = (int64_t)c.n_q_heads * c.head_dim, kvd = (int64_t)c.n_kv_heads * c.head_dim;
  add("embed", c.vocab, d);
  for (int l = 0; l < c.n_layers; ++l) {
    std::string p = "l" + std::to_string(l) + ".";
    add(p + "g1", d, 1);
    add(p + "w_qkv", qd + 2 * kvd, d);
    add(p + "w_o", d, qd);
    add(p + "g2", d, 1);
    add(p + "w_gu", 2 * (int64_t)c.d_ffn, d);
    add(p + "w_d", d, c.d_ffn);
  }
  add("gf", d, 1);
  add("lm_head", c.vocab, d);
  e->blob_elems = off;
  e->host_blob_elems = e->tied ? off - (int64_t)c.vocab * d : off;
  e->streamed_weight_bytes = (int64_t)e->esz * (off - (int64_t)c.vocab * d);
}

int check_cfg(const pl_model_cfg &c) {
  if (c.n_layers < 0 || c.d_model <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.d_ffn <= 0 || c.vocab <= 0)
    return fail(PL_E_INVAL, "non-positive model dimension");
  if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return fail(PL_E_INVAL, "head_dim must be 32, 64 or 128");
  if (c.n_q_heads % c.n_kv_heads || c.n_q_heads / c.n_kv_heads > 16)
    return fail(PL_E_INVAL, "n_q_heads must be a multiple of n_kv_heads with at most 16 query heads per kv head");
  if (c.d_model % 256 || c.d_ffn % 256 || (c.n_q_heads * c.head_dim) % 256 || c.d_model > 8192)
    return fail(PL_E_INVAL, "d_model (<= 8192), d_ffn and n_q_heads*head_dim must be multiples of 256");
  if (c.vocab % 32) return fail(PL_E_INVAL, "vocab must be a multiple of 32");
  if (c.max_batch < 1 || c.max_batch > 512) return fail(PL_E_INVAL, "max_batch must be in [1, 512]");
  if (c.max_context < 1) return fail(PL_E_INVAL, "max_context must be positive");
  if (c.kv_page_tokens < 0 || c.kv_page_tokens % 32) return fail(PL_E_INVAL, "kv_page_tokens must be a multiple of 32");
  if (c.n_weight_buffers != 1 && c.n_weight_buffers != 2) return fail(PL_E_INVAL, "n_weight_buffers must be 1 or 2");
  if (!(c.rope_theta > 0) || !(c.rms_eps >= 0)) return fail(PL_E_INVAL, "bad rope_theta / rms_eps");
  if (c.dtype != PL_BF16 && c.dtype != PL_F32) return fail(PL_E_INVAL, "dtype must be PL_BF16 or PL_F32");
  if (c.kv_pool_tokens < 0) return fail(PL_E_INVAL, "kv_pool_tokens must be >= 0 (0 = size the pool from free memory)");
  // the GEMM kernels address a matrix through one 32-bit buffer descriptor
  const int64_t qd = (int64_t)c.n_q_heads * c.head_dim, kvd = (int64_t)c.n_kv_heads * c.head_dim;
  const int64_t biggest = std::max(std::max((int64_t)c.vocab, 2 * (int64_t)c.d_ffn), qd + 2 * kvd) * c.d_model;
  if (biggest * 2 >= pl::GEMM_MAX_OPERAND_BYTES || (int64_t)c.d_model * std::max(qd, (int64_t)c.d_ffn) * 2 >= pl::GEMM_MAX_OPERAND_BYTES)
    return fail(PL_E_INVAL, "a weight matrix would reach %lld bytes; the GEMM kernels address at most 2 GiB per matrix",
                (long long)(biggest * 2));
  return PL_OK;
}

// device memory an automatically sized KV pool leaves to the caller
constexpr int64_t KV_AUTO_RESERVE_BYTES = (int64_t)6 << 30;

void set_pool_pages(pl_engine *e, int64_t n_pages) {
  e->n_pages = n_pages;
  e->layer_stride = e->page_stride * n_pages;
  e->free_pages.clear();
  e->free_pages.reserve(n_pages);
  for (int64_t p = n_pages - 1; p >= 0; --p) e->free_pages.push_back((int32_t)p);   // page 0 is handed out first
  e->st.kv_pages_total = n_pages;
}

template <typename T>
int dev_alloc(T **p, int64_t n_elems) {
  if (n_elems <= 0) n_elems = 1;
  hipError_t err = hipMalloc((void **)p, (size_t)n_elems * sizeof(T));
  if (err != hipSuccess) return fail(PL_E_NOMEM, "hipMalloc of %lld bytes failed: %s", (long long)(n_elems * sizeof(T)), hipGetErrorString(err));
  return PL_OK;
}

int alloc_work(pl_engine *e, pl_engine::Work &w, int64_t R, int64_t parts_elems, bool pinned_image) {
  const pl_model_cfg &c = e->cfg;
  const int64_t d = c.d_model, qd = (int64_t)c.n_q_heads * c.head_dim;
  const int64_t wide = e->esz / 2;   // the activation buffers are declared bf16; the fp32 build needs twice the bytes
  int rc;
  w.rows_cap = (int)R;
  if ((rc = dev_alloc(&w.meta_d, e->meta_bytes))) return rc;
  if ((rc = dev_alloc(&w.h, R * d))) return rc;
  if ((rc = dev_alloc(&w.a, R * d * wide))) return rc;
  if ((rc = dev_alloc(&w.parts, parts_elems))) return rc;
  if ((rc = dev_alloc(&w.q_rot, R * qd * wide))) return rc;
  if ((rc = dev_alloc(&w.attn_out, R * qd * wide))) return rc;
  if ((rc = dev_alloc(&w.mid, R * c.d_ffn * wide))) return rc;
  if ((rc = dev_alloc(&w.cs, R * c.head_dim))) return rc;
  if ((rc = dev_alloc(&w.ctx_len, R))) return rc;
  if ((rc = dev_alloc(&w.pt, (int64_t)c.max_batch * e->pages_per_seq))) return rc;
  const int64_t np = R * c.n_kv_heads * e->attn_max_chunks * e->G;
  if ((rc = dev_alloc(&w.attn_po, np * c.head_dim))) return rc;
  if ((rc = dev_alloc(&w.attn_pml, np * 2))) return rc;
  if ((rc = dev_alloc(&w.attn_work, pl::attention_worklist_ints((int)R, e->attn_max_chunks)))) return rc;
  if (pinned_image) HIP_TRY(hipHostMalloc((void **)&w.meta_h, (size_t)e->meta_bytes, hipHostMallocDefault));
  return PL_OK;
}

void free_work(pl_engine::Work &w) {
  void *dev[] = {w.meta_d, w.h, w.a, w.parts, w.q_rot, w.attn_out, w.mid, w.cs, w.ctx_len, w.pt, w.attn_po, w.attn_pml, w.attn_work};
  for (void *p : dev)
    if (p) (void)hipFree(p);
  w = pl_engine::Work{};
}

constexpr int PASS_RING = 8;   // host metadata images of cache-only passes that may wait on the device at once

int alloc_device(pl_engine *e) {
  const pl_model_cfg &c = e->cfg;
  HIP_TRY(hipSetDevice(c.device));
  HIP_TRY(hipStreamCreateWithFlags(&e->s_dec, hipStreamNonBlocking));
  HIP_TRY(hipStreamCreateWithFlags(&e->s_copy, hipStreamNonBlocking));
  HIP_TRY(hipStreamCreateWithFlags(&e->wk[1].stream, hipStreamNonBlocking));
  e->wk[0].stream = e->s_dec;
  HIP_TRY(hipEventCreate(&e->ev_a));
  HIP_TRY(hipEventCreate(&e->ev_b));
  HIP_TRY(hipEventCreate(&e->ev_c));
  HIP_TRY(hipEventCreate(&e->ev_staged));
  HIP_TRY(hipEventCreate(&e->ev_copy0));
  HIP_TRY(hipEventCreateWithFlags(&e->ev_pre_last, hipEventDisableTiming));
  for (auto &ev : e->ev_pre_buf) HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
  int rc;
  for (int b = 0; b < c.n_weight_buffers; ++b)
    if ((rc = dev_alloc(&e->wbuf[b], e->blob_elems * e->esz))) return rc;
  const int B = c.max_batch;
  const int64_t d = c.d_model, qd = (int64_t)c.n_q_heads * c.head_dim, kvd = (int64_t)c.n_kv_heads * c.head_dim;
  const int64_t wq = qd + 2 * kvd;
  // K splits are fixed by max_batch alone: a pass of any row count adds up every element in the same order
  e->ks_qkv = pl::gemm_pick_split(B, (int)wq, (int)d, 0);
  e->ks_o = pl::gemm_pick_split(B, (int)d, (int)qd, 0);
  e->ks_gu = pl::gemm_pick_split(B, 2 * c.d_ffn, (int)d, 1);
  e->ks_d = pl::gemm_pick_split(B, (int)d, c.d_ffn, 0);
  e->ks_lm = pl::GemmSplit{1, c.vocab, 1};
  const int64_t R = e->rows_cap;   // rows of the activation buffers (cache-only passes take up to 256 rows)
  int64_t parts = std::max(std::max(std::max(e->ks_qkv.splits * wq, e->ks_o.splits * d), e->ks_d.splits * d) * R,
                           pl::gemm_workspace_elems((int)R, 2 * c.d_ffn, e->ks_gu));
  if (e->f32) parts = R * std::max(wq, 2 * (int64_t)c.d_ffn);   // the fp32 build keeps whole products there
  // the chunk length is fixed by max_batch alone, so a sequence's attention result never depends on
  // how many rows a pass holds
  e->attn_chunk = pl::attention_chunk_tokens(B, c.n_kv_heads, c.max_context);
  e->attn_max_chunks = (c.max_context + e->attn_chunk - 1) / e->attn_chunk;
  if ((rc = alloc_work(e, e->wk[0], R, parts, true))) return rc;
  if ((rc = alloc_work(e, e->wk[1], R, parts, false))) return rc;
  e->ring.resize(PASS_RING);
  for (auto &im : e->ring) {
    HIP_TRY(hipHostMalloc((void **)&im.meta_h, (size_t)e->meta_bytes, hipHostMallocDefault));
    HIP_TRY(hipEventCreate(&im.ev_begin));
    HIP_TRY(hipEventCreate(&im.ev_end));
  }
  e->ev_slot.resize(B);
  for (auto &ev : e->ev_slot) HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
  if ((rc = dev_alloc(&e->logits, (int64_t)B * c.vocab))) return rc;
  if ((rc = dev_alloc(&e->tok_d, B))) return rc;
  if ((rc = dev_alloc(&e->lp_d, B))) return rc;
  char *ws = nullptr;
  if ((rc = dev_alloc(&ws, pl::sample_workspace_bytes(B, c.vocab)))) return rc;
  e->samp_ws = ws;
  // the KV pool comes last: with kv_pool_tokens == 0 it takes what is left of the device memory, minus
  // a reserve for the caller, up to the most the slots could ever use
  if (e->n_pages == 0) {
    size_t free_b = 0, total_b = 0;
    HIP_TRY(hipMemGetInfo(&free_b, &total_b));
    const int64_t page_bytes = e->page_stride * e->esz * std::max(c.n_layers, 1);
    const int64_t avail = (int64_t)free_b - KV_AUTO_RESERVE_BYTES;
    const int64_t most = (int64_t)B * e->pages_per_seq;
    e->n_pages = std::min(avail > 0 ? avail / page_bytes : 0, most);
    if (e->n_pages < 1) return fail(PL_E_NOMEM, "no device memory left for a KV pool (%lld bytes free)", (long long)free_b);
    set_pool_pages(e, e->n_pages);
  }
  const int64_t pool_elems = e->layer_stride * c.n_layers;
  if ((rc = dev_alloc(&e->kv_pool, pool_elems * e->esz))) return rc;
  // Every position a kernel may touch must hold a finite value: masked soft-max weights are
  // exactly 0, and 0 * finite stays 0.
  HIP_TRY(hipMemsetAsync(e->kv_pool, 0, (size_t)pool_elems * e->esz, e->s_dec));
  HIP_TRY(hipHostMalloc((void **)&e->pt_h, (size_t)B * e->pages_per_seq * 4, hipHostMallocDefault));
  HIP_TRY(hipHostMalloc((void **)&e->tok_h, (size_t)B * 4, hipHostMallocDefault));
  HIP_TRY(hipHostMalloc((void **)&e->lp_h, (size_t)B * 4, hipHostMallocDefault));
  memset(e->pt_h, 0, (size_t)B * e->pages_per_seq * 4);
  HIP_TRY(hipStreamSynchronize(e->s_dec));
  return PL_OK;
}

LayerW layer_weights(const pl_engine *e, int l) {
  const bf16_t *base = (const bf16_t *)e->wbuf[e->active_buf];
  const Tensor *t = &e->layout[1 + (size_t)l * 6];
  return LayerW{base + t[0].offset, base + t[1].offset, base + t[2].offset,
                base + t[3].offset, base + t[4].offset, base + t[5].offset};
}

// The fixed kernel sequence of one decode step over n rows (rows = occupied slots, slot order).
enum { CAT_OTHER = 0, CAT_ATTN = 1, CAT_GEMM = 2, CAT_SAMPLE = 3 };

// Close the segment of work enqueued since the previous mark and attribute it to `cat`.
void mark(pl_engine *e, int cat, bool attention_edge = false) {
  if (!e->profile || (e->profile == 1 && !attention_edge)) return;
  if (e->prof_n == e->prof_ev.size()) {
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) return;
    e->prof_ev.push_back(ev);
    e->prof_cat.push_back(cat);
  }
  e->prof_cat[e->prof_n] = cat;
  (void)hipEventRecord(e->prof_ev[e->prof_n++], e->s_dec);
}

// The same step in the fp32 test build: plain kernels, whole products in `parts`, no K split, no
// attention chunks.  Same order of operations as the definition: embed, per layer norm, q|k|v, rotary,
// append, attention, +W_o, norm, SwiGLU, +W_d, final norm, LM head, sampler.
int enqueue_step_f32(pl_engine *e, pl_engine::Work &w, int n, bool prefill) {
  const pl_model_cfg &c = e->cfg;
  hipStream_t s = w.stream;
  if (!prefill) e->prof_n = 0;
  const float *base = (const float *)e->wbuf[e->active_buf];
  auto T = [&](size_t i) { return base + e->layout[i].offset; };
  const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, wq = qd + 2 * kvd;
  const size_t last = e->layout.size() - 1;
  float *a = (float *)w.a, *q_rot = (float *)w.q_rot, *attn_out = (float *)w.attn_out, *mid = (float *)w.mid;
  int rc = 0;
  rc |= pl::launch_rope_tables(w.m_pos(true), w.cs, w.ctx_len, n, c.head_dim, c.rope_theta, s);
  rc |= pl::f32_launch_norm(T(0), w.m_input(true), c.vocab, nullptr, c.n_layers ? T(1) : T(last - 1), w.h, a, n, d, c.rms_eps, s);
  for (int l = 0; l < c.n_layers && !rc; ++l) {
    const size_t t0 = 1 + (size_t)l * 6;   // g1, w_qkv, w_o, g2, w_gu, w_d
    float *kv_layer = (float *)e->kv_pool + (int64_t)l * e->layer_stride;
    rc |= pl::f32_launch_gemm(a, T(t0 + 1), w.parts, n, wq, d, s);
    rc |= pl::f32_launch_rope_append(w.parts, w.cs, w.m_pos(true), w.m_row_slot(true), w.pt, q_rot, kv_layer, n,
                                     c.n_q_heads, c.n_kv_heads, c.head_dim, e->page_tokens, e->pages_per_seq, s);
    if (prefill && l + 1 == c.n_layers) break;
    rc |= pl::f32_launch_attention(q_rot, kv_layer, w.pt, w.m_pos(true), w.m_row_slot(true), attn_out, n, c.n_q_heads,
                                   c.n_kv_heads, c.head_dim, e->page_tokens, e->pages_per_seq, s);
    rc |= pl::f32_launch_gemm(attn_out, T(t0 + 2), w.parts, n, d, qd, s);
    rc |= pl::f32_launch_norm(nullptr, nullptr, 0, w.parts, T(t0 + 3), w.h, a, n, d, c.rms_eps, s);
    rc |= pl::f32_launch_gemm(a, T(t0 + 4), w.parts, n, 2 * c.d_ffn, d, s);
    rc |= pl::f32_launch_swiglu(w.parts, mid, n, c.d_ffn, s);
    rc |= pl::f32_launch_gemm(mid, T(t0 + 5), w.parts, n, d, c.d_ffn, s);
    rc |= pl::f32_launch_norm(nullptr, nullptr, 0, w.parts, l + 1 < c.n_layers ? T(t0 + 6) : T(last - 1), w.h, a, n, d,
                              c.rms_eps, s);
  }
  if (prefill) return rc ? fail(PL_E_HIP, "kernel launch failed: %s", hipGetErrorString(hipGetLastError())) : PL_OK;
  rc |= pl::f32_launch_gemm(a, T(last), e->logits, n, c.vocab, d, s);
  pl::SampleParams sp{};
  sp.logits = e->logits; sp.n = n; sp.vocab = c.vocab; sp.seq_id = w.m_seq_id(true);
  sp.position = w.m_pos(true); sp.inv_t = w.m_inv_t(true); sp.forced = w.m_forced(true);
  sp.seed = c.seed; sp.token = e->tok_d; sp.logprob = e->lp_d; sp.workspace = e->samp_ws;
  rc |= pl::launch_sample(sp, s);
  return rc ? fail(PL_E_HIP, "kernel launch failed: %s", hipGetErrorString(hipGetLastError())) : PL_OK;
}

// prefill: cache-only pass; only the keys and values the rows leave in the cache are wanted, so the
// last layer stops after its append and there is no LM head or sampler.  Runs on the work set's stream.
int enqueue_step(pl_engine *e, pl_engine::Work &w, int n, bool prefill = false) {
  const pl_model_cfg &c = e->cfg;
  hipStream_t s = w.stream;
  if (e->f32) return enqueue_step_f32(e, w, n, prefill);
  const bool timed = !prefill;   // the per-group timers describe decode steps only
  if (timed) { e->prof_n = 0; mark(e, CAT_OTHER); }
  const bf16_t *base = (const bf16_t *)e->wbuf[e->active_buf];
  const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, wq = qd + 2 * kvd;
  const bf16_t *embed = base + e->layout.front().offset;
  const bf16_t *gf = base + e->layout[e->layout.size() - 2].offset;
  const bf16_t *lm = base + e->layout.back().offset;
  int rc = 0;
  rc |= pl::launch_rope_tables(w.m_pos(true), w.cs, w.ctx_len, n, c.head_dim, c.rope_theta, s);
  rc |= pl::launch_attention_worklist(w.ctx_len, w.m_row_slot(true), w.pt, w.attn_work, n, e->attn_max_chunks,
                                      e->attn_chunk, e->page_tokens, e->pages_per_seq, s);
  const bf16_t *g_first = c.n_layers ? layer_weights(e, 0).g1 : gf;
  rc |= pl::launch_embed_rmsnorm(embed, g_first, w.m_input(true), nullptr, w.m_row_slot(true), w.h, w.a, n,
                                 d, c.vocab, c.rms_eps, s);
  for (int l = 0; l < c.n_layers && !rc; ++l) {
    const LayerW lw = layer_weights(e, l);
    bf16_t *kv_layer = (bf16_t *)e->kv_pool + (int64_t)l * e->layer_stride;
    if (timed) mark(e, CAT_OTHER);
    rc |= pl::launch_gemm(w.a, lw.w_qkv, w.parts, nullptr, n, wq, d, 0, e->ks_qkv, s);
    if (timed) mark(e, CAT_GEMM);
    rc |= pl::launch_rope_append(w.parts, e->ks_qkv.splits, w.cs, w.m_pos(true), w.m_row_slot(true), w.pt,
                                 w.q_rot, kv_layer, n, c.n_q_heads, c.n_kv_heads, c.head_dim, e->page_tokens,
                                 e->pages_per_seq, s);
    pl::AttnParams ap{};
    ap.q = w.q_rot; ap.kv = kv_layer; ap.page_table = w.pt; ap.ctx_len = w.ctx_len;
    ap.row_slot = w.m_row_slot(true); ap.out = w.attn_out; ap.part_o = w.attn_po; ap.part_ml = w.attn_pml;
    ap.n_seq = n; ap.Hq = c.n_q_heads; ap.Hkv = c.n_kv_heads; ap.hd = c.head_dim;
    ap.page_tokens = e->page_tokens; ap.pages_per_seq = e->pages_per_seq; ap.chunk = e->attn_chunk;
    ap.max_chunks = e->attn_max_chunks;
    ap.work = w.attn_work; ap.max_items = w.attn_items;
    ap.multi = pl::attention_multi_list(w.attn_work, n, e->attn_max_chunks); ap.max_multi = w.attn_multi;
    if (prefill && l + 1 == c.n_layers) break;
    if (timed && e->profile) {   // the timers bracket the decode kernel alone; the merge kernel counts as "other"
      mark(e, CAT_OTHER, true);
      rc |= pl::launch_attention(ap, s, 1);
      mark(e, CAT_ATTN, true);
      rc |= pl::launch_attention(ap, s, 2);
      mark(e, CAT_OTHER);
    } else {
      rc |= pl::launch_attention(ap, s);
    }
    rc |= pl::launch_gemm(w.attn_out, lw.w_o, w.parts, nullptr, n, d, qd, 0, e->ks_o, s);
    if (timed) mark(e, CAT_GEMM);
    rc |= pl::launch_resid_rmsnorm(w.h, w.parts, e->ks_o.splits, lw.g2, w.a, n, d, c.rms_eps, s);
    if (timed) mark(e, CAT_OTHER);
    rc |= pl::launch_gemm(w.a, lw.w_gu, w.mid, w.parts, n, 2 * c.d_ffn, d, 1, e->ks_gu, s);
    rc |= pl::launch_gemm(w.mid, lw.w_d, w.parts, nullptr, n, d, c.d_ffn, 0, e->ks_d, s);
    if (timed) mark(e, CAT_GEMM);
    const bf16_t *g_next = (l + 1 < c.n_layers) ? layer_weights(e, l + 1).g1 : gf;
    rc |= pl::launch_resid_rmsnorm(w.h, w.parts, e->ks_d.splits, g_next, w.a, n, d, c.rms_eps, s);
  }
  if (prefill) return rc ? fail(PL_E_HIP, "kernel launch failed: %s", hipGetErrorString(hipGetLastError())) : PL_OK;
  mark(e, CAT_OTHER);
  rc |= pl::launch_gemm(w.a, lm, e->logits, nullptr, n, c.vocab, d, 0, e->ks_lm, s);
  mark(e, CAT_GEMM);
  pl::SampleParams sp{};
  sp.logits = e->logits; sp.n = n; sp.vocab = c.vocab; sp.seq_id = w.m_seq_id(true);
  sp.position = w.m_pos(true); sp.inv_t = w.m_inv_t(true); sp.forced = w.m_forced(true);
  sp.seed = c.seed; sp.token = e->tok_d; sp.logprob = e->lp_d; sp.workspace = e->samp_ws;
  sp.last_tok = nullptr; sp.row_slot = nullptr;
  rc |= pl::launch_sample(sp, s);
  mark(e, CAT_SAMPLE);
  return rc ? fail(PL_E_HIP, "kernel launch failed: %s", hipGetErrorString(hipGetLastError())) : PL_OK;
}

constexpr size_t MAX_STEP_GRAPHS = 32;

void drop_graph(pl_engine::StepGraph &g) {
  if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (g.graph) (void)hipGraphDestroy(g.graph);
  g = pl_engine::StepGraph{};
}

// Run the kernels of a decode step (or of a cache-only pass) for n rows on the work set's stream: as
// the replay of a captured graph when one may be used (no per-kernel timers on the decode step), launch
// by launch otherwise.
int run_step(pl_engine *e, pl_engine::Work &w, int n, bool prefill = false) {
  if (!e->use_graphs || (!prefill && e->profile != 0)) return enqueue_step(e, w, n, prefill);
  const int set = prefill ? 1 : 0;
  // grid bounds of the attention kernels in coarse steps, so that few shapes occur; workgroups beyond
  // the lists' real lengths (which the kernels read from device memory) leave at once
  w.attn_items = std::min((w.attn_items + 63) / 64 * 64, n * e->attn_max_chunks);
  if (w.attn_multi) w.attn_multi = std::min((w.attn_multi + 15) / 16 * 16, n);
  pl_engine::StepGraph *g = nullptr;
  for (auto &x : e->graphs)
    if (x.n == n && x.buf == e->active_buf && x.items == w.attn_items && x.multi == w.attn_multi && x.set == set) { g = &x; break; }
  if (!g) {
    if (e->graphs.size() >= MAX_STEP_GRAPHS) {   // evict the least recently used
      size_t lru = 0;
      for (size_t i = 1; i < e->graphs.size(); ++i)
        if (e->graphs[i].last_use < e->graphs[lru].last_use) lru = i;
      drop_graph(e->graphs[lru]);
      e->graphs.erase(e->graphs.begin() + lru);
    }
    pl_engine::StepGraph ng;
    ng.n = n; ng.buf = e->active_buf; ng.items = w.attn_items; ng.multi = w.attn_multi; ng.set = set;
    HIP_TRY(hipStreamBeginCapture(w.stream, hipStreamCaptureModeThreadLocal));
    const int rc = enqueue_step(e, w, n, prefill);
    const hipError_t ce = hipStreamEndCapture(w.stream, &ng.graph);
    hipError_t ie = hipSuccess;
    if (!rc && ce == hipSuccess) ie = hipGraphInstantiate(&ng.exec, ng.graph, nullptr, nullptr, 0);
    if (rc || ce != hipSuccess || ie != hipSuccess) {
      // Nothing was executed while capturing.  If the runtime cannot capture or instantiate this
      // sequence, the engine goes on launching kernel by kernel (same results) for the rest of its life.
      drop_graph(ng);
      (void)hipGetLastError();
      if (rc) return rc;
      e->use_graphs = false;
      return enqueue_step(e, w, n, prefill);
    }
    e->graphs.push_back(ng);
    g = &e->graphs.back();
  }
  g->last_use = ++e->graph_clock;
  HIP_TRY(hipGraphLaunch(g->exec, w.stream));
  return PL_OK;
}

// Tied embeddings: the LM head of weight buffer `buf` is the embedding table, stored once more in the
// layout the LM-head GEMM streams.  Enqueued behind the copy that brought the blob in.
int tie_lm_head(pl_engine *e, int buf, hipStream_t s) {
  if (!e->tied) return PL_OK;
  const pl_model_cfg &c = e->cfg;
  char *base = e->wbuf[buf];
  const int64_t eo = e->layout.front().offset, lo = e->layout.back().offset;
  if (pl::launch_tie_lm_head(base + eo * e->esz, base + lo * e->esz, c.vocab, c.d_model, e->f32, s))
    return fail(PL_E_HIP, "LM-head tie launch failed");
  return PL_OK;
}

void activate_staged(pl_engine *e) {
  if (e->cfg.n_weight_buffers == 2) e->active_buf ^= 1;
  e->version = e->staged_version;
  e->staged = false;
  e->st.swaps++;
}

int admit(pl_engine *e, uint64_t seq_id, const int32_t *prompt, int32_t n_prompt, int32_t max_new, float temp,
          int32_t context_len, int32_t n_emitted, int32_t last_token, int32_t *out_slot) {
  const pl_model_cfg &c = e->cfg;
  if (n_prompt < 1 || max_new < 1 || !(temp > 0.f) || !std::isfinite(temp))
    return fail(PL_E_INVAL, "need n_prompt >= 1, max_new >= 1, temperature > 0");
  if ((int64_t)n_prompt + max_new - 1 > c.max_context) return fail(PL_E_CTX, "n_prompt + max_new - 1 exceeds max_context");
  const bool need_prompt = context_len < n_prompt;
  if (need_prompt && !prompt) return fail(PL_E_INVAL, "prompt is NULL");
  if (context_len < 0 || context_len > n_prompt + max_new - 1 || n_emitted < 0 || n_emitted >= max_new)
    return fail(PL_E_INVAL, "inconsistent context_len / n_emitted");
  if (prompt)
    for (int i = 0; i < n_prompt; ++i)
      if (prompt[i] < 0 || prompt[i] >= c.vocab) return fail(PL_E_INVAL, "prompt token %d out of range", prompt[i]);
  if (context_len >= n_prompt && (last_token < 0 || last_token >= c.vocab)) return fail(PL_E_INVAL, "last_token out of range");
  int slot = -1;
  for (int i = 0; i < c.max_batch; ++i)
    if (!e->seqs[i].active) { slot = i; break; }
  if (slot < 0) return fail(PL_E_NOSLOT, "all %d slots are occupied", c.max_batch);
  // pages for what is already cached (or, for a fresh sequence, for its prompt)
  const int64_t need_tok = std::max<int64_t>(context_len, n_prompt);
  const int64_t want_pages = (need_tok + e->page_tokens - 1) / e->page_tokens;
  const int64_t need_pages = want_pages;
  if ((int64_t)e->free_pages.size() < want_pages) return fail(PL_E_NOKV, "KV pool cannot hold the prompt (%lld pages free)", (long long)e->free_pages.size());
  Seq &q = e->seqs[slot];
  q = Seq{};
  q.active = true;
  q.seq_id = seq_id;
  if (prompt) q.prompt.assign(prompt, prompt + n_prompt);
  q.n_prompt = n_prompt;
  q.max_new = max_new;
  q.inv_t = 1.0f / temp;
  q.pos = context_len;
  q.hist_known = context_len == 0;
  q.n_emitted = n_emitted;
  q.next_input = last_token;
  for (int64_t i = 0; i < need_pages; ++i) {
    q.pages.push_back(e->free_pages.back());
    e->free_pages.pop_back();
    if (e->pt_h) e->pt_h[(int64_t)slot * e->pages_per_seq + i] = q.pages.back();
  }
  e->pt_dirty = true;
  if (out_slot) *out_slot = slot;
  return PL_OK;
}

// Add the GPU time of finished cache-only passes to the counters they belong to.
void harvest_passes(pl_engine *e) {
  for (auto &im : e->ring) {
    if (!im.pending || hipEventQuery(im.ev_end) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, im.ev_begin, im.ev_end) == hipSuccess && im.ms_into) *im.ms_into += ms;
    im.pending = false;
  }
  (void)hipGetLastError();
}

// Wait for every cache-only pass enqueued so far; slots whose prompts were being read join the batch.
int drain_passes(pl_engine *e) {
  if (e->dry) {
    for (Seq &q : e->seqs) q.reading = false;
    return PL_OK;
  }
  if (e->pre_pending) {
    HIP_TRY(hipStreamSynchronize(e->wk[1].stream));
    e->pre_pending = false;
    e->pre_buf_pending[0] = e->pre_buf_pending[1] = false;
  }
  harvest_passes(e);
  for (Seq &q : e->seqs) q.reading = false;
  return PL_OK;
}

// Cache-only passes: rows (slot, position, token) go through the decode kernels in prefill mode, in
// groups of up to 256, on the second work set's stream; the rows of one slot must come in position
// order, because a row attends to the keys and values that earlier rows of its slot (in this or an
// earlier group) leave.  Returns once everything is enqueued; the caller waits (or records an event).
int run_kv_passes(pl_engine *e, const std::vector<int32_t> &slots, const std::vector<int32_t> &positions,
                  const std::vector<int32_t> &tokens, double *ms_total, uint64_t *passes) {
  const pl_model_cfg &c = e->cfg;
  const int rows_max = 256;
  pl_engine::Work &w = e->wk[1];
  if (!e->dry) HIP_TRY(hipSetDevice(c.device));
  const size_t total = slots.size();
  for (size_t r0 = 0; r0 < total; r0 += rows_max) {
    const int n = (int)std::min<size_t>(rows_max, total - r0);
    if (!e->dry) {
      // next host image of the ring; if its previous pass has not run yet, wait for it
      pl_engine::PassImage &im = e->ring[e->ring_next];
      e->ring_next = (e->ring_next + 1) % e->ring.size();
      if (im.pending) {
        HIP_TRY(hipEventSynchronize(im.ev_end));
        harvest_passes(e);
      }
      w.meta_h = im.meta_h;
      int items = 0, multi = 0;
      int32_t *row_slot = w.m_row_slot(false), *pos = w.m_pos(false), *inp = w.m_input(false), *frc = w.m_forced(false);
      float *inv_t = w.m_inv_t(false);
      uint64_t *sid = w.m_seq_id(false);
      for (int r = 0; r < n; ++r) {
        const Seq &q = e->seqs[slots[r0 + r]];
        row_slot[r] = slots[r0 + r];
        pos[r] = positions[r0 + r];
        inp[r] = tokens[r0 + r];
        frc[r] = -1;
        inv_t[r] = q.inv_t;
        sid[r] = q.seq_id;
        items += (pos[r] + 1 + e->attn_chunk - 1) / e->attn_chunk;
        multi += pos[r] + 1 > e->attn_chunk;
      }
      w.attn_items = items;
      w.attn_multi = multi;
      hipStream_t s = w.stream;
      // The page table goes up on this stream into this set's own device copy (no device buffer is ever
      // written from two streams); the rows of the slots being read do not change while they are read.
      // The dirty flag stays: the decode stream sends the table to its own copy.
      if (r0 == 0)
        HIP_TRY(hipMemcpyAsync(w.pt, e->pt_h, (size_t)c.max_batch * e->pages_per_seq * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(hipMemcpyAsync(w.meta_d, w.meta_h, (size_t)e->meta_bytes, hipMemcpyHostToDevice, s));
      HIP_TRY(hipEventRecord(im.ev_begin, s));
      int rc = run_step(e, w, n, true);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(im.ev_end, s));
      im.pending = true;
      im.ms_into = ms_total;
      e->pre_pending = true;
    }
    ++*passes;
  }
  if (!e->dry && total) {
    HIP_TRY(hipEventRecord(e->ev_pre_last, w.stream));
    HIP_TRY(hipEventRecord(e->ev_pre_buf[e->active_buf], w.stream));
    e->pre_buf_pending[e->active_buf] = true;
  }
  return PL_OK;
}

// "KV cache recomputed" variant of Sec. 5.1: after a flip, replay every token each sequence has read
// so far under the new weights, overwriting its cached keys and values in place.
int recompute_all_kv(pl_engine *e) {
  int rc = drain_passes(e);   // prompts still being read in the background finish first
  if (rc) return rc;
  std::vector<int32_t> slots, positions, tokens;
  for (int s = 0; s < e->cfg.max_batch; ++s) {
    const Seq &q = e->seqs[s];
    if (!q.active) continue;
    for (int p = 0; p < q.pos; ++p) {
      slots.push_back(s);
      positions.push_back(p);
      tokens.push_back(q.hist[p]);
    }
  }
  rc = run_kv_passes(e, slots, positions, tokens, &e->st.recompute_ms, &e->st.recompute_passes);
  if (rc) return rc;
  if ((rc = drain_passes(e))) return rc;
  e->st.recompute_positions += slots.size();
  return PL_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
extern "C" {

const char *pl_last_error(void) { return g_err; }

int pl_create(const pl_model_cfg *cfg, pl_engine **out) {
  if (!cfg || !out) return fail(PL_E_INVAL, "NULL argument");
  *out = nullptr;
  int rc = check_cfg(*cfg);
  if (rc) return rc;
  pl_engine *e = new (std::nothrow) pl_engine();
  if (!e) return fail(PL_E_NOMEM, "out of host memory");
  e->cfg = *cfg;
  e->dry = cfg->device == PL_DEVICE_NONE;
  e->f32 = cfg->dtype == PL_F32;
  e->esz = e->f32 ? 4 : 2;
  e->tied = cfg->tie_embeddings != 0;
  e->G = cfg->n_q_heads / cfg->n_kv_heads;
  e->page_tokens = cfg->kv_page_tokens ? cfg->kv_page_tokens : 128;
  e->pages_per_seq = (cfg->max_context + e->page_tokens - 1) / e->page_tokens;
  e->page_stride = (int64_t)cfg->n_kv_heads * 2 * e->page_tokens * cfg->head_dim;
  int64_t n_pages = cfg->kv_pool_tokens / e->page_tokens;
  if (cfg->kv_pool_tokens == 0)   // automatic: a bookkeeping-only engine gets the most its slots can use
    n_pages = e->dry ? (int64_t)cfg->max_batch * e->pages_per_seq : 0;
  else if (n_pages < 1) {
    delete e;
    return fail(PL_E_INVAL, "kv_pool_tokens must hold at least one page");
  }
  if (n_pages > 0x7FFFFFFF) {
    delete e;
    return fail(PL_E_INVAL, "KV pool of more than 2^31 pages");
  }
  build_layout(e);
  e->seqs.resize(cfg->max_batch);
  set_pool_pages(e, n_pages);
  e->rows_cap = std::max(cfg->max_batch, 256);
  e->meta_bytes = (int64_t)e->rows_cap * (4 * 5 + 8);
  e->wk[0].rows_cap = e->wk[1].rows_cap = e->rows_cap;
  if (e->dry) {
    e->wk[0].meta_h = (char *)calloc(1, (size_t)e->meta_bytes);
    if (!e->wk[0].meta_h) { delete e; return fail(PL_E_NOMEM, "out of host memory"); }
  } else {
    if (cfg->device < 0) { delete e; return fail(PL_E_INVAL, "bad device"); }
    rc = alloc_device(e);
    if (rc) { pl_destroy(e); return rc; }
  }
  *out = e;
  return PL_OK;
}

void pl_destroy(pl_engine *e) {
  if (!e) return;
  if (e->dry) {
    free(e->wk[0].meta_h);
  } else {
    (void)hipSetDevice(e->cfg.device);
    if (e->s_dec) (void)hipStreamSynchronize(e->s_dec);
    if (e->s_copy) (void)hipStreamSynchronize(e->s_copy);
    if (e->wk[1].stream) (void)hipStreamSynchronize(e->wk[1].stream);
    void *dev[] = {e->wbuf[0], e->wbuf[1], e->kv_pool, e->logits, e->tok_d, e->lp_d, e->samp_ws};
    for (void *p : dev)
      if (p) (void)hipFree(p);
    void *hst[] = {e->pt_h, e->wk[0].meta_h, e->tok_h, e->lp_h};
    for (void *p : hst)
      if (p) (void)hipHostFree(p);
    for (auto &g : e->graphs) drop_graph(g);
    hipStream_t s_pre = e->wk[1].stream;
    free_work(e->wk[0]);
    free_work(e->wk[1]);
    for (auto &im : e->ring) {
      if (im.meta_h) (void)hipHostFree(im.meta_h);
      if (im.ev_begin) (void)hipEventDestroy(im.ev_begin);
      if (im.ev_end) (void)hipEventDestroy(im.ev_end);
    }
    for (hipEvent_t ev : e->ev_slot)
      if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : e->prof_ev) (void)hipEventDestroy(ev);
    hipEvent_t evs[] = {e->ev_a, e->ev_b, e->ev_c, e->ev_staged, e->ev_copy0, e->ev_pre_last, e->ev_pre_buf[0], e->ev_pre_buf[1]};
    for (hipEvent_t ev : evs)
      if (ev) (void)hipEventDestroy(ev);
    if (e->s_dec) (void)hipStreamDestroy(e->s_dec);
    if (e->s_copy) (void)hipStreamDestroy(e->s_copy);
    if (s_pre) (void)hipStreamDestroy(s_pre);
  }
  delete e;
}

// the caller's blob ends before the LM head when that is tied to the embedding table
int32_t pl_weight_count(const pl_engine *e) { return e ? (int32_t)e->layout.size() - (e->tied ? 1 : 0) : 0; }

int pl_weight_layout(const pl_engine *e, int32_t idx, const char **name, int64_t *offset_elems, int64_t shape[2]) {
  if (!e || idx < 0 || idx >= pl_weight_count(e)) return fail(PL_E_INVAL, "tensor index out of range");
  const Tensor &t = e->layout[idx];
  if (name) *name = t.name.c_str();
  if (offset_elems) *offset_elems = t.offset;
  if (shape) { shape[0] = t.rows; shape[1] = t.cols; }
  return PL_OK;
}

int64_t pl_weight_nbytes(const pl_engine *e) { return e ? e->host_blob_elems * e->esz : 0; }

int pl_pack_weights(const pl_engine *e, const char *name, const void *src, int32_t src_is_f32, void *blob) {
  if (!e || !name || !src || !blob) return fail(PL_E_INVAL, "NULL argument");
  const pl_model_cfg &c = e->cfg;
  const int64_t d = c.d_model, qd = (int64_t)c.n_q_heads * c.head_dim, kvd = (int64_t)c.n_kv_heads * c.head_dim;
  // source tensor -> (blob tensor, rows and columns of the source, where its rows go)
  std::string target = name;
  int64_t rows = 0, cols = d, row0 = 0;
  int interleave = -1;   // 0 / 1: gate / up rows of the 32-row interleaved w_gu
  const size_t dot = target.find('.');
  const std::string leaf = dot == std::string::npos ? target : target.substr(dot + 1);
  const std::string pre = dot == std::string::npos ? "" : target.substr(0, dot + 1);
  if (dot == std::string::npos) {
    if (leaf == "embed" || leaf == "lm_head") rows = c.vocab;
    else if (leaf == "gf") { rows = d; cols = 1; }
    else return fail(PL_E_INVAL, "unknown tensor '%s'", name);
  } else if (leaf == "g1" || leaf == "g2") { rows = d; cols = 1; }
  else if (leaf == "wq") { rows = qd; target = pre + "w_qkv"; }
  else if (leaf == "wk") { rows = kvd; row0 = qd; target = pre + "w_qkv"; }
  else if (leaf == "wv") { rows = kvd; row0 = qd + kvd; target = pre + "w_qkv"; }
  else if (leaf == "wo") { rows = d; cols = qd; target = pre + "w_o"; }
  else if (leaf == "wg") { rows = c.d_ffn; interleave = 0; target = pre + "w_gu"; }
  else if (leaf == "wu") { rows = c.d_ffn; interleave = 1; target = pre + "w_gu"; }
  else if (leaf == "wd") { rows = d; cols = c.d_ffn; target = pre + "w_d"; }
  else return fail(PL_E_INVAL, "unknown tensor '%s'", name);
  const Tensor *t = nullptr;
  for (const Tensor &x : e->layout)
    if (x.name == target) { t = &x; break; }
  if (!t) return fail(PL_E_INVAL, "unknown tensor '%s'", name);
  if (e->tied && t->name == "lm_head") return fail(PL_E_INVAL, "the LM head is tied to the embedding table; the blob holds no lm_head");
  if (e->f32) {   // test build: fp32, row-major, rows placed at row0 (gate rows first, then up rows)
    if (!src_is_f32) return fail(PL_E_INVAL, "the fp32 build packs fp32 sources");
    if (interleave == 1) row0 = c.d_ffn;
    memcpy((float *)blob + t->offset + row0 * cols, src, (size_t)(rows * cols) * 4);
    return PL_OK;
  }
  uint16_t *dst = (uint16_t *)blob + t->offset;
  auto bits = [&](int64_t i) -> uint16_t {
    return src_is_f32 ? f32_to_bf16_bits(((const float *)src)[i]) : ((const uint16_t *)src)[i];
  };
  if (t->cols == 1 || t->name == "embed") {   // stored as they are
    for (int64_t i = 0; i < rows * cols; ++i) dst[i] = bits(i);
    return PL_OK;
  }
  const int64_t row_blocks = t->rows / 32;
  for (int64_t r = 0; r < rows; ++r) {
    const int64_t R = interleave < 0 ? row0 + r : 64 * (r / 32) + 32 * interleave + r % 32;
    for (int64_t k = 0; k < cols; ++k) {
      const int64_t o = ((k / 64) * row_blocks + R / 32) * 2048 + ((k % 32) / 8) * 512 + ((k % 64) / 32) * 256 + (R % 32) * 8 + k % 8;
      dst[o] = bits(r * cols + k);
    }
  }
  return PL_OK;
}

int pl_load_weights(pl_engine *e, const void *src, int64_t nbytes) {
  if (!e || !src) return fail(PL_E_INVAL, "NULL argument");
  if (nbytes != e->host_blob_elems * e->esz) return fail(PL_E_INVAL, "weight blob is %lld bytes, expected %lld", (long long)nbytes, (long long)(e->host_blob_elems * e->esz));
  if (e->staged) return fail(PL_E_BUSY, "a weight update is staged");
  if (!e->dry) {
    HIP_TRY(hipSetDevice(e->cfg.device));
    HIP_TRY(hipStreamSynchronize(e->s_dec));
    HIP_TRY(hipStreamSynchronize(e->wk[1].stream));   // a prompt read in the background finishes under the old weights
    HIP_TRY(hipMemcpy(e->wbuf[e->active_buf], src, (size_t)nbytes, hipMemcpyDefault));
    int rc = tie_lm_head(e, e->active_buf, e->s_dec);
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(e->s_dec));
  }
  if (e->loaded) { e->version++; e->st.swaps++; }
  e->loaded = true;
  return PL_OK;
}

int pl_swap_weights(pl_engine *e, const void *src, int64_t nbytes, uint32_t flags, uint32_t *out_new_version) {
  if (!e || !src) return fail(PL_E_INVAL, "NULL argument");
  if (flags & ~(PL_SWAP_WAIT | PL_SWAP_RECOMPUTE_KV)) return fail(PL_E_INVAL, "unknown flags");
  if (flags & PL_SWAP_RECOMPUTE_KV)
    for (const Seq &q : e->seqs)
      if (q.active && !q.hist_known) return fail(PL_E_STATE, "a sequence was admitted without its token history; its cache cannot be recomputed");
  if (nbytes != e->host_blob_elems * e->esz) return fail(PL_E_INVAL, "weight blob is %lld bytes, expected %lld", (long long)nbytes, (long long)(e->host_blob_elems * e->esz));
  if (!e->loaded) return fail(PL_E_STATE, "no weights loaded yet");
  if (e->staged) return fail(PL_E_BUSY, "the previous weight update is not active yet");
  e->staged_version = e->version + 1;
  e->staged_wait = (flags & PL_SWAP_WAIT) != 0;
  e->staged_recompute = (flags & PL_SWAP_RECOMPUTE_KV) != 0;
  if (!e->dry) {
    HIP_TRY(hipSetDevice(e->cfg.device));
    if (e->cfg.n_weight_buffers == 2) {
      // Steps are synchronous, so no decode kernel is reading the inactive buffer now; a prompt whose
      // reading was enqueued before the last flip may still be: the copy waits for the last such pass
      // (passes enqueued since the flip read the active buffer and do not hold the copy up).
      const int tgt = e->active_buf ^ 1;
      if (e->pre_buf_pending[tgt]) {
        if (hipEventQuery(e->ev_pre_buf[tgt]) == hipSuccess) e->pre_buf_pending[tgt] = false;
        else HIP_TRY(hipStreamWaitEvent(e->s_copy, e->ev_pre_buf[tgt], 0));
        (void)hipGetLastError();
      }
      HIP_TRY(hipEventRecord(e->ev_copy0, e->s_copy));
      HIP_TRY(hipMemcpyAsync(e->wbuf[e->active_buf ^ 1], src, (size_t)nbytes, hipMemcpyDefault, e->s_copy));
      int rc = tie_lm_head(e, e->active_buf ^ 1, e->s_copy);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(e->ev_staged, e->s_copy));
    } else {
      HIP_TRY(hipStreamSynchronize(e->wk[1].stream));
      HIP_TRY(hipEventRecord(e->ev_copy0, e->s_dec));
      HIP_TRY(hipMemcpyAsync(e->wbuf[0], src, (size_t)nbytes, hipMemcpyDefault, e->s_dec));
      int rc = tie_lm_head(e, 0, e->s_dec);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(e->ev_staged, e->s_dec));
      HIP_TRY(hipStreamSynchronize(e->s_dec));
      e->staged_wait = true;
    }
  }
  e->staged = true;
  if (out_new_version) *out_new_version = e->staged_version;
  return PL_OK;
}

int pl_swap_poll(pl_engine *e, int32_t *staged_ready, uint32_t *active_version) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  int ready = 0;
  if (e->staged) {
    if (e->dry) ready = 1;
    else {
      hipError_t q = hipEventQuery(e->ev_staged);
      if (q == hipSuccess) ready = 1;
      else if (q != hipErrorNotReady) return fail(PL_E_HIP, "hipEventQuery: %s", hipGetErrorString(q));
    }
  }
  if (staged_ready) *staged_ready = ready;
  if (active_version) *active_version = e->version;
  return PL_OK;
}

int pl_add_sequence(pl_engine *e, uint64_t seq_id, const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                    float temperature, int32_t *out_slot) {
  if (!e || !prompt) return fail(PL_E_INVAL, "NULL argument");
  return admit(e, seq_id, prompt, n_prompt, max_new, temperature, 0, 0, -1, out_slot);
}

int pl_debug_add_sequence_at(pl_engine *e, uint64_t seq_id, const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                             float temperature, int32_t context_len, int32_t n_emitted, int32_t last_token,
                             int32_t *out_slot) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  return admit(e, seq_id, prompt, n_prompt, max_new, temperature, context_len, n_emitted, last_token, out_slot);
}

int pl_debug_set_history(pl_engine *e, int32_t slot, const int32_t *tokens, int32_t n) {
  if (!e || !tokens) return fail(PL_E_INVAL, "NULL argument");
  if (slot < 0 || slot >= e->cfg.max_batch || !e->seqs[slot].active) return fail(PL_E_STATE, "slot %d is idle", slot);
  Seq &q = e->seqs[slot];
  if (n != q.pos) return fail(PL_E_INVAL, "history must cover the %d positions read so far", q.pos);
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= e->cfg.vocab) return fail(PL_E_INVAL, "token %d out of range", tokens[i]);
  q.hist.assign(tokens, tokens + n);
  q.hist_known = true;
  return PL_OK;
}

int pl_retire_sequence(pl_engine *e, int32_t slot) {
  if (!e || slot < 0 || slot >= e->cfg.max_batch) return fail(PL_E_INVAL, "slot out of range");
  Seq &q = e->seqs[slot];
  if (!q.active) return fail(PL_E_STATE, "slot %d is idle", slot);
  if (q.reading && !e->dry) {   // its pages are still being written
    HIP_TRY(hipSetDevice(e->cfg.device));
    HIP_TRY(hipEventSynchronize(e->ev_slot[slot]));
  }
  for (int32_t p : q.pages) e->free_pages.push_back(p);
  q = Seq{};
  return PL_OK;
}

int32_t pl_num_active(const pl_engine *e) {
  int n = 0;
  if (e)
    for (auto &q : e->seqs) n += q.active;
  return n;
}

static double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

int pl_decode_step(pl_engine *e, const int32_t *forced, pl_step_out *out) {
  if (!e || !out) return fail(PL_E_INVAL, "NULL argument");
  const double t_enter = now_ms();
  if (!e->loaded) return fail(PL_E_STATE, "no weights loaded");
  const pl_model_cfg &c = e->cfg;
  // 1. validate: nothing below may fail half-way
  // an update that rebuilds the caches may become active in this step: background reading ends first
  if (e->staged && e->staged_recompute) {
    int rc = drain_passes(e);
    if (rc) return rc;
  }
  // slots whose prompt is being read in the background join the batch once that is done; if nothing
  // else is in flight the step waits for the first of them instead of returning empty-handed
  int n_reading = 0, n_ready = 0;
  for (int s = 0; s < c.max_batch; ++s) {
    Seq &q = e->seqs[s];
    if (!q.active) continue;
    if (q.reading) {
      if (e->dry) q.reading = false;
      else {
        hipError_t qy = hipEventQuery(e->ev_slot[s]);
        if (qy == hipSuccess) q.reading = false;
        else if (qy != hipErrorNotReady) return fail(PL_E_HIP, "hipEventQuery: %s", hipGetErrorString(qy));
      }
    }
    if (q.reading) ++n_reading; else ++n_ready;
  }
  if (n_reading && !n_ready) {
    for (int s = 0; s < c.max_batch; ++s) {
      Seq &q = e->seqs[s];
      if (!q.active || !q.reading) continue;
      HIP_TRY(hipSetDevice(c.device));
      HIP_TRY(hipEventSynchronize(e->ev_slot[s]));   // slots were enqueued in this order on one stream
      q.reading = false;
      break;
    }
  }
  if (!e->dry && !n_reading && e->pre_pending && hipEventQuery(e->ev_pre_last) == hipSuccess) e->pre_pending = false;
  bool shared_gpu = e->pre_pending;   // a cache-only pass may run beside this step's kernels
  int n = 0;
  int64_t new_pages = 0;
  for (int s = 0; s < c.max_batch; ++s) {
    const Seq &q = e->seqs[s];
    if (!q.active || q.reading) continue;
    if (q.n_emitted >= q.max_new) return fail(PL_E_STATE, "slot %d has finished; retire it", s);
    if (q.pos >= c.max_context) return fail(PL_E_CTX, "slot %d is at max_context", s);
    if (forced && forced[s] >= c.vocab) return fail(PL_E_INVAL, "forced token out of range");
    if (q.pos / e->page_tokens >= (int)q.pages.size()) ++new_pages;
    ++n;
  }
  if (new_pages > (int64_t)e->free_pages.size()) return fail(PL_E_NOKV, "KV pool exhausted: %lld pages needed, %lld free", (long long)new_pages, (long long)e->free_pages.size());
  out->n = n;
  out->step_ms = 0.f;
  out->swap_stall_ms = 0.f;
  e->last_n = n;
  if (n == 0) return PL_OK;

  // 2. in-flight weight update: flips only here, between two steps
  bool timed_stall = false;
  if (e->staged && e->staged_recompute)
    // a slot admitted after the request may lack its history: refuse before anything changes (the
    // update stays staged; the caller supplies the history or retires the slot and steps again)
    for (const Seq &q : e->seqs)
      if (q.active && (!q.hist_known || (int)q.hist.size() < q.pos))
        return fail(PL_E_STATE, "a slot admitted after the update was requested has no token history; its cache cannot be recomputed");
  if (e->staged) {
    if (e->dry) {
      activate_staged(e);
    } else if (e->staged_wait) {
      HIP_TRY(hipEventRecord(e->ev_c, e->s_dec));
      HIP_TRY(hipStreamWaitEvent(e->s_dec, e->ev_staged, 0));
      timed_stall = true;
      activate_staged(e);
    } else {
      hipError_t qy = hipEventQuery(e->ev_staged);
      if (qy == hipSuccess) activate_staged(e);
      else if (qy != hipErrorNotReady) return fail(PL_E_HIP, "hipEventQuery: %s", hipGetErrorString(qy));
    }
    if (!e->staged && !e->dry && e->poison_inactive && c.n_weight_buffers == 2) {
      // Nothing may read the old weights after the flip: with every element a bf16 NaN, a kernel that
      // still does shows up in the logits.  The next staging copy overwrites the buffer; it cannot start
      // before this step has ended (steps are synchronous).  A prompt being read in the background was
      // enqueued under the old weights and is entitled to them: the fill waits for the last such pass.
      if (e->pre_buf_pending[e->active_buf ^ 1]) HIP_TRY(hipStreamWaitEvent(e->s_dec, e->ev_pre_buf[e->active_buf ^ 1], 0));
      if (pl::launch_fill_u32((uint32_t *)e->wbuf[e->active_buf ^ 1], e->f32 ? 0x7FC00000u : 0x7FC07FC0u,
                              e->blob_elems * e->esz / 4, e->s_dec))
        return fail(PL_E_HIP, "fill launch failed");
    }
    if (!e->staged && !e->dry) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, e->ev_copy0, e->ev_staged) == hipSuccess) e->st.last_swap_copy_ms = ms;
      (void)hipGetLastError();
    }
    if (!e->staged && e->staged_recompute) {

      // the update asked for the caches to be rebuilt under the new weights: do it now, before the
      // first token is produced from them; the time counts as this step's stall
      e->staged_recompute = false;
      if (!e->dry && !timed_stall) {
        HIP_TRY(hipEventRecord(e->ev_c, e->s_dec));
        timed_stall = true;
      }
      int rc = recompute_all_kv(e);
      if (rc) return rc;
    }
  }

  if (e->staged && !e->dry) shared_gpu = true;   // the staging copy of an update is still writing to HBM beside this step

  // 3. pages and per-step metadata
  pl_engine::Work &w = e->wk[0];
  int32_t *row_slot = w.m_row_slot(false), *pos = w.m_pos(false), *inp = w.m_input(false), *frc = w.m_forced(false);
  float *inv_t = w.m_inv_t(false);
  uint64_t *sid = w.m_seq_id(false);
  int r = 0;
  double kv_tokens = 0;
  int items = 0, multi = 0;
  for (int s = 0; s < c.max_batch; ++s) {
    Seq &q = e->seqs[s];
    if (!q.active || q.reading) continue;
    if (q.pos / e->page_tokens >= (int)q.pages.size()) {
      q.pages.push_back(e->free_pages.back());
      e->free_pages.pop_back();
      if (e->pt_h) e->pt_h[(int64_t)s * e->pages_per_seq + q.pages.size() - 1] = q.pages.back();
      e->pt_dirty = true;
    }
    row_slot[r] = s;
    pos[r] = q.pos;
    inp[r] = q.pos < q.n_prompt && !q.prompt.empty() ? q.prompt[q.pos] : q.next_input;
    frc[r] = forced ? forced[s] : -1;
    if (frc[r] < -1) frc[r] = -1;
    inv_t[r] = q.inv_t;
    sid[r] = q.seq_id;
    kv_tokens += q.pos;
    items += (q.pos + 1 + e->attn_chunk - 1) / e->attn_chunk;
    multi += q.pos + 1 > e->attn_chunk;
    ++r;
  }

  w.attn_items = items;
  w.attn_multi = multi;

  // 4. run
  if (!e->dry) {
    HIP_TRY(hipSetDevice(c.device));
    hipStream_t s = e->s_dec;
    if (e->pt_dirty) {
      HIP_TRY(hipMemcpyAsync(w.pt, e->pt_h, (size_t)c.max_batch * e->pages_per_seq * 4, hipMemcpyHostToDevice, s));
      e->pt_dirty = false;
    }
    HIP_TRY(hipMemcpyAsync(w.meta_d, w.meta_h, (size_t)e->meta_bytes, hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(e->ev_a, s));
    e->prof_n = 0;   // a replayed graph records no per-kernel events: nothing of an earlier step may be counted again
    int rc = run_step(e, w, n);
    if (rc) return rc;
    HIP_TRY(hipEventRecord(e->ev_b, s));
    HIP_TRY(hipMemcpyAsync(e->tok_h, e->tok_d, (size_t)n * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(e->lp_h, e->lp_d, (size_t)n * 4, hipMemcpyDeviceToHost, s));
    const double t_enq = now_ms();
    HIP_TRY(hipStreamSynchronize(s));
    e->st.host_enqueue_ms += t_enq - t_enter;
    e->st.host_wait_ms += now_ms() - t_enq;
    HIP_TRY(hipEventElapsedTime(&out->step_ms, e->ev_a, e->ev_b));
    for (size_t i = 1; i < e->prof_n; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, e->prof_ev[i - 1], e->prof_ev[i]) != hipSuccess) continue;
      switch (e->prof_cat[i]) {
        case CAT_ATTN:
          e->st.attn_ms += ms; e->st.attn_launches++; e->st.attn_kv_bytes += (kv_tokens + n) * 4.0 * c.n_kv_heads * c.head_dim;
          if (shared_gpu) { e->st.attn_shared_ms += ms; e->st.attn_shared_launches++; e->st.attn_shared_kv_bytes += (kv_tokens + n) * 4.0 * c.n_kv_heads * c.head_dim; }
          break;
        case CAT_GEMM: e->st.gemm_ms += ms; break;
        case CAT_SAMPLE: e->st.sample_ms += ms; break;
        default: e->st.other_ms += ms;
      }
    }
    if (e->prof_n && e->profile == 2) e->st.gemm_launches += 4 * (uint64_t)c.n_layers + 1;
    if (timed_stall) {
      float t_total = 0.f;
      HIP_TRY(hipEventElapsedTime(&t_total, e->ev_c, e->ev_a));
      out->swap_stall_ms = t_total;
    }
  }

  // 5. outputs and bookkeeping
  r = 0;
  for (int s = 0; s < c.max_batch; ++s) {
    Seq &q = e->seqs[s];
    if (!q.active || q.reading) continue;
    const int32_t tok = e->dry ? (frc[r] >= 0 ? frc[r] : -1) : e->tok_h[r];
    const float lp = e->dry ? NAN : e->lp_h[r];
    const bool emitted = q.pos >= q.n_prompt - 1;
    if (emitted) { q.n_emitted++; q.next_input = tok; e->st.tokens_emitted++; }
    const bool fin = emitted && q.n_emitted >= q.max_new;
    if (out->slot) out->slot[r] = s;
    if (out->seq_id) out->seq_id[r] = q.seq_id;
    if (out->token) out->token[r] = tok;
    if (out->logprob) out->logprob[r] = lp;
    if (out->weight_version) out->weight_version[r] = e->version;
    if (out->position) out->position[r] = q.pos;
    if (out->emitted) out->emitted[r] = emitted;
    if (out->finished) out->finished[r] = fin;
    if (q.hist_known) q.hist.push_back(inp[r]);
    q.pos++;
    ++r;
  }
  e->st.steps++;
  e->st.slot_steps += n;
  e->st.gpu_ms_total += out->step_ms;
  const double kvb = 2.0 * c.n_layers * c.n_kv_heads * c.head_dim * e->esz;
  e->st.algorithmic_bytes += (double)e->streamed_weight_bytes + (kv_tokens + n) * kvb;
  return PL_OK;
}

// Enqueue the reading of a slot's prompt (all positions not read yet, except the last) on the
// cache-only stream; the slot is marked as reading and its event recorded.
static int start_prefill(pl_engine *e, int32_t slot, int32_t *out_positions) {
  if (out_positions) *out_positions = 0;
  if (!e->loaded) return fail(PL_E_STATE, "no weights loaded");
  const pl_model_cfg &c = e->cfg;
  if (slot < 0 || slot >= c.max_batch || !e->seqs[slot].active) return fail(PL_E_STATE, "slot %d is idle", slot);
  Seq &q = e->seqs[slot];
  if (q.reading) return fail(PL_E_BUSY, "slot %d is already reading its prompt", slot);
  const int first = q.pos, last = q.n_prompt - 1;   // positions [first, last) are read here
  if (first >= last) return PL_OK;
  if ((int)q.prompt.size() < q.n_prompt) return fail(PL_E_STATE, "slot %d holds no prompt", slot);
  if ((int64_t)q.pages.size() * e->page_tokens < last) return fail(PL_E_STATE, "slot %d has no pages for its prompt", slot);
  std::vector<int32_t> slots(last - first, slot), positions, tokens;
  for (int p = first; p < last; ++p) { positions.push_back(p); tokens.push_back(q.prompt[p]); }
  int rc = run_kv_passes(e, slots, positions, tokens, &e->st.prefill_ms, &e->st.prefill_passes);
  if (rc) return rc;
  if (!e->dry) HIP_TRY(hipEventRecord(e->ev_slot[slot], e->wk[1].stream));
  e->st.prefill_positions += last - first;
  if (q.hist_known) q.hist.insert(q.hist.end(), tokens.begin(), tokens.end());
  q.pos = last;
  q.reading = true;
  if (out_positions) *out_positions = last - first;
  return PL_OK;
}

int pl_prefill(pl_engine *e, int32_t slot, int32_t *out_positions) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  // a slot whose prompt is already being read in the background: nothing is left to read, wait for it
  const bool already = slot >= 0 && slot < e->cfg.max_batch && e->seqs[slot].active && e->seqs[slot].reading;
  if (already && out_positions) *out_positions = 0;
  int rc = already ? PL_OK : start_prefill(e, slot, out_positions);
  if (rc) return rc;
  Seq &q = e->seqs[slot];
  if (q.reading) {
    if (!e->dry) {
      HIP_TRY(hipEventSynchronize(e->ev_slot[slot]));
      harvest_passes(e);
    }
    q.reading = false;
  }
  e->last_n = 0;
  return PL_OK;
}

int pl_prefill_async(pl_engine *e, int32_t slot, int32_t *out_positions) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  return start_prefill(e, slot, out_positions);
}

int pl_get_stats(pl_engine *e, pl_stats *out) {
  if (!e || !out) return fail(PL_E_INVAL, "NULL argument");
  if (!e->dry) harvest_passes(e);
  e->st.active_version = e->version;
  e->st.kv_pages_free = (int64_t)e->free_pages.size();
  *out = e->st;
  return PL_OK;
}

int pl_debug_get_logits(pl_engine *e, float *out, int64_t out_elems) {
  if (!e || !out) return fail(PL_E_INVAL, "NULL argument");
  if (e->dry) return fail(PL_E_STATE, "bookkeeping-only engine computes no logits");
  if (out_elems < (int64_t)e->last_n * e->cfg.vocab) return fail(PL_E_INVAL, "output buffer too small");
  HIP_TRY(hipSetDevice(e->cfg.device));
  HIP_TRY(hipMemcpy(out, e->logits, (size_t)e->last_n * e->cfg.vocab * 4, hipMemcpyDeviceToHost));
  return PL_OK;
}

static int kv_xfer(pl_engine *e, int32_t slot, int32_t layer, float *k, float *v, const float *k_in,
                   const float *v_in, int32_t n_ctx, bool write) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  if (e->dry) return fail(PL_E_STATE, "bookkeeping-only engine holds no KV");
  const pl_model_cfg &c = e->cfg;
  if (slot < 0 || slot >= c.max_batch || layer < 0 || layer >= c.n_layers) return fail(PL_E_INVAL, "slot or layer out of range");
  Seq &q = e->seqs[slot];
  if (!q.active) return fail(PL_E_STATE, "slot %d is idle", slot);
  if (n_ctx < 0 || (int64_t)n_ctx > (int64_t)q.pages.size() * e->page_tokens) return fail(PL_E_INVAL, "n_ctx exceeds the slot's pages");
  HIP_TRY(hipSetDevice(c.device));
  HIP_TRY(hipStreamSynchronize(e->s_dec));
  HIP_TRY(hipStreamSynchronize(e->wk[1].stream));
  const int hd = c.head_dim, Hkv = c.n_kv_heads, ptok = e->page_tokens;
  if (e->f32) {   // fp32 pages: [kv head][K | V][token][hd]
    std::vector<float> img((size_t)e->page_stride);
    for (int p0 = 0; p0 < n_ctx; p0 += ptok) {
      float *dev = (float *)e->kv_pool + (int64_t)layer * e->layer_stride + (int64_t)q.pages[p0 / ptok] * e->page_stride;
      HIP_TRY(hipMemcpy(img.data(), dev, img.size() * 4, hipMemcpyDeviceToHost));
      const int cnt = std::min(ptok, n_ctx - p0);
      for (int t = 0; t < cnt; ++t)
        for (int g = 0; g < Hkv; ++g)
          for (int d = 0; d < hd; ++d) {
            const int64_t ci = ((int64_t)(p0 + t) * Hkv + g) * hd + d;
            float *kb = img.data() + ((int64_t)g * 2 * ptok + t) * hd + d, *vb = kb + (int64_t)ptok * hd;
            if (write) { *kb = k_in[ci]; *vb = v_in[ci]; }
            else { k[ci] = *kb; v[ci] = *vb; }
          }
      if (write) HIP_TRY(hipMemcpy(dev, img.data(), img.size() * 4, hipMemcpyHostToDevice));
    }
    return PL_OK;
  }
  std::vector<uint16_t> img((size_t)e->page_stride);
  for (int p0 = 0; p0 < n_ctx; p0 += ptok) {
    bf16_t *dev = (bf16_t *)e->kv_pool + (int64_t)layer * e->layer_stride + (int64_t)q.pages[p0 / ptok] * e->page_stride;
    HIP_TRY(hipMemcpy(img.data(), dev, img.size() * 2, hipMemcpyDeviceToHost));
    const int cnt = std::min(ptok, n_ctx - p0);
    for (int t = 0; t < cnt; ++t)
      for (int g = 0; g < Hkv; ++g) {
        uint16_t *kb = img.data() + (int64_t)g * 2 * ptok * hd, *vb = kb + (int64_t)ptok * hd;
        for (int d = 0; d < hd; ++d) {
          const int64_t ci = ((int64_t)(p0 + t) * Hkv + g) * hd + d;
          if (write) {
            kb[pl::k_elem_offset(t, d, hd)] = f32_to_bf16_bits(k_in[ci]);
            vb[pl::v_elem_offset(t, d, hd)] = f32_to_bf16_bits(v_in[ci]);
          } else {
            k[ci] = bf16_bits_to_f32(kb[pl::k_elem_offset(t, d, hd)]);
            v[ci] = bf16_bits_to_f32(vb[pl::v_elem_offset(t, d, hd)]);
          }
        }
      }
    if (write) HIP_TRY(hipMemcpy(dev, img.data(), img.size() * 2, hipMemcpyHostToDevice));
  }
  return PL_OK;
}

int pl_debug_read_kv(pl_engine *e, int32_t slot, int32_t layer, float *k_out, float *v_out, int32_t n_ctx) {
  if (!k_out || !v_out) return fail(PL_E_INVAL, "NULL argument");
  return kv_xfer(e, slot, layer, k_out, v_out, nullptr, nullptr, n_ctx, false);
}

int pl_debug_write_kv(pl_engine *e, int32_t slot, int32_t layer, const float *k_in, const float *v_in, int32_t n_ctx) {
  if (!k_in || !v_in) return fail(PL_E_INVAL, "NULL argument");
  return kv_xfer(e, slot, layer, nullptr, nullptr, k_in, v_in, n_ctx, true);
}

int pl_debug_set_profile(pl_engine *e, int32_t level) {
  if (!e || level < 0 || level > 2) return fail(PL_E_INVAL, "bad argument");
  e->profile = e->dry ? 0 : level;
  return PL_OK;
}

int pl_debug_set_graphs(pl_engine *e, int32_t on) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  e->use_graphs = on != 0;
  return PL_OK;
}

int pl_debug_set_poison(pl_engine *e, int32_t on) {
  if (!e) return fail(PL_E_INVAL, "NULL argument");
  e->poison_inactive = on != 0;
  return PL_OK;
}

int pl_debug_kv_pool(pl_engine *e, void **device_ptr, int64_t *nbytes) {
  if (!e || !device_ptr || !nbytes) return fail(PL_E_INVAL, "NULL argument");
  if (e->dry) return fail(PL_E_STATE, "bookkeeping-only engine holds no KV");
  *device_ptr = e->kv_pool;
  *nbytes = e->layer_stride * e->cfg.n_layers * e->esz;
  return PL_OK;
}

// ---- kernel-level entry points ---------------------------------------------------------------------

int64_t pl_attention_workspace_bytes(int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t hd, int32_t max_ctx) {
  if (n_seq < 1 || n_q_heads < 1 || n_kv_heads < 1 || hd < 1 || max_ctx < 1) return 0;
  const int chunk = pl::attention_chunk_tokens(n_seq, n_kv_heads, max_ctx);
  const int64_t max_chunks = (max_ctx + chunk - 1) / chunk;
  return (int64_t)n_seq * n_q_heads * max_chunks * (hd + 2) * 4 + pl::attention_worklist_ints(n_seq, (int)max_chunks) * 4 + 32;
}

int pl_attention_decode(const void *q, const void *kv_pages, const int32_t *page_table, const int32_t *ctx_len,
                        void *out, void *workspace, int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t hd,
                        int32_t page_tokens, int32_t pages_per_seq, int32_t max_ctx, void *stream) {
  if (!q || !kv_pages || !page_table || !ctx_len || !out || !workspace) return fail(PL_E_INVAL, "NULL argument");
  if (n_seq < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || n_q_heads / n_kv_heads > 16) return fail(PL_E_INVAL, "bad head counts");
  if (hd != 32 && hd != 64 && hd != 128) return fail(PL_E_INVAL, "head_dim must be 32, 64 or 128");
  if (page_tokens < 32 || page_tokens % 32 || pages_per_seq < 1 || max_ctx < 1 || max_ctx > (int64_t)pages_per_seq * page_tokens)
    return fail(PL_E_INVAL, "bad page geometry");
  pl::AttnParams p{};
  p.q = (const bf16_t *)q; p.kv = (const bf16_t *)kv_pages; p.page_table = page_table; p.ctx_len = ctx_len;
  p.row_slot = nullptr; p.out = (bf16_t *)out;
  p.n_seq = n_seq; p.Hq = n_q_heads; p.Hkv = n_kv_heads; p.hd = hd; p.page_tokens = page_tokens;
  p.pages_per_seq = pages_per_seq;
  p.chunk = pl::attention_chunk_tokens(n_seq, n_kv_heads, max_ctx);
  p.max_chunks = (max_ctx + p.chunk - 1) / p.chunk;
  const int64_t np = (int64_t)n_seq * n_q_heads * p.max_chunks;
  p.part_o = (float *)workspace;
  p.part_ml = p.part_o + np * hd;
  int32_t *work = (int32_t *)(((uintptr_t)(p.part_ml + np * 2) + 31) & ~(uintptr_t)31);   // records are read 16 bytes at a time
  p.work = work;
  p.multi = pl::attention_multi_list(work, n_seq, p.max_chunks);
  p.max_items = n_seq * p.max_chunks;
  p.max_multi = p.max_chunks > 1 ? n_seq : 0;
  if (n_seq > 1024) return fail(PL_E_INVAL, "at most 1024 sequences per launch");
  if (pl::launch_attention_worklist(ctx_len, nullptr, page_table, work, n_seq, p.max_chunks, p.chunk, page_tokens, pages_per_seq, (hipStream_t)stream)) return fail(PL_E_HIP, "attention launch failed");
  if (pl::launch_attention(p, (hipStream_t)stream)) return fail(PL_E_HIP, "attention launch failed");
  return PL_OK;
}

int pl_is_ess(const float *logp_pi, const float *logp_mu, const int64_t *seq_offsets, int32_t n_seq, float c,
              float *w_out, double *seq_sums, double *ess_seq, double *totals, void *stream) {
  if (!logp_pi || !logp_mu || !seq_offsets || !seq_sums || !ess_seq || !totals) return fail(PL_E_INVAL, "NULL argument");
  if (n_seq < 1) return fail(PL_E_INVAL, "n_seq must be positive");
  if (!(c > 0.f)) return fail(PL_E_INVAL, "the truncation level c must be positive");
  if (pl::launch_is_ess(logp_pi, logp_mu, seq_offsets, n_seq, (double)c, w_out, seq_sums, ess_seq, totals, (hipStream_t)stream))
    return fail(PL_E_HIP, "importance-weight launch failed");
  return PL_OK;
}

int pl_kv_pack_host(uint16_t *pages_host, const int32_t *page_ids, const float *k, const float *v, int32_t first_pos,
                    int32_t n, int32_t n_kv_heads, int32_t hd, int32_t page_tokens) {
  if (!pages_host || !page_ids || !k || !v) return fail(PL_E_INVAL, "NULL argument");
  if (first_pos < 0 || n < 0 || n_kv_heads < 1 || page_tokens < 32 || page_tokens % 32 || (hd != 32 && hd != 64 && hd != 128))
    return fail(PL_E_INVAL, "bad geometry");
  const int64_t head_elems = (int64_t)2 * page_tokens * hd;
  for (int i = 0; i < n; ++i) {
    const int p = first_pos + i, t = p % page_tokens;
    const int64_t page = page_ids[p / page_tokens];
    for (int g = 0; g < n_kv_heads; ++g) {
      uint16_t *kb = pages_host + (page * n_kv_heads + g) * head_elems, *vb = kb + (int64_t)page_tokens * hd;
      for (int d = 0; d < hd; ++d) {
        const int64_t ci = ((int64_t)i * n_kv_heads + g) * hd + d;
        kb[pl::k_elem_offset(t, d, hd)] = f32_to_bf16_bits(k[ci]);
        vb[pl::v_elem_offset(t, d, hd)] = f32_to_bf16_bits(v[ci]);
      }
    }
  }
  return PL_OK;
}

int pl_gemm_bf16(const void *x, const void *w, void *y, int32_t M, int32_t N, int32_t K, int32_t mode, int32_t splits,
                 void *stream) {
  if (!x || !w || !y) return fail(PL_E_INVAL, "NULL argument");
  if (mode == 1 && splits != 1) return fail(PL_E_INVAL, "the SwiGLU product takes splits = 1");
  int rc = pl::launch_gemm((const bf16_t *)x, (const bf16_t *)w, y, nullptr, M, N, K, mode, pl::GemmSplit{splits, N, 1}, (hipStream_t)stream);
  if (rc == -1) return fail(PL_E_INVAL, "unsupported GEMM shape M=%d N=%d K=%d mode=%d splits=%d", M, N, K, mode, splits);
  if (rc) return fail(PL_E_HIP, "GEMM launch failed");
  return PL_OK;
}

int pl_debug_gemm_cfg(int32_t cfg, const void *x, const void *w, void *y, void *ws, int32_t M, int32_t N, int32_t K,
                      int32_t mode, int32_t splits, int32_t n_begin, int32_t n_end, int32_t paired, void *stream) {
  if (!x || !w || !y) return fail(PL_E_INVAL, "NULL argument");
  int rc = pl::launch_gemm_cfg(cfg, (const bf16_t *)x, (const bf16_t *)w, y, (float *)ws, M, N, K, mode, splits, n_begin,
                               n_end, paired != 0, (hipStream_t)stream);
  if (rc == -1) return fail(PL_E_INVAL, "unsupported GEMM launch cfg=%d M=%d N=%d K=%d mode=%d splits=%d [%d, %d)", cfg, M, N, K, mode, splits, n_begin, n_end);
  if (rc) return fail(PL_E_HIP, "GEMM launch failed");
  return PL_OK;
}

int pl_debug_gemm_plan(int32_t M_max, int32_t N, int32_t K, int32_t mode, int32_t *splits, int32_t *n_main,
                       int32_t *rem_splits, int64_t *ws_elems) {
  if (M_max < 1 || M_max > 512 || N < 32 || K < 256 || (mode != 0 && mode != 1)) return fail(PL_E_INVAL, "unsupported GEMM shape");
  const pl::GemmSplit ks = pl::gemm_pick_split(M_max, N, K, mode);
  if (splits) *splits = ks.splits;
  if (n_main) *n_main = ks.n_main;
  if (rem_splits) *rem_splits = ks.rem_splits;
  if (ws_elems) *ws_elems = mode == 1 ? pl::gemm_workspace_elems(M_max, N, ks) : 0;   // mode 0 keeps its slices in y
  return PL_OK;
}

int pl_debug_gemm_planned(const void *x, const void *w, void *y, void *ws, int32_t M_max, int32_t M, int32_t N, int32_t K,
                          int32_t mode, void *stream) {
  if (!x || !w || !y) return fail(PL_E_INVAL, "NULL argument");
  if (M_max < 1 || M_max > 512 || M < 1 || M > M_max || N < 32 || K < 256 || (mode != 0 && mode != 1))
    return fail(PL_E_INVAL, "unsupported GEMM shape");
  const pl::GemmSplit ks = pl::gemm_pick_split(M_max, N, K, mode);
  if (!ws && mode == 1 && pl::gemm_workspace_elems(M_max, N, ks) > 0) return fail(PL_E_INVAL, "this plan needs a workspace");
  int rc = pl::launch_gemm((const bf16_t *)x, (const bf16_t *)w, y, (float *)ws, M, N, K, mode, ks, (hipStream_t)stream);
  if (rc == -1) return fail(PL_E_INVAL, "unsupported GEMM shape M=%d N=%d K=%d mode=%d", M, N, K, mode);
  if (rc) return fail(PL_E_HIP, "GEMM launch failed");
  return PL_OK;
}

int64_t pl_debug_stream_read(const void *device_ptr, int64_t nbytes, int32_t nontemporal, void *stream) {
  if (!device_ptr || nbytes < (int64_t)16 * 8192 * 2048) return fail(PL_E_INVAL, "need a device buffer of at least 256 MiB");
  int64_t r = pl::launch_stream_read(device_ptr, nbytes, nullptr, nontemporal != 0, (hipStream_t)stream);
  if (r < 0) return fail(PL_E_HIP, "stream read launch failed");
  return r;
}

int64_t pl_sample_workspace_bytes(int32_t n, int32_t vocab) {
  if (n < 1 || vocab < 1) return 0;
  return pl::sample_workspace_bytes(n, vocab);
}

int pl_sample(const float *logits, int32_t n, int32_t vocab, const uint64_t *seq_id, const int32_t *position,
              const float *inv_temperature, const int32_t *forced, uint64_t seed, int32_t *token, float *logprob,
              void *workspace, void *stream) {
  if (!logits || !seq_id || !position || !inv_temperature || !token || !logprob || !workspace) return fail(PL_E_INVAL, "NULL argument");
  if (n < 1 || vocab < 4 || vocab % 4) return fail(PL_E_INVAL, "need n >= 1 and vocab a positive multiple of 4");
  pl::SampleParams p{};
  p.logits = logits; p.n = n; p.vocab = vocab; p.seq_id = seq_id; p.position = position; p.inv_t = inv_temperature;
  p.forced = forced; p.seed = seed; p.token = token; p.logprob = logprob; p.workspace = workspace;
  if (pl::launch_sample(p, (hipStream_t)stream)) return fail(PL_E_HIP, "sampler launch failed");
  return PL_OK;
}

int pl_sample_static(const float *logits, int32_t n, int32_t vocab, const uint64_t *seq_id, const int32_t *position,
                     const float *inv_temperature, const int32_t *forced, uint64_t seed, int32_t *token, float *logprob,
                     void *stream) {
  if (!logits || !seq_id || !position || !inv_temperature || !token || !logprob) return fail(PL_E_INVAL, "NULL argument");
  if (n < 1 || vocab < 4 || vocab % 4) return fail(PL_E_INVAL, "need n >= 1 and vocab a positive multiple of 4");
  void *ws = nullptr;
  const int rc = pl::sample_static_workspace(n, vocab, &ws);
  if (rc == -1) {
    int mr = 0, mv = 0;
    pl::sample_static_limits(&mr, &mv);
    return fail(PL_E_INVAL, "pl_sample_static serves at most %d rows and a vocabulary of %d; got n = %d, vocab = %d", mr, mv, n, vocab);
  }
  if (rc) return fail(PL_E_HIP, "hipGetSymbolAddress of the sampler's scratch array failed");
  pl::SampleParams p{};
  p.logits = logits; p.n = n; p.vocab = vocab; p.seq_id = seq_id; p.position = position; p.inv_t = inv_temperature;
  p.forced = forced; p.seed = seed; p.token = token; p.logprob = logprob; p.workspace = ws;
  if (pl::launch_sample(p, (hipStream_t)stream)) return fail(PL_E_HIP, "sampler launch failed");
  return PL_OK;
}

}  // extern "C"
