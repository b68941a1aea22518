/*
 * pl.h - C ABI of the constant-batch decode engine with in-flight weight updates (gfx950).
 *
 * The engine is the generation side of the Actor loop of the PipelineRL paper (Alg. 2): keep H
 * sequences in flight, produce one token per sequence per step, refill a slot as soon as its
 * sequence finishes, and take a new set of weights between two steps without discarding any
 * sequence's key/value history (Sec. 4; Sec. 5.1 for the stale-cache semantics).  Every emitted
 * token carries the log-probability it had under the weights that sampled it (the behaviour
 * policy mu of the truncated importance-sampling estimator, Sec. 2.1) and the version number of
 * those weights (token lag, Fig. 3).
 *
 * Conventions
 *   - Every function returns a pl_status (0 = success, negative = error) unless stated otherwise;
 *     nothing throws or aborts across this boundary.  pl_last_error() returns a NUL-terminated
 *     message owned by the library, valid until the next call on the same thread.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device memory on
 *     the engine's GPU.  The caller owns every buffer it passes; the engine copies what it keeps.
 *   - An engine is bound to one GPU and must be driven from one host thread at a time.
 *   - All floating-point storage on the device is bf16 unless stated; accumulation is fp32.
 */
#ifndef PL_H
#define PL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PL_OK = 0,
  PL_E_INVAL = -1,  /* bad configuration, shape, size, pointer or temperature <= 0          */
  PL_E_NOSLOT = -2, /* all max_batch slots are occupied                                      */
  PL_E_NOKV = -3,   /* KV page pool exhausted; the engine state is unchanged                 */
  PL_E_BUSY = -4,   /* a weight update is still being staged                                 */
  PL_E_STATE = -5,  /* call not valid in this state (idle slot, no weights loaded, ...)      */
  PL_E_CTX = -6,    /* sequence would grow past max_context                                  */
  PL_E_HIP = -7,    /* a HIP call failed; the engine should be destroyed                     */
  PL_E_NOMEM = -8   /* host or device allocation failed                                      */
} pl_status;

#define PL_SWAP_ASYNC 0u /* stage in the background; flip at the first step boundary once staged */
#define PL_SWAP_WAIT 1u  /* the next step waits for the staging copy, then flips                  */
#define PL_SWAP_RECOMPUTE_KV 2u /* or-ed in: at the flip, rebuild every sequence's cache under the new weights */
#define PL_DEVICE_NONE (-1) /* bookkeeping-only engine: no GPU is touched, no token is computed  */
#define PL_BF16 0 /* the engine proper: bf16 weights, KV cache and activations, fp32 accumulation   */
#define PL_F32 1  /* test build: everything in fp32 through plain kernels (see pl_model_cfg.dtype) */

typedef struct pl_engine pl_engine;

/* Decoder shape and engine capacity.  The network is a pre-norm decoder with RMSNorm, rotary
 * positions (half-split pairing: element i rotates with element i + head_dim/2, angle
 * pos * rope_theta^(-2i/head_dim)), grouped-query attention (query head h reads kv head
 * h / (n_q_heads / n_kv_heads)), SwiGLU feed-forward, untied LM head, no biases. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta; /* e.g. 1e4 */
  float rms_eps;    /* added to the mean square inside the root, e.g. 1e-6 */
  int32_t max_batch;      /* H of Alg. 2: number of slots */
  int32_t max_context;    /* cap on prompt + generated positions of one sequence */
  int64_t kv_pool_tokens; /* capacity of the paged KV pool, in token positions (all layers); 0 = what is
                             left of the device memory after the weights and work buffers, minus a
                             6 GiB reserve for the caller, at most max_batch * max_context */
  int32_t kv_page_tokens; /* tokens per page: multiple of 32; 0 selects 128 */
  int32_t n_weight_buffers; /* 2: in-flight updates are staged into the inactive buffer; 1: updates
                               overwrite the only buffer and always block */
  uint64_t seed;          /* sampler key */
  int32_t device;         /* HIP device ordinal, or PL_DEVICE_NONE */
  int32_t dtype;          /* PL_BF16 (0), or PL_F32: the test build, in which weights, KV cache and
                             activations are fp32 and every step runs through plain, untuned kernels, so
                             that the engine around them (slots, pages, positions, head mapping, update
                             protocol, sampler keying) can be held to 1e-4 against the oracle.  Its blob
                             has the same tensors in the same order, 4 bytes per element, every matrix
                             row-major [out, in], "l<l>.w_gu" = all gate rows then all up rows
                             (pl_pack_weights produces it).  Same calls, same semantics; slow. */
  int32_t tie_embeddings; /* 0: untied LM head (default).  1: the LM head is the embedding table: the blob
                             ends after "gf" (pl_weight_count / pl_weight_layout / pl_weight_nbytes do not
                             list an lm_head), and every load or update derives the LM head's streaming
                             layout from the table on the device, behind the copy that brought the blob in */
} pl_model_cfg;

/* Result of one decode step: one entry per occupied slot, in slot order.  Arrays are caller
 * allocated with room for max_batch entries; any of the array pointers may be NULL. */
typedef struct {
  int32_t n;                /* out: number of entries */
  int32_t *slot;            /* out: slot index */
  uint64_t *seq_id;         /* out: caller's sequence id */
  int32_t *token;           /* out: token produced by this step (sampled or forced) */
  float *logprob;           /* out: log softmax(logits / T)[token] under the step's weights */
  uint32_t *weight_version; /* out: version of the weights that produced the token */
  int32_t *position;        /* out: position of the token that was consumed (0-based) */
  uint8_t *emitted;         /* out: 1 if `token` is a generated token, 0 while the prompt is read */
  uint8_t *finished;        /* out: 1 if this was the sequence's last token (max_new reached) */
  float step_ms;            /* out: GPU time of the step on the decode stream */
  float swap_stall_ms;      /* out: time this step spent waiting for a staged weight copy */
} pl_step_out;

typedef struct {
  uint64_t steps;             /* decode steps run */
  uint64_t tokens_emitted;    /* generated tokens */
  uint64_t slot_steps;        /* sum over steps of occupied slots (prompt reading included) */
  uint64_t swaps;             /* weight updates that became active */
  double gpu_ms_total;        /* sum of step_ms */
  double algorithmic_bytes;   /* sum over steps of streamed weight bytes + KV bytes read + written */
  float last_swap_copy_ms;    /* duration of the last staging copy */
  uint32_t active_version;
  int64_t kv_pages_free, kv_pages_total;
  /* filled while profiling is on (pl_debug_set_profile): GPU time between HIP events recorded on the
   * decode stream around each kernel group, summed over steps */
  double attn_ms, gemm_ms, sample_ms, other_ms;
  uint64_t attn_launches, gemm_launches; /* launches of the decode-attention kernel (one per layer per step; the kernel
                                          * that merges the chunks of long rows is timed under other_ms), GEMM launches */
  double attn_kv_bytes;                  /* K/V bytes those attention launches had to read */
  /* the part of the three attention figures above that was measured in steps during which a background
   * cache-only pass (pl_prefill_async) or the staging copy of an update was in flight, i.e. while the
   * kernel shared the GPU or its memory */
  double attn_shared_ms, attn_shared_kv_bytes;
  uint64_t attn_shared_launches;
  /* host time inside pl_decode_step, summed over steps: from entry until the step's work is enqueued,
   * and from then until its results have arrived */
  double host_enqueue_ms, host_wait_ms;
  /* batched prompt reading (pl_prefill); not part of steps / slot_steps / gpu_ms_total above */
  uint64_t prefill_passes, prefill_positions;
  double prefill_ms;
  /* cache recomputation after updates staged with PL_SWAP_RECOMPUTE_KV (its time is also part of
   * that step's swap_stall_ms) */
  uint64_t recompute_passes, recompute_positions;
  double recompute_ms;
} pl_stats;

/* ---- engine life cycle --------------------------------------------------------------------- */

/* Create an engine: allocates weight buffer(s), the KV page pool and work buffers on cfg->device.
 * PL_E_INVAL if a shape is unsupported (head_dim not in {32, 64, 128}, n_q_heads not a multiple
 * of n_kv_heads or group > 16, d_model, d_ffn or n_q_heads*head_dim not a multiple of 256, a weight
 * matrix of 2 GiB or more, ...); PL_E_NOMEM if an allocation fails (nothing is leaked). */
int pl_create(const pl_model_cfg *cfg, pl_engine **out);
void pl_destroy(pl_engine *e);
const char *pl_last_error(void);

/* ---- weights --------------------------------------------------------------------------------
 * Weights travel as one flat bf16 blob.  pl_weight_layout enumerates its tensors: for idx in
 * [0, pl_weight_count) it returns the tensor's name, element offset into the blob and shape
 * [rows, cols] (cols = 1 for gains).  Tensors, in order: "embed" [vocab, d]; per layer l:
 * "l<l>.g1" [d], "l<l>.w_qkv" [(Hq + 2 Hkv) hd, d] (rows: all q heads, all k heads, all v heads),
 * "l<l>.w_o" [d, Hq hd], "l<l>.g2" [d], "l<l>.w_gu" [2 F, d] (gate and up rows interleaved in
 * blocks of 32: rows [64 t, 64 t + 32) are gate rows 32 t .., rows [64 t + 32, 64 t + 64) the
 * matching up rows), "l<l>.w_d" [d, F]; then "gf" [d] and "lm_head" [vocab, d].  Every matrix W is
 * [out_features, in_features] (y = x W^T).  "embed" is row-major.  All other matrices are stored in
 * MFMA operand order, so that a wavefront streams its rows with contiguous 1 KiB loads and all
 * workgroups together read W plane by plane: in blocks of 32 rows x 64 columns, block (r / 32, c / 64)
 * at element offset ((c / 64) (rows / 32) + r / 32) 2048 (column-block major), and inside a block
 * element (r, c) at ((c % 32) / 8) 512 + ((c % 64) / 32) 256 + (r % 32) 8 + c % 8. */
int32_t pl_weight_count(const pl_engine *e);
int pl_weight_layout(const pl_engine *e, int32_t idx, const char **name, int64_t *offset_elems,
                     int64_t shape[2]);
int64_t pl_weight_nbytes(const pl_engine *e);

/* Host helper (layout only, no device access): write one source tensor into its place in a host
 * image `blob` (pl_weight_nbytes bytes) of the flat blob described above (or of the fp32 test
 * build's blob, whose sources must be fp32).  `name` is "embed", "gf",
 * "lm_head", or "l<l>.<t>" with t one of g1, g2 (gains, [d]), wq [Hq hd, d], wk, wv [Hkv hd, d],
 * wo [d, Hq hd], wg, wu [F, d], wd [d, F]; `src` is the tensor row-major [out_features, in_features],
 * fp32 if src_is_f32 (rounded to bf16, nearest even) or bf16 bit patterns otherwise.  The row
 * concatenation q|k|v, the 32-row gate/up interleave and the operand ordering are applied here, so a
 * caller never needs the formulas.  PL_E_INVAL for an unknown name. */
int pl_pack_weights(const pl_engine *e, const char *name, const void *src, int32_t src_is_f32, void *blob);

/* Blocking load of version 0 (or a blocking replacement of the active buffer, version + 1, if
 * weights are already loaded).  src: host or device pointer to pl_weight_nbytes bytes. */
int pl_load_weights(pl_engine *e, const void *src, int64_t nbytes);

/* In-flight weight update ("mu <- receive_weight_update()", Alg. 2).  Starts copying the blob at
 * src (host - pinned for a truly asynchronous copy - or device memory) into the inactive buffer
 * on a side stream and returns at once.  The engine flips to the new buffer only between two
 * decode steps: with PL_SWAP_WAIT at the very next step (which first waits for the copy), with
 * PL_SWAP_ASYNC at the first step that finds the copy complete.  No KV page is touched: tokens
 * produced after the flip are conditioned on keys/values computed under older weights (Sec. 5.1).
 * src must stay valid and unmodified until the flip.  *out_new_version receives the version the
 * new weights will carry.  PL_E_BUSY if an update is already staged and not yet active;
 * PL_E_STATE before pl_load_weights.  With n_weight_buffers == 1 the copy overwrites the active
 * buffer on the decode stream and the call returns when it is done.
 * flags | PL_SWAP_RECOMPUTE_KV selects the "KV cache recomputed" variant of Sec. 5.1 instead: at the
 * flip, before the step produces anything, every token each occupied slot has read so far is replayed
 * under the new weights (batched passes through the decode kernels) and its keys and values are
 * overwritten in place, so later tokens are conditioned on a fresh cache.  The time is reported in that
 * step's swap_stall_ms and in pl_stats.recompute_ms.  PL_E_STATE if a slot was admitted mid-life
 * without its token history (pl_debug_add_sequence_at without pl_debug_set_history). */
int pl_swap_weights(pl_engine *e, const void *src, int64_t nbytes, uint32_t flags,
                    uint32_t *out_new_version);
int pl_swap_poll(pl_engine *e, int32_t *staged_ready, uint32_t *active_version);

/* ---- sequences (Alg. 2: pop finished, refill to H) ------------------------------------------- */

/* Admit a sequence into the lowest free slot.  The engine copies the prompt.  The sequence reads
 * its prompt one token per step (positions 0 .. n_prompt-1); the step that reads the last prompt
 * token emits the first generated token; it is finished after max_new emitted tokens.
 * PL_E_CTX if n_prompt + max_new - 1 > max_context; PL_E_NOKV if the pool cannot hold the
 * prompt; PL_E_NOSLOT if the batch is full; PL_E_INVAL for temperature <= 0, empty prompt,
 * token out of range. */
int pl_add_sequence(pl_engine *e, uint64_t seq_id, const int32_t *prompt, int32_t n_prompt,
                    int32_t max_new, float temperature, int32_t *out_slot);
/* Batched prompt reading on refill ("add prompts", Alg. 2): reads the positions of the slot's prompt
 * that have not been read yet, except the last one, in passes of up to 256 positions
 * through the same kernels as a decode step (rows = consecutive positions of one sequence, causal
 * because row i attends to positions <= its own), under the active weights.  It leaves exactly the
 * keys and values that reading those tokens one per step would leave (up to bf16 rounding of
 * identical arithmetic: same kernels, same per-row operation order) and emits nothing; the next
 * pl_decode_step reads the last prompt token and produces the first generated token.
 * *out_positions (may be NULL) receives the number of positions read (0 if none were left).
 * Blocks until done (on a slot that pl_prefill_async is already reading: until that reading is done).
 * PL_E_STATE if the slot is idle or before pl_load_weights. */
int pl_prefill(pl_engine *e, int32_t slot, int32_t *out_positions);
/* The same reading, in the background: the passes are enqueued on a stream of their own and the call
 * returns at once, so decode steps of the other slots go on meanwhile (the passes are GEMM-bound, the
 * decode step mostly waits for K/V bytes; the two overlap on the GPU).  Until its passes have finished
 * the slot takes no part in decode steps: pl_decode_step leaves it out (its entry is simply missing
 * from that step's output) and includes it from the first step that finds the reading complete; a
 * step with no other occupied slot waits for it.  What a sequence produces does not depend on when it
 * joins: its cache, logits and draws are those of pl_prefill.  The prompt is read under the weights
 * active at this call even if an update becomes active meanwhile (the next staging copy waits for the
 * passes that still read the old buffer).  pl_retire_sequence on such a slot waits for its passes;
 * an update with PL_SWAP_RECOMPUTE_KV waits for all of them.  PL_E_BUSY if the slot is already reading. */
int pl_prefill_async(pl_engine *e, int32_t slot, int32_t *out_positions);
/* Free a slot and its KV pages (finished or not).  PL_E_STATE if the slot is idle. */
int pl_retire_sequence(pl_engine *e, int32_t slot);
int32_t pl_num_active(const pl_engine *e);

/* ---- the step ("generate next tokens with mu", Alg. 2) ---------------------------------------
 * One token for every occupied slot.  forced (host, may be NULL): forced[slot] >= 0 replaces the
 * token this step would sample for that slot (teacher forcing; its log-prob is still recorded and
 * it is what the next step consumes); -1 samples.  Blocks until the step's outputs are in `out`.
 * Sampling is Gumbel-max over logits / T with Philox4x32-10 noise keyed by (seed; seq_id,
 * position, vocabulary index), so a sequence's draws do not depend on its slot or neighbours.
 * PL_E_NOKV if a sequence needs a new page and none is free (nothing is executed). */
int pl_decode_step(pl_engine *e, const int32_t *forced, pl_step_out *out);

int pl_get_stats(pl_engine *e, pl_stats *out);

/* ---- test and benchmark hooks -----------------------------------------------------------------*/

/* fp32 logits [n, vocab] of the last step (host out), rows in the order of that step's entries. */
int pl_debug_get_logits(pl_engine *e, float *out, int64_t out_elems);
/* Keys (after rotation) and values of one slot and layer as host fp32 [n_ctx, n_kv_heads, hd]. */
int pl_debug_read_kv(pl_engine *e, int32_t slot, int32_t layer, float *k_out, float *v_out,
                     int32_t n_ctx);
int pl_debug_write_kv(pl_engine *e, int32_t slot, int32_t layer, const float *k_in,
                      const float *v_in, int32_t n_ctx);
/* Admit a sequence as if it had already run for `context_len` positions (>= n_prompt - 1 ... the
 * prompt is not needed then and may be NULL when context_len >= n_prompt): pages for
 * context_len positions are allocated, their contents left as they are in the pool; n_emitted
 * tokens count as generated; last_token is what the next step consumes. */
int pl_debug_add_sequence_at(pl_engine *e, uint64_t seq_id, const int32_t *prompt, int32_t n_prompt,
                             int32_t max_new, float temperature, int32_t context_len,
                             int32_t n_emitted, int32_t last_token, int32_t *out_slot);
/* Tokens read at positions [0, n) of a slot admitted with pl_debug_add_sequence_at (n must equal its
 * context length), so that its cache can be recomputed after an update. */
int pl_debug_set_history(pl_engine *e, int32_t slot, const int32_t *tokens, int32_t n);
/* Per-kernel-group timing with HIP events recorded on the decode stream, accumulated into pl_stats:
 * level 0 off; 1 around the attention launches only (attn_ms, attn_launches, attn_kv_bytes; everything
 * else lands in other_ms); 2 around every group (attention, GEMMs, sampler, rest).  Each event costs a
 * little GPU time between kernels, which is why level 1 exists. */
int pl_debug_set_profile(pl_engine *e, int32_t level);
/* A decode step replays its kernel sequence from a captured HIP graph (one per launch shape; on by
 * default, not used while pl_debug_set_profile is on).  on = 0 makes every step launch its kernels one
 * by one instead; results are identical either way. */
int pl_debug_set_graphs(pl_engine *e, int32_t on);
/* Debugging aid for the double-buffered update: when on, the step that flips to the new weights
 * first fills the buffer that just went inactive with bf16 NaN, so any kernel that still reads the
 * old weights after the flip shows up as NaN logits.  Costs one fill of the blob per update. */
int pl_debug_set_poison(pl_engine *e, int32_t on);
/* Device pointer and size of the KV page pool (to fill it with synthetic values). */
int pl_debug_kv_pool(pl_engine *e, void **device_ptr, int64_t *nbytes);

/* One launch of one tile configuration of the GEMM kernel over output columns [n_begin, n_end) (tuning
 * and tests).  cfg: 0 32x256, 1 64x256, 2 128x256, 3 64x128, 4 128x128, 5 256x128, 6 64x64, 7 128x64,
 * 8 32x128 (rows x columns of a workgroup's tile; 6-8 mode 0 only), 9 128x64 and 10 256x64 with the
 * wavefronts stacked along the rows.  mode and splits as in pl_gemm_bf16, except that mode 1 accepts
 * splits > 1: the partial sums then go to ws (device fp32 [splits, M, n_end - n_begin]) and a second
 * kernel applies the SwiGLU to their sum.  paired != 0 (splits = 1 only) lays the grid out so that the
 * row tiles of one column tile run on the same XCD at the same time.  PL_E_INVAL (nothing launched)
 * for shapes the configuration does not cover. */
int pl_debug_gemm_cfg(int32_t cfg, const void *x, const void *w, void *y, void *ws, int32_t M, int32_t N, int32_t K,
                      int32_t mode, int32_t splits, int32_t n_begin, int32_t n_end, int32_t paired, void *stream);

/* The K split an engine of max_batch = M_max fixes for the product [*, K] x [N, K]^T (mode as in
 * pl_gemm_bf16): columns [0, n_main) in `splits` slices, columns [n_main, N) in `rem_splits` (mode 0:
 * n_main = N), and the fp32 elements of workspace a mode-1 product then needs (0: none).  Any output
 * pointer may be NULL. */
int pl_debug_gemm_plan(int32_t M_max, int32_t N, int32_t K, int32_t mode, int32_t *splits, int32_t *n_main,
                       int32_t *rem_splits, int64_t *ws_elems);
/* The product of M <= M_max rows launched exactly as such an engine launches it for a pass of M rows
 * (tile shapes from M, K split from M_max).  mode 0: y is device fp32 [splits, M, N]; mode 1: y is device
 * bf16 [M, N / 2], ws device fp32 of ws_elems (may be NULL when that is 0).  Outputs of the same x rows
 * are bit-identical for every M <= M_max.  PL_E_INVAL (nothing launched) for unsupported shapes. */
int pl_debug_gemm_planned(const void *x, const void *w, void *y, void *ws, int32_t M_max, int32_t M, int32_t N, int32_t K,
                          int32_t mode, void *stream);

/* Launch a kernel that only reads the device buffer (contiguous 16-byte loads, 8 in flight per lane;
 * ordinary loads, or non-temporal ones if `nontemporal` is non-zero) on `stream`; returns the number of bytes it reads (a multiple of 256 MiB, <= nbytes) or a negative
 * pl_status.  Timed by the caller, it gives the read bandwidth HBM delivers on this board. */
int64_t pl_debug_stream_read(const void *device_ptr, int64_t nbytes, int32_t nontemporal, void *stream);

/* ---- kernel-level entry points (device pointers; `stream` is a hipStream_t or NULL) ----------- */

/* Ragged grouped-query decode attention over a paged bf16 cache: for every sequence b < n_seq and
 * query head h, out[b, h, :] = sum_j softmax_j(q[b, h] . K_b[j, h / group] / sqrt(hd)) V_b[j, h / group],
 * j < ctx_len[b].
 *   q          device bf16 [n_seq, n_q_heads, hd]
 *   kv_pages   device bf16 page pool of one layer; page p, kv head g starts at element
 *              (p * n_kv_heads + g) * 2 * page_tokens * hd: first the K block, then the V block.
 *              Within a page, tokens are grouped in runs of 32 (t = 32 r + u).  K block element
 *              (t, d): ((r * 2 + T) * (hd / 8) + d / 8) * 128 + R * 8 + d % 8 with T = (u / 4) % 2,
 *              R = (u / 8) * 4 + u % 4.  V block element (t, d): page_tokens * hd offset, then
 *              ((r * (hd / 16) + d / 16) * 4 + u / 8) * 128 + (d % 16) * 8 + u % 8.
 *   page_table device int32 [n_seq, pages_per_seq]; ctx_len device int32 [n_seq] (0 = skip row)
 *   out        device bf16 [n_seq, n_q_heads, hd]
 *   workspace  device, at least pl_attention_workspace_bytes(...) bytes
 * max_ctx bounds ctx_len (sizes the launch).  Positions at or beyond ctx_len inside the last page
 * must hold finite values.  Up to three launches on `stream` (work list from ctx_len and page_table, the
 * attention proper, and, when max_ctx allows sequences of several chunks, their merge); the caller owns every buffer, the
 * workspace holds nothing of value afterwards.  PL_E_INVAL (nothing launched) for n_seq outside
 * [1, 1024], head_dim not in {32, 64, 128}, more than 16 query heads per kv head, page_tokens not a
 * multiple of 32, or max_ctx beyond pages_per_seq * page_tokens. */
int64_t pl_attention_workspace_bytes(int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t hd,
                                     int32_t max_ctx);
int pl_attention_decode(const void *q, const void *kv_pages, const int32_t *page_table,
                        const int32_t *ctx_len, void *out, void *workspace, int32_t n_seq,
                        int32_t n_q_heads, int32_t n_kv_heads, int32_t hd, int32_t page_tokens,
                        int32_t pages_per_seq, int32_t max_ctx, void *stream);
/* Host helper: scatter fp32 [n, n_kv_heads, hd] keys and values of consecutive positions
 * first_pos .. first_pos + n - 1 of one sequence into host images of its pages (same layout as
 * above; `pages_host` is the host copy of the layer's pool, page ids taken from page_ids). */
int pl_kv_pack_host(uint16_t *pages_host, const int32_t *page_ids, const float *k, const float *v,
                    int32_t first_pos, int32_t n, int32_t n_kv_heads, int32_t hd, int32_t page_tokens);

/* y = x W^T with bf16 inputs and fp32 accumulation.  x device bf16 [M, K] row-major; w device bf16
 * [N, K] in MFMA operand order (see pl_weight_layout); K a multiple of 256, N a multiple of 32,
 * 1 <= M <= 512, and both x and w below 2 GiB (PL_E_INVAL otherwise: the kernels address an operand
 * through one 32-bit buffer descriptor).
 *   mode 0: y device fp32 [splits, M, N]; slice s holds the partial sum over columns
 *           [256 s c, min(256 (s + 1) c, K)), c = ceil((K / 256) / splits); their sum over s is the
 *           product.  1 <= splits <= K / 256 and no slice may be empty.
 *   mode 1: SwiGLU: w holds gate/up rows interleaved in blocks of 32 (see pl_weight_layout);
 *           y device bf16 [M, N / 2] = silu(gate) * up; splits must be 1. */
int pl_gemm_bf16(const void *x, const void *w, void *y, int32_t M, int32_t N, int32_t K,
                 int32_t mode, int32_t splits, void *stream);

/* Log-softmax + Gumbel-max sampler over fp32 logits (the decision is taken in fp32 with the
 * operation order given in the sampler specification).  All arrays device memory:
 * logits fp32 [n, vocab]; seq_id uint64 [n]; position int32 [n]; inv_temperature fp32 [n];
 * forced int32 [n] (-1 = sample); token int32 [n] out; logprob fp32 [n] out; workspace at least
 * pl_sample_workspace_bytes(n, vocab). */
int64_t pl_sample_workspace_bytes(int32_t n, int32_t vocab);
int pl_sample(const float *logits, int32_t n, int32_t vocab, const uint64_t *seq_id,
              const int32_t *position, const float *inv_temperature, const int32_t *forced,
              uint64_t seed, int32_t *token, float *logprob, void *workspace, void *stream);

/* pl_sample for callers that cannot allocate or carry a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments and results as pl_sample, but the
 * per-slice partial results live in a 256 KiB array in the library's own device image (one copy per
 * GPU, held until the process ends), so the call allocates nothing and takes no workspace.  Limits:
 * n <= 512 rows and vocab <= 262144; beyond them PL_E_INVAL and nothing is launched.  All calls on one
 * GPU share that array: calls that overlap in time on the same GPU (different streams or threads) race
 * and must be serialised by the caller; nothing needs clearing between calls (every partial a launch
 * reads was written by that launch). */
int pl_sample_static(const float *logits, int32_t n, int32_t vocab, const uint64_t *seq_id,
                     const int32_t *position, const float *inv_temperature, const int32_t *forced,
                     uint64_t seed, int32_t *token, float *logprob, void *stream);

/* Trainer-side use of the recorded log-probs (Sec. 2.1): truncated token-level importance weights
 * w_i = min(c, exp(logp_pi[i] - logp_mu[i])) (the paper clamps at c = 5) and the normalised effective
 * sample size (sum w)^2 / (N sum w^2) (Sec. 2.1, ESS), per sequence of a packed batch and over all its
 * tokens.  All device pointers:
 *   logp_pi, logp_mu  fp32 [n_tokens]: log-prob of each token under the current policy and the
 *                     behaviour log-prob the engine recorded for it
 *   seq_offsets       int64 [n_seq + 1], non-decreasing: sequence s owns tokens [off[s], off[s+1])
 *   w_out             fp32 [n_tokens] or NULL
 *   seq_sums          fp64 [n_seq, 2]: sum w and sum w^2 of each sequence
 *   ess_seq           fp64 [n_seq]: normalised ESS of each sequence (NaN for an empty one)
 *   totals            fp64 [3]: sum w, sum w^2 and normalised ESS over all tokens
 * fp64 arithmetic, fixed reduction order (bit-reproducible).  PL_E_INVAL for c <= 0 or n_seq < 1.
 * Asynchronous on `stream`; the caller owns every buffer. */
int pl_is_ess(const float *logp_pi, const float *logp_mu, const int64_t *seq_offsets, int32_t n_seq, float c,
              float *w_out, double *seq_sums, double *ess_seq, double *totals, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PL_H */
