/* Host logic of the engine under AddressSanitizer / UndefinedBehaviorSanitizer: a plain C program that
 * drives bookkeeping-only engines (device = PL_DEVICE_NONE, no GPU touched) through the C ABI: slot table,
 * page accounting, prompt reading, weight-update protocol, weight packing, error paths.  Built and run by
 * tests/test_host_sanitized.py; any sanitizer report or failed check makes it exit non-zero. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/pl.h"

#define CHECK(cond)                                                                    \
  do {                                                                                 \
    if (!(cond)) {                                                                     \
      fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, pl_last_error()); \
      exit(1);                                                                         \
    }                                                                                  \
  } while (0)

static pl_model_cfg tiny(int32_t batch, int32_t ctx, int64_t pool, int32_t page) {
  pl_model_cfg c;
  memset(&c, 0, sizeof c);
  c.n_layers = 2; c.d_model = 256; c.n_q_heads = 8; c.n_kv_heads = 2; c.head_dim = 32; c.d_ffn = 1024; c.vocab = 4096;
  c.rope_theta = 1e4f; c.rms_eps = 1e-6f; c.max_batch = batch; c.max_context = ctx; c.kv_pool_tokens = pool;
  c.kv_page_tokens = page; c.n_weight_buffers = 2; c.seed = 7; c.device = PL_DEVICE_NONE;
  return c;
}

typedef struct {
  int32_t *slot, *token, *position; uint64_t *seq_id; float *logprob; uint32_t *version; uint8_t *emitted, *finished;
  pl_step_out out;
} outbuf;

static outbuf make_out(int n) {
  outbuf b;
  b.slot = malloc(n * 4); b.token = malloc(n * 4); b.position = malloc(n * 4); b.seq_id = malloc(n * 8);
  b.logprob = malloc(n * 4); b.version = malloc(n * 4); b.emitted = malloc(n); b.finished = malloc(n);
  memset(&b.out, 0, sizeof b.out);
  b.out.slot = b.slot; b.out.token = b.token; b.out.position = b.position; b.out.seq_id = b.seq_id;
  b.out.logprob = b.logprob; b.out.weight_version = b.version; b.out.emitted = b.emitted; b.out.finished = b.finished;
  return b;
}
static void free_out(outbuf *b) {
  free(b->slot); free(b->token); free(b->position); free(b->seq_id); free(b->logprob); free(b->version);
  free(b->emitted); free(b->finished);
}

static void life_cycle(int32_t batch) {
  pl_model_cfg c = tiny(batch, 128, 0, 32);             /* pool sized automatically */
  pl_engine *e = NULL;
  CHECK(pl_create(&c, &e) == PL_OK && e);
  const int64_t nbytes = pl_weight_nbytes(e);
  uint16_t *blob = calloc(nbytes / 2, 2);
  /* every source tensor through the packing helper, fp32 and bf16 sources */
  for (int32_t i = 0; i < pl_weight_count(e); ++i) {
    const char *name; int64_t off, shp[2];
    CHECK(pl_weight_layout(e, i, &name, &off, shp) == PL_OK);
    CHECK(off >= 0 && (off + shp[0] * shp[1]) * 2 <= nbytes);
  }
  const char *mats[] = {"embed", "lm_head", "l0.wq", "l0.wk", "l0.wv", "l0.wo", "l0.wg", "l0.wu", "l0.wd",
                        "l1.wq", "l1.wk", "l1.wv", "l1.wo", "l1.wg", "l1.wu", "l1.wd"};
  const int64_t rows[] = {4096, 4096, 256, 64, 64, 256, 1024, 1024, 256, 256, 64, 64, 256, 1024, 1024, 256};
  const int64_t cols[] = {256, 256, 256, 256, 256, 256, 256, 256, 1024, 256, 256, 256, 256, 256, 256, 1024};
  for (int t = 0; t < 16; ++t) {
    float *src = malloc(rows[t] * cols[t] * 4);
    for (int64_t i = 0; i < rows[t] * cols[t]; ++i) src[i] = (float)((i * 2654435761u) % 1000) * 1e-3f - 0.5f;
    CHECK(pl_pack_weights(e, mats[t], src, 1, blob) == PL_OK);
    free(src);
  }
  uint16_t gains[256];
  for (int i = 0; i < 256; ++i) gains[i] = 0x3F80;
  const char *gn[] = {"l0.g1", "l0.g2", "l1.g1", "l1.g2", "gf"};
  for (int t = 0; t < 5; ++t) CHECK(pl_pack_weights(e, gn[t], gains, 0, blob) == PL_OK);
  CHECK(pl_pack_weights(e, "l2.wq", gains, 0, blob) == PL_E_INVAL);
  CHECK(pl_pack_weights(e, "nonsense", gains, 0, blob) == PL_E_INVAL);

  outbuf ob = make_out(batch);
  CHECK(pl_decode_step(e, NULL, &ob.out) == PL_E_STATE);          /* no weights yet */
  CHECK(pl_load_weights(e, blob, nbytes - 2) == PL_E_INVAL);
  CHECK(pl_load_weights(e, blob, nbytes) == PL_OK);
  int32_t prompt[100];
  for (int i = 0; i < 100; ++i) prompt[i] = (i * 37) % 4096;
  int32_t slot = -1, npos = -1;
  CHECK(pl_add_sequence(e, 1, prompt, 100, 40, 1.0f, &slot) == PL_E_CTX);
  CHECK(pl_add_sequence(e, 1, prompt, 0, 4, 1.0f, &slot) == PL_E_INVAL);
  CHECK(pl_add_sequence(e, 1, prompt, 4, 4, 0.0f, &slot) == PL_E_INVAL);
  for (int32_t b = 0; b < batch; ++b) {
    CHECK(pl_add_sequence(e, 100 + b, prompt, 20 + b % 7, 5 + b % 3, 1.0f, &slot) == PL_OK && slot == b);
    if (b % 3 == 0) CHECK(pl_prefill(e, slot, &npos) == PL_OK && npos == 20 + b % 7 - 1);
    if (b % 3 == 1) {
      CHECK(pl_prefill_async(e, slot, &npos) == PL_OK && npos == 20 + b % 7 - 1);
      CHECK(pl_prefill_async(e, slot, &npos) == PL_E_BUSY);
    }
  }
  CHECK(pl_add_sequence(e, 9, prompt, 4, 4, 1.0f, &slot) == PL_E_NOSLOT);
  CHECK(pl_num_active(e) == batch);
  uint32_t ver = 0;
  int32_t *forced = malloc(batch * 4);
  long emitted = 0, steps = 0;
  uint32_t seen_version = 0;
  while (pl_num_active(e) > 0 && steps < 400) {
    if (steps == 3) CHECK(pl_swap_weights(e, blob, nbytes, PL_SWAP_ASYNC, &ver) == PL_OK && ver == 1);
    if (steps == 4) CHECK(pl_swap_weights(e, blob, nbytes, PL_SWAP_WAIT, &ver) == PL_OK && ver == 2);
    if (steps == 5) CHECK(pl_swap_weights(e, blob, nbytes, PL_SWAP_WAIT | PL_SWAP_RECOMPUTE_KV, &ver) == PL_OK && ver == 3);
    if (steps == 5) CHECK(pl_swap_weights(e, blob, nbytes, PL_SWAP_WAIT, &ver) == PL_E_BUSY);
    for (int32_t b = 0; b < batch; ++b) forced[b] = (steps % 2) ? (int32_t)((b * 13 + steps) % 4096) : -1;
    CHECK(pl_decode_step(e, forced, &ob.out) == PL_OK);
    CHECK(ob.out.n == pl_num_active(e));
    for (int32_t i = 0; i < ob.out.n; ++i) {
      CHECK(ob.version[i] >= seen_version && ob.version[i] == ob.version[0]);   /* one version per step, never going back */
      seen_version = ob.version[i];
      CHECK(ob.slot[i] >= 0 && ob.slot[i] < batch && ob.position[i] >= 0 && ob.position[i] < 128);
      emitted += ob.emitted[i];
      if (ob.finished[i]) CHECK(pl_retire_sequence(e, ob.slot[i]) == PL_OK);
    }
    ++steps;
  }
  CHECK(pl_num_active(e) == 0 && emitted > 0);
  pl_stats st;
  CHECK(pl_get_stats(e, &st) == PL_OK);
  CHECK(st.kv_pages_free == st.kv_pages_total && st.swaps == seen_version && st.tokens_emitted == (uint64_t)emitted);
  CHECK(batch < 3 || seen_version == 3);
  CHECK(pl_retire_sequence(e, 0) == PL_E_STATE);
  CHECK(pl_retire_sequence(e, batch) == PL_E_INVAL);
  /* mid-life admission hook and history */
  CHECK(pl_debug_add_sequence_at(e, 77, NULL, 16, 64, 1.0f, 70, 55, 3, &slot) == PL_OK);
  CHECK(pl_debug_set_history(e, slot, prompt, 69) == PL_E_INVAL);
  CHECK(pl_debug_set_history(e, slot, prompt, 70) == PL_OK);
  CHECK(pl_decode_step(e, NULL, &ob.out) == PL_OK && ob.out.n == 1 && ob.position[0] == 70);
  free(forced);
  free_out(&ob);
  free(blob);
  pl_destroy(e);
}

static void pool_exhaustion(void) {
  pl_model_cfg c = tiny(4, 128, 96, 32);                /* three pages */
  pl_engine *e = NULL;
  CHECK(pl_create(&c, &e) == PL_OK);
  uint16_t *blob = calloc(pl_weight_nbytes(e) / 2, 2);
  CHECK(pl_load_weights(e, blob, pl_weight_nbytes(e)) == PL_OK);
  int32_t prompt[64] = {0}, slot;
  CHECK(pl_add_sequence(e, 1, prompt, 60, 60, 1.0f, &slot) == PL_OK);       /* two pages */
  CHECK(pl_add_sequence(e, 2, prompt, 40, 10, 1.0f, &slot) == PL_E_NOKV);    /* would need two more */
  CHECK(pl_add_sequence(e, 2, prompt, 30, 60, 1.0f, &slot) == PL_OK);       /* one page */
  outbuf ob = make_out(4);
  int rc = PL_OK, steps = 0;
  while ((rc = pl_decode_step(e, NULL, &ob.out)) == PL_OK && steps < 200) ++steps;
  CHECK(rc == PL_E_NOKV && steps > 0);                  /* growth ran the pool dry; the engine is unchanged */
  CHECK(pl_retire_sequence(e, 1) == PL_OK);
  CHECK(pl_decode_step(e, NULL, &ob.out) == PL_OK && ob.out.n == 1);
  free_out(&ob);
  free(blob);
  pl_destroy(e);
}

static void bad_configurations(void) {
  pl_engine *e = NULL;
  pl_model_cfg c = tiny(4, 128, 256, 32);
  c.head_dim = 48;
  CHECK(pl_create(&c, &e) == PL_E_INVAL && e == NULL);
  c = tiny(4, 128, 256, 48);
  CHECK(pl_create(&c, &e) == PL_E_INVAL);
  c = tiny(0, 128, 256, 32);
  CHECK(pl_create(&c, &e) == PL_E_INVAL);
  c = tiny(4, 128, -1, 32);
  CHECK(pl_create(&c, &e) == PL_E_INVAL);
  c = tiny(4, 128, 256, 32);
  c.d_model = 8192; c.vocab = 131072 + 32; c.n_q_heads = 64; c.n_kv_heads = 8; c.head_dim = 128; c.d_ffn = 8192;
  CHECK(pl_create(&c, &e) == PL_E_INVAL);               /* a matrix the GEMM cannot address */
  CHECK(pl_create(NULL, &e) == PL_E_INVAL);
  CHECK(pl_weight_nbytes(NULL) == 0 && pl_weight_count(NULL) == 0 && pl_num_active(NULL) == 0);
  pl_destroy(NULL);
}

static void build_variants(void) {
  /* fp32 test build and tied embeddings: blob sizes, layout enumeration, packing */
  for (int variant = 0; variant < 4; ++variant) {
    pl_model_cfg c = tiny(3, 64, 0, 32);
    c.dtype = variant & 1 ? PL_F32 : PL_BF16;
    c.tie_embeddings = variant >> 1;
    pl_engine *e = NULL;
    CHECK(pl_create(&c, &e) == PL_OK);
    const int64_t nbytes = pl_weight_nbytes(e), esz = c.dtype == PL_F32 ? 4 : 2;
    int64_t elems = 0;
    for (int32_t i = 0; i < pl_weight_count(e); ++i) {
      const char *name; int64_t off, shp[2];
      CHECK(pl_weight_layout(e, i, &name, &off, shp) == PL_OK && off == elems);
      elems += shp[0] * shp[1];
      CHECK(!(c.tie_embeddings && strcmp(name, "lm_head") == 0));
    }
    CHECK(elems * esz == nbytes);
    char *blob = calloc(nbytes, 1);
    float *src = malloc(4096 * 256 * 4);
    for (int i = 0; i < 4096 * 256; ++i) src[i] = (float)(i % 97) * 0.01f;
    CHECK(pl_pack_weights(e, "embed", src, 1, blob) == PL_OK);
    CHECK(pl_pack_weights(e, "l1.wu", src, 1, blob) == PL_OK);
    CHECK(pl_pack_weights(e, "l0.wk", src, 1, blob) == PL_OK);
    CHECK(pl_pack_weights(e, "lm_head", src, 1, blob) == (c.tie_embeddings ? PL_E_INVAL : PL_OK));
    if (c.dtype == PL_F32) CHECK(pl_pack_weights(e, "l0.wq", src, 0, blob) == PL_E_INVAL);   /* fp32 sources only */
    CHECK(pl_load_weights(e, blob, nbytes) == PL_OK);
    free(src);
    free(blob);
    pl_destroy(e);
  }
}

int main(void) {
  build_variants();
  const int32_t batches[] = {1, 3, 4, 64, 257, 511};
  for (unsigned i = 0; i < sizeof batches / sizeof *batches; ++i) life_cycle(batches[i]);
  pool_exhaustion();
  bad_configurations();
  puts("host logic clean under the sanitizers");
  return 0;
}
