/* Host-side exercise of the C ABI for a sanitizer build (AddressSanitizer + UBSan on host code
 * only): configuration checks, layout arithmetic at the largest supported sizes, NULL and
 * out-of-range arguments.  Needs no GPU: every call here is decided on the host, and a context
 * cannot be created without a device.  Prints "ok" and exits 0; a sanitizer report makes the
 * process exit non-zero.  Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>
#include "mkv.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static mkv_config base_config(void) {
  mkv_config c;
  memset(&c, 0, sizeof c);
  c.n_layers = 1; c.batch = 2; c.n_q_heads = 8; c.n_kv_heads = 2; c.head_dim = 64; c.dtype = MKV_F32;
  c.max_prefill = 256; c.decode_budget = 64; c.evict_trigger = 72; c.recent_window = 8; c.alpha = 0.9f;
  return c;
}

int main(void) {
  mkv_config c = base_config();
  size_t need = mkv_required_bytes(&c);
  CHECK(need > 0);
  CHECK(mkv_required_bytes(NULL) == 0);

  /* every field at a bad value: refused, with a message, before anything touches a device */
  {
    mkv_ctx* ctx = (mkv_ctx*)0x1;
    mkv_config b;
#define BAD(stmt) do { b = base_config(); stmt; CHECK(mkv_required_bytes(&b) == 0); \
                       CHECK(mkv_create(&b, &ctx) == MKV_ERR_ARG); CHECK(ctx == NULL); \
                       CHECK(strlen(mkv_last_error(NULL)) > 0); } while (0)
    BAD(b.n_q_heads = 7); BAD(b.head_dim = 96); BAD(b.dtype = 5); BAD(b.decode_budget = 0);
    BAD(b.evict_trigger = 63); BAD(b.recent_window = 65); BAD(b.alpha = 1.5f); BAD(b.alpha = -0.1f);
    BAD(b.batch = 0); BAD(b.n_layers = 0); BAD(b.score_mode = 3); BAD(b.split_keys = 100);
    BAD(b.evict_trigger = MKV_NEVER_EVICT);
    BAD(b.evict_trigger = MKV_NEVER_EVICT; b.decode_capacity = 64);
    BAD(b.decode_capacity = 70); BAD(b.decode_budget = 20000; b.evict_trigger = 20000);
    BAD(b.batch = 5000); BAD(b.max_prefill = 1 << 24); BAD(b.softmax_scale = -1.0f);
    BAD(b.arena = (void*)12345; b.arena_bytes = (size_t)1 << 30);
    BAD(b.max_q_len = 17); BAD(b.max_q_len = 4);               /* multi-query needs bf16 x 128 */
    BAD(b.attn_variant = 99); BAD(b.groups_per_cu = 99); BAD(b.n_kv_heads = 0);
    BAD(b.evict_trigger = 2147483000; b.decode_capacity = 0);  /* trigger + 1 beyond the supported pool */
    CHECK(mkv_create(&c, NULL) == MKV_ERR_ARG);
    CHECK(mkv_create(NULL, &ctx) == MKV_ERR_ARG);
  }

  /* layout arithmetic at the largest supported sizes (64-bit offsets, no overflow) */
  {
    mkv_config big = base_config();
    big.n_layers = 32; big.batch = 32; big.n_q_heads = 32; big.n_kv_heads = 8; big.head_dim = 128;
    big.dtype = MKV_BF16; big.max_prefill = 16384; big.decode_budget = 4096; big.evict_trigger = 4159;
    big.recent_window = 128;
    size_t kv = (size_t)32 * 32 * (16384 + 4160) * 4096;
    size_t got = mkv_required_bytes(&big);
    CHECK(got > kv && got < kv + kv / 50);
    big.n_layers = 64; big.batch = 1024; big.max_prefill = 1 << 20; big.decode_budget = 16000;
    big.evict_trigger = 16383; big.recent_window = 16000; big.max_q_len = 16; big.decode_capacity = 16384;
    big.evict_trigger = 16384 - 16;
    got = mkv_required_bytes(&big);
    CHECK(got > (size_t)1 << 40);                               /* far beyond any device, still computed */
    big.score_mode = MKV_SCORE_PER_KV_HEAD;
    CHECK(mkv_required_bytes(&big) > got);
    /* the paper's cadence on a bf16 x 128 layer: deferred compaction adds its spare slots */
    mkv_config cad = base_config();
    cad.dtype = MKV_BF16; cad.head_dim = 128; cad.decode_budget = 512; cad.evict_trigger = 512;
    size_t with_room = mkv_required_bytes(&cad);
    cad.decode_capacity = 513;
    CHECK(with_room > mkv_required_bytes(&cad));
    cad.decode_budget = cad.evict_trigger = 16383; cad.decode_capacity = 0; cad.recent_window = 0;
    CHECK(mkv_required_bytes(&cad) > 0);                        /* no room left for spare slots: still valid */
  }

  /* NULL contexts and pointers */
  CHECK(mkv_destroy(NULL) == MKV_OK);
  CHECK(mkv_evict(NULL, 0, 0) == MKV_ERR_ARG);
  CHECK(mkv_get_lens(NULL, 0, 0, NULL, NULL, NULL) == MKV_ERR_ARG);
  CHECK(mkv_decode_step(NULL, 0, NULL, NULL, NULL, NULL, NULL) == MKV_ERR_ARG);
  CHECK(mkv_decode_step_static(NULL, 0, NULL, NULL, NULL, NULL, NULL) == MKV_ERR_ARG);
  CHECK(mkv_decode_step_multi(NULL, 0, 1, NULL, NULL, NULL, NULL, NULL) == MKV_ERR_ARG);
  CHECK(mkv_prefill_append(NULL, 0, 0, NULL, NULL, 0) == MKV_ERR_ARG);
  CHECK(mkv_prefill_compress(NULL, 0, 0, NULL, 1) == MKV_ERR_ARG);
  CHECK(mkv_project_append(NULL, 0, NULL, NULL, NULL, 256, NULL, 1e4f, NULL) == MKV_ERR_ARG);
  CHECK(mkv_read_scores(NULL, 0, 0, NULL, NULL, 0, NULL) == MKV_ERR_ARG);
  CHECK(mkv_read_slots(NULL, 0, 0, NULL, NULL, NULL, 0, NULL, NULL) == MKV_ERR_ARG);
  CHECK(mkv_write_scores(NULL, 0, 0, NULL, 0) == MKV_ERR_ARG);
  CHECK(mkv_load_decode(NULL, 0, 0, NULL, NULL, NULL, NULL, 0, 0) == MKV_ERR_ARG);
  CHECK(mkv_read_kv(NULL, 0, 0, 0, 0, NULL, NULL, 0, NULL) == MKV_ERR_ARG);
  CHECK(mkv_read_probs(NULL, 0, 0, NULL, NULL, 0, NULL) == MKV_ERR_ARG);
  CHECK(mkv_set_score_view(NULL, 0) == MKV_ERR_ARG);
  CHECK(mkv_set_profiling(NULL, 1) == MKV_ERR_ARG);
  CHECK(mkv_read_profile(NULL, NULL, NULL) == MKV_ERR_ARG);

  /* a valid configuration on a machine without a device: an error code, never a crash */
  {
    mkv_ctx* ctx = NULL;
    int rc = mkv_create(&c, &ctx);
    if (rc == MKV_OK) { CHECK(ctx != NULL); CHECK(mkv_destroy(ctx) == MKV_OK); }
    else { CHECK(ctx == NULL); CHECK(rc == MKV_ERR_NOMEM || rc == MKV_ERR_HIP); CHECK(strlen(mkv_last_error(NULL)) > 0); }
  }
  if (failures) { printf("%d checks failed\n", failures); return 1; }
  printf("ok\n");
  return 0;
}
