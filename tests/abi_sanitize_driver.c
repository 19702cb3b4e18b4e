/* Host-side misuse battery for the C ABI of libgta, meant to be linked against objects whose HOST code
 * was built with -fsanitize=address,undefined (tests/test_abi_sanitized.py does that): every call below
 * is refused by the validation layer before anything touches a device, so it runs on a box without a
 * GPU; the sanitizers watch the validation and workspace-sizing code while it handles NULL pointers,
 * misaligned pointers, extreme sizes and inconsistent cache descriptions.  Exit status 0 = every call
 * returned the expected status (a sanitizer report aborts the program by itself). */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "gta.h"

static int failures = 0;
#define EXPECT(call, want)                                                                  \
  do {                                                                                      \
    long long got_ = (long long)(call);                                                     \
    if (got_ != (long long)(want)) {                                                        \
      fprintf(stderr, "line %d: %s = %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); \
      ++failures;                                                                           \
    }                                                                                       \
  } while (0)

static gta_config base_config(void) {
  gta_config c;
  memset(&c, 0, sizeof c);
  c.d_model = 256; c.n_heads = 8; c.n_qgroups = 2; c.n_kgroups = 2; c.n_cgroups = 1;
  c.head_dim = 32; c.latent_dim = 64; c.dtype = GTA_F32; c.rope = 0; c.rope_base = 10000.f;
  c.gate = GTA_GATE_SIGMOID; c.softmax_scale = 0.f;
  return c;
}

int main(void) {
  void *fake = (void *)(uintptr_t)4096;          /* never dereferenced: validation fails first */
  void *odd = (void *)(uintptr_t)(4096 + 4);
  gta_config cfg = base_config();
  gta_weights w = {fake, fake, fake, fake, fake, NULL};
  gta_cache cache;
  memset(&cache, 0, sizeof cache);
  cache.k = fake; cache.c = fake; cache.seq_lens = (int32_t *)fake; cache.status = (int32_t *)fake;
  cache.max_batch = 2; cache.max_seq = 64;
  const size_t big = (size_t)1 << 40;

  /* configurations */
  EXPECT(gta_uses_tuned_kernels(NULL, GTA_MODE_PREFILL), GTA_ERR_NULL);
  EXPECT(gta_uses_tuned_kernels(&cfg, GTA_MODE_PREFILL), 0);
  EXPECT(gta_uses_tuned_kernels(&cfg, 99), GTA_ERR_DTYPE);
  { gta_config c = cfg; c.n_qgroups = 3; EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_DECODE), GTA_ERR_SHAPE); }
  { gta_config c = cfg; c.latent_dim = 16; EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_DECODE), GTA_ERR_SHAPE); }
  { gta_config c = cfg; c.dtype = 7; EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_DECODE), GTA_ERR_DTYPE); }
  { gta_config c = cfg; c.gate = 42; EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_DECODE), GTA_ERR_DTYPE); }
  { gta_config c = cfg; c.d_model = INT32_MAX; c.n_heads = INT32_MAX - 1; c.n_qgroups = INT32_MAX - 1; c.n_kgroups = INT32_MAX - 1;
    c.n_cgroups = INT32_MAX - 1; c.head_dim = INT32_MAX; c.latent_dim = INT32_MAX;
    EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_PREFILL) < 0, 1); }     /* no overflow on the way to the refusal */
  { gta_config c = cfg; c.softmax_scale = -1.f; EXPECT(gta_uses_tuned_kernels(&c, GTA_MODE_PREFILL), GTA_ERR_SHAPE); }

  /* workspace sizing */
  EXPECT(gta_workspace_bytes(NULL, GTA_MODE_PREFILL, 1, 128, 128, 0), 0);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_PREFILL, 0, 128, 128, 0), 0);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_PREFILL, 1, -5, 128, 0), 0);
  EXPECT(gta_workspace_bytes(&cfg, 17, 1, 128, 128, 0), 0);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_PREFILL, 1, 128, 128, 0) > 0, 1);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_PREFILL_CHUNK, 4, 4096, 2048, 0) > 0, 1);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_DECODE, 65535, 0, INT32_MAX, 1024) > 0, 1);
  EXPECT(gta_workspace_bytes(&cfg, GTA_MODE_PREFILL, 65535, INT32_MAX, INT32_MAX, 0) > 0, 1);

  /* prefill */
  EXPECT(gta_prefill(&cfg, &w, NULL, NULL, 1, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_NULL);
  EXPECT(gta_prefill(&cfg, NULL, fake, NULL, 1, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_NULL);
  EXPECT(gta_prefill(&cfg, &w, odd, NULL, 1, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_ALIGN);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 0, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 3, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 1, (int64_t)INT32_MAX + 1, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 1, 128, 128, NULL, NULL, fake, fake, 16, NULL), GTA_ERR_WORKSPACE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 1, 128, 128, NULL, NULL, fake, NULL, 0, NULL), GTA_ERR_WORKSPACE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 1, 128, 128, &cache, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_prefill(&cfg, &w, fake, NULL, 1, 0, 0, NULL, NULL, fake, fake, big, NULL), GTA_OK);   /* nothing to do */
  { gta_weights wn = w; wn.wk = NULL; EXPECT(gta_prefill(&cfg, &wn, fake, NULL, 1, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_NULL); }
  { gta_weights wn = w; wn.wo = odd; EXPECT(gta_prefill(&cfg, &wn, fake, NULL, 1, 128, 128, NULL, NULL, fake, fake, big, NULL), GTA_ERR_ALIGN); }

  /* chunked prefill */
  EXPECT(gta_prefill_chunk(&cfg, &w, fake, NULL, 1, 16, 16, NULL, NULL, fake, fake, big, NULL), GTA_ERR_NULL);
  EXPECT(gta_prefill_chunk(&cfg, &w, fake, NULL, 1, 128, 128, &cache, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_prefill_chunk(&cfg, &w, fake, NULL, 1, 16, 16, &cache, NULL, fake, fake, 16, NULL), GTA_ERR_WORKSPACE);
  EXPECT(gta_prefill_chunk(&cfg, &w, fake, NULL, 3, 16, 16, &cache, NULL, fake, fake, big, NULL), GTA_ERR_SHAPE);

  /* decode, with and without a workspace of the caller */
  EXPECT(gta_decode(&cfg, &w, fake, 1, NULL, NULL, fake, 0, fake, big, NULL), GTA_ERR_NULL);
  EXPECT(gta_decode(&cfg, &w, fake, 3, &cache, NULL, fake, 0, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_decode(&cfg, &w, fake, 1, &cache, NULL, fake, -1, fake, big, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_decode(&cfg, &w, fake, 1, &cache, NULL, odd, 0, fake, big, NULL), GTA_ERR_ALIGN);
  EXPECT(gta_decode(&cfg, &w, fake, 1, &cache, NULL, fake, 0, fake, 16, NULL), GTA_ERR_WORKSPACE);
  { gta_cache p = cache; p.block_table = (const int32_t *)fake; p.page_size = 16; p.pages_per_slot = 3; p.num_pages = 8;
    EXPECT(gta_decode(&cfg, &w, fake, 1, &p, NULL, fake, 0, fake, big, NULL), GTA_ERR_SHAPE); }    /* 16 * 3 != 64 */
  { gta_cache p = cache; p.block_table = (const int32_t *)fake; p.page_size = 16; p.pages_per_slot = 4; p.num_pages = 0;
    EXPECT(gta_decode(&cfg, &w, fake, 1, &p, NULL, fake, 0, fake, big, NULL), GTA_ERR_SHAPE); }
  { gta_cache p = cache; p.block_table = (const int32_t *)((uintptr_t)fake + 2); p.page_size = 16; p.pages_per_slot = 4; p.num_pages = 8;
    EXPECT(gta_decode(&cfg, &w, fake, 1, &p, NULL, fake, 0, fake, big, NULL), GTA_ERR_ALIGN); }
  { gta_cache p = cache; p.max_seq = 0; EXPECT(gta_decode(&cfg, &w, fake, 1, &p, NULL, fake, 0, fake, big, NULL), GTA_ERR_SHAPE); }
  { gta_config c = cfg; c.d_model = 1 << 20; c.n_heads = 1 << 12; c.n_qgroups = 1 << 12; c.n_kgroups = 1 << 12; c.n_cgroups = 1; c.head_dim = 128;
    c.latent_dim = 1 << 12; gta_cache p = cache; p.max_batch = 65535; p.max_seq = 1 << 20;    /* far more scratch than the fixed array */
    EXPECT(gta_decode_static(&c, &w, fake, 65535, &p, NULL, fake, 0, NULL), GTA_ERR_WORKSPACE); }
  EXPECT(gta_decode_static(&cfg, &w, fake, 1, NULL, NULL, fake, 0, NULL) < 0, 1);

  /* append and the stage entry points */
  EXPECT(gta_cache_append(&cfg, &cache, NULL, fake, NULL, (const int32_t *)fake, 1, 1, NULL), GTA_ERR_NULL);
  EXPECT(gta_cache_append(&cfg, &cache, NULL, fake, fake, (const int32_t *)fake, 1, -1, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_cache_append(&cfg, &cache, NULL, odd, fake, (const int32_t *)fake, 1, 1, NULL), GTA_ERR_ALIGN);
  EXPECT(gta_prefill_attention(&cfg, fake, fake, NULL, NULL, 1, 128, 128, fake, NULL), GTA_ERR_NULL);
  EXPECT(gta_prefill_attention(&cfg, fake, fake, fake, NULL, 1, 0, 0, fake, NULL), GTA_OK);
  EXPECT(gta_prefill_projection(&cfg, &w, fake, NULL, 1, 128, 128, fake, fake, fake, fake, fake, big, NULL), GTA_ERR_UNSUPPORTED);
  EXPECT(gta_prefill_decoder(&cfg, &w, fake, NULL, 128, fake, NULL), GTA_ERR_NULL);
  EXPECT(gta_output_projection(&cfg, &w, fake, 128, fake, NULL), GTA_ERR_NULL);      /* no W_O given */
  EXPECT(gta_decode_attention(&cfg, NULL, &cache, NULL, 1, 0, fake, big, NULL), GTA_ERR_NULL);
  EXPECT(gta_decode_combine(&cfg, &cache, NULL, 1, 0, fake, 16, (float *)fake, NULL), GTA_ERR_WORKSPACE);
  EXPECT(gta_calibration_copy(fake, fake, 24, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_calibration_copy(fake, fake, 0, NULL), GTA_OK);
  EXPECT(gta_calibration_read(fake, 1 << 20, 7, fake, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_calibration_mfma(0, 1, 0, fake, NULL), GTA_ERR_SHAPE);
  EXPECT(gta_calibration_mfma(4, 1, 7, fake, NULL), GTA_ERR_DTYPE);
  EXPECT(strcmp(gta_strerror(GTA_ERR_WORKSPACE), "workspace missing or too small"), 0);
  EXPECT(strcmp(gta_strerror(-99), "unknown gta_status"), 0);

  if (failures) { fprintf(stderr, "%d unexpected status value(s)\n", failures); return 1; }
  printf("abi sanitize driver: all calls refused as expected\n");
  return 0;
}
