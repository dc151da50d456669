/* Host-side exercise of libmixkvq's C ABI for a build with AddressSanitizer and UndefinedBehaviorSanitizer on the
 * host code (tests/test_library_host.py compiles csrc/api.hip that way, links this driver against it and runs it).
 * Only host logic runs: configuration checks, record layout, buffer sizes, the handle, the token-count state machine
 * and its error paths.  Device pointers are made-up addresses that nothing dereferences on the host.  Where no GPU is
 * present a call that has to enqueue a kernel fails inside HIP; the driver then checks that the call reports
 * MIXKVQ_EHIP and leaves the token counts as they were.  Where a GPU is present those calls are skipped (the made-up
 * addresses must never reach a kernel). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "mixkvq.h"

extern int hipGetDeviceCount(int* count);

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      exit(1);                                                               \
    }                                                                        \
  } while (0)

static mixkvq_config base_config(void) {
  mixkvq_config c;
  memset(&c, 0, sizeof(c));
  c.B = 3; c.Hq = 14; c.Hkv = 2; c.D = 128; c.T_max = 512; c.Gk = 128; c.Gv = 128; c.R = 128; c.k4 = 16; c.k16 = 0;
  c.tau16 = c.tau4 = 1.0;
  return c;
}

static mixkvq_buffers fake_buffers(void) {
  mixkvq_buffers b;
  b.blocks = (void*)(uintptr_t)0x100000000000ull;
  b.res_k = (void*)(uintptr_t)0x110000000000ull;
  b.res_v = (void*)(uintptr_t)0x120000000000ull;
  b.qacc = (void*)(uintptr_t)0x130000000000ull;
  b.workspace = (void*)(uintptr_t)0x140000000000ull;
  return b;
}

int main(void) {
  int n_dev = 0;
  const int have_gpu = hipGetDeviceCount(&n_dev) == 0 && n_dev > 0;

  /* configuration checks and layout */
  mixkvq_config cfg = base_config();
  mixkvq_block_layout_t lay;
  CHECK(mixkvq_block_layout(&cfg, &lay) == MIXKVQ_OK);
  CHECK(lay.rec_bytes == 9760 && lay.NL == 112 && lay.Wlo == 7 && lay.W4 == 2 && lay.NG == 1 && lay.NVG == 1);
  CHECK(mixkvq_block_layout(NULL, &lay) == MIXKVQ_EINVAL && mixkvq_block_layout(&cfg, NULL) == MIXKVQ_EINVAL);
  {
    mixkvq_config bad = cfg;
    bad.D = 64;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
    bad = cfg; bad.Hq = 15;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
    bad = cfg; bad.k4 = 12;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
    bad = cfg; bad.T_max = 500;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
    bad = cfg; bad.policy = 1; bad.tau16 = -1.0;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
    bad = cfg; bad.R = 256; bad.T_max = 1024;      /* two records per block */
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_OK && lay.NG == 1);
    bad = cfg; bad.B = 1 << 21;
    CHECK(mixkvq_block_layout(&bad, &lay) == MIXKVQ_EINVAL);
  }
  mixkvq_sizes sz;
  CHECK(mixkvq_cache_sizes(&cfg, &sz) == MIXKVQ_OK);
  CHECK(sz.blocks >= (uint64_t)6 * 4 * 9760 && sz.blocks % 256 == 0 && sz.res_k == sz.res_v && sz.workspace % 256 == 0);

  /* handle */
  mixkvq_buffers bufs = fake_buffers();
  mixkvq_cache* c = NULL;
  {
    mixkvq_buffers misaligned = bufs;
    misaligned.qacc = (void*)((uintptr_t)bufs.qacc + 8);
    CHECK(mixkvq_cache_create(&cfg, &misaligned, &c) == MIXKVQ_EINVAL && c == NULL);
    misaligned = bufs; misaligned.blocks = NULL;
    CHECK(mixkvq_cache_create(&cfg, &misaligned, &c) == MIXKVQ_EINVAL && c == NULL);
  }
  CHECK(mixkvq_cache_create(&cfg, &bufs, &c) == MIXKVQ_OK && c != NULL);
  int64_t nq = -1; int32_t nr = -1, ns = -1;
  CHECK(mixkvq_cache_state(c, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0 && ns == 0);
  CHECK(mixkvq_cache_state(c, NULL, NULL, NULL) == MIXKVQ_OK);
  CHECK(mixkvq_cache_state_seq(c, 3, &nq, &nr, &ns) == MIXKVQ_EINVAL && mixkvq_cache_state_seq(c, -1, &nq, &nr, &ns) == MIXKVQ_EINVAL);
  CHECK(mixkvq_decode_path(c) == MIXKVQ_PATH_NONE && mixkvq_decode_path(NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_set_timing_events(c, (void*)8, NULL) == MIXKVQ_EINVAL && mixkvq_set_timing_events(c, NULL, NULL) == MIXKVQ_OK);

  /* argument checks that come before any launch */
  const int64_t st3[3] = {2 * 600 * 128, 600 * 128, 128};
  const int64_t st_bad[3] = {2 * 600 * 128, 600 * 128, 132};
  void* kv = (void*)(uintptr_t)0x150000000000ull;
  void* q = (void*)(uintptr_t)0x160000000000ull;
  void* out = (void*)(uintptr_t)0x170000000000ull;
  CHECK(mixkvq_quantize_append(c, kv, kv, -1, st3, NULL, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_quantize_append(c, kv, kv, 0, st3, NULL, NULL) == MIXKVQ_OK);
  CHECK(mixkvq_quantize_append(c, NULL, kv, 5, st3, NULL, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_quantize_append(c, (char*)kv + 2, kv, 5, st3, NULL, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_quantize_append(c, kv, kv, 5, st_bad, NULL, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_quantize_append(c, kv, kv, 512 + 129, st3, NULL, NULL) == MIXKVQ_ECAPACITY);   /* 5 blocks > T_max / R = 4 */
  CHECK(mixkvq_decode_attention(c, q, out, NULL, 0.f, 0, NULL) == MIXKVQ_EEMPTY);
  CHECK(mixkvq_decode_attention_noalloc(c, q, out, NULL, 0.f, 0, NULL) == MIXKVQ_EEMPTY);
  CHECK(mixkvq_decode_attention(c, NULL, out, NULL, 0.f, 0, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_select_channels(c, NULL, 4, NULL, kv, 16, st3, (uint8_t*)out, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_select_channels(c, NULL, 0, NULL, kv, 0, st3, (uint8_t*)out, NULL) == MIXKVQ_EINVAL);
  CHECK(mixkvq_cache_state(c, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0 && ns == 0);
  CHECK(mixkvq_cache_set_block_table(c, (const int32_t*)out) == MIXKVQ_OK && mixkvq_cache_set_block_table(c, NULL) == MIXKVQ_OK);

  /* every code has a message */
  for (int code = 0; code >= -8; --code) CHECK(mixkvq_strerror(code) != NULL && strlen(mixkvq_strerror(code)) > 0);

  if (!have_gpu) {
    /* no device: a call that must enqueue a kernel fails in HIP; the host counts stay as they were */
    int rc = mixkvq_quantize_append(c, kv, kv, 300, st3, NULL, NULL);
    CHECK(rc == MIXKVQ_EHIP);
    CHECK(strstr(mixkvq_strerror(rc), "HIP error") != NULL);
    CHECK(mixkvq_cache_state(c, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0 && ns == 0);
    for (int b = 0; b < cfg.B; ++b)
      CHECK(mixkvq_cache_state_seq(c, b, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0 && ns == 0);
    const int64_t st2[2] = {600 * 128, 128};
    CHECK(mixkvq_quantize_append_seq(c, 1, kv, kv, 40, st2, NULL, NULL) == MIXKVQ_EHIP);
    CHECK(mixkvq_cache_state(c, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0);      /* still in lock-step, still empty */
    CHECK(mixkvq_decode_step(c, kv, kv, st3, q, out, NULL, 0.f, 1, NULL) == MIXKVQ_EHIP);
    CHECK(mixkvq_cache_state(c, &nq, &nr, &ns) == MIXKVQ_OK && nq == 0 && nr == 0);
    CHECK(mixkvq_cache_reset(c, NULL) == MIXKVQ_EHIP);
  }
  mixkvq_cache_destroy(c);
  mixkvq_cache_destroy(NULL);

  /* a batch too large for per-sequence calls */
  {
    mixkvq_config big = base_config();
    big.B = 300;
    mixkvq_cache* cb = NULL;
    CHECK(mixkvq_cache_create(&big, &bufs, &cb) == MIXKVQ_OK);
    const int64_t st2[2] = {600 * 128, 128};
    CHECK(mixkvq_quantize_append_seq(cb, 1, kv, kv, 40, st2, NULL, NULL) == MIXKVQ_EINVAL);
    CHECK(mixkvq_cache_reset_seq(cb, 1, NULL) == MIXKVQ_EINVAL);
    mixkvq_cache_destroy(cb);
  }
  printf("host shim driver: ok (%s)\n", have_gpu ? "GPU present: launch paths skipped" : "no GPU: launch failures checked");
  return 0;
}
