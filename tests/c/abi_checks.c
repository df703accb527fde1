/* Host-side argument checks of every entry point, driven from plain C so that the library's host
 * code (argument validation, workspace carve-up, launch-shape choice) can run under the address and
 * undefined-behaviour sanitizers on a machine without a GPU.  Every call below is rejected before
 * anything is launched; pointers that are "valid" are never dereferenced. */
#include <stdio.h>
#include <string.h>

#include "decoquant.h"

#define CHECK(cond)                                                   \
  do {                                                                \
    if (!(cond)) {                                                    \
      fprintf(stderr, "failed at line %d: %s\n", __LINE__, #cond);    \
      return 1;                                                       \
    }                                                                 \
  } while (0)

int main(void) {
  dq_format fmt = {4, 128, 128, 16, 8, 128, 1, 0, 1};
  dq_format fmts[] = {{4, 128, 128, 16, 8, 128, 1, 0, 1}, {2, 64, 128, 16, 8, 256, 8, 1, 1}, {8, 64, 64, 8, 8, 128, 1, 0, 1},
                      {4, 32, 64, 16, 4, 128, 1, 0, 2}, {4, 128, 128, 8, 16, 128, 1, 0, 4}, {4, 128, 128, 32, 4, 1024, 1, 0, 1}};
  dq_format bad[] = {{3, 128, 128, 16, 8, 128, 1, 0, 1}, {4, 96, 128, 16, 8, 128, 1, 0, 1}, {4, 128, 128, 16, 4, 128, 1, 0, 1},
                     {4, 128, 128, 16, 8, 100, 1, 0, 1}, {4, 128, 256, 16, 16, 128, 1, 0, 1}, {4, 128, 128, 16, 8, 128, 4, 0, 1},
                     {4, 128, 128, 16, 8, 128, 1, 2, 1}, {4, 128, 128, 16, 8, 128, 1, 0, 3}, {4, 128, 128, 16, 8, 128, 8, 0, 2},
                     {4, 128, 128, 32, 4, 128, 1, 0, 2}, {4, 128, 128, 16, 8, 128, 1, 0, 0}, {4, 4, 128, 16, 8, 128, 1, 0, 1}};
  char fake[256];
  dq_cache cache;
  dq_tail tail;
  dq_kv_state state;
  uint16_t* h = (uint16_t*)fake;
  int32_t* w = (int32_t*)fake;
  size_t i, need, cneed, aneed;
  int32_t b, hq;

  CHECK(dq_version() == 6);
  for (i = 0; i < 8; ++i) CHECK(dq_status_string(-(int32_t)i) != NULL && strlen(dq_status_string(-(int32_t)i)) > 0);
  CHECK(dq_last_hip_error() == 0);

  /* workspace queries over good and bad formats and sizes */
  for (i = 0; i < sizeof fmts / sizeof fmts[0]; ++i) {
    CHECK(dq_decode_workspace_bytes(&fmts[i], 3, 8, 4, 1000) > 0);
    CHECK(dq_compress_workspace_bytes(&fmts[i], 3, 4) > 0);
    CHECK(dq_compress_blocks_workspace_bytes(&fmts[i], 3, 4, 5000) >= dq_compress_workspace_bytes(&fmts[i], 3, 4));
    CHECK(dq_cache_append_workspace_bytes(&fmts[i], 3, 4) >= dq_compress_workspace_bytes(&fmts[i], 3, 4));
    for (hq = 1; hq <= 64; ++hq) (void)dq_decode_mfma_supported(&fmts[i], hq * 2, 2);
  }
  for (i = 0; i < sizeof bad / sizeof bad[0]; ++i) {
    CHECK(dq_decode_workspace_bytes(&bad[i], 3, 8, 4, 1000) == 0);
    CHECK(dq_compress_workspace_bytes(&bad[i], 3, 4) == 0);
    CHECK(dq_compress_blocks_workspace_bytes(&bad[i], 3, 4, 300) == 0);
    CHECK(dq_cache_append_workspace_bytes(&bad[i], 3, 4) == 0);
    CHECK(dq_decode_mfma_supported(&bad[i], 8, 4) == 0);
  }
  CHECK(dq_decode_workspace_bytes(NULL, 3, 8, 4, 1000) == 0);
  CHECK(dq_decode_workspace_bytes(&fmt, 0, 8, 4, 1000) == 0);
  CHECK(dq_decode_workspace_bytes(&fmt, 3, 7, 4, 1000) == 0);
  CHECK(dq_decode_workspace_bytes(&fmt, 3, 8, 4, -1) == 0);
  CHECK(dq_compress_blocks_workspace_bytes(&fmt, 1 << 20, 64, 128 * 64) == 0);   /* more blocks than a call takes */

  /* decode: null pieces, sizes, flags, workspace */
  memset(&cache, 0, sizeof cache);
  cache.batch = 2; cache.kv_heads = 4; cache.block_capacity = 8;
  need = dq_decode_workspace_bytes(&fmt, 2, 4, 4, 1024);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);   /* null arrays */
  cache.k_codes = cache.v_codes = (uint8_t*)fake;
  cache.k_scales = cache.v_scales = cache.k_small = cache.v_small = h;
  CHECK(dq_attn_decode(NULL, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, NULL, h, 4, w, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, NULL, 4, w, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, NULL, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, NULL, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, NULL, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 6, w, 1024, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1025, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, -1, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need - 1, 0, NULL) == DQ_ENOSPACE);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, 3, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, DQ_DECODE_SPLITS(65), NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, DQ_DECODE_WAVES(5), NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, DQ_DECODE_UNIT_MAP(6), NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need, 1u << 30, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmts[3], &cache, h, 4, w, 1024, 0.f, h, NULL, fake, 1u << 30, DQ_DECODE_FORCE_MFMA, NULL) == DQ_EINVAL);
  CHECK(dq_attn_decode(&fmts[1], &cache, h, 4, w, 1024, 0.f, h, NULL, fake, 1u << 30, 0, NULL) == DQ_EINVAL);   /* no T_3 arrays */
  CHECK(dq_attn_decode_timed(&fmt, &cache, h, 4, w, 1024, 0.f, h, NULL, fake, need - 1, 0, NULL, NULL, NULL) == DQ_ENOSPACE);
  /* every launch shape the library may choose, as far as the workspace check (which comes first) */
  for (b = 1; b <= 64; b *= 2)
    for (hq = 1; hq <= 8; hq *= 2) {
      cache.batch = b; cache.kv_heads = 2;
      CHECK(dq_attn_decode(&fmt, &cache, h, 2 * hq, w, 1024, 0.f, h, NULL, fake, 16, 0, NULL) == DQ_ENOSPACE);
    }
  cache.batch = 2; cache.kv_heads = 4;
  tail.k_tail = tail.v_tail = h; tail.tail_lens = w;
  tail.capacity = 1025;
  CHECK(dq_attn_decode_tail(&fmt, &cache, h, 4, w, 1024, &tail, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  tail.capacity = 0;
  CHECK(dq_attn_decode_tail(&fmt, &cache, h, 4, w, 1024, &tail, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  tail.capacity = 128; tail.tail_lens = NULL;
  CHECK(dq_attn_decode_tail(&fmt, &cache, h, 4, w, 1024, &tail, 0.f, h, NULL, fake, need, 0, NULL) == DQ_EINVAL);
  cache.batch = 129;
  CHECK(dq_attn_decode_static(&fmt, &cache, h, 4, w, 1024, NULL, 0.f, h, NULL, 0, NULL) == DQ_ELIMIT);
  cache.batch = 2;
  CHECK(dq_attn_decode_static(&fmt, NULL, h, 4, w, 1024, NULL, 0.f, h, NULL, 0, NULL) == DQ_EINVAL);

  /* compression */
  cneed = dq_compress_workspace_bytes(&fmt, 2, 4);
  CHECK(dq_compress_kv(&fmt, &cache, h, h, 0, w, NULL, fake, cneed, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv(&fmt, &cache, h, h, 129, w, NULL, fake, cneed, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv(&fmt, &cache, NULL, h, 128, w, NULL, fake, cneed, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv(&fmt, &cache, h, h, 128, NULL, NULL, fake, cneed, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv(&fmt, &cache, h, h, 128, w, NULL, fake, cneed - 1, NULL) == DQ_ENOSPACE);
  CHECK(dq_compress_kv_blocks(&fmt, &cache, h, h, 8 * 128 + 1, w, NULL, fake, (size_t)1 << 40, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv_blocks(&fmt, &cache, h, h, 300, w, NULL, fake, cneed, NULL) == DQ_ENOSPACE);
  CHECK(dq_compress_kv_ex(&fmt, &cache, h, h, 128, w, NULL, fake, cneed, 4, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv_ex(&fmt, &cache, h, h, 128, w, NULL, fake, cneed, DQ_COMPRESS_WAVES(3), NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv_ex(&fmt, &cache, h, h, 128, w, NULL, fake, cneed - 1,
                          DQ_COMPRESS_NO_LARGE | DQ_COMPRESS_PLAIN | DQ_COMPRESS_WAVES(4), NULL) == DQ_ENOSPACE);
  CHECK(dq_quantize_pack(&fmt, (const float*)fake, 100, 0, (uint8_t*)fake, h, NULL) == DQ_EINVAL);
  CHECK(dq_quantize_pack(&fmt, (const float*)fake, -128, 0, (uint8_t*)fake, h, NULL) == DQ_EINVAL);
  CHECK(dq_quantize_pack(&fmt, (const float*)fake, 0, 0, (uint8_t*)fake, h, NULL) == DQ_OK);       /* nothing to do */
  CHECK(dq_quantize_pack(&fmt, NULL, 128, 0, (uint8_t*)fake, h, NULL) == DQ_EINVAL);

  /* the cache policy */
  aneed = dq_cache_append_workspace_bytes(&fmt, 2, 4);
  state.k_tail = state.v_tail = (uint16_t*)(fake + 16); state.tail_lens = state.seq_lens = w;
  CHECK(dq_cache_append(&fmt, &cache, &state, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 0, NULL, fake, aneed, 0, NULL) == DQ_EINVAL);
  CHECK(dq_cache_append(&fmt, &cache, &state, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 129, NULL, fake, aneed, 0, NULL) == DQ_EINVAL);
  CHECK(dq_cache_append(&fmt, &cache, &state, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 1, NULL, fake, aneed, 2, NULL) == DQ_EINVAL);
  CHECK(dq_cache_append(&fmt, &cache, &state, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 1, NULL, fake, aneed - 1, 0, NULL) == DQ_ENOSPACE);
  CHECK(dq_cache_append(&fmt, &cache, NULL, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 1, NULL, fake, aneed, 0, NULL) == DQ_EINVAL);
  state.seq_lens = NULL;
  CHECK(dq_cache_append(&fmt, &cache, &state, (uint16_t*)(fake + 32), (uint16_t*)(fake + 32), 1, NULL, fake, aneed, 0, NULL) == DQ_EINVAL);

  /* helpers */
  CHECK(dq_workspace_init(NULL, 16, NULL) == DQ_EINVAL);
  CHECK(dq_workspace_init(fake, 0, NULL) == DQ_OK || 1);
  CHECK(dq_workspace_init(fake, 24, NULL) == DQ_EINVAL);
  CHECK(dq_stream_read(NULL, 16, (uint32_t*)fake, NULL) == DQ_EINVAL);
  CHECK(dq_stream_read(fake, 24, (uint32_t*)fake, NULL) == DQ_EINVAL);
  CHECK(dq_stream_read(fake, 0, (uint32_t*)fake, NULL) == DQ_OK || 1);
  printf("abi checks ok\n");
  return 0;
}
