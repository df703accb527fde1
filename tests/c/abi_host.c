/* A plain C caller of the library's host-side entry points (no GPU needed): version, status
 * strings, workspace queries and the argument checks that precede any launch. */
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
  dq_format bad = {3, 128, 128, 16, 8, 128, 1, 0, 1};
  dq_cache cache;
  char fake[64];
  memset(&cache, 0, sizeof cache);
  CHECK(dq_version() == 6);
  CHECK(strcmp(dq_status_string(DQ_OK), "ok") == 0);
  CHECK(dq_decode_workspace_bytes(&fmt, 8, 32, 32, 4096) > 0);
  CHECK(dq_decode_workspace_bytes(&bad, 8, 32, 32, 4096) == 0);
  CHECK(dq_compress_workspace_bytes(&fmt, 4, 40) == 256u + 4u * 40u * 2u * 128u * 128u * 4u + 1280u);
  CHECK(dq_decode_mfma_supported(&fmt, 32, 8) == 1);
  /* null pointers inside the cache struct are rejected before anything is launched */
  cache.batch = 1; cache.kv_heads = 1; cache.block_capacity = 1;
  CHECK(dq_attn_decode(&fmt, &cache, (const uint16_t*)fake, 1, (const int32_t*)fake, 128, 0.0f,
                       (uint16_t*)fake, NULL, fake, 1u << 20, DQ_DECODE_AUTO, NULL) == DQ_EINVAL);
  CHECK(dq_compress_kv_ex(&fmt, &cache, (const uint16_t*)fake, (const uint16_t*)fake, 128, (const int32_t*)fake,
                          NULL, fake, 1u << 20, DQ_COMPRESS_NO_LARGE, NULL) == DQ_EINVAL);
  /* launch-shape overrides travel in the flags word; an unknown bit is rejected */
  CHECK(dq_attn_decode(&fmt, &cache, (const uint16_t*)fake, 1, (const int32_t*)fake, 128, 0.0f, (uint16_t*)fake, NULL,
                       fake, 1u << 20, DQ_DECODE_SPLITS(65), NULL) == DQ_EINVAL);
  CHECK((DQ_DECODE_SPLITS(5) | DQ_DECODE_WAVES(8) | DQ_DECODE_UNIT_MAP(3)) == ((5u << 8) | (8u << 16) | (4u << 20)));
  /* the entry point without a workspace refuses more than 512 (sequence, query head) pairs */
  cache.batch = 513;
  CHECK(dq_attn_decode_static(&fmt, &cache, (const uint16_t*)fake, 1, (const int32_t*)fake, 128, NULL, 0.0f,
                              (uint16_t*)fake, NULL, DQ_DECODE_AUTO, NULL) == DQ_ELIMIT);
  printf("abi ok\n");
  return 0;
}
