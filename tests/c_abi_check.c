/* A plain C client of include/lkv.h: proves that the header is C, that the library links from C, and
 * that the calls which need no GPU behave as the header says.  Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>

#include "lkv.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      fprintf(stderr, "line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                  \
    }                                                            \
  } while (0)

int main(void) {
  int32_t lens[2] = {1000, 37};
  lkv_cache cache;
  lkv_scorer scorer;
  size_t ws;

  CHECK(strstr(lkv_version(), "gfx950") != NULL);

  memset(&cache, 0, sizeof(cache));
  cache.n_seq = 2;
  cache.n_layers = 3;
  cache.n_kv_heads = 2;
  cache.n_q_heads = 8;
  cache.head_dim = 128;
  cache.seq_len = lens;

  /* host arithmetic only: the normaliser pairs of the window scorer, at least 8 bytes per key row and head */
  ws = lkv_score_window_workspace_bytes(&cache);
  CHECK(ws % 256 == 0);
  CHECK(ws >= (size_t)6 * (1000 + 37) * 8);
  CHECK(ws <= (size_t)6 * (1000 + 37 + 2 * 128) * 16 + 6 * 128 * 4 * 2 + 4 * 256);
  CHECK(lkv_score_window_workspace_bytes(NULL) == 0);
  CHECK(lkv_masked_decode_workspace_bytes(&cache) > 0);
  CHECK(lkv_decode_workspace_bytes(12, 300, 8, 2) % 256 == 0);
  CHECK(lkv_masked_attn_backward_workspace_bytes(8, 2, 100) > 0);
  CHECK(lkv_soft_topk_max_n(0) == 1 << 22);

  /* every call that takes a context refuses a null one before touching the GPU */
  memset(&scorer, 0, sizeof(scorer));
  CHECK(lkv_score(NULL, &cache, &scorer, NULL, NULL) == LKV_ERR_INVALID_ARG);
  CHECK(lkv_score_window(NULL, &cache, NULL, NULL, 32, 7, LKV_POOL_MAX, 0.1f, NULL, NULL, 0, NULL) == LKV_ERR_INVALID_ARG);
  CHECK(lkv_select(NULL, &cache, NULL, NULL, NULL, NULL, NULL) == LKV_ERR_INVALID_ARG);
  CHECK(lkv_soft_topk_backward(NULL, NULL, 0, 1, 1.0, NULL, NULL, NULL, NULL, NULL) == LKV_ERR_INVALID_ARG);
  CHECK(strcmp(lkv_last_error(NULL), "context is NULL") == 0);
  lkv_destroy(NULL);

  puts("c abi ok");
  return 0;
}
