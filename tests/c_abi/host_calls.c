/* A plain C99 caller of libindexmem: the header compiles as C, the library links from C, and the
 * host-only calls behave as the header says (no GPU is touched: every call here returns before
 * anything is enqueued). */
#include <stdio.h>
#include <string.h>

#include "indexmem.h"

#define CHECK(cond)                                            \
  do {                                                         \
    if (!(cond)) {                                             \
      printf("FAILED line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                \
    }                                                          \
  } while (0)

int main(void) {
  im_config c;
  memset(&c, 0, sizeof c);
  c.batch = 2; c.n_q_heads = 32; c.n_kv_heads = 8; c.head_dim = 128; c.capacity = 512;
  c.n_idx_heads = 8; c.idx_dim = 64; c.mem_dim = 128; c.gate_in_dim = 32 * 128; c.n_sink = 4;
  c.n_recent = 0; c.fold_block = 64; c.max_queries = 16; c.head_shared = 0;
  c.rms_eps = 1e-6f; c.mem_eps = 1e-6f; c.softmax_scale = 0.08838834764f;

  const size_t ws = im_workspace_bytes(&c);
  CHECK(ws > 0 && ws % 256 == 0);
  CHECK(im_workspace_bytes(NULL) == 0);

  im_handle* h = NULL;
  /* a fake, aligned workspace address: im_create is host-only and never dereferences it */
  CHECK(im_create(&c, (void*)(size_t)(1u << 20), ws, &h) == IM_OK && h != NULL);
  im_handle* h2 = NULL;
  CHECK(im_create(&c, (void*)(size_t)(1u << 20), ws - 256, &h2) != IM_OK);   /* workspace too small */

  /* NULL arguments are turned into errors with a text, before any launch */
  CHECK(im_index_score(h, NULL, NULL, NULL, NULL, NULL, 1, NULL, NULL) == IM_ERR_INVALID_ARG);
  CHECK(strlen(im_last_error(h)) > 0);
  CHECK(im_set_max_live(h, 0) == IM_ERR_INVALID_ARG);
  CHECK(im_set_max_live(h, 513) == IM_ERR_INVALID_ARG);
  CHECK(im_set_max_live(h, 300) == IM_OK);

  /* the allocation-free entry point validates on the host too, and says what the limit is */
  c.batch = 64; c.capacity = 1 << 20;
  CHECK(im_decode_attn_with_readout_static(&c, 1 << 20, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == IM_ERR_INVALID_ARG);

  im_destroy(h);
  printf("ok %lu\n", (unsigned long)ws);
  return 0;
}
