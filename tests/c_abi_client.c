/* A client of the C ABI written in plain C (C99, no Python, no C++): shows that heddle.h is a C
 * header and that the library links and runs from C.  Host-only context: block manager and
 * split-K planner.  The expected plan is the first hand-worked example of
 * tests/golden/plan_worked_examples.json (derivation there); the block ids follow from the stack
 * rule stated in heddle.h.  Prints "ok" and exits 0, or names the first check that failed. */
#include <stdio.h>
#include <string.h>

#include "heddle.h"

#define CHECK(cond)                                            \
  do {                                                         \
    if (!(cond)) {                                             \
      printf("failed at line %d: %s\n", __LINE__, #cond);      \
      return 1;                                                \
    }                                                          \
  } while (0)

static int same(const int32_t* a, const int32_t* b, int n) { return memcmp(a, b, sizeof(int32_t) * (size_t)n) == 0; }

int main(void) {
  heddle_config cfg;
  heddle_ctx* ctx = NULL;
  memset(&cfg, 0, sizeof(cfg));
  cfg.n_q_heads = 8;
  cfg.n_kv_heads = 2;
  cfg.head_dim = 128;
  cfg.block_tokens = HEDDLE_BLOCK_TOKENS;
  cfg.n_blocks = 6;
  cfg.device = -1;
  cfg.n_cu = 4;
  cfg.wg_per_cu = 2;
  cfg.min_chunk_blk = 2;
  cfg.tile_blk = 2;
  cfg.max_split = 3;
  CHECK(heddle_version() >= 1);
  CHECK(heddle_ctx_create(&cfg, &ctx) == HEDDLE_OK && ctx != NULL);

  /* block manager: a fresh pool hands out 0, 1, 2, ...; the block freed last comes back first;
     a block with two holders survives the first free */
  {
    int32_t ids[6], free_now = -1;
    const int32_t first[4] = {0, 1, 2, 3};
    const int32_t give_back[2] = {1, 3};
    const int32_t again[3] = {3, 1, 4};
    const int32_t shared[1] = {0};
    CHECK(heddle_kv_alloc(ctx, 4, ids) == HEDDLE_OK && same(ids, first, 4));
    CHECK(heddle_kv_alloc(ctx, 3, ids) == HEDDLE_E_NOMEM);
    CHECK(heddle_kv_free(ctx, 2, give_back) == HEDDLE_OK);
    CHECK(heddle_kv_free(ctx, 2, give_back) == HEDDLE_E_INVAL);
    CHECK(heddle_kv_alloc(ctx, 3, ids) == HEDDLE_OK && same(ids, again, 3));
    CHECK(heddle_kv_retain(ctx, 1, shared) == HEDDLE_OK);
    CHECK(heddle_kv_free(ctx, 1, shared) == HEDDLE_OK);
    CHECK(heddle_kv_num_free(ctx, &free_now) == HEDDLE_OK && free_now == 1);
    CHECK(heddle_kv_free(ctx, 1, shared) == HEDDLE_OK);
    CHECK(heddle_kv_num_free(ctx, &free_now) == HEDDLE_OK && free_now == 2);
    CHECK(heddle_kv_alloc(ctx, 1, ids) == HEDDLE_OK && ids[0] == 0);
  }

  /* split-K plan of the hand-worked example */
  {
    const int32_t lens[5] = {100, 1000, 16, 5000, 1};
    const int32_t want_nsplit[5] = {1, 1, 1, 3, 1};
    const int32_t want_part_off[6] = {0, 1, 2, 3, 6, 7};
    const int32_t want_b[7] = {3, 3, 3, 1, 0, 2, 4};
    const int32_t want_s[7] = {0, 1, 2, 0, 0, 0, 0};
    const int32_t want_begin[7] = {0, 106, 212, 0, 0, 0, 0};
    const int32_t want_end[7] = {106, 212, 313, 63, 7, 1, 1};
    int32_t b[15], s[15], begin[15], end[15], nsplit[5], part_off[6];
    heddle_plan plan;
    memset(&plan, 0, sizeof(plan));
    plan.cap_items = 15;
    plan.item_b = b;
    plan.item_s = s;
    plan.item_blk_begin = begin;
    plan.item_blk_end = end;
    plan.nsplit = nsplit;
    plan.part_off = part_off;
    CHECK(heddle_plan_decode(ctx, 5, lens, &plan) == HEDDLE_OK);
    CHECK(plan.n_items == 7 && plan.chunk == 98);
    CHECK(same(nsplit, want_nsplit, 5) && same(part_off, want_part_off, 6));
    CHECK(same(b, want_b, 7) && same(s, want_s, 7) && same(begin, want_begin, 7) && same(end, want_end, 7));
    plan.cap_items = 6;
    CHECK(heddle_plan_decode(ctx, 5, lens, &plan) == HEDDLE_E_NOMEM);
  }

  /* no device behind this context: attention calls say so instead of touching a GPU */
  {
    heddle_decode_args args;
    memset(&args, 0, sizeof(args));
    CHECK(heddle_attn_decode(ctx, &args, NULL) == HEDDLE_E_UNSUPPORTED);
    CHECK(heddle_ctx_set_kv_pool(ctx, &args) == HEDDLE_E_INVAL);
    CHECK(strcmp(heddle_strerror(HEDDLE_OK), "ok") == 0);
  }
  CHECK(heddle_ctx_destroy(ctx) == HEDDLE_OK);
  printf("ok\n");
  return 0;
}
