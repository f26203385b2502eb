/*
 * heddle.h - C ABI of the trajectory-generation attention path on MI355X (gfx950).
 *
 * What it covers.  In agentic RL rollout an LLM agent produces multi-step
 * trajectories, alternating token generation with tool calls (paper Sec. 2.1);
 * a trajectory keeps its KV cache while it waits for a tool or is preempted
 * (Sec. 4.2, "Preemptive Execution"; Algorithm 1), the cache is paged (Sec. 9,
 * PagedAttention), and a worker runs a batch of trajectories whose lengths are
 * long-tailed (Sec. 1, Sec. 2.2).  The two GPU operations of that generation
 * step are exported here:
 *
 *   heddle_attn_decode   one new token for every live trajectory of the batch
 *   heddle_attn_append   a tool-output chunk appended onto the retained cache
 *                        (the "tool-output prefill" of Sec. 8)
 *
 * together with the block manager of the paged pool (heddle_kv_alloc/free) and
 * the host-side planners whose output the tests compare bit for bit.
 *
 * Attention is scaled dot-product attention with grouped query heads:
 *   out[j] = sum_t softmax_t(scale * q[j] . K[t][j / G]) * V[t][j / G],  G = n_q / n_kv.
 * bf16 inputs and outputs, fp32 accumulation.
 *
 * Memory layout (all device pointers are caller-owned; the library allocates
 * only its own context, a small pinned staging ring and grow-only scratch):
 *   kv_pool    bf16 [n_blocks][n_kv_heads][2][16 * head_dim]; per (block, kv head) a K tile,
 *              token-major [16][head_dim], followed by a V tile stored transposed,
 *              [head_dim][16] (the 16 tokens of one head-dim element are contiguous)
 *   block table in CSR form: token position p of trajectory b is stored in
 *              block  block_ids[row_off[b] + p / 16], slot p % 16
 *              (a row may be longer than its trajectory needs; entries behind the
 *              needed blocks are never read as addresses)
 *   q / out    bf16 [rows][n_q_heads][head_dim]
 *   k / v rows bf16 [rows][n_kv_heads][head_dim]
 * Slots past a trajectory's length and blocks outside every table may hold
 * anything (NaN included) and never influence a result.
 *
 * Conventions.  Every function returns HEDDLE_OK (0) or a negative code; no
 * exceptions, no abort, nothing printed.  Arguments are validated before any
 * device work is enqueued, so a failing call has no device side effect.
 * Calls that take a stream are asynchronous on it and do not synchronise it.
 * The library's scratch (plan image, split-K partials, pinned staging ring) is
 * sized by heddle_ctx_reserve; a call that needs more than is there - no
 * reservation was made, or the batch is larger than the reserved one -
 * synchronises the device once and reallocates, so a serving loop reserves for
 * its largest batch after creating the context and never meets that case.
 * Host arrays are consumed before the call returns.  Every attention call plans
 * its work on the host from the lengths it is given and uploads that plan, so a
 * call is not something to capture into a HIP graph and replay: a replay would
 * run the plan of the captured lengths.
 * A context is not thread-safe.  All its stream-taking calls (attention, pack,
 * unpack, copy) share its scratch and are therefore ordered: a call issued on
 * another stream than the call before it first makes its stream wait, on the
 * device, for the work this context has enqueued on the previous stream (one
 * event record and one stream wait; the host does not block).  Work that should
 * overlap - staging a preempted trajectory's cache on a side stream while decode
 * runs - uses a second context over the same pool.  A stream that a context has
 * been used on must stay alive until the context's next call has returned or the
 * context is destroyed.
 * Device pointers of queries, outputs, K/V rows, staging buffers and the pool must
 * be 16-byte aligned (else HEDDLE_E_INVAL).  Block ids in the needed part of a
 * device table are trusted: the library cannot see them; where it is also given
 * the host copy (heddle_attn_decode_shared, pack, unpack, copy) ids outside the
 * pool are HEDDLE_E_INVAL.
 */
#ifndef HEDDLE_H
#define HEDDLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HEDDLE_OK             0
#define HEDDLE_E_INVAL       (-1)  /* bad argument, bad block id, table too short, ... */
#define HEDDLE_E_NOMEM       (-2)  /* pool exhausted / caller array too small / malloc failed */
#define HEDDLE_E_HIP         (-3)  /* a HIP runtime call failed */
#define HEDDLE_E_UNSUPPORTED (-4)  /* shape outside what the kernels are built for */

#define HEDDLE_BLOCK_TOKENS  16
#define HEDDLE_MAX_CONTEXT   131072   /* tokens per trajectory */

typedef struct heddle_ctx heddle_ctx;

typedef struct heddle_config {
  int32_t n_q_heads;      /* multiple of n_kv_heads; query heads per kv head G = n_q/n_kv: with head_dim
                             128 any G from 1 to 32 (decode for G other than 1, 2, 4, 8 needs tile_blk
                             to be a multiple of 4); with head_dim 64 G in {1,2,4,8} (every call; chunks
                             of a few rows run in the kernel for long chunks there).
                             Else HEDDLE_E_UNSUPPORTED. */
  int32_t n_kv_heads;
  int32_t head_dim;       /* 64 or 128 */
  int32_t block_tokens;   /* must be 16 */
  int32_t n_blocks;       /* pool capacity in blocks (>= 1) */
  int32_t device;         /* HIP device ordinal; -1 = host-only context: block manager and
                             planners work, attention calls return HEDDLE_E_UNSUPPORTED */
  void*   kv_pool;        /* DEVICE, caller-owned, layout above; may be NULL iff device == -1 */
  /* split-K planner parameters; 0 selects the default in brackets */
  int32_t n_cu;           /* [compute units of the device; 256 if host-only] */
  int32_t wg_per_cu;      /* [4]  work items wanted per CU */
  int32_t min_chunk_blk;  /* [16] smallest split, in blocks */
  int32_t tile_blk;       /* [4]  splits start at multiples of this many blocks */
  int32_t max_split;      /* [64] most splits per trajectory */
  float   scale;          /* 0 selects 1/sqrt(head_dim) */
  /* shared-prefix planner parameters (heddle_plan_decode_shared); 0 selects the default */
  int32_t min_share_blk;    /* [4] fewest common leading blocks that make two trajectories a group */
  int32_t group_wg_per_cu;  /* [1] work items wanted per CU for the shared-prefix kernel */
  /* split-K of small append batches (heddle_plan_append_split); 0 selects the default */
  int32_t append_wg_per_cu; /* [2] workgroups of the append kernel that fit on a CU */
  int32_t append_min_steps; /* [4] smallest part, in 64-key steps */
} heddle_config;

/* Creates a context.  *out is written only on success.  With device >= 0 the
 * device is queried and a small pinned staging ring is allocated. */
int heddle_ctx_create(const heddle_config* cfg, heddle_ctx** out);
/* Synchronises the device if the context has enqueued work, frees everything it owns. */
int heddle_ctx_destroy(heddle_ctx* ctx);
/* Points the context at another pool of the same shape (n_blocks, n_kv_heads,
 * head_dim, layout above): DEVICE, caller-owned.  A model keeps one pool per
 * layer while block table, lengths and block manager are common to all layers
 * (a token has the same position in each), so one context serves them in turn.
 * Calls already enqueued keep the pool they were issued with.  NULL or a
 * host-only context -> INVAL. */
int heddle_ctx_set_kv_pool(heddle_ctx* ctx, void* kv_pool);
/* Sizes the context's scratch for batches of up to max_trajectories trajectories in a
 * decode step and, if max_chunk_rows > 0, appends of up to max_chunk_rows chunk rows in
 * total over at most max_trajectories trajectories; with_shared_prefix != 0 also covers
 * heddle_attn_decode_shared (a partial slot per member and prefix part: more memory).
 * The sizes are upper bounds derived from the plan rules, so no call within these limits
 * allocates or synchronises.  May synchronise the device itself (it replaces buffers that
 * enqueued work may still read): call it after creation or between steps, not inside one.
 * Never shrinks.  Errors: max_trajectories < 1, max_chunk_rows < 0 -> INVAL; host-only
 * context -> UNSUPPORTED; allocation failure -> NOMEM. */
int heddle_ctx_reserve(heddle_ctx* ctx, int32_t max_trajectories, int32_t max_chunk_rows, int32_t with_shared_prefix);

/* ---- block manager of the paged pool (host only, O(n), all-or-nothing) ----
 * A trajectory's blocks stay allocated across tool calls and preemption
 * (Sec. 4.2) and are returned when it finishes.  Stack discipline: a fresh
 * context hands out 0,1,2,...; free pushes ids in the order given; alloc pops,
 * most recently freed first.  A block may have several holders: the samples
 * of one prompt (Sec. 7, "Workloads") name the prompt's blocks in their tables
 * (what heddle_attn_decode_shared reads once per group).  alloc gives a block
 * one holder, retain adds one, free takes one away; the block goes back on
 * the stack when its last holder frees it, in the order of that free call.
 *   alloc:  n < 0 -> INVAL; fewer than n free -> NOMEM; nothing changes on error.
 *   retain: any id out of range, not allocated, or repeated in the call -> INVAL,
 *           nothing changes.
 *   free:   the same conditions -> INVAL, nothing changes. */
int heddle_kv_alloc(heddle_ctx* ctx, int32_t n, int32_t* out_block_ids /* HOST [n] */);
int heddle_kv_retain(heddle_ctx* ctx, int32_t n, const int32_t* block_ids /* HOST [n] */);
int heddle_kv_free(heddle_ctx* ctx, int32_t n, const int32_t* block_ids /* HOST [n] */);
int heddle_kv_num_free(const heddle_ctx* ctx, int32_t* out);

/* ---- split-K plan for decode (host only) ----------------------------------
 * Spreads the batch over the GPU: a long-tail trajectory (Sec. 2.2) is cut into
 * several work items so that no compute unit is left streaming one straggler
 * alone; items are ordered longest first (the LPT idea of Sec. 4.2).  Rule, all
 * integer: nblk = ceil(len/16); W = sum nblk; target = max(1, n_cu*wg_per_cu /
 * n_kv_heads); chunk = max(ceil(W/target), min_chunk_blk) rounded up to a
 * multiple of tile_blk; per trajectory ns = min(ceil(nblk/chunk), max_split),
 * per = ceil(nblk/ns) rounded up to tile_blk, nsplit = ceil(nblk/per); split k
 * covers blocks [k*per, min((k+1)*per, nblk)); partial slot = part_off[b] + k;
 * items sorted by (-(blk_end-blk_begin), b, k).
 * All arrays are HOST memory owned by the caller.  cap_items must be at least
 * the number of items (never more than B*max_split), else NOMEM. */
typedef struct heddle_plan {
  int32_t  cap_items;        /* in  */
  int32_t  n_items;          /* out */
  int32_t  chunk;            /* out, in blocks */
  int32_t* item_b;           /* out [n_items] trajectory of the item */
  int32_t* item_s;           /* out [n_items] split index within the trajectory */
  int32_t* item_blk_begin;   /* out [n_items] first logical block */
  int32_t* item_blk_end;     /* out [n_items] one past the last logical block */
  int32_t* nsplit;           /* out [B] */
  int32_t* part_off;         /* out [B+1] */
} heddle_plan;
int heddle_plan_decode(const heddle_ctx* ctx, int32_t B, const int32_t* len_host, heddle_plan* plan);

/* ---- work order of append (host only) --------------------------------------
 * One tile per (trajectory, tile_rows consecutive chunk rows); cost of a tile =
 * number of keys its last row sees = L_b + min(row0 + tile_rows, C_b); tiles are
 * sorted by (-extent, b, row0).  tile_rows <= 0 selects the kernel's own tile
 * height for this context.  Arrays are HOST, cap_tiles >= sum ceil(C_b/tile_rows). */
typedef struct heddle_append_plan {
  int32_t  cap_tiles;        /* in  */
  int32_t  n_tiles;          /* out */
  int32_t  tile_rows;        /* out: the tile height used */
  int32_t* tile_b;           /* out [n_tiles] */
  int32_t* tile_row0;        /* out [n_tiles] first chunk row of the tile */
  int32_t* tile_rows_n;      /* out [n_tiles] rows in the tile (< tile_rows only at a chunk's end) */
  int32_t* tile_extent;      /* out [n_tiles] */
} heddle_append_plan;
int heddle_plan_append(const heddle_ctx* ctx, int32_t B, const int32_t* ctx_len_host,
                       const int32_t* cu_chunk_host, int32_t tile_rows, heddle_append_plan* plan);

/* ---- split-K of a small append batch (host only) ------------------------------
 * A tile with many more keys than an even share of the batch (one long trajectory
 * with a short chunk; the long tail of a speculative-decoding verify step, a few
 * tokens per trajectory, Sec. 8) would keep one workgroup busy long after the rest;
 * its keys are cut into parts that run as separate work items and are merged per
 * row afterwards, as in decode.  Rule (integer), tiles as produced by
 * heddle_plan_append, index t in that order:
 *  1. S_t = ceil(extent_t / 64); slots = n_cu * append_wg_per_cu.
 *  2. W = sum S_t, target = max(1, slots / n_kv_heads), chunk = max(ceil(W /
 *     target), append_min_steps); per tile ns = min(ceil(S/chunk), max_split), per =
 *     ceil(S/ns), n = ceil(S/per); while n > 1 and (n-1)*per*64 > L_b + row0: n -= 1
 *     (the tile's first row must see a key of the last part: no row of a part is an
 *     empty softmax).  Part k < n-1 covers steps [k*per, (k+1)*per), the last part
 *     [(n-1)*per, S).
 *  3. a tile with n > 1 owns rows_n * n partial slots from part_base_t (assigned in
 *     tile order); row r, part k -> part_base_t + r*n + k.
 *  4. items (t, k) sorted by (-(step_end - step_begin), b_t, step_begin, row0_t): equally
 *     long parts of one trajectory's tiles over the same keys run side by side.
 * heddle_attn_append applies this rule itself; the function exposes it for checking. */
typedef struct heddle_append_split_plan {
  int32_t  cap_tiles, cap_items;            /* in  */
  int32_t  n_tiles, n_items, n_slots, tile_rows;   /* out */
  int32_t* tile_b; int32_t* tile_row0; int32_t* tile_rows_n; int32_t* tile_extent;   /* [n_tiles] */
  int32_t* tile_nsplit; int32_t* tile_part_base;                                     /* [n_tiles] */
  int32_t* item_tile; int32_t* item_k; int32_t* item_step_begin; int32_t* item_step_end;   /* [n_items] */
} heddle_append_split_plan;
int heddle_plan_append_split(const heddle_ctx* ctx, int32_t B, const int32_t* ctx_len_host,
                             const int32_t* cu_chunk_host, int32_t tile_rows, heddle_append_split_plan* plan);

/* ---- decode: one query token per trajectory ---------------------------------
 * len[b] counts the KV rows the query sees, the new token's own row included.
 * If k_new/v_new are given, row b is first stored at position len[b]-1 (the
 * table must cover it); otherwise the caller has stored it already.
 * Errors: B < 1, len < 1 or > HEDDLE_MAX_CONTEXT, a table row shorter than
 * ceil(len/16) blocks, NULL required pointer -> INVAL. */
typedef struct heddle_decode_args {
  int32_t        B;
  const int32_t* len_host;       /* HOST   [B] */
  const int32_t* row_off_host;   /* HOST   [B+1] CSR offsets (validation and planning) */
  const int32_t* row_off;        /* DEVICE [B+1] same values */
  const int32_t* block_ids;      /* DEVICE [row_off[B]] physical block of each logical block */
  const void*    q;              /* DEVICE bf16 [B][n_q][d] */
  const void*    k_new;          /* DEVICE bf16 [B][n_kv][d] or NULL */
  const void*    v_new;          /* DEVICE bf16 [B][n_kv][d] or NULL (both or neither) */
  void*          out;            /* DEVICE bf16 [B][n_q][d] */
  float*         lse;            /* DEVICE f32  [B][n_q] natural-log sum of exponentials, or NULL */
} heddle_decode_args;
int heddle_attn_decode(heddle_ctx* ctx, const heddle_decode_args* args, void* hip_stream);

/* ---- decode without allocation ----------------------------------------------
 * For callers that cannot allocate device memory while they run: code inside a HIP
 * graph capture, a serving loop that must not stall on the allocator, a harness that
 * forbids hipMalloc.  Same arguments, result and errors as heddle_attn_decode, same
 * kernels; the plan image and the split-K partials live in a static device array of
 * the library (64 KiB + 16 MiB, one copy per GPU that loads the library, held until
 * the process ends) instead of the context's grow-only scratch.  The call makes no
 * hipMalloc, hipFree, hipHostMalloc or other allocating HIP call and does not
 * synchronise for memory; the pinned staging ring it copies the plan from was sized
 * for it when the context was created.
 * Limits: plan image 8*n_items + 4*B + 1 <= 16384 words and partials
 * n_items * n_q_heads * (head_dim + 4) * 4 bytes <= 16 MiB (n_items as returned by
 * heddle_plan_decode; 992 items at 32 query heads of 128).  A larger call returns
 * HEDDLE_E_NOMEM before anything is enqueued, heddle_last_error_detail() says which
 * limit.  Nothing in the array has to start at zero (every partial that is read was
 * written by the same call).  All contexts of a GPU share its array: two such calls
 * that overlap in time on one GPU (different streams, or different contexts) race
 * and give wrong results; calls on one stream are ordered and safe. */
int heddle_attn_decode_static(heddle_ctx* ctx, const heddle_decode_args* args, void* hip_stream);

/* ---- decode with shared prefixes --------------------------------------------
 * The samples of one prompt (16 per prompt in the paper's rollouts, Sec. 7
 * "Workloads") start with the same tokens, and a prefix-cache hit (Sec. 2.3,
 * cache-affinity placement) lets their block-table rows name the same physical
 * blocks for that prefix.  This variant of the decode step reads such a prefix
 * once per group instead of once per trajectory; the result is the same
 * attention, defined by each trajectory's own table row.
 * Plan rule (integer; extends the rule of heddle_plan_decode):
 *  1. nblk[b] = ceil(len[b]/16); shareable[b] = (len[b]-1)/16, the blocks wholly
 *     before the step's own row (the block that row is written to is never shared).
 *  2. Walking b upwards, the first trajectory with shareable >= 1 whose first block
 *     id is new leads that id; a later trajectory with the same first id joins the
 *     leader's group iff lcp >= min_share_blk, lcp = number of leading table entries
 *     equal to the leader's, capped by both shareable counts and, in a context whose
 *     decode steps run on the matrix-core kernel (see below), rounded down to a
 *     multiple of 4.  A group exists iff
 *     someone joined; prefix p_g = min lcp of the joined; members ascending;
 *     groups numbered by ascending leader.
 *  3. chunk from W = sum_b (nblk[b] - prefix[b]) as in heddle_plan_decode; chunk_g
 *     likewise from Wg = sum_g p_g * ceil(members_g / tile_members) with target_g =
 *     max(1, n_cu * group_wg_per_cu / n_kv_heads); tile_members = 128 / G.
 *  4. cut(n, c): ns = min(ceil(n/c), max_split); per = ceil(n/ns) rounded up to
 *     tile_blk; count = ceil(n/per).
 *  5. group g: cut(p_g, chunk_g) -> parts k over leader blocks [k*per, min((k+1)*per,
 *     p_g)), each crossed with member tiles of tile_members consecutive members
 *     (group items, sorted by (-(blk_end-blk_begin), g, k, tile)).
 *  6. trajectory b: cut(nblk[b]-prefix[b], chunk) -> parts over [prefix[b] + k*per, ...)
 *     with slot = parts_g + k; nsplit[b] = parts_g + count; items sorted as before.
 * All arrays HOST, caller-owned; capacities too small -> NOMEM.  On a shape the
 * matrix-core kernel is not built for (head_dim other than 64 and 128) no groups are formed. */
typedef struct heddle_shared_plan {
  int32_t  cap_items, cap_gitems, cap_groups;          /* in  */
  int32_t  n_items, n_gitems, n_groups, chunk, chunk_g; /* out */
  int32_t* item_b;  int32_t* item_s;  int32_t* item_blk_begin;  int32_t* item_blk_end;   /* [n_items]  */
  int32_t* gitem_g; int32_t* gitem_k; int32_t* gitem_blk_begin; int32_t* gitem_blk_end;  /* [n_gitems] */
  int32_t* gitem_m0; int32_t* gitem_mn;   /* [n_gitems] members[member_off[g] + m0 .. + mn) */
  int32_t* group_leader; int32_t* group_prefix; int32_t* group_parts;   /* [n_groups] */
  int32_t* member_off;       /* [n_groups + 1] */
  int32_t* members;          /* [B] (member_off[n_groups] used) */
  int32_t* traj_group;       /* [B] group of the trajectory or -1 */
  int32_t* traj_prefix;      /* [B] shared blocks of the trajectory (0 outside groups) */
  int32_t* nsplit;           /* [B] */
  int32_t* part_off;         /* [B+1] */
} heddle_shared_plan;
int heddle_plan_decode_shared(const heddle_ctx* ctx, int32_t B, const int32_t* len_host,
                              const int32_t* row_off_host, const int32_t* block_ids_host,
                              heddle_shared_plan* plan);

/* Kernel routing of both decode entry points (stated here because it shows in the plan):
 * with head_dim 128 and tile_blk a multiple of 4, contexts with 8 query heads per kv head,
 * or with a number of them other than 1, 2, 4, 8, read the blocks of a decode step with
 * the matrix-core kernel for short-row tiles, which starts at multiples of 64 keys; all
 * other contexts use the packed-dot split-K kernel.
 *
 * Same arguments, results and errors as heddle_attn_decode, plus the HOST copy of
 * the block table (block_ids_host [row_off_host[B]], read before the call returns)
 * from which the groups are found.  Two trajectories may name the same physical
 * block only in positions wholly below both lengths. */
int heddle_attn_decode_shared(heddle_ctx* ctx, const heddle_decode_args* args, const int32_t* block_ids_host,
                              void* hip_stream);

/* ---- append: a chunk of C_b >= 1 new tokens per trajectory ------------------
 * The chunk's K/V rows are stored at positions L_b .. L_b+C_b-1 (the table must
 * already cover L_b + C_b tokens), then chunk row i attends to positions
 * 0 .. L_b+i: the whole retained context plus the chunk causally, itself
 * included.  L_b = 0 is legal (first prompt).  With k and v both NULL the caller
 * has stored the chunk's rows already (as with k_new / v_new of decode) and the
 * call only attends.
 * Errors: B < 1, C_b < 1, L_b < 0, L_b + C_b > HEDDLE_MAX_CONTEXT, table too
 * short, a required pointer NULL, only one of k and v given -> INVAL. */
typedef struct heddle_append_args {
  int32_t        B;
  const int32_t* ctx_len_host;   /* HOST   [B] L_b */
  const int32_t* cu_chunk_host;  /* HOST   [B+1] prefix sums of C_b, cu[0] = 0 */
  const int32_t* row_off_host;   /* HOST   [B+1] */
  const int32_t* row_off;        /* DEVICE [B+1] */
  const int32_t* block_ids;      /* DEVICE [row_off[B]] */
  const void*    q;              /* DEVICE bf16 [sum C][n_q][d] */
  const void*    k;              /* DEVICE bf16 [sum C][n_kv][d] or NULL */
  const void*    v;              /* DEVICE bf16 [sum C][n_kv][d] or NULL (both or neither) */
  void*          out;            /* DEVICE bf16 [sum C][n_q][d] */
  float*         lse;            /* DEVICE f32  [sum C][n_q] or NULL */
} heddle_append_args;
int heddle_attn_append(heddle_ctx* ctx, const heddle_append_args* args, void* hip_stream);

/* ---- pack / unpack: a trajectory's cache as one contiguous buffer -----------
 * Staging form of a cache that leaves the pool or enters it: a preempted
 * trajectory keeps its cache for its next step (Sec. 4.2), a trajectory that is
 * reassigned moves its cache to the worker that takes it (Sec. 5.3).  pack
 * copies the n pool blocks block_ids[0..n), in that order, into staging
 * (DEVICE, n * block_bytes, block_bytes = n_kv_heads * 2 * 16 * head_dim * 2);
 * unpack copies staging block i into pool block block_ids[i] (ids distinct).
 * Whole blocks move bit for bit, the slots past the trajectory's length
 * included.  block_ids is a HOST array, read before the call returns.
 * Errors: an id outside [0, n_blocks), a repeated id in unpack, n < 0 or a NULL
 * pointer with n > 0 -> INVAL; a context without a device -> UNSUPPORTED. */
int heddle_kv_pack(heddle_ctx* ctx, int32_t n, const int32_t* block_ids_host, void* staging, void* hip_stream);
int heddle_kv_unpack(heddle_ctx* ctx, int32_t n, const int32_t* block_ids_host, const void* staging,
                     void* hip_stream);

/* Copies whole blocks inside the pool, bit for bit: block dst[i] becomes a copy of
 * block src[i].  For a sample that continues a shared prompt (16 samples per prompt,
 * Sec. 7 "Workloads"): it names the prompt's whole blocks in its own table
 * (heddle_kv_retain) and takes a copy of the partly filled last block, which it will
 * write to.  Both lists are HOST arrays, read before the call returns; the copy is
 * enqueued on the stream.
 * Errors: an id outside [0, n_blocks), a destination named twice or also named as a
 * source, n < 0 or a NULL list with n > 0 -> INVAL; no device -> UNSUPPORTED. */
int heddle_kv_copy(heddle_ctx* ctx, int32_t n, const int32_t* src_block_ids_host, const int32_t* dst_block_ids_host,
                   void* hip_stream);

/* ---- trajectory placement (host only, no context) -----------------------------
 * Presorted dynamic programming of Sec. 5.2: n trajectories in DESCENDING length
 * order are split into at most m contiguous runs, one per worker, minimising
 *   max over workers of  (L_first * T) * F[size]          (Eq. 2 under Lemma 1)
 * with dp[i][1] = L_1 T F(i), dp[i][j] = min_k max(dp[k][j-1], L_{k+1} T F(i-k))   (Eq. 3).
 * F is a table over group sizes 0 .. F_len-1 and must reach the total member count.
 * count (or NULL = all ones) gives members per element, for bundled short
 * trajectories; a group's size is the sum of its elements' counts.  min(n, m) workers
 * get a non-empty run, the rest size 0; among equal optima the smallest split index k
 * wins at every step.  sizes_out [m] = elements per worker, longest trajectories first.
 * mode 0: when F is non-decreasing the minimum over k is found at the crossing of
 * the two monotone terms (O(n m log n)), else by the full scan; mode 1: always the
 * full scan of Eq. 3 (O(n^2 m)).  Both give the same result bit for bit.
 * Errors: lengths not descending, count < 1, F too short, m < 1, NULL -> INVAL. */
int heddle_placement_dp(int32_t n, const double* len_desc, const int32_t* count, int32_t m, const double* F,
                        int32_t F_len, double T, int32_t mode, int32_t* sizes_out, double* makespan_out);

/* Bundles the short tail of the sorted list (Sec. 5.2: trajectories under a threshold
 * are merged after the sort to shrink n): an element is one trajectory of length >=
 * threshold, or up to `bundle` consecutive shorter ones.  first_out / count_out [n]. */
int heddle_placement_aggregate(int32_t n, const double* len_desc, double threshold, int32_t bundle,
                               int32_t* first_out, int32_t* count_out, int32_t* n_elems_out);

/* Interference factor from a profile (Sec. 5.2, "Interference Factor"): step_time[i] is
 * the time of one decode step at batch size batch_sizes[i] (strictly increasing).
 * t(s) interpolates linearly (flat below the first point, last slope continued);
 * F_out[s] = t(s) / t(1) for s = 1..n under a running maximum, F_out[0] = 0. */
int heddle_interference_table(int32_t n_prof, const double* batch_sizes, const double* step_time, int32_t n,
                              double* F_out /* [n+1] */);

/* Simulator of one worker's group: all trajectories decode concurrently, a step with
 * a of them active takes t(a), a trajectory of length L leaves after L steps.
 * *time_out = total time in the profile's unit. */
int heddle_simulate_group(int32_t n, const int32_t* lengths, int32_t n_prof, const double* batch_sizes,
                          const double* step_time, double* time_out);

const char* heddle_strerror(int code);
/* Text of the HIP call that made the calling thread's last HEDDLE_E_HIP, or of the limit that its
 * last heddle_attn_decode_static call exceeded (empty if neither happened yet). */
const char* heddle_last_error_detail(void);
int heddle_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HEDDLE_H */
