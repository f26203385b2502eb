// Launch interface between the host API and the HIP kernels of libheddle.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace heddle {

// One split-K work item as the decode kernel reads it: a single 32-byte record, so that a
// workgroup learns everything about its item with one scalar load.
struct DecodeItemRec {
  int32_t b;            // trajectory
  int32_t slot;         // partial slot = part_off[b] + split index
  int32_t blk_begin;    // logical blocks [blk_begin, blk_end) of the trajectory
  int32_t blk_end;
  int32_t len;          // context length of the trajectory
  int32_t table_off;    // row_off[b]: start of its row in block_ids
  int32_t nsplit;       // items of the trajectory
  int32_t pad;
};

struct DecodeTrajRec {
  int32_t part_off;     // first partial slot of the trajectory
  int32_t nsplit;
};

// Arguments of the split-K decode pass.  Pointers are device-accessible memory.
struct DecodeLaunch {
  const uint16_t* pool;        // bf16 [n_blocks][n_kv]{K tile [16][d], V tile [d][16]}
  const int32_t* block_ids;    // CSR block table
  const DecodeItemRec* items;  // [n_items] longest first
  const DecodeTrajRec* trajs;  // [B]
  const int32_t* out_row;      // combine only: output row of record i, or nullptr for row i
  const uint16_t* q;           // bf16 [B][n_q][d]
  float* part_acc;             // f32 [n_parts][n_q][d]   unnormalised sum of p * v
  float* part_ml;              // f32 [n_parts][n_q][4]   (max logit in log2 units, sum of bf16-rounded p,
                               //                          sum of unrounded p, unused)
  uint16_t* out;               // bf16 [B][n_q][d]
  float* lse;                  // f32 [B][n_q] or nullptr
  int32_t B, n_items, n_q_heads, n_kv_heads, head_dim;
  float scale_log2;            // softmax scale times log2(e)
};

// Returns hipSuccess or the launch error; HEDDLE_E_UNSUPPORTED shapes are rejected by the caller.
bool decode_shape_supported(int32_t group, int32_t head_dim);
hipError_t launch_decode_splitk(const DecodeLaunch& a, hipStream_t stream);
hipError_t launch_decode_combine(const DecodeLaunch& a, hipStream_t stream);

// Scatter of new K/V rows into the paged pool.  Row i (of n_rows) belongs to trajectory
// row_traj[i] ... expressed through cu_rows: trajectory b owns rows [cu_rows[b], cu_rows[b+1])
// and its first row goes to token position first_pos[b].
struct KvWriteLaunch {
  uint16_t* pool;
  const int32_t* row_off;
  const int32_t* block_ids;
  const int32_t* first_pos;    // [B] device
  const int32_t* cu_rows;      // [B+1] device
  const int32_t* cu_wblk;      // [B+1] device: prefix sums of the pool blocks each trajectory's rows touch
  const uint16_t* k;           // bf16 [n_rows][n_kv][d]
  const uint16_t* v;
  int32_t B, n_rows, n_wblk, n_kv_heads, head_dim;
  int32_t one_row_each;        // 1: trajectory b brings exactly row b (a decode step); cu_rows and cu_wblk are
                               // not read then
};
hipError_t launch_kv_write(const KvWriteLaunch& a, hipStream_t stream);

// One work item of the append pass (32-byte record): 128/G consecutive chunk rows of one
// trajectory against a range of the keys they see.  An item that covers all keys of its tile
// (nsplit == 1) writes the final rows; otherwise it writes a split-K partial per (row, head) into
// slot slot0 + row_in_tile * nsplit, and decode_combine_kernel merges the parts of each row.
struct AppendItemRec {
  int32_t b;            // trajectory
  int32_t row0;         // first chunk row of the tile
  int32_t rows_n;       // rows in the tile
  int32_t key_end;      // keys [64 * step_begin, key_end) are processed (key_end <= L_b + row0 + rows_n)
  int32_t step_begin;   // first 64-key step of the item
  int32_t slot0;        // partial slot of row 0 of the tile for this part
  int32_t nsplit;       // parts of the tile
  int32_t pad;
};

// Arguments of the causal chunked-append attention pass.  All pointers are device memory.
struct AppendLaunch {
  const uint16_t* pool;
  const int32_t* row_off;
  const int32_t* block_ids;
  const int32_t* ctx_len;      // [B]   tokens retained before the chunk
  const int32_t* cu_chunk;     // [B+1] prefix sums of chunk lengths
  const AppendItemRec* items;  // [n_items] longest first
  const uint16_t* q;           // bf16 [sum C][n_q][d]
  uint16_t* out;               // bf16 [sum C][n_q][d]
  float* lse;                  // f32 [sum C][n_q] or nullptr
  float* part_acc;             // as in DecodeLaunch; used by items with nsplit > 1
  float* part_ml;
  int32_t n_items, n_q_heads, n_kv_heads, head_dim;
  float scale_log2;
};
// One shared-prefix work item: the query rows of up to 128/G member trajectories of a group
// against blocks [blk_begin, blk_end) of the prefix all of them share (32-byte record).
struct GroupItemRec {
  int32_t table_off;    // start of the group leader's row in block_ids
  int32_t blk_begin;    // logical blocks of the shared prefix covered by this item
  int32_t blk_end;
  int32_t part;         // partial slot of this item within each member: trajs[b].part_off + part
  int32_t member_off;   // members[member_off .. member_off + n_members) are the item's trajectories
  int32_t n_members;
  int32_t pad[2];
};

static_assert(sizeof(DecodeItemRec) == 32 && sizeof(AppendItemRec) == 32 && sizeof(GroupItemRec) == 32,
              "work item records are 32 bytes: the plan image reserves 8 words for each");

// Arguments of the shared-prefix pass of a decode step: same matrix-core kernel as append, no
// causal edge, and the result is a split-K partial per (member, query head) that the combine
// kernel merges with the partials of the member's private blocks.
struct GroupLaunch {
  const uint16_t* pool;
  const int32_t* block_ids;
  const GroupItemRec* items;   // [n_items] longest first
  const int32_t* members;
  const DecodeTrajRec* trajs;  // [B]
  const uint16_t* q;           // bf16 [B][n_q][d]
  float* part_acc;             // as in DecodeLaunch
  float* part_ml;
  int32_t n_items, n_q_heads, n_kv_heads, head_dim;
  float scale_log2;
};
hipError_t launch_group_attn(const GroupLaunch& a, hipStream_t stream);

bool append_shape_supported(int32_t group, int32_t head_dim);
int32_t append_tile_rows(int32_t group);   // chunk rows per workgroup tile
hipError_t launch_append_attn(const AppendLaunch& a, hipStream_t stream);
// Same arguments for items whose tile has at most narrow_tile_rows(G) chunk rows (32 query rows
// per kv head): the four waves split the keys instead of the rows, nothing is staged in LDS.
inline bool narrow_shape_supported(int32_t group, int32_t head_dim) {   // what launch_narrow_attn accepts
  return head_dim == 128 && group >= 1 && group <= 32;
}
int32_t narrow_tile_rows(int32_t group);
hipError_t launch_narrow_attn(const AppendLaunch& a, hipStream_t stream);

// Copies n whole blocks pool[ids[i]] -> staging[i] (pack) or staging[i] -> pool[ids[i]] (unpack);
// ids is a device array, block_bytes a multiple of 4096.
hipError_t launch_kv_move(bool pack, void* pool, void* staging, const int32_t* ids, int32_t n, int64_t block_bytes,
                          hipStream_t stream);

// Copies n whole blocks inside the pool: block ids[n + i] becomes a copy of block ids[i] (ids is a
// device array of 2n entries; no destination may also be a source or appear twice).
hipError_t launch_kv_copy(void* pool, const int32_t* ids, int32_t n, int64_t block_bytes, hipStream_t stream);

hipError_t launch_stream_read(const void* src, uint64_t bytes, uint32_t* sink, hipStream_t stream);

// Copies n_vec 16-byte pieces from pinned host memory (src, device-visible) to device memory in a
// kernel on the caller's stream.  With rows != nullptr the same launch also stores one new K/V row
// per trajectory (rows->one_row_each must be set); rows->first_pos must then point into memory
// that is already valid when the kernel starts (the pinned image, not the copy's destination).
hipError_t launch_plan_copy(const void* src, void* dst, size_t n_vec, const KvWriteLaunch* rows, hipStream_t stream);

}  // namespace heddle
