// Internal declarations shared by the host and device translation units of libheddle.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "heddle.h"

namespace heddle {

// ---------------------------------------------------------------- block manager
// Stack allocator of 16-token blocks (paper Sec. 4.2: caches outlive tool calls
// and preemption, so blocks are only returned when a trajectory ends).
class BlockManager {
 public:
  explicit BlockManager(int32_t n_blocks);
  int alloc(int32_t n, int32_t* out);
  int retain(int32_t n, const int32_t* ids);
  int release(int32_t n, const int32_t* ids);
  int32_t num_free() const { return static_cast<int32_t>(stack_.size()); }

 private:
  enum : uint8_t { kFree = 0, kHeld = 1, kMarked = 2 };
  // Validates a list (every id in range, held, named once) by marking; restores the marks.
  bool valid_held_list(int32_t n, const int32_t* ids);
  std::vector<int32_t> stack_;    // top = back
  std::vector<uint8_t> state_;
  std::vector<int32_t> holders_;  // per block: trajectories that name it (0 = free)
};

// ---------------------------------------------------------------- planners
struct PlanParams {
  int32_t n_kv_heads, n_cu, wg_per_cu, min_chunk_blk, tile_blk, max_split;
};

struct DecodeItem {
  int32_t b, s, blk_begin, blk_end;
};

// Split-K plan (rule in heddle.h).  items sorted longest first; nsplit [B]; part_off [B+1].
void plan_decode(const PlanParams& p, int32_t B, const int32_t* len, std::vector<DecodeItem>& items,
                 std::vector<int32_t>& nsplit, std::vector<int32_t>& part_off, int32_t& chunk);

// Decode plan with shared prefixes: trajectories whose block-table rows start with the same
// physical blocks form a group; the group's prefix is read once (group items, processed by the
// matrix-core kernel for all members at a time), every member's remaining blocks are ordinary
// decode items (rule in heddle.h).
struct GroupItem {
  int32_t g, k, blk_begin, blk_end, m0, mn;   // members[member_off[g] + m0 .. + mn)
};
struct SharedPlan {
  int32_t chunk = 0, chunk_g = 0;
  std::vector<int32_t> group_leader, group_prefix, group_parts, member_off, members;
  std::vector<int32_t> traj_group, traj_prefix, nsplit, part_off;
  std::vector<DecodeItem> items;     // s = slot within the trajectory (prefix parts come first)
  std::vector<GroupItem> gitems;
};
void plan_decode_shared(const PlanParams& p, int32_t min_share_blk, int32_t group_wg_per_cu, int32_t tile_members,
                        int32_t prefix_align, int32_t B, const int32_t* len, const int32_t* row_off,
                        const int32_t* block_ids, SharedPlan& out);

struct AppendTile {
  int32_t b, row0, rows, extent;
};
void plan_append(int32_t B, const int32_t* ctx_len, const int32_t* cu_chunk, int32_t tile_rows,
                 std::vector<AppendTile>& tiles);

// Split-K of an append batch that is too small to fill the GPU: the keys of a tile are cut at
// multiples of 64 (one main-loop step of the kernel) into parts (rule in heddle.h).
constexpr int32_t kAppendStepKeys = 64;
struct AppendItem {
  int32_t tile, k, step_begin, step_end;
};
struct AppendSplit {
  std::vector<int32_t> nsplit, part_base;   // per tile, in plan order
  int32_t n_slots = 0;
  std::vector<AppendItem> items;            // longest first
};
void split_append_tiles(const PlanParams& p, int32_t append_wg_per_cu, int32_t min_steps,
                        const std::vector<AppendTile>& tiles, const int32_t* ctx_len, AppendSplit& out);

}  // namespace heddle
