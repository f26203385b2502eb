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
  int release(int32_t n, const int32_t* ids);
  int32_t num_free() const { return static_cast<int32_t>(stack_.size()); }

 private:
  enum : uint8_t { kFree = 0, kHeld = 1, kMarked = 2 };
  std::vector<int32_t> stack_;  // top = back
  std::vector<uint8_t> state_;
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

struct AppendTile {
  int32_t b, row0, rows, extent;
};
void plan_append(int32_t B, const int32_t* ctx_len, const int32_t* cu_chunk, int32_t tile_rows,
                 std::vector<AppendTile>& tiles);

}  // namespace heddle
