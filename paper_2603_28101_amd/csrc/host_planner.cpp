// Host-side planners: split-K partition of a decode batch, and tile order of an append batch.
#include <algorithm>

#include "heddle_internal.h"

namespace heddle {

namespace {
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t m) { return ceil_div(a, m) * m; }
}  // namespace

void plan_decode(const PlanParams& p, int32_t B, const int32_t* len, std::vector<DecodeItem>& items,
                 std::vector<int32_t>& nsplit, std::vector<int32_t>& part_off, int32_t& chunk) {
  items.clear();
  nsplit.assign(static_cast<size_t>(B), 0);
  part_off.assign(static_cast<size_t>(B) + 1, 0);

  int64_t total_blocks = 0;
  for (int32_t b = 0; b < B; ++b) total_blocks += ceil_div(len[b], HEDDLE_BLOCK_TOKENS);

  const int64_t target = std::max<int64_t>(1, (int64_t)p.n_cu * p.wg_per_cu / p.n_kv_heads);
  const int64_t chunk64 =
      round_up(std::max<int64_t>(ceil_div(total_blocks, target), p.min_chunk_blk), p.tile_blk);
  chunk = static_cast<int32_t>(chunk64);

  for (int32_t b = 0; b < B; ++b) {
    const int64_t nblk = ceil_div(len[b], HEDDLE_BLOCK_TOKENS);
    const int64_t want = std::min<int64_t>(ceil_div(nblk, chunk64), p.max_split);
    const int64_t per = round_up(ceil_div(nblk, want), p.tile_blk);
    const int64_t n = ceil_div(nblk, per);
    nsplit[b] = static_cast<int32_t>(n);
    part_off[b + 1] = part_off[b] + static_cast<int32_t>(n);
    for (int64_t k = 0; k < n; ++k) {
      DecodeItem it;
      it.b = b;
      it.s = static_cast<int32_t>(k);
      it.blk_begin = static_cast<int32_t>(k * per);
      it.blk_end = static_cast<int32_t>(std::min((k + 1) * per, nblk));
      items.push_back(it);
    }
  }
  // longest first; (b, s) ascending among equals.  Items were generated in (b, s)
  // order, so a stable sort on size alone gives exactly that order.
  std::stable_sort(items.begin(), items.end(), [](const DecodeItem& x, const DecodeItem& y) {
    return (x.blk_end - x.blk_begin) > (y.blk_end - y.blk_begin);
  });
}

void plan_append(int32_t B, const int32_t* ctx_len, const int32_t* cu_chunk, int32_t tile_rows,
                 std::vector<AppendTile>& tiles) {
  tiles.clear();
  for (int32_t b = 0; b < B; ++b) {
    const int32_t C = cu_chunk[b + 1] - cu_chunk[b];
    for (int32_t r0 = 0; r0 < C; r0 += tile_rows) {
      AppendTile t;
      t.b = b;
      t.row0 = r0;
      t.rows = std::min(tile_rows, C - r0);
      t.extent = ctx_len[b] + r0 + t.rows;
      tiles.push_back(t);
    }
  }
  std::stable_sort(tiles.begin(), tiles.end(),
                   [](const AppendTile& x, const AppendTile& y) { return x.extent > y.extent; });
}

}  // namespace heddle
