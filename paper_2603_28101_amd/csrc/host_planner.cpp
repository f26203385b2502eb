// Host-side planners: split-K partition of a decode batch, and tile order of an append batch.
#include <algorithm>
#include <unordered_map>

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
  // longest first; (b, s) ascending among equals.  The key is total, so an in-place sort gives
  // one order and the call takes no work buffer from the heap.
  std::sort(items.begin(), items.end(), [](const DecodeItem& x, const DecodeItem& y) {
    const int32_t nx = x.blk_end - x.blk_begin, ny = y.blk_end - y.blk_begin;
    if (nx != ny) return nx > ny;
    if (x.b != y.b) return x.b < y.b;
    return x.s < y.s;
  });
}

void plan_decode_shared(const PlanParams& p, int32_t min_share_blk, int32_t group_wg_per_cu, int32_t tile_members,
                        int32_t prefix_align, int32_t B, const int32_t* len, const int32_t* row_off,
                        const int32_t* block_ids, SharedPlan& out) {
  const size_t nB = static_cast<size_t>(B);
  out.group_leader.clear();
  out.group_prefix.clear();
  out.group_parts.clear();
  out.members.clear();
  out.member_off.assign(1, 0);
  out.traj_group.assign(nB, -1);
  out.traj_prefix.assign(nB, 0);
  out.nsplit.assign(nB, 0);
  out.part_off.assign(nB + 1, 0);
  out.items.clear();
  out.gitems.clear();

  // ---- who shares with whom: leader = first trajectory seen with a given first block id
  std::unordered_map<int32_t, int32_t> leader_of_id;
  std::vector<int32_t> leader(nB, -1), lcp(nB, 0), n_joined(nB, 0), min_lcp(nB, 0);
  for (int32_t b = 0; b < B; ++b) {
    const int32_t share_b = (len[b] - 1) / HEDDLE_BLOCK_TOKENS;
    if (share_b < 1) continue;
    auto [it, fresh] = leader_of_id.try_emplace(block_ids[row_off[b]], b);
    if (fresh) continue;
    const int32_t a = it->second;
    const int32_t cap = std::min(share_b, (len[a] - 1) / HEDDLE_BLOCK_TOKENS);
    const int32_t* ra = block_ids + row_off[a];
    const int32_t* rb = block_ids + row_off[b];
    int32_t n = 0;
    while (n < cap && ra[n] == rb[n]) ++n;
    n = n / prefix_align * prefix_align;      // shared prefixes end where the private blocks' kernel may start
    if (n < min_share_blk || n < 1) continue;
    leader[b] = a;
    lcp[b] = n;
    min_lcp[a] = n_joined[a] == 0 ? n : std::min(min_lcp[a], n);
    ++n_joined[a];
  }
  // groups in ascending order of their leader; members ascending (leader first, it is the smallest)
  std::vector<int32_t> group_of_leader(nB, -1);
  for (int32_t a = 0; a < B; ++a) {
    if (n_joined[a] == 0) continue;
    group_of_leader[a] = static_cast<int32_t>(out.group_leader.size());
    out.group_leader.push_back(a);
    out.group_prefix.push_back(min_lcp[a]);
    out.member_off.push_back(out.member_off.back() + 1 + n_joined[a]);
  }
  out.members.assign(static_cast<size_t>(out.member_off.back()), 0);
  std::vector<int32_t> fill(out.group_leader.size(), 0);
  for (int32_t b = 0; b < B; ++b) {
    const int32_t g = n_joined[b] > 0 ? group_of_leader[b] : (leader[b] >= 0 ? group_of_leader[leader[b]] : -1);
    if (g < 0) continue;
    out.members[static_cast<size_t>(out.member_off[g] + fill[g]++)] = b;
    out.traj_group[b] = g;
    out.traj_prefix[b] = out.group_prefix[g];
  }

  // ---- chunk sizes: private blocks for the decode kernel, shared blocks for the group kernel
  int64_t work = 0, work_g = 0;
  for (int32_t b = 0; b < B; ++b) work += ceil_div(len[b], HEDDLE_BLOCK_TOKENS) - out.traj_prefix[b];
  for (size_t g = 0; g < out.group_leader.size(); ++g)
    work_g += static_cast<int64_t>(out.group_prefix[g]) * ceil_div(out.member_off[g + 1] - out.member_off[g], tile_members);
  const int64_t target = std::max<int64_t>(1, (int64_t)p.n_cu * p.wg_per_cu / p.n_kv_heads);
  const int64_t target_g = std::max<int64_t>(1, (int64_t)p.n_cu * group_wg_per_cu / p.n_kv_heads);
  const int64_t chunk = round_up(std::max<int64_t>(ceil_div(work, target), p.min_chunk_blk), p.tile_blk);
  const int64_t chunk_g = round_up(std::max<int64_t>(ceil_div(work_g, target_g), p.min_chunk_blk), p.tile_blk);
  out.chunk = static_cast<int32_t>(chunk);
  out.chunk_g = static_cast<int32_t>(chunk_g);
  auto cut = [&](int64_t n, int64_t c, int64_t& per) {
    const int64_t want = std::min<int64_t>(ceil_div(n, c), p.max_split);
    per = round_up(ceil_div(n, want), p.tile_blk);
    return ceil_div(n, per);
  };

  for (size_t g = 0; g < out.group_leader.size(); ++g) {
    const int64_t pre = out.group_prefix[g];
    int64_t per = 0;
    const int64_t cnt = cut(pre, chunk_g, per);
    out.group_parts.push_back(static_cast<int32_t>(cnt));
    const int32_t n_mem = out.member_off[g + 1] - out.member_off[g];
    for (int64_t k = 0; k < cnt; ++k)
      for (int32_t m0 = 0; m0 < n_mem; m0 += tile_members) {
        GroupItem it;
        it.g = static_cast<int32_t>(g);
        it.k = static_cast<int32_t>(k);
        it.blk_begin = static_cast<int32_t>(k * per);
        it.blk_end = static_cast<int32_t>(std::min((k + 1) * per, pre));
        it.m0 = m0;
        it.mn = std::min(tile_members, n_mem - m0);
        out.gitems.push_back(it);
      }
  }
  std::stable_sort(out.gitems.begin(), out.gitems.end(), [](const GroupItem& x, const GroupItem& y) {
    return (x.blk_end - x.blk_begin) > (y.blk_end - y.blk_begin);
  });

  for (int32_t b = 0; b < B; ++b) {
    const int32_t g = out.traj_group[b];
    const int32_t before = g >= 0 ? out.group_parts[static_cast<size_t>(g)] : 0;
    const int64_t nblk = ceil_div(len[b], HEDDLE_BLOCK_TOKENS);
    const int64_t first = out.traj_prefix[b];
    int64_t per = 0;
    const int64_t cnt = cut(nblk - first, chunk, per);
    out.nsplit[b] = before + static_cast<int32_t>(cnt);
    out.part_off[b + 1] = out.part_off[b] + out.nsplit[b];
    for (int64_t k = 0; k < cnt; ++k) {
      DecodeItem it;
      it.b = b;
      it.s = before + static_cast<int32_t>(k);
      it.blk_begin = static_cast<int32_t>(first + k * per);
      it.blk_end = static_cast<int32_t>(std::min(first + (k + 1) * per, nblk));
      out.items.push_back(it);
    }
  }
  std::stable_sort(out.items.begin(), out.items.end(), [](const DecodeItem& x, const DecodeItem& y) {
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

void split_append_tiles(const PlanParams& p, int32_t append_wg_per_cu, int32_t min_steps,
                        const std::vector<AppendTile>& tiles, const int32_t* ctx_len, AppendSplit& out) {
  const size_t n = tiles.size();
  out.nsplit.assign(n, 1);
  out.part_base.assign(n, 0);
  out.items.clear();
  out.n_slots = 0;
  std::vector<int64_t> steps(n), per(n);
  int64_t work = 0;
  for (size_t t = 0; t < n; ++t) {
    steps[t] = per[t] = ceil_div(tiles[t].extent, kAppendStepKeys);
    work += steps[t];
  }
  const int64_t slots = static_cast<int64_t>(p.n_cu) * append_wg_per_cu;
  const int64_t target = std::max<int64_t>(1, slots / p.n_kv_heads);
  const int64_t chunk = std::max<int64_t>(ceil_div(work, target), min_steps);
  for (size_t t = 0; t < n; ++t) {
    const int64_t want = std::min<int64_t>(ceil_div(steps[t], chunk), p.max_split);
    const int64_t each = ceil_div(steps[t], want);
    int64_t parts = ceil_div(steps[t], each);
    // the first row of the tile must see a key of the last part (with parts of one or two steps
    // more than one part may lie behind what that row sees)
    const int64_t first_row_pos = static_cast<int64_t>(ctx_len[tiles[t].b]) + tiles[t].row0;
    while (parts > 1 && (parts - 1) * each * kAppendStepKeys > first_row_pos) --parts;
    out.nsplit[t] = static_cast<int32_t>(parts);
    per[t] = each;
  }
  for (size_t t = 0; t < n; ++t) {
    const int32_t parts = out.nsplit[t];
    if (parts > 1) {
      out.part_base[t] = out.n_slots;
      out.n_slots += tiles[t].rows * parts;
    }
    for (int32_t k = 0; k < parts; ++k) {
      AppendItem it;
      it.tile = static_cast<int32_t>(t);
      it.k = k;
      it.step_begin = static_cast<int32_t>(k * per[t]);
      it.step_end = static_cast<int32_t>(k == parts - 1 ? steps[t] : (k + 1) * per[t]);
      out.items.push_back(it);
    }
  }
  // longest first; among equals by (trajectory, first step, first row): parts of different tiles of
  // one trajectory that cover the same keys become neighbours and share those keys in cache
  std::sort(out.items.begin(), out.items.end(), [&tiles](const AppendItem& x, const AppendItem& y) {
    const int32_t lx = x.step_end - x.step_begin, ly = y.step_end - y.step_begin;
    if (lx != ly) return lx > ly;
    const AppendTile& tx = tiles[static_cast<size_t>(x.tile)];
    const AppendTile& ty = tiles[static_cast<size_t>(y.tile)];
    if (tx.b != ty.b) return tx.b < ty.b;
    if (x.step_begin != y.step_begin) return x.step_begin < y.step_begin;
    return tx.row0 < ty.row0;
  });
}

}  // namespace heddle
