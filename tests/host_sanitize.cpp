// Drives the host side of the library (block manager, planners, placement) with random and
// extreme inputs under AddressSanitizer and UndefinedBehaviorSanitizer.  Built and run by
// tests/test_host_abi.py from the same sources the library is built from; a memory error or an
// overflow ends the program with the sanitizer's report, a broken invariant with a message.
// The values themselves are compared with the oracle elsewhere: here only "every block is
// covered exactly once" style facts are checked, so that the run has something to fail on
// besides the sanitizers.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <numeric>
#include <vector>

#include "heddle_internal.h"

using namespace heddle;

namespace {

uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint64_t rnd() {  // splitmix64
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
int32_t between(int32_t lo, int32_t hi) { return lo + static_cast<int32_t>(rnd() % static_cast<uint64_t>(hi - lo + 1)); }

#define REQUIRE(cond)                                                   \
  do {                                                                  \
    if (!(cond)) {                                                      \
      std::printf("failed at line %d: %s\n", __LINE__, #cond);          \
      std::exit(1);                                                     \
    }                                                                   \
  } while (0)

int32_t draw_len() {
  switch (rnd() % 5) {
    case 0: return between(1, 40);
    case 1: return 16 * between(1, 300) + between(-1, 1);
    case 2: return between(1, 5000);
    case 3: return between(60000, HEDDLE_MAX_CONTEXT);
    default: return rnd() % 2 ? 1 : HEDDLE_MAX_CONTEXT;
  }
}

PlanParams draw_params() {
  PlanParams p;
  p.n_kv_heads = between(1, 16);
  p.n_cu = between(1, 304);
  p.wg_per_cu = between(1, 8);
  p.min_chunk_blk = between(1, 64);
  p.tile_blk = between(1, 8);
  p.max_split = between(1, 64);
  return p;
}

void manager() {
  for (int round = 0; round < 200; ++round) {
    const int32_t n = between(1, 50);
    BlockManager m(n);
    std::vector<int32_t> holders(static_cast<size_t>(n), 0), ids(80);
    for (int step = 0; step < 300; ++step) {
      const int op = static_cast<int>(rnd() % 4);
      const int32_t k = between(-1, 12);
      if (op == 0) {
        const int rc = m.alloc(k, ids.data());
        if (rc == HEDDLE_OK)
          for (int32_t i = 0; i < k; ++i) {
            REQUIRE(ids[i] >= 0 && ids[i] < n && holders[ids[i]] == 0);
            holders[ids[i]] = 1;
          }
      } else {
        for (int32_t i = 0; i < k; ++i) ids[i] = between(-2, n + 1);     // often invalid, often repeated
        bool valid = k >= 0;
        for (int32_t i = 0; i < k && valid; ++i) {
          valid = ids[i] >= 0 && ids[i] < n && holders[ids[i]] > 0;
          for (int32_t j = 0; j < i && valid; ++j) valid = ids[j] != ids[i];
        }
        const int rc = op == 1 ? m.retain(k, ids.data()) : m.release(k, ids.data());
        REQUIRE((rc == HEDDLE_OK) == valid);
        if (valid)
          for (int32_t i = 0; i < k; ++i) holders[ids[i]] += op == 1 ? 1 : -1;
      }
      int32_t free_now = 0;
      for (int32_t h : holders) free_now += h == 0;
      REQUIRE(m.num_free() == free_now);
    }
  }
}

void decode_plans() {
  std::vector<DecodeItem> items;
  std::vector<int32_t> nsplit, part_off, covered;
  for (int round = 0; round < 2000; ++round) {
    const PlanParams p = draw_params();
    const int32_t B = round % 50 == 0 ? between(500, 2000) : between(1, 70);
    std::vector<int32_t> len(static_cast<size_t>(B));
    for (int32_t& l : len) l = draw_len();
    int32_t chunk = 0;
    plan_decode(p, B, len.data(), items, nsplit, part_off, chunk);
    REQUIRE(chunk >= 1 && static_cast<int32_t>(nsplit.size()) == B && static_cast<int32_t>(part_off.size()) == B + 1);
    covered.assign(static_cast<size_t>(B), 0);
    for (const DecodeItem& it : items) {
      REQUIRE(it.b >= 0 && it.b < B && it.s >= 0 && it.s < nsplit[it.b] && it.blk_begin < it.blk_end);
      covered[it.b] += it.blk_end - it.blk_begin;
    }
    for (int32_t b = 0; b < B; ++b) {
      REQUIRE(covered[b] == (len[b] + 15) / 16 && nsplit[b] >= 1 && nsplit[b] <= p.max_split);
      REQUIRE(part_off[b + 1] == part_off[b] + nsplit[b]);
    }
  }
}

void shared_plans() {
  SharedPlan sp;
  for (int round = 0; round < 1500; ++round) {
    PlanParams p = draw_params();
    const int32_t align = rnd() % 2 ? 1 : 4;
    if (align == 4) p.tile_blk = 4 * between(1, 2);
    const int32_t B = between(1, 60);
    std::vector<int32_t> len(static_cast<size_t>(B)), row_off(static_cast<size_t>(B) + 1, 0), ids;
    int32_t next_id = 0;
    std::vector<std::vector<int32_t>> prompts(static_cast<size_t>(between(1, 5)));
    for (auto& pr : prompts) {
      pr.resize(static_cast<size_t>(between(1, 200)));
      for (int32_t& id : pr) id = next_id++;
    }
    for (int32_t b = 0; b < B; ++b) {
      len[b] = std::min(draw_len(), 20000);
      const int32_t nblk = (len[b] + 15) / 16 + between(0, 2);          // rows may be longer than needed
      const auto& pr = prompts[rnd() % prompts.size()];
      const int32_t shared = rnd() % 3 == 0 ? 0 : std::min<int32_t>(static_cast<int32_t>(pr.size()), nblk);
      for (int32_t i = 0; i < nblk; ++i) ids.push_back(i < shared ? pr[i] : next_id++);
      row_off[b + 1] = static_cast<int32_t>(ids.size());
    }
    plan_decode_shared(p, between(1, 16), between(1, 2), between(1, 128), align, B, len.data(), row_off.data(),
                       ids.data(), sp);
    std::vector<int32_t> covered(static_cast<size_t>(B), 0);
    for (const DecodeItem& it : sp.items) {
      REQUIRE(it.b >= 0 && it.b < B && it.blk_begin >= sp.traj_prefix[it.b] && it.blk_begin < it.blk_end);
      covered[it.b] += it.blk_end - it.blk_begin;
    }
    for (int32_t b = 0; b < B; ++b) {
      REQUIRE(covered[b] + sp.traj_prefix[b] == (len[b] + 15) / 16);
      REQUIRE(sp.traj_prefix[b] % align == 0 && sp.traj_prefix[b] <= (len[b] - 1) / 16);
      REQUIRE(sp.part_off[b + 1] == sp.part_off[b] + sp.nsplit[b]);
    }
    for (const GroupItem& it : sp.gitems) {
      REQUIRE(it.g >= 0 && it.g < static_cast<int32_t>(sp.group_leader.size()));
      REQUIRE(it.blk_begin < it.blk_end && it.blk_end <= sp.group_prefix[it.g] && it.mn >= 1);
      REQUIRE(sp.member_off[it.g] + it.m0 + it.mn <= sp.member_off[it.g + 1]);
    }
  }
}

void append_plans() {
  std::vector<AppendTile> tiles;
  AppendSplit split;
  for (int round = 0; round < 1500; ++round) {
    const PlanParams p = draw_params();
    const int32_t B = between(1, 40), tile_rows = between(1, 128);
    std::vector<int32_t> L(static_cast<size_t>(B)), cu(static_cast<size_t>(B) + 1, 0);
    for (int32_t b = 0; b < B; ++b) {
      const int32_t C = rnd() % 4 == 0 ? between(1, 8) : between(1, 1500);
      L[b] = std::min(rnd() % 4 == 0 ? 0 : draw_len(), HEDDLE_MAX_CONTEXT - C);
      cu[b + 1] = cu[b] + C;
    }
    plan_append(B, L.data(), cu.data(), tile_rows, tiles);
    int64_t rows = 0;
    for (const AppendTile& t : tiles) {
      REQUIRE(t.b >= 0 && t.b < B && t.rows >= 1 && t.rows <= tile_rows && t.extent == L[t.b] + t.row0 + t.rows);
      rows += t.rows;
    }
    REQUIRE(rows == cu[B]);
    split_append_tiles(p, between(1, 4), between(1, 8), tiles, L.data(), split);
    REQUIRE(split.nsplit.size() == tiles.size() && split.part_base.size() == tiles.size());
    std::vector<int32_t> steps(tiles.size(), 0);
    for (const AppendItem& it : split.items) {
      REQUIRE(it.tile >= 0 && it.tile < static_cast<int32_t>(tiles.size()) && it.step_begin < it.step_end);
      REQUIRE(it.k >= 0 && it.k < split.nsplit[it.tile]);
      steps[it.tile] += it.step_end - it.step_begin;
    }
    for (size_t t = 0; t < tiles.size(); ++t) REQUIRE(steps[t] == (tiles[t].extent + kAppendStepKeys - 1) / kAppendStepKeys);
  }
}

void placement() {
  for (int round = 0; round < 200; ++round) {
    const int32_t n = between(1, 60), m = between(1, 12);
    std::vector<double> len(static_cast<size_t>(n)), F(static_cast<size_t>(n) * 12 + 2);
    for (double& l : len) l = static_cast<double>(draw_len());
    std::sort(len.rbegin(), len.rend());
    std::vector<int32_t> count(static_cast<size_t>(n));
    int64_t total = 0;
    for (int32_t& c : count) total += (c = between(1, 12));
    const bool monotone = rnd() % 2;
    for (size_t s = 0; s < F.size(); ++s)
      F[s] = monotone ? 1.0 + 0.01 * static_cast<double>(s) : 1.0 + static_cast<double>(rnd() % 100) / 50.0;
    std::vector<int32_t> sizes(static_cast<size_t>(m), -1);
    double makespan = -1.0;
    const int rc = heddle_placement_dp(n, len.data(), count.data(), m, F.data(), static_cast<int32_t>(total) + 1, 2.0,
                                       static_cast<int32_t>(rnd() % 2), sizes.data(), &makespan);
    REQUIRE(rc == HEDDLE_OK && makespan > 0.0);
    int32_t placed = 0;
    for (int32_t j = 0; j < m; ++j) {
      REQUIRE(j < std::min(n, m) ? sizes[j] >= 1 : sizes[j] == 0);
      placed += sizes[j];
    }
    REQUIRE(placed == n);
    REQUIRE(heddle_placement_dp(n, len.data(), count.data(), m, F.data(), static_cast<int32_t>(total), 2.0, 0,
                                sizes.data(), &makespan) == HEDDLE_E_INVAL);        // F one entry short
  }
}

}  // namespace

int main() {
  manager();
  decode_plans();
  shared_plans();
  append_plans();
  placement();
  std::printf("ok\n");
  return 0;
}
