"""Split-K partition plan for batched decode, and work order for append.
TEST INFRASTRUCTURE ONLY (see package docstring).

A plan is a heuristic, not a unique answer, so this file follows the written
rule step by step and the C++ planner must reproduce it bit for bit.  The rule
is motivated by the paper's straggler observation (Sec. 1, Sec. 2.2: the
longest trajectory dominates) and borrows the longest-processing-time-first
ordering the paper uses for its scheduler (Sec. 4.2).

Rule (all integer arithmetic; BT = 16 tokens per block):
  1. nblk[b] = ceil(len[b] / BT);  W = sum nblk
  2. target  = max(1, floor(n_cu * wg_per_cu / n_kv_heads))   items wanted per kv head
  3. chunk   = max(ceil(W / target), min_chunk_blk), rounded up to a multiple of tile_blk
  4. per trajectory: ns = min(ceil(nblk / chunk), max_split);
     per = ceil(nblk / ns) rounded up to a multiple of tile_blk;
     nsplit = ceil(nblk / per)
  5. split k covers blocks [k*per, min((k+1)*per, nblk))
  6. part_off = exclusive prefix sum of nsplit; slot of (b, k) = part_off[b] + k
  7. items = all (b, k) sorted by (-(blk_end - blk_begin), b, k)
"""
from __future__ import annotations

import numpy as np

BLOCK_TOKENS = 16

DEFAULTS = dict(n_cu=256, wg_per_cu=4, min_chunk_blk=16, tile_blk=4, max_split=64)


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def _round_up(a: int, m: int) -> int:
    return _ceil_div(a, m) * m


def plan_decode(lens, n_kv_heads: int, n_cu=256, wg_per_cu=4, min_chunk_blk=16,
                tile_blk=4, max_split=64):
    lens = [int(x) for x in lens]
    B = len(lens)
    nblk = [_ceil_div(n, BLOCK_TOKENS) for n in lens]
    W = sum(nblk)
    target = max(1, (n_cu * wg_per_cu) // n_kv_heads)
    chunk = _round_up(max(_ceil_div(W, target), min_chunk_blk), tile_blk)

    nsplit, part_off, items = [], [0], []
    for b in range(B):
        ns = min(_ceil_div(nblk[b], chunk), max_split)
        per = _round_up(_ceil_div(nblk[b], ns), tile_blk)
        n = _ceil_div(nblk[b], per)
        nsplit.append(n)
        part_off.append(part_off[-1] + n)
        for k in range(n):
            lo, hi = k * per, min((k + 1) * per, nblk[b])
            items.append((-(hi - lo), b, k, lo, hi))
    items.sort()
    i32 = lambda v: np.asarray(v, dtype=np.int32)
    return dict(
        chunk=chunk,
        n_items=len(items),
        item_b=i32([it[1] for it in items]),
        item_s=i32([it[2] for it in items]),
        item_blk_begin=i32([it[3] for it in items]),
        item_blk_end=i32([it[4] for it in items]),
        nsplit=i32(nsplit),
        part_off=i32(part_off),
    )


def plan_append(ctx_lens, chunk_lens, tile_rows: int):
    """Work order of the append kernel: one tile per (trajectory, group of
    tile_rows consecutive chunk rows); the tile's cost is the number of keys its
    last row sees, extent = L_b + min((t+1)*tile_rows, C_b).  Tiles are sorted
    by (-extent, b, t), longest first.  Returns int32 arrays tile_b, tile_row0,
    tile_rows_n, tile_extent."""
    tiles = []
    for b, (L, C) in enumerate(zip(ctx_lens, chunk_lens)):
        L, C = int(L), int(C)
        for t in range(_ceil_div(C, tile_rows)):
            r0 = t * tile_rows
            r1 = min(r0 + tile_rows, C)
            tiles.append((-(L + r1), b, t, r0, r1 - r0))
    tiles.sort()
    i32 = lambda v: np.asarray(v, dtype=np.int32)
    return dict(
        n_tiles=len(tiles),
        tile_b=i32([t[1] for t in tiles]),
        tile_row0=i32([t[3] for t in tiles]),
        tile_rows_n=i32([t[4] for t in tiles]),
        tile_extent=i32([-t[0] for t in tiles]),
    )


def plan_decode_shared(lens, row_off, block_ids, n_kv_heads: int, tile_members: int, n_cu=256,
                       wg_per_cu=4, min_chunk_blk=16, tile_blk=4, max_split=64, min_share_blk=4,
                       group_wg_per_cu=1, prefix_align=1):
    """Split-K plan for a decode step in which trajectories whose block-table rows begin with
    the same physical blocks (the samples of one prompt, Sec. 7 Workloads; a prefix-cache hit
    in the sense of Sec. 2.3) read that shared prefix once per group instead of once each.

    Rule (all integer arithmetic; BT = 16):
      1. nblk[b] = ceil(len[b]/BT); shareable[b] = (len[b]-1) // BT: blocks wholly before the
         position of the step's own row (the block that row is written to is never shared).
      2. Walk b upwards.  The first trajectory whose first block id has not been seen is the
         leader of that id.  For a later trajectory with the same first id, lcp = number of
         leading table entries equal to the leader's, capped by both shareable counts and
         rounded down to a multiple of prefix_align (the kernel that reads the private blocks
         of some head shapes starts only at such blocks); it joins
         the leader's group iff lcp >= min_share_blk.  A group exists iff someone joined; its
         prefix p = min lcp over the joined; members = leader + joined, ascending b.
         Groups are numbered by ascending leader.  prefix[b] = p for members, else 0.
      3. Private work W = sum_b (nblk[b] - prefix[b]); target and chunk from W as in plan_decode.
         Shared work Wg = sum_g p_g * ceil(|members_g| / tile_members);
         target_g = max(1, floor(n_cu * group_wg_per_cu / n_kv_heads));
         chunk_g = max(ceil(Wg / target_g), min_chunk_blk) rounded up to a multiple of tile_blk.
      4. cut(n, c) -> (per, count): ns = min(ceil(n/c), max_split); per = ceil(n/ns) rounded up
         to a multiple of tile_blk; count = ceil(n/per).
      5. Group g: (per, np_g) = cut(p_g, chunk_g); prefix part k covers blocks
         [k*per, min((k+1)*per, p_g)) of the leader's row.  Members are cut into tiles of
         tile_members consecutive members.  Group items (g, k, t) carry (blk_begin, blk_end,
         first member index, member count).
      6. Trajectory b: n = nblk[b] - prefix[b] (>= 1); (per, ns_b) = cut(n, chunk); suffix part k covers
         [prefix[b] + k*per, min(prefix[b] + (k+1)*per, nblk[b])) and has slot np_g + k
         (np_g = 0 outside groups).  nsplit[b] = np_g + ns_b; part_off = exclusive prefix sum.
      7. decode items sorted by (-(blk_end-blk_begin), b, slot); group items sorted by
         (-(blk_end-blk_begin), g, k, t).
    """
    lens = [int(x) for x in lens]
    row_off = [int(x) for x in row_off]
    B = len(lens)
    nblk = [_ceil_div(n, BLOCK_TOKENS) for n in lens]
    shareable = [(n - 1) // BLOCK_TOKENS for n in lens]

    leader_of_id, joined, lcp_of = {}, {}, {}
    for b in range(B):
        if shareable[b] < 1:
            continue
        first = int(block_ids[row_off[b]])
        if first not in leader_of_id:
            leader_of_id[first] = b
            continue
        a = leader_of_id[first]
        cap = min(shareable[a], shareable[b])
        n = 0
        while n < cap and int(block_ids[row_off[a] + n]) == int(block_ids[row_off[b] + n]):
            n += 1
        n = (n // prefix_align) * prefix_align
        if n >= min_share_blk and n >= 1:
            joined.setdefault(a, []).append(b)
            lcp_of[b] = n
    leaders = sorted(joined)
    group_leader, group_prefix, group_members = [], [], []
    traj_group, prefix = [-1] * B, [0] * B
    for g, a in enumerate(leaders):
        p = min(lcp_of[b] for b in joined[a])
        members = [a] + joined[a]
        group_leader.append(a)
        group_prefix.append(p)
        group_members.append(members)
        for b in members:
            traj_group[b], prefix[b] = g, p

    W = sum(nblk[b] - prefix[b] for b in range(B))
    target = max(1, (n_cu * wg_per_cu) // n_kv_heads)
    chunk = _round_up(max(_ceil_div(W, target), min_chunk_blk), tile_blk)
    Wg = sum(p * _ceil_div(len(m), tile_members) for p, m in zip(group_prefix, group_members))
    target_g = max(1, (n_cu * group_wg_per_cu) // n_kv_heads)
    chunk_g = _round_up(max(_ceil_div(Wg, target_g), min_chunk_blk), tile_blk)

    def cut(n, c):
        ns = min(_ceil_div(n, c), max_split)
        per = _round_up(_ceil_div(n, ns), tile_blk)
        return per, _ceil_div(n, per)

    gitems, group_parts = [], []
    for g, p in enumerate(group_prefix):
        per, cnt = cut(p, chunk_g)
        group_parts.append(cnt)
        n_mem = len(group_members[g])
        for k in range(cnt):
            lo, hi = k * per, min((k + 1) * per, p)
            for t in range(_ceil_div(n_mem, tile_members)):
                m0 = t * tile_members
                gitems.append((-(hi - lo), g, k, t, lo, hi, m0, min(tile_members, n_mem - m0)))
    gitems.sort()

    nsplit, part_off, items = [], [0], []
    for b in range(B):
        npg = group_parts[traj_group[b]] if traj_group[b] >= 0 else 0
        n = nblk[b] - prefix[b]
        per, cnt = cut(n, chunk)
        nsplit.append(npg + cnt)
        part_off.append(part_off[-1] + npg + cnt)
        for k in range(cnt):
            lo, hi = prefix[b] + k * per, min(prefix[b] + (k + 1) * per, nblk[b])
            items.append((-(hi - lo), b, npg + k, lo, hi))
    items.sort()

    i32 = lambda v: np.asarray(v, dtype=np.int32)
    member_off = [0]
    for m in group_members:
        member_off.append(member_off[-1] + len(m))
    return dict(
        chunk=chunk,
        chunk_g=chunk_g,
        n_groups=len(leaders),
        group_leader=i32(group_leader),
        group_prefix=i32(group_prefix),
        group_parts=i32(group_parts),
        member_off=i32(member_off),
        members=i32([b for m in group_members for b in m]),
        traj_group=i32(traj_group),
        traj_prefix=i32(prefix),
        n_items=len(items),
        item_b=i32([it[1] for it in items]),
        item_s=i32([it[2] for it in items]),
        item_blk_begin=i32([it[3] for it in items]),
        item_blk_end=i32([it[4] for it in items]),
        n_gitems=len(gitems),
        gitem_g=i32([it[1] for it in gitems]),
        gitem_k=i32([it[2] for it in gitems]),
        gitem_blk_begin=i32([it[4] for it in gitems]),
        gitem_blk_end=i32([it[5] for it in gitems]),
        gitem_m0=i32([it[6] for it in gitems]),
        gitem_mn=i32([it[7] for it in gitems]),
        nsplit=i32(nsplit),
        part_off=i32(part_off),
    )


APPEND_STEP_KEYS = 64     # keys per main-loop step of the append kernel; parts are cut at these


def split_append_tiles(plan, ctx_lens, n_kv_heads: int, n_cu=256, append_wg_per_cu=2, min_steps=4,
                       max_split=64):
    """Split-K for append: a tile whose keys are many more than an even share of the batch (one
    long trajectory with a short chunk; the long tail of a speculative-decoding verify step of a
    few tokens per trajectory, Sec. 8) has its keys cut into parts that run as separate work
    items and are merged afterwards, as in decode.

    Rule (integer; `plan` is the output of plan_append, tiles in its order, index t):
      1. S_t = ceil(extent_t / 64) steps; slots = n_cu * append_wg_per_cu.
      2. W = sum S_t, target = max(1, slots // n_kv_heads),
         chunk = max(ceil(W / target), min_steps).  Per tile ns = min(ceil(S/chunk), max_split),
         per = ceil(S / ns), n = ceil(S / per); while n > 1 and (n-1) * per * 64 > L_b + row0:
         n -= 1 (the first row of the tile must see a key of the last part, or that row's share
         of the part would be an empty softmax).  Part k < n-1 covers steps [k*per, (k+1)*per),
         the last part [(n-1)*per, S).
      3. Tiles with n > 1 own rows_n * n partial slots from part_base_t on (bases assigned in
         tile order); row r of the tile, part k -> slot part_base_t + r*n + k.
      4. items (t, k) sorted by (-(step_end - step_begin), b_t, step_begin, row0_t): among equally
         long items, those of one trajectory that cover the same keys (parts of its different
         tiles) are neighbours, run at the same time and share the K/V they read in cache.
    Returns tile_nsplit[n_tiles], tile_part_base[n_tiles], n_slots, and item arrays
    item_tile, item_k, item_step_begin, item_step_end."""
    n_tiles = int(plan["n_tiles"])
    S = [_ceil_div(int(e), APPEND_STEP_KEYS) for e in plan["tile_extent"]]
    slots = n_cu * append_wg_per_cu
    nsplit, per_of = [1] * n_tiles, list(S)
    W = sum(S)
    target = max(1, slots // n_kv_heads)
    chunk = max(_ceil_div(W, target), min_steps)
    for t in range(n_tiles):
        ns = min(_ceil_div(S[t], chunk), max_split)
        per = _ceil_div(S[t], ns)
        n = _ceil_div(S[t], per)
        first_row_pos = int(ctx_lens[int(plan["tile_b"][t])]) + int(plan["tile_row0"][t])
        while n > 1 and (n - 1) * per * APPEND_STEP_KEYS > first_row_pos:
            n -= 1
        nsplit[t], per_of[t] = n, per
    base, part_base, items = 0, [], []
    for t in range(n_tiles):
        part_base.append(base if nsplit[t] > 1 else 0)
        if nsplit[t] > 1:
            base += int(plan["tile_rows_n"][t]) * nsplit[t]
        for k in range(nsplit[t]):
            lo = k * per_of[t]
            hi = S[t] if k == nsplit[t] - 1 else (k + 1) * per_of[t]
            items.append((-(hi - lo), int(plan["tile_b"][t]), lo, int(plan["tile_row0"][t]), t, k, hi))
    items.sort()
    i32 = lambda v: np.asarray(v, dtype=np.int32)
    return dict(
        tile_nsplit=i32(nsplit), tile_part_base=i32(part_base), n_slots=base, n_items=len(items),
        item_tile=i32([it[4] for it in items]), item_k=i32([it[5] for it in items]),
        item_step_begin=i32([it[2] for it in items]), item_step_end=i32([it[6] for it in items]),
    )
