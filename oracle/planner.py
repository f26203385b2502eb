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
