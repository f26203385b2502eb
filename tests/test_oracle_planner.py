"""Pins of the oracle's split-K planner, append ordering and block manager (no GPU)."""
import json
import os

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import planner as op
from oracle.kv_manager import KVManager

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def test_plan_hand_worked_examples():
    for ex in load("plan_worked_examples.json")["examples"]:
        p = dict(ex["params"])
        plan = op.plan_decode(ex["lens"], p.pop("n_kv_heads"), **p)
        assert plan["chunk"] == ex["chunk"]
        for key in ("nsplit", "part_off", "item_b", "item_s", "item_blk_begin", "item_blk_end"):
            assert plan[key].tolist() == ex[key], key


def test_plan_named_workload_figures():
    g = load("plan_worked_examples.json")["named_workloads_seed0"]
    for cfg in (1, 2, 3, 4):
        lens, _ = hw.workload_lengths(cfg, 0)
        plan = op.plan_decode(lens, hw.WORKLOADS[cfg].n_kv_heads, **op.DEFAULTS)
        assert int(((lens + 15) // 16).sum()) == g[str(cfg)]["W"]
        assert plan["chunk"] == g[str(cfg)]["chunk"]
        assert plan["n_items"] == g[str(cfg)]["n_items"]
        assert int(plan["nsplit"].max()) == g[str(cfg)]["max_nsplit"]


def check_plan_invariants(lens, plan, tile_blk, max_split):
    B = len(lens)
    nblk = [(int(n) + 15) // 16 for n in lens]
    assert plan["part_off"][0] == 0 and plan["part_off"][B] == plan["n_items"]
    cover = {b: [] for b in range(B)}
    for i in range(plan["n_items"]):
        b, k = int(plan["item_b"][i]), int(plan["item_s"][i])
        lo, hi = int(plan["item_blk_begin"][i]), int(plan["item_blk_end"][i])
        assert 0 <= lo < hi <= nblk[b]
        assert lo % tile_blk == 0
        cover[b].append((k, lo, hi))
    for b in range(B):
        parts = sorted(cover[b])
        assert [p[0] for p in parts] == list(range(len(parts)))
        assert len(parts) == plan["nsplit"][b] <= max_split
        assert plan["part_off"][b + 1] - plan["part_off"][b] == len(parts)
        assert parts[0][1] == 0 and parts[-1][2] == nblk[b]
        for a, c in zip(parts, parts[1:]):
            assert a[2] == c[1]
        sizes = [p[2] - p[1] for p in parts]
        assert all(s == sizes[0] for s in sizes[:-1]) and sizes[-1] <= sizes[0]
    keys = [(-(int(plan["item_blk_end"][i]) - int(plan["item_blk_begin"][i])), int(plan["item_b"][i]),
             int(plan["item_s"][i])) for i in range(plan["n_items"])]
    assert keys == sorted(keys)


def test_plan_invariants_random_long_tail():
    rng = np.random.default_rng(5)
    for trial in range(300):
        B = int(rng.integers(1, 40))
        lens = np.clip(np.rint(np.exp(rng.normal(np.log(2000), 1.5, B))), 1, 131072).astype(int)
        kw = dict(n_cu=int(rng.integers(1, 300)), wg_per_cu=int(rng.integers(1, 9)),
                  min_chunk_blk=int(rng.integers(1, 40)), tile_blk=int(rng.choice([1, 2, 4, 8])),
                  max_split=int(rng.integers(1, 70)))
        n_kv = int(rng.choice([1, 2, 8]))
        plan = op.plan_decode(lens, n_kv, **kw)
        check_plan_invariants(lens, plan, kw["tile_blk"], kw["max_split"])
        # a trajectory that needs no more than max_split chunks gets no item larger than the chunk
        for i in range(plan["n_items"]):
            b = int(plan["item_b"][i])
            if -(-((int(lens[b]) + 15) // 16) // plan["chunk"]) <= kw["max_split"]:
                assert plan["item_blk_end"][i] - plan["item_blk_begin"][i] <= plan["chunk"]


def test_plan_exhaustive_small():
    for a in range(1, 70, 3):
        for b in range(1, 200, 7):
            lens = [a, b, 200 - b + 1]
            plan = op.plan_decode(lens, 1, n_cu=2, wg_per_cu=3, min_chunk_blk=1, tile_blk=2, max_split=4)
            check_plan_invariants(lens, plan, 2, 4)


def test_stragglers_are_spread():
    lens, _ = hw.workload_lengths(4, 0)
    plan = op.plan_decode(lens, 8, **op.DEFAULTS)
    sizes = (plan["item_blk_end"] - plan["item_blk_begin"]).astype(int)
    # the 13 tail trajectories hold most of the blocks but no single item holds more than a chunk
    assert sizes.max() <= plan["chunk"] < ((lens.max() + 15) // 16) // 4
    assert (plan["nsplit"][-13:] >= 5).all()


def test_append_order_invariants_and_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(50):
        B = int(rng.integers(1, 9))
        L = rng.integers(0, 5000, B)
        C = rng.integers(1, 300, B)
        R = int(rng.choice([16, 32, 64]))
        plan = op.plan_append(L, C, R)
        seen = set()
        for i in range(plan["n_tiles"]):
            b, r0, n, ext = (int(plan[k][i]) for k in ("tile_b", "tile_row0", "tile_rows_n", "tile_extent"))
            assert r0 % R == 0 and 1 <= n <= R and r0 + n <= C[b]
            assert n == R or r0 + n == C[b]
            assert ext == L[b] + r0 + n
            seen.add((b, r0))
        assert len(seen) == plan["n_tiles"] == sum(-(-int(c) // R) for c in C)
        ext = plan["tile_extent"].astype(int)
        assert (np.diff(ext) <= 0).all()
        # ties broken by (b, row0)
        keys = [(-int(e), int(b), int(r)) for e, b, r in zip(ext, plan["tile_b"], plan["tile_row0"])]
        assert keys == sorted(keys)


def test_append_order_hand_example():
    plan = op.plan_append([100, 0], [40, 33], 32)
    # tiles: b0: rows 0-31 (extent 132), rows 32-39 (extent 140); b1: rows 0-31 (32), 32 (33)
    assert plan["tile_b"].tolist() == [0, 0, 1, 1]
    assert plan["tile_row0"].tolist() == [32, 0, 32, 0]
    assert plan["tile_rows_n"].tolist() == [8, 32, 1, 32]
    assert plan["tile_extent"].tolist() == [140, 132, 33, 32]


# ------------------------------------------------------------- block manager

def replay(trace):
    m = KVManager(trace["n_blocks"])
    for op_ in trace["ops"]:
        if op_[0] == "alloc":
            code, ids = m.alloc(op_[1])
            assert (code, ids) == (op_[2], op_[3]), op_
        elif op_[0] == "free":
            assert m.free(op_[1]) == op_[2], op_
        elif op_[0] == "retain":
            assert m.retain(op_[1]) == op_[2], op_
        else:
            assert m.num_free() == op_[1], op_


def test_manager_hand_written_traces():
    for tr in load("kv_manager_traces.json")["traces"]:
        replay(tr)


def test_manager_conservation_random():
    rng = np.random.default_rng(0)
    m = KVManager(50)
    held = []
    for _ in range(2000):
        if rng.random() < 0.5:
            n = int(rng.integers(0, 12))
            before = m.num_free()
            code, ids = m.alloc(n)
            if n > before:
                assert code == -2 and m.num_free() == before
            else:
                assert code == 0 and len(set(ids)) == n and not (set(ids) & set(held))
                held += ids
        elif held:
            k = int(rng.integers(1, len(held) + 1))
            idx = rng.permutation(len(held))[:k]
            ids = [held[i] for i in idx]
            assert m.free(ids) == 0
            held = [h for i, h in enumerate(held) if i not in set(idx.tolist())]
            # most recently freed comes back first
            code, got = m.alloc(1)
            assert got == [ids[-1]]
            held += got
        assert m.num_free() + len(held) == 50


def test_manager_holders_random():
    """With retain in the mix: a block is on the stack exactly when nobody holds it, and a block comes
    back when as many frees as (1 + retains) have named it."""
    rng = np.random.default_rng(3)
    m = KVManager(40)
    count = {}                                   # block -> holders, kept here independently
    for _ in range(3000):
        r = rng.random()
        if r < 0.4:
            code, ids = m.alloc(int(rng.integers(0, 6)))
            if code == 0:
                for i in ids:
                    assert i not in count
                    count[i] = 1
        elif count:
            held = sorted(count)
            k = int(rng.integers(1, len(held) + 1))
            ids = [held[i] for i in rng.permutation(len(held))[:k]]
            if r < 0.6:
                assert m.retain(ids) == 0
                for i in ids:
                    count[i] += 1
            else:
                assert m.free(ids) == 0
                back = [i for i in ids if count[i] == 1]
                for i in ids:
                    count[i] -= 1
                    if count[i] == 0:
                        del count[i]
                if back:                         # the last block that lost its last holder is on top
                    code, got = m.alloc(1)
                    assert code == 0 and got == [back[-1]]
                    count[got[0]] = 1
        assert m.num_free() + len(count) == 40
        assert all(m.is_free[i] == (i not in count) for i in range(40))


# ---------------------------------------------------------------- shared-prefix decode plan
SHARED_KEYS = ("group_leader", "group_prefix", "group_parts", "member_off", "members", "traj_group",
               "traj_prefix", "nsplit", "part_off", "item_b", "item_s", "item_blk_begin", "item_blk_end",
               "gitem_g", "gitem_k", "gitem_blk_begin", "gitem_blk_end", "gitem_m0", "gitem_mn")


def csr(tables):
    row_off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int32)
    ids = np.asarray([x for t in tables for x in t], dtype=np.int32)
    return row_off, ids


def test_shared_plan_hand_worked_examples():
    for ex in load("shared_plan_worked_examples.json")["examples"]:
        row_off, ids = csr(ex["tables"])
        plan = op.plan_decode_shared(ex["lens"], row_off, ids, **ex["params"])
        assert plan["chunk"] == ex["chunk"] and plan["chunk_g"] == ex["chunk_g"]
        for k in SHARED_KEYS:
            assert plan[k].tolist() == ex[k], k


def check_shared_invariants(lens, row_off, ids, plan, tile_members, tile_blk, max_split, min_share_blk):
    """What any valid shared plan must satisfy, whatever rule produced it."""
    B = len(lens)
    nblk = [-(-int(n) // 16) for n in lens]
    covered = [np.zeros(n, dtype=np.int32) for n in nblk]
    slots = [set() for _ in range(B)]
    # private items
    for b, s, lo, hi in zip(plan["item_b"], plan["item_s"], plan["item_blk_begin"], plan["item_blk_end"]):
        assert plan["traj_prefix"][b] <= lo < hi <= nblk[b]
        covered[b][lo:hi] += 1
        assert s not in slots[b]
        slots[b].add(int(s))
    # group items: every member of the tile is covered through the leader's blocks, which it shares
    for g, k, lo, hi, m0, mn in zip(plan["gitem_g"], plan["gitem_k"], plan["gitem_blk_begin"],
                                    plan["gitem_blk_end"], plan["gitem_m0"], plan["gitem_mn"]):
        p = int(plan["group_prefix"][g])
        assert 0 <= lo < hi <= p and lo % tile_blk == 0 and 1 <= mn <= tile_members
        mem = plan["members"][plan["member_off"][g]:plan["member_off"][g + 1]]
        leader = int(plan["group_leader"][g])
        assert mem[0] == leader and list(mem) == sorted(mem)
        for b in mem[m0:m0 + mn]:
            assert plan["traj_group"][b] == g and plan["traj_prefix"][b] == p
            assert p >= min_share_blk and p * 16 <= int(lens[b]) - 1      # never the block of the step's own row
            assert np.array_equal(ids[row_off[b]:row_off[b] + p], ids[row_off[leader]:row_off[leader] + p])
            covered[b][lo:hi] += 1
            slots[b].add(int(k))
    for b in range(B):
        assert (covered[b] == 1).all(), f"trajectory {b}: every block exactly once"
        assert slots[b] == set(range(int(plan["nsplit"][b])))
        assert plan["part_off"][b + 1] - plan["part_off"][b] == plan["nsplit"][b]
        if plan["traj_group"][b] < 0:
            assert plan["traj_prefix"][b] == 0
    for g in range(plan["n_groups"]):
        assert plan["group_parts"][g] <= max_split
        assert plan["member_off"][g + 1] - plan["member_off"][g] >= 2
    d = plan["item_blk_end"] - plan["item_blk_begin"]
    assert (np.diff(d) <= 0).all()
    dg = plan["gitem_blk_end"] - plan["gitem_blk_begin"]
    assert (np.diff(dg) <= 0).all()


def random_shared_tables(rng, B, n_groups, max_len):
    """Block tables in which random subsets of trajectories share random numbers of leading
    blocks (sometimes diverging early, sometimes sharing only the first id)."""
    lens = rng.integers(1, max_len, B)
    nblk = -(-lens // 16)
    next_id = [1000]

    def fresh(n):
        out = list(range(next_id[0], next_id[0] + n))
        next_id[0] += n
        return out

    prompts = [fresh(int(rng.integers(1, max_len // 16 + 2))) for _ in range(n_groups)]
    tables = []
    for b in range(B):
        g = int(rng.integers(-1, n_groups))
        if g < 0:
            tables.append(fresh(int(nblk[b])))
            continue
        share = int(rng.integers(1, len(prompts[g]) + 1))
        share = min(share, (int(lens[b]) - 1) // 16 + int(rng.integers(0, 2)), int(nblk[b]))   # sometimes one too many
        tables.append(prompts[g][:share] + fresh(int(nblk[b]) - share))
    return lens.astype(np.int32), tables


def test_shared_plan_invariants_random():
    rng = np.random.default_rng(77)
    for trial in range(60):
        B = int(rng.integers(1, 40))
        lens, tables = random_shared_tables(rng, B, int(rng.integers(1, 5)), int(rng.choice([64, 400, 3000])))
        row_off, ids = csr(tables)
        prm = dict(n_kv_heads=int(rng.choice([1, 2, 8])), tile_members=int(rng.choice([2, 16, 32])),
                   n_cu=int(rng.choice([2, 16, 256])), wg_per_cu=int(rng.integers(1, 5)),
                   min_chunk_blk=int(rng.choice([1, 4, 16])), tile_blk=int(rng.choice([1, 2, 4])),
                   max_split=int(rng.choice([2, 8, 64])), min_share_blk=int(rng.choice([1, 2, 4])),
                   group_wg_per_cu=int(rng.integers(1, 3)))
        plan = op.plan_decode_shared(lens, row_off, ids, **prm)
        check_shared_invariants(lens, row_off, ids, plan, prm["tile_members"], prm["tile_blk"], prm["max_split"],
                                prm["min_share_blk"])
        # prefixes that must end at multiples of 4 blocks (a kernel that starts at multiples of 64 keys reads
        # the private blocks): still a valid plan, every prefix a multiple of 4, and with tile_blk = 4
        # every private item starts at a multiple of 4.  (A prefix may come out longer than without the
        # constraint: a member that shared fewer than 4 blocks no longer joins and no longer shortens it.)
        prm4 = dict(prm, tile_blk=4, prefix_align=4)
        plan4 = op.plan_decode_shared(lens, row_off, ids, **prm4)
        check_shared_invariants(lens, row_off, ids, plan4, prm["tile_members"], 4, prm["max_split"], prm["min_share_blk"])
        assert (plan4["group_prefix"] % 4 == 0).all() and (plan4["item_blk_begin"] % 4 == 0).all()


def test_shared_plan_without_sharing_is_the_plain_plan():
    rng = np.random.default_rng(5)
    lens = rng.integers(1, 9000, 30).astype(np.int32)
    tables = []
    nxt = 0
    for n in lens:
        k = -(-int(n) // 16)
        tables.append(list(range(nxt, nxt + k)))
        nxt += k
    row_off, ids = csr(tables)
    a = op.plan_decode(lens, 8)
    b = op.plan_decode_shared(lens, row_off, ids, 8, 32)
    assert b["n_groups"] == 0 and b["n_gitems"] == 0 and a["chunk"] == b["chunk"]
    for k in ("item_b", "item_s", "item_blk_begin", "item_blk_end", "nsplit", "part_off"):
        assert np.array_equal(a[k], b[k]), k


def test_shared_plan_named_workload():
    """Workload 6: the 8 prompts are found with exactly their whole shared blocks, 16 members each."""
    lens, group_of, prompt = hw.draw_group_lengths(np.random.default_rng([6, 0]))
    # tables with sharing, built here from the definition (ids need not be permuted for the plan)
    tables, nxt = [], 10_000
    for b in range(len(lens)):
        p = int(prompt[group_of[b]]) // 16
        n = -(-int(lens[b]) // 16)
        tables.append([int(group_of[b]) * 1000 + i for i in range(p)] + list(range(nxt, nxt + n - p)))
        nxt += n - p
    row_off, ids = csr(tables)
    plan = op.plan_decode_shared(lens, row_off, ids, 8, 32)
    assert plan["n_groups"] == 8
    assert sorted(plan["group_prefix"].tolist()) == sorted((prompt // 16).tolist())
    assert (np.diff(plan["member_off"]) == 16).all()
    check_shared_invariants(lens, row_off, ids, plan, 32, 4, 64, 4)


# ------------------------------------------------------------- split-K of small append batches

def test_append_split_hand_example():
    # one trajectory, L = 1000, C = 5, tile height 32: one tile, extent 1005 -> S = 16 steps.
    # n_kv = 2, n_cu = 4, 2 per CU: slots 8 > 1*2 tiles -> split.  W = 16, target = 8 // 2 = 4,
    # chunk = max(ceil(16/4), 2) = 4; ns = 4, per = 4, n = 4; last part starts at key 3*4*64 = 768
    # <= 1000 -> stays 4.  Slots: 5 rows * 4 parts = 20.
    plan = op.plan_append([1000], [5], 32)
    sp = op.split_append_tiles(plan, [1000], 2, n_cu=4, append_wg_per_cu=2, min_steps=2, max_split=8)
    assert sp["tile_nsplit"].tolist() == [4] and sp["tile_part_base"].tolist() == [0] and sp["n_slots"] == 20
    assert sp["item_k"].tolist() == [0, 1, 2, 3]
    assert sp["item_step_begin"].tolist() == [0, 4, 8, 12] and sp["item_step_end"].tolist() == [4, 8, 12, 16]
    # L = 60, C = 100 (tile rows 0-31: extent 92 -> 2 steps; rows 32-63: extent 124 -> 2; 64-95: 156 -> 3;
    # 96-99: extent 160 -> 3 steps).  With chunk 1 the tile of rows 0-31 would get 2 parts, the second
    # starting at key 64 > L + row0 = 60: merged back into one; rows 64-95 would get 3, the third
    # starting at key 128 > 124: two.
    plan = op.plan_append([60], [100], 32)
    sp = op.split_append_tiles(plan, [60], 1, n_cu=64, append_wg_per_cu=2, min_steps=1, max_split=8)
    by_row0 = {int(r): int(n) for r, n in zip(plan["tile_row0"], sp["tile_nsplit"])}
    assert by_row0 == {0: 1, 32: 2, 64: 2, 96: 3}
    # L = 31, C = 106 in one tile of 128 rows: extent 137 -> S = 3 steps.  n_kv = 2, 256 CUs x 4: target 512,
    # chunk = max(ceil(3/512), 1) = 1; ns = 3, per = 1, n = 3.  The first row sees keys 0..31 only: the third
    # part would start at key 128, the second at key 64, both behind it -> n = 3 -> 2 -> 1, the tile stays whole.
    plan = op.plan_append([31], [106], 128)
    sp = op.split_append_tiles(plan, [31], 2, n_cu=256, append_wg_per_cu=4, min_steps=1)
    assert sp["tile_nsplit"].tolist() == [1] and sp["n_slots"] == 0
    assert sp["item_step_begin"].tolist() == [0] and sp["item_step_end"].tolist() == [3]
    # the same tile behind L = 70: the first row sees keys 0..70, the second part (from key 64) stays, the
    # third (from key 128) is merged into it
    plan = op.plan_append([70], [106], 128)
    sp = op.split_append_tiles(plan, [70], 2, n_cu=256, append_wg_per_cu=4, min_steps=1)
    assert sp["tile_nsplit"].tolist() == [2] and sp["n_slots"] == 2 * 106
    assert sorted(zip(sp["item_step_begin"].tolist(), sp["item_step_end"].tolist())) == [(0, 1), (1, 3)]


def test_append_split_invariants():
    rng = np.random.default_rng(21)
    for trial in range(400):
        B = int(rng.integers(1, 6))
        L = rng.integers(0, int(rng.choice([40, 300, 20000])), B)      # short contexts under tall tiles included
        C = rng.integers(1, int(rng.choice([70, 400])), B)
        R = int(rng.choice([16, 32, 128]))
        n_kv = int(rng.choice([1, 2, 8]))
        prm = dict(n_cu=int(rng.choice([4, 64, 256])), append_wg_per_cu=int(rng.integers(1, 5)),
                   min_steps=int(rng.choice([1, 2, 4, 8])), max_split=int(rng.choice([2, 16, 64])))
        plan = op.plan_append(L, C, R)
        sp = op.split_append_tiles(plan, L, n_kv, **prm)
        used = np.zeros(sp["n_slots"], dtype=np.int32)
        for t in range(plan["n_tiles"]):
            S = -(-int(plan["tile_extent"][t]) // 64)
            n = int(sp["tile_nsplit"][t])
            assert 1 <= n <= prm["max_split"]
            parts = sorted((int(k), int(lo), int(hi)) for tt, k, lo, hi in
                           zip(sp["item_tile"], sp["item_k"], sp["item_step_begin"], sp["item_step_end"]) if tt == t)
            assert [p[0] for p in parts] == list(range(n))
            assert parts[0][1] == 0 and parts[-1][2] == S
            assert all(parts[i][2] == parts[i + 1][1] and parts[i][1] < parts[i][2] for i in range(n - 1))
            # the first row of the tile sees at least one key of every part
            assert parts[-1][1] * 64 <= int(L[plan["tile_b"][t]]) + int(plan["tile_row0"][t])
            if n > 1:
                rows = int(plan["tile_rows_n"][t])
                used[sp["tile_part_base"][t]: sp["tile_part_base"][t] + rows * n] += 1
        assert (used == 1).all()
        d = sp["item_step_end"] - sp["item_step_begin"]
        assert (np.diff(d) <= 0).all()


def test_append_split_spreads_stragglers_only():
    # many equal tiles: an even share each, nothing to split
    plan = op.plan_append([4000] * 200, [32] * 200, 32)
    sp = op.split_append_tiles(plan, [4000] * 200, 8)
    assert (sp["tile_nsplit"] == 1).all() and sp["n_slots"] == 0
    # the large append workload: only tiles far above the average are cut, into a few parts
    L, C = hw.workload_lengths(5, 0)
    plan = op.plan_append(L, C, 32)
    sp = op.split_append_tiles(plan, L, 8)
    assert sp["tile_nsplit"].max() <= 4 and (sp["tile_nsplit"] == 1).sum() > plan["n_tiles"] // 2
    plan = op.plan_append([120000], [8], 32)
    sp = op.split_append_tiles(plan, [120000], 8)
    assert sp["tile_nsplit"][0] >= 32           # one tile x 8 kv heads alone would use 8 of 512 slots


def test_shared_plan_prefix_alignment_hand_example():
    """Worked by hand.  Tables (block ids): trajectories 0-2 begin with the same 21 blocks 100..120,
    trajectory 3 with the first 3 of them only, trajectories 4-5 with the same 7 blocks 200..206; every
    length leaves those blocks wholly before the step's own row.  With prefix_align = 4 the common
    prefixes 21 and 7 are used as 20 and 4; trajectory 3 (3 common blocks -> 0) stays alone, and with it
    out of the way group 0's prefix is 20 (without alignment its lcp of 3 < min_share_blk = 4 would have
    kept it out as well, and the prefix would be 21)."""
    def own(n, base):
        return list(range(base, base + n))
    tables = [own(21, 100) + own(2, 1000), own(21, 100) + own(9, 1100), own(21, 100) + own(1, 1200),
              own(3, 100) + own(30, 1300), own(7, 200) + own(1, 1400), own(7, 200) + own(5, 1500)]
    lens = [16 * 22 + 3, 16 * 29 + 16, 16 * 21 + 1, 16 * 32 + 7, 16 * 7 + 2, 16 * 11 + 9]
    row_off, ids = csr(tables)
    free = op.plan_decode_shared(lens, row_off, ids, 2, 25, n_cu=4, wg_per_cu=2)
    assert free["group_prefix"].tolist() == [21, 7] and free["traj_prefix"].tolist() == [21, 21, 21, 0, 7, 7]
    plan = op.plan_decode_shared(lens, row_off, ids, 2, 25, n_cu=4, wg_per_cu=2, prefix_align=4)
    assert plan["n_groups"] == 2 and plan["group_prefix"].tolist() == [20, 4]
    assert plan["traj_prefix"].tolist() == [20, 20, 20, 0, 4, 4]
    assert plan["members"].tolist() == [0, 1, 2, 4, 5]
    # private work W = (23-20) + (30-20) + (22-20) + 33 + (8-4) + (12-4) = 60 blocks; target = 4*2/2 = 4;
    # chunk = max(ceil(60/4), 16) = 16; trajectory 3 (33 blocks): ns = 3, per = ceil(33/3) = 11 -> 12,
    # parts [0,12) [12,24) [24,33); everybody else one private part starting at the prefix
    assert plan["chunk"] == 16
    t3 = [(int(lo), int(hi)) for b, lo, hi in zip(plan["item_b"], plan["item_blk_begin"], plan["item_blk_end"]) if b == 3]
    assert sorted(t3) == [(0, 12), (12, 24), (24, 33)]
    starts = {int(b): int(lo) for b, lo in zip(plan["item_b"], plan["item_blk_begin"]) if b != 3}
    assert starts == {0: 20, 1: 20, 2: 20, 4: 4, 5: 4}
    check_shared_invariants(lens, row_off, ids, plan, 25, 4, 64, 4)
