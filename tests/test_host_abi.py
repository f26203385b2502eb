"""Host side of the C ABI (no GPU): symbols, block manager, planners, error paths.

The C++ planner and block manager are compared bit for bit with the oracle's."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

import heddle_workloads as hw
import paper_2603_28101_amd as heddle
from oracle import planner as op
from oracle.kv_manager import KVManager

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["heddle.h", "heddle_debug.h"]
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in headers)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(heddle_[a-z_]+)\s*\(", text)))
    assert {"heddle_kv_alloc", "heddle_kv_free", "heddle_attn_decode", "heddle_attn_append",
            "heddle_plan_decode", "heddle_ctx_create", "heddle_ctx_reserve", "heddle_attn_decode_static",
            "heddle_timing_enable", "heddle_stream_read"} <= set(names)
    lib = ctypes.CDLL(heddle.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    assert lib.heddle_version() >= 1


def host_ctx(n_q=32, n_kv=8, d=128, n_blocks=64, **kw):
    return heddle.Context(n_q, n_kv, d, n_blocks, **kw)


def test_strerror_and_create_errors():
    assert heddle.lib.heddle_strerror(0) == b"ok"
    assert b"invalid" in heddle.lib.heddle_strerror(heddle.E_INVAL)
    for bad in (dict(n_q=6, n_kv=4), dict(n_blocks=0), dict(d=7)):
        with pytest.raises(heddle.HeddleError) as e:
            host_ctx(**bad)
        assert e.value.code == heddle.E_INVAL
    with pytest.raises(heddle.HeddleError):     # device context without a pool
        heddle.Context(8, 2, 64, 4, kv_pool=None, device=0)


def test_attention_on_host_only_context_is_refused():
    c = host_ctx()
    with pytest.raises(heddle.HeddleError) as e:
        c.attn_decode([5], [0, 1], 0x1000, 0x1000, 0x1000, 0x1000, stream=0)
    assert e.value.code == heddle.E_UNSUPPORTED


# ------------------------------------------------------------- block manager

def test_manager_golden_traces_on_library():
    traces = json.load(open(os.path.join(GOLDEN, "kv_manager_traces.json")))["traces"]
    for tr in traces:
        c = host_ctx(n_blocks=tr["n_blocks"])
        for o in tr["ops"]:
            if o[0] == "alloc":
                if o[2] == 0:
                    assert c.kv_alloc(o[1]).tolist() == o[3], o
                else:
                    with pytest.raises(heddle.HeddleError) as e:
                        c.kv_alloc(o[1])
                    assert e.value.code == o[2], o
            elif o[0] in ("free", "retain"):
                call = c.kv_free if o[0] == "free" else c.kv_retain
                if o[2] == 0:
                    call(o[1])
                else:
                    with pytest.raises(heddle.HeddleError) as e:
                        call(o[1])
                    assert e.value.code == o[2], o
            else:
                assert c.kv_num_free() == o[1], o


def test_manager_random_scripts_match_oracle():
    rng = np.random.default_rng(1)
    for trial in range(20):
        n = int(rng.integers(1, 200))
        c, m = host_ctx(n_blocks=n), KVManager(n)
        held = []
        for step in range(400):
            r = rng.random()
            if r < 0.45:
                k = int(rng.integers(0, n // 2 + 2))
                code, ids = m.alloc(k)
                try:
                    got = c.kv_alloc(k).tolist()
                    assert code == 0 and got == ids
                    held += ids
                except heddle.HeddleError as e:
                    assert e.code == code != 0
            elif r < 0.9 and held:
                distinct = sorted(set(held))
                k = int(rng.integers(1, len(distinct) + 1))
                idx = rng.permutation(len(distinct))[:k].tolist()
                ids = [distinct[i] for i in idx]
                if rng.random() < 0.15:          # corrupt: duplicate / foreign / out of range
                    ids = ids + [ids[0]] if rng.random() < 0.5 else ids + [int(rng.integers(-3, n + 3))]
                retain = rng.random() < 0.3      # one more holder, or one fewer
                code = m.retain(ids) if retain else m.free(ids)
                try:
                    (c.kv_retain if retain else c.kv_free)(ids)
                    assert code == 0
                    for i in ids:                # `held` lists a block once per holder
                        held.append(i) if retain else held.remove(i)
                except heddle.HeddleError as e:
                    assert e.code == code != 0
            assert c.kv_num_free() == m.num_free()


# ------------------------------------------------------------------ planners

def same_plan(a, b):
    assert a["chunk"] == b["chunk"] and a["n_items"] == b["n_items"]
    for k in ("item_b", "item_s", "item_blk_begin", "item_blk_end", "nsplit", "part_off"):
        assert np.array_equal(a[k], b[k]), k
        assert a[k].dtype == np.int32


def test_plan_golden_examples_on_library():
    for ex in json.load(open(os.path.join(GOLDEN, "plan_worked_examples.json")))["examples"]:
        p = dict(ex["params"])
        c = heddle.Context(p["n_kv_heads"], p["n_kv_heads"], 128, 4, n_cu=p["n_cu"], wg_per_cu=p["wg_per_cu"],
                           min_chunk_blk=p["min_chunk_blk"], tile_blk=p["tile_blk"], max_split=p["max_split"])
        plan = c.plan_decode(ex["lens"])
        assert plan["chunk"] == ex["chunk"]
        for key in ("nsplit", "part_off", "item_b", "item_s", "item_blk_begin", "item_blk_end"):
            assert plan[key].tolist() == ex[key], key


def test_plan_named_workloads_match_oracle():
    for cfg in (1, 2, 3, 4):
        w = hw.WORKLOADS[cfg]
        for seed in (0, 1, 2):
            lens, _ = hw.workload_lengths(cfg, seed)
            c = host_ctx(w.n_q_heads, w.n_kv_heads, w.head_dim, n_cu=256)
            same_plan(c.plan_decode(lens), op.plan_decode(lens, w.n_kv_heads, **op.DEFAULTS))


def test_plan_exhaustive_small_matches_oracle():
    kw = dict(n_cu=2, wg_per_cu=3, min_chunk_blk=1, tile_blk=2, max_split=4)
    c = heddle.Context(1, 1, 64, 4, **kw)
    for a in range(1, 201, 9):
        for b in range(1, 201, 5):
            for d in (1, 16, 17, 200):
                lens = [a, b, d]
                same_plan(c.plan_decode(lens), op.plan_decode(lens, 1, **kw))


def test_plan_random_long_tail_matches_oracle():
    rng = np.random.default_rng(7)
    for trial in range(400):
        B = int(rng.integers(1, 300))
        lens = np.clip(np.rint(np.exp(rng.normal(np.log(3000), 1.4, B))), 1, 131072).astype(np.int64)
        kw = dict(n_cu=int(rng.integers(1, 400)), wg_per_cu=int(rng.integers(1, 9)),
                  min_chunk_blk=int(rng.integers(1, 64)), tile_blk=int(rng.choice([1, 2, 4, 8])),
                  max_split=int(rng.integers(1, 80)))
        n_kv = int(rng.choice([1, 2, 4, 8]))
        c = heddle.Context(n_kv, n_kv, 128, 4, **kw)
        same_plan(c.plan_decode(lens), op.plan_decode(lens, n_kv, **kw))


def test_plan_errors():
    c = host_ctx()
    for lens in ([0], [5, -1], [131073]):
        with pytest.raises(heddle.HeddleError) as e:
            c.plan_decode(lens)
        assert e.value.code == heddle.E_INVAL
    c.plan_decode([131072])


def test_append_order_matches_oracle():
    rng = np.random.default_rng(9)
    c = host_ctx()
    for trial in range(100):
        B = int(rng.integers(1, 40))
        L = rng.integers(0, 60000, B)
        Cn = rng.integers(1, 1025, B)
        cu = np.concatenate([[0], np.cumsum(Cn)])
        R = int(rng.choice([16, 32, 64]))
        a, b = c.plan_append(L, cu, R), op.plan_append(L, Cn, R)
        assert a["n_tiles"] == b["n_tiles"] and a["tile_rows"] == R
        for k in ("tile_b", "tile_row0", "tile_rows_n", "tile_extent"):
            assert np.array_equal(a[k], b[k]), k
    # default tile height: 128 MFMA rows shared by the G heads of a group
    assert c.plan_append([10], [0, 100])["tile_rows"] == 32
    with pytest.raises(heddle.HeddleError):
        c.plan_append([10], [0, 0], 32)          # empty chunk
    with pytest.raises(heddle.HeddleError):
        c.plan_append([-1], [0, 4], 32)


# ------------------------------------------------------------------ shared-prefix decode plan

def test_shared_plan_matches_oracle_on_random_tables():
    from tests.test_oracle_planner import SHARED_KEYS, csr, random_shared_tables
    rng = np.random.default_rng(123)
    for trial in range(80):
        B = int(rng.integers(1, 90))
        lens, tables = random_shared_tables(rng, B, int(rng.integers(1, 4)), int(rng.choice([64, 400, 3000])))
        row_off, ids = csr(tables)
        G = int(rng.choice([1, 2, 4, 8, 3, 5, 6, 7, 12]))
        n_kv = int(rng.choice([1, 2, 8]))
        prm = dict(n_cu=int(rng.choice([2, 16, 256])), wg_per_cu=int(rng.integers(1, 5)),
                   min_chunk_blk=int(rng.choice([1, 4, 16])), tile_blk=int(rng.choice([1, 2, 4])),
                   max_split=int(rng.choice([2, 8, 64])), min_share_blk=int(rng.choice([1, 2, 4])),
                   group_wg_per_cu=int(rng.integers(1, 3)))
        c = heddle.Context(n_kv * G, n_kv, 128, 4, **prm)
        got = c.plan_decode_shared(lens, row_off, ids)
        oracle_prm = dict(prm)
        if G not in (1, 2, 4, 8):
            # the private blocks of such head shapes are read by a kernel that starts at multiples of 4
            # blocks: prefixes end there, and a plan whose parts need not start there forms no group
            oracle_prm["prefix_align"] = 4
            if prm["tile_blk"] % 4 != 0:
                oracle_prm["min_share_blk"] = 2 ** 31 - 1
        elif G == 8 and prm["tile_blk"] % 4 == 0:
            # 8 query heads per kv head decode on that kernel too when the plan is on its 64-key grid
            oracle_prm["prefix_align"] = 4
        ref = op.plan_decode_shared(lens, row_off, ids, n_kv, 128 // G, **oracle_prm)
        assert (got["chunk"], got["chunk_g"], got["n_groups"]) == (ref["chunk"], ref["chunk_g"], ref["n_groups"])
        for k in SHARED_KEYS:
            assert np.array_equal(got[k][: len(ref[k])], ref[k]), (trial, k)


def test_shared_plan_on_unsupported_head_dim_forms_no_groups():
    from tests.test_oracle_planner import csr
    tables = [[1, 2, 3, 4, 5, 6, 10], [1, 2, 3, 4, 5, 6, 11]]
    row_off, ids = csr(tables)
    c = heddle.Context(8, 2, 32, 32)          # host-only context; no kernel is built for head_dim 32
    plan = c.plan_decode_shared([100, 100], row_off, ids)
    assert plan["n_groups"] == 0 and plan["n_gitems"] == 0
    same_plan({**c.plan_decode([100, 100])}, {**plan, "n_items": plan["n_items"]})


def test_shared_plan_errors():
    from tests.test_oracle_planner import csr
    row_off, ids = csr([[1, 2], [1, 3]])
    c = host_ctx()
    with pytest.raises(heddle.HeddleError):
        c.plan_decode_shared([0, 20], row_off, ids)            # length < 1
    with pytest.raises(heddle.HeddleError):
        c.plan_decode_shared([40, 20], row_off, ids)           # table row too short


def test_ids_outside_the_pool_behind_the_needed_blocks_never_reach_a_work_item():
    """A table row may be longer than its trajectory needs; the entries behind the needed blocks may
    be anything (-1, INT32_MAX, an id just past the pool).  The work items the library builds from
    the lengths name logical blocks below ceil(len/16) only, and the group search compares needed
    entries only: the plans are those of the exact table, in both the library and the oracle."""
    from tests.test_oracle_planner import SHARED_KEYS, csr
    lens = np.array([330, 500, 421, 17, 2100], dtype=np.int32)
    need = [-(-int(n) // 16) for n in lens]
    prompt = list(range(100, 120))                        # trajectories 0-2 share 20 blocks
    nxt = iter(range(200, 1000))
    rows = [(prompt if b < 3 else []) + [next(nxt) for _ in range(need[b] - (20 if b < 3 else 0))] for b in range(5)]
    junk = [-1, 2 ** 31 - 1, 1000, -(2 ** 31)]
    padded = [r + junk[: 1 + b % 4] for b, r in enumerate(rows)]
    for G in (4, 5):
        c = heddle.Context(2 * G, 2, 128, 1000, n_cu=8)
        exact_off, exact_ids = csr(rows)
        pad_off, pad_ids = csr(padded)
        exact = c.plan_decode_shared(lens, exact_off, exact_ids)
        dirty = c.plan_decode_shared(lens, pad_off, pad_ids)
        assert exact["n_groups"] == 1 and dirty["n_groups"] == 1
        for k in SHARED_KEYS:
            assert np.array_equal(exact[k], dirty[k]), k
        assert (dirty["item_blk_end"] <= np.asarray(need)[dirty["item_b"]]).all()
        assert (dirty["gitem_blk_end"] <= dirty["group_prefix"][dirty["gitem_g"]]).all()
        assert (dirty["group_prefix"] <= (lens[dirty["group_leader"]] - 1) // 16).all()
        kw = dict(prefix_align=4) if G == 5 else {}
        ref = op.plan_decode_shared(lens, pad_off, pad_ids, 2, 128 // G, n_cu=8, **kw)
        for k in SHARED_KEYS:
            assert np.array_equal(dirty[k][: len(ref[k])], ref[k]), k
        plain = c.plan_decode(lens)
        assert (plain["item_blk_end"] <= np.asarray(need)[plain["item_b"]]).all()
        tiles = c.plan_append(lens - 3, np.arange(6, dtype=np.int32) * 3)
        assert (tiles["tile_extent"] <= lens[tiles["tile_b"]]).all()


# ------------------------------------------------------------------ placement (Sec. 5.2)

def test_placement_golden_examples_on_library():
    for ex in json.load(open(os.path.join(GOLDEN, "placement_worked_examples.json")))["examples"]:
        for full_scan in (False, True):
            mk, sizes = heddle.placement_dp(ex["lengths"], ex["m"], ex["F"], ex["T"], full_scan=full_scan)
            assert mk == ex["makespan"] and sizes.tolist() == ex["sizes"]


def test_placement_matches_oracle_bit_for_bit():
    from oracle import placement as pl
    rng = np.random.default_rng(11)
    for trial in range(120):
        n, m = int(rng.integers(0, 60)), int(rng.integers(1, 12))
        kind = trial % 4
        if kind == 0:       # many ties: few distinct lengths, flat stretches in F
            L = sorted(rng.choice([5, 9, 9, 30], n).tolist(), reverse=True)
            F = np.concatenate([[0.0], 1.0 + np.cumsum(rng.choice([0.0, 0.0, 0.5], max(n, 1)))])
        elif kind == 1:     # long tail, smooth F
            L = sorted(rng.lognormal(7, 1.2, n).tolist(), reverse=True)
            F = np.concatenate([[0.0], 1.0 + np.cumsum(rng.uniform(0, 0.3, max(n, 1)))])
        elif kind == 2:     # F that is not monotone: the library must fall back to the full scan
            L = sorted(rng.integers(1, 500, n).tolist(), reverse=True)
            F = np.concatenate([[0.0], rng.uniform(0.5, 3.0, max(n, 1))])
        else:               # bundled elements
            L = sorted(rng.integers(1, 500, n).tolist(), reverse=True)
            F = np.concatenate([[0.0], 1.0 + np.cumsum(rng.uniform(0, 0.3, 4 * max(n, 1)))])
        counts = rng.integers(1, 5, n).tolist() if kind == 3 else None
        T = float(rng.uniform(0.1, 3.0))
        ref_mk, ref_sizes = pl.placement_dp(L, m, F.tolist(), T, counts)
        for full_scan in (False, True):
            mk, sizes = heddle.placement_dp(L, m, F, T, counts, full_scan=full_scan)
            assert mk == ref_mk and sizes.tolist() == ref_sizes, (trial, full_scan)


def test_placement_helpers_match_oracle():
    from oracle import placement as pl
    rng = np.random.default_rng(12)
    for trial in range(40):
        n = int(rng.integers(0, 40))
        L = sorted(rng.integers(1, 100, n).tolist(), reverse=True)
        thr, bundle = int(rng.integers(0, 100)), int(rng.integers(0, 6))
        f, c = heddle.placement_aggregate(L, thr, bundle)
        rf, rc = pl.aggregate_short(L, thr, bundle)
        assert f.tolist() == rf and c.tolist() == rc
        k = int(rng.integers(1, 6))
        bs = np.cumsum(rng.integers(1, 9, k)).astype(float)
        ts = rng.uniform(1.0, 50.0, k)
        assert heddle.interference_table(bs, ts, 70).tolist() == pl.interference_table(bs, ts, 70)
        lens = rng.integers(0, 300, n)
        assert heddle.simulate_group(lens, bs, ts) == pl.simulate_group(lens, bs, ts)


def test_placement_errors():
    F = [0.0, 1.0, 2.0, 3.0]
    with pytest.raises(heddle.HeddleError):
        heddle.placement_dp([1, 2, 3], 2, F)                 # ascending
    with pytest.raises(heddle.HeddleError):
        heddle.placement_dp([3, 2, 1], 0, F)                 # no worker
    with pytest.raises(heddle.HeddleError):
        heddle.placement_dp([3, 2, 1], 2, F[:3])             # F does not reach size 3
    with pytest.raises(heddle.HeddleError):
        heddle.placement_dp([3, 2, 1], 2, F, counts=[1, 0, 1])
    with pytest.raises(heddle.HeddleError):
        heddle.interference_table([2, 2], [1.0, 2.0], 4)


# ------------------------------------------------------------------ split-K of small append batches

def test_append_split_matches_oracle():
    rng = np.random.default_rng(31)
    for trial in range(300):
        B = int(rng.integers(1, 6))
        L = rng.integers(0, int(rng.choice([40, 300, 20000])), B).astype(np.int32)   # short contexts under tall tiles too
        Cn = rng.integers(1, int(rng.choice([70, 400])), B)
        cu = np.concatenate([[0], np.cumsum(Cn)]).astype(np.int32)
        G = int(rng.choice([1, 4, 8]))
        n_kv = int(rng.choice([1, 2, 8]))
        prm = dict(n_cu=int(rng.choice([4, 64, 256])), append_wg_per_cu=int(rng.integers(1, 5)),
                   append_min_steps=int(rng.choice([1, 2, 4, 8])), max_split=int(rng.choice([2, 16, 64])))
        c = heddle.Context(n_kv * G, n_kv, 128, 4, **prm)
        got = c.plan_append_split(L, cu)
        plan = op.plan_append(L, Cn, 128 // G)
        ref = op.split_append_tiles(plan, L, n_kv, n_cu=prm["n_cu"], append_wg_per_cu=prm["append_wg_per_cu"],
                                    min_steps=prm["append_min_steps"], max_split=prm["max_split"])
        assert got["n_slots"] == ref["n_slots"] and got["n_items"] == ref["n_items"]
        for k in ("tile_b", "tile_row0", "tile_rows_n", "tile_extent"):
            assert np.array_equal(got[k], plan[k]), k
        for k in ("tile_nsplit", "tile_part_base", "item_tile", "item_k", "item_step_begin", "item_step_end"):
            assert np.array_equal(got[k], ref[k]), (trial, k)


def test_plain_c_client_compiles_links_and_runs(tmp_path):
    """heddle.h is a C header: a C99 program (strict warnings) links against the library and gets the
    hand-worked plan and the block ids the stack rule gives."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "c_abi_client")
    libdir = os.path.dirname(heddle.lib_path())
    cmd = [cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, "-L", libdir, "-lheddle",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert ran.returncode == 0 and ran.stdout.strip() == "ok", ran.stdout + ran.stderr


def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    """Block manager, planners and placement, built from the library's own sources with
    -fsanitize=address,undefined, driven with random and extreme inputs (tests/host_sanitize.cpp)."""
    import shutil
    import subprocess
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    csrc = os.path.join(ROOT, "paper_2603_28101_amd", "csrc")
    exe = str(tmp_path / "host_sanitize")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-D_GLIBCXX_ASSERTIONS", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host_sanitize.cpp")]
    cmd += [os.path.join(csrc, f) for f in ("host_manager.cpp", "host_planner.cpp", "host_placement.cpp")]
    built = subprocess.run(cmd + ["-o", exe], capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-3000:]
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    if ran.returncode != 0 and ("ASan runtime does not come first" in ran.stderr or "Shadow memory" in ran.stderr):
        pytest.skip("the sanitizer runtime cannot start in this environment")
    assert ran.returncode == 0 and ran.stdout.strip().endswith("ok"), (ran.stdout + ran.stderr)[-3000:]
