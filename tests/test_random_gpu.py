"""Seeded random batches through decode, append and shared-prefix decode against the float64 oracle:
head shapes, batch sizes, length mixes (many tiny, a few long, lengths on and next to block, tile
and chunk boundaries) and planner parameters are drawn per seed, so that combinations nobody
wrote down by hand are exercised too.  Every case prints its draw before it runs.  Needs the GPU."""
import os

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, bf16_to_host_bits, bits_to_f64, torch_mod)

pytestmark = pytest.mark.gpu

# more seeds per test for an occasional longer run: HEDDLE_RANDOM_CASES=100 python -m pytest tests/test_random_gpu.py
# (HEDDLE_RANDOM_FIRST=1000 starts them at seed 1000)
EXTRA = int(os.environ.get("HEDDLE_RANDOM_CASES", "0"))
FIRST = int(os.environ.get("HEDDLE_RANDOM_FIRST", "0"))


def seeds(default):
    return range(FIRST, FIRST + max(default, EXTRA))

HEAD_SHAPES = [(1, 1, 128), (2, 2, 64), (2, 1, 128), (4, 1, 128), (8, 2, 128), (8, 1, 128), (16, 2, 128),
               (16, 4, 64), (32, 8, 128), (8, 8, 64), (6, 3, 128), (10, 2, 128), (40, 8, 128), (6, 2, 128),
               (14, 2, 128), (24, 2, 128), (32, 1, 128)]
POW2 = (1, 2, 4, 8)
EDGE_LENGTHS = np.array([1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513,
                         1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097])


def draw_lengths(rng, n, longest):
    """A long-tailed mix: mostly short, some on boundaries, a few long."""
    kind = rng.integers(0, 4, n)
    out = np.empty(n, dtype=np.int64)
    out[kind == 0] = rng.integers(1, 40, int((kind == 0).sum()))
    out[kind == 1] = rng.choice(EDGE_LENGTHS, int((kind == 1).sum()))
    out[kind == 2] = np.clip(np.rint(np.exp(rng.normal(np.log(300), 1.0, int((kind == 2).sum())))), 1, longest)
    out[kind == 3] = rng.integers(longest // 2, longest + 1, int((kind == 3).sum()))
    return np.minimum(out, longest).astype(np.int32)


def draw_plan_kw(rng):
    if rng.integers(0, 3) == 0:
        return {}
    return dict(n_cu=int(rng.choice([1, 4, 16, 64, 256])), wg_per_cu=int(rng.choice([1, 2, 4, 8])),
                min_chunk_blk=int(rng.choice([1, 4, 16, 32])), tile_blk=int(rng.choice([1, 4, 8])),
                max_split=int(rng.choice([1, 2, 5, 64])))


@pytest.mark.parametrize("seed", seeds(12))
def test_random_decode(seed):
    rng = np.random.default_rng([101, seed])
    n_q, n_kv, d = HEAD_SHAPES[int(rng.integers(0, len(HEAD_SHAPES)))]
    B = int(rng.integers(1, 33))
    lens = draw_lengths(rng, B, int(rng.choice([300, 3000, 9000])))
    kw = draw_plan_kw(rng)
    if n_q // n_kv not in POW2 and kw:
        kw["tile_blk"] = 4 * int(rng.integers(1, 3))          # the matrix-core kernel cuts keys at multiples of 64
    write_row = bool(rng.integers(0, 2))
    print(f"random decode seed {seed}: heads {n_q}/{n_kv} d {d} B {B} lens {lens.tolist()} plan {kw} "
          f"write_row {write_row}", flush=True)
    c = hw.build_case(entropy=[101, seed], lens=lens, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d, threads=4)
    dc = DeviceCase(c, **kw)
    pool = c["pool"].copy()
    k_new = v_new = None
    if write_row:
        from tests.gpu_util import to_dev_bf16
        k_bits = hw.f32_to_bf16_bits(rng.standard_normal((B, n_kv, d), dtype=np.float32))
        v_bits = hw.f32_to_bf16_bits(rng.standard_normal((B, n_kv, d), dtype=np.float32))
        for b in range(B):
            oa.write_kv(pool, c["row_off"], c["block_ids"], [int(lens[b]) - 1], b, k_bits[b:b + 1], v_bits[b:b + 1])
        k_new, v_new = to_dev_bf16(k_bits), to_dev_bf16(v_bits)
    out, lse = dc.decode(k_new=k_new, v_new=v_new)
    # with 8 query heads per kv head and d = 128 the step may run on the matrix cores, whose
    # bound is the one for the append kernels
    centered = None if (n_q // n_kv not in (1, 2, 4) and d == 128) else True
    ref, ref_lse, spread = oa.decode(pool, c["row_off"], c["block_ids"], lens, c["q"], n_kv, with_spread=True,
                                     centered=centered)
    assert_close(out, ref, f"random decode {seed}", spread)
    assert_lse_close(lse, ref_lse, f"random decode lse {seed}")
    if write_row:
        assert np.array_equal(dc.pool_bits(), pool), "pool after the new rows differs from the oracle's"


@pytest.mark.parametrize("seed", seeds(10))
def test_random_append(seed):
    rng = np.random.default_rng([102, seed])
    shapes = [s for s in HEAD_SHAPES if s[2] == 128 or s[0] // s[1] in POW2]
    n_q, n_kv, d = shapes[int(rng.integers(0, len(shapes)))]
    B = int(rng.integers(1, 13))
    L = draw_lengths(rng, B, int(rng.choice([200, 2000, 6000])))
    L[rng.integers(0, 2, B) == 0] //= 3                      # some short or empty contexts
    mode = int(rng.integers(0, 3))
    C = {0: rng.integers(1, 9, B),                          # verify-like chunks
         1: rng.integers(1, 200, B),                         # tool outputs
         2: rng.choice(EDGE_LENGTHS[:17], B)}[mode].astype(np.int32)
    kw = {} if rng.integers(0, 2) else dict(n_cu=int(rng.choice([2, 16, 256])),
                                            append_wg_per_cu=int(rng.choice([1, 2, 4])),
                                            append_min_steps=int(rng.choice([1, 2, 4, 8])))
    if kw and rng.integers(0, 2):
        kw["max_split"] = int(rng.choice([1, 2, 5, 64]))
    print(f"random append seed {seed}: heads {n_q}/{n_kv} B {B} L {L.tolist()} C {C.tolist()} ctx {kw}", flush=True)
    c = hw.build_case(entropy=[102, seed], lens=L, chunk_lens=C, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d,
                      threads=4)
    dc = DeviceCase(c, **kw)
    out, lse = dc.append()
    pool = c["pool"].copy()
    ref, ref_lse, spread = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"], c["k_new"],
                                     c["v_new"], n_kv, with_spread=True, centered=None)
    assert np.array_equal(dc.pool_bits(), pool), "pool after append differs from the oracle's"
    assert_close(out, ref, f"random append {seed}", spread)
    assert_lse_close(lse, ref_lse, f"random append lse {seed}")


@pytest.mark.parametrize("seed", seeds(3))
def test_random_append_tall(seed):
    """Chunks of a few hundred rows (many row tiles per trajectory, each cut over its keys when
    the planner's parameters say so) behind contexts from empty to a few thousand tokens."""
    rng = np.random.default_rng([105, seed])
    shapes = [s for s in HEAD_SHAPES if s[2] == 128 or s[0] // s[1] in POW2]
    n_q, n_kv, d = shapes[int(rng.integers(0, len(shapes)))]
    B = int(rng.integers(1, 3))
    L = rng.integers(0, int(rng.choice([70, 600, 2000])), B).astype(np.int32)
    C = rng.integers(130, 400, B).astype(np.int32)
    kw = {} if rng.integers(0, 3) == 0 else dict(n_cu=int(rng.choice([16, 256])),
                                                 append_wg_per_cu=int(rng.choice([1, 2, 4])),
                                                 append_min_steps=int(rng.choice([1, 2, 4])),
                                                 max_split=int(rng.choice([2, 5, 64])))
    print(f"random tall append seed {seed}: heads {n_q}/{n_kv} d {d} L {L.tolist()} C {C.tolist()} ctx {kw}", flush=True)
    c = hw.build_case(entropy=[105, seed], lens=L, chunk_lens=C, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d,
                      threads=4)
    dc = DeviceCase(c, **kw)
    out, lse = dc.append()
    pool = c["pool"].copy()
    ref, ref_lse, spread = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"], c["k_new"],
                                     c["v_new"], n_kv, with_spread=True, centered=None)
    assert np.array_equal(dc.pool_bits(), pool), "pool after append differs from the oracle's"
    assert_close(out, ref, f"random tall append {seed}", spread)
    assert_lse_close(lse, ref_lse, f"random tall append lse {seed}")


@pytest.mark.parametrize("seed", seeds(8))
def test_random_shared_decode(seed):
    rng = np.random.default_rng([103, seed])
    n_q, n_kv, d = [(8, 2, 128), (4, 1, 128), (16, 2, 128), (32, 8, 128), (2, 2, 128), (10, 2, 128), (40, 8, 128),
                    (6, 2, 128), (8, 2, 64), (16, 4, 64)][int(rng.integers(0, 10))]
    n_groups = int(rng.integers(1, 5))
    group_of, lens, shared = [], [], []
    for g in range(n_groups):
        members = int(rng.integers(2, 20))
        blocks = int(rng.choice([1, 3, 4, 5, 17, 40, 130]))
        shared.append(blocks)
        for _ in range(members):
            group_of.append(g)
            lens.append(blocks * 16 + int(rng.integers(1, 400)))
    for _ in range(int(rng.integers(0, 6))):                 # trajectories of no group
        group_of.append(-1)
        lens.append(int(rng.integers(1, 3000)))
    order = rng.permutation(len(lens))
    group_of, lens = np.asarray(group_of)[order], np.asarray(lens, dtype=np.int32)[order]
    kw = {} if rng.integers(0, 2) else dict(min_share_blk=int(rng.choice([1, 4, 16])),
                                            group_wg_per_cu=int(rng.choice([1, 2])), n_cu=int(rng.choice([4, 64, 256])))
    if kw and rng.integers(0, 2):
        kw.update(wg_per_cu=int(rng.choice([1, 2, 4, 8])), min_chunk_blk=int(rng.choice([1, 4, 16, 32])),
                  max_split=int(rng.choice([1, 2, 5, 64])))
        if n_q // n_kv in (1, 2, 4) or d == 64:
            kw["tile_blk"] = int(rng.choice([1, 4, 8]))       # the matrix-core kernel needs multiples of 4
        else:
            kw["tile_blk"] = int(rng.choice([4, 8]))
    print(f"random shared decode seed {seed}: heads {n_q}/{n_kv} groups {shared} members "
          f"{np.bincount(group_of[group_of >= 0]).tolist()} B {len(lens)} ctx {kw}", flush=True)
    c = hw.build_case(entropy=[103, seed], lens=lens, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d,
                      group_of=group_of, shared_blocks=np.asarray(shared), threads=4)
    dc = DeviceCase(c, **kw)
    dc.ctx.attn_decode_shared(c["lens"], c["row_off"], c["block_ids"], dc.row_off, dc.block_ids, dc.q, dc.out, dc.lse)
    torch_mod().cuda.synchronize()
    out, lse = bits_to_f64(bf16_to_host_bits(dc.out)), dc.lse.cpu().numpy().astype(np.float64)
    ref, ref_lse, spread = oa.decode(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"], n_kv,
                                     with_spread=True, centered=None)
    assert_close(out, ref, f"random shared decode {seed}", spread)
    assert_lse_close(lse, ref_lse, f"random shared decode lse {seed}")
