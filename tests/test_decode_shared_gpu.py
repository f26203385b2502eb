"""Parity of heddle_attn_decode_shared (decode that reads a prefix shared by several trajectories
once per group) with the float64 oracle, which knows nothing of sharing: it evaluates every
trajectory over its own block-table row.  Needs the GPU."""
import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from oracle import planner as op
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, bf16_to_host_bits, bits_to_f64,
                            to_dev_bf16, torch_mod)

pytestmark = pytest.mark.gpu


def shared_case(seed, lens, group_of, shared_blocks, n_q=8, n_kv=2, d=128, **kw):
    return hw.build_case(entropy=[9, seed], lens=np.asarray(lens), n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d,
                         group_of=np.asarray(group_of), shared_blocks=np.asarray(shared_blocks), threads=4, **kw)


def run_shared(dc, k_new=None, v_new=None, lens=None):
    c = dc.case
    dc.ctx.attn_decode_shared(c["lens"] if lens is None else lens, c["row_off"], c["block_ids"], dc.row_off,
                              dc.block_ids, dc.q, dc.out, dc.lse, k_new, v_new)
    torch_mod().cuda.synchronize()
    return bits_to_f64(bf16_to_host_bits(dc.out)), dc.lse.cpu().numpy().astype(np.float64)


def oracle_decode(c, lens=None, pool=None):
    # the shared part takes the unrounded weight sum as denominator, the private parts the rounded
    # one: the bound is the one for "some keys each way"
    return oa.decode(c["pool"] if pool is None else pool, c["row_off"], c["block_ids"],
                     c["lens"] if lens is None else lens, c["q"], c["n_kv_heads"], with_spread=True, centered=None)


@pytest.mark.parametrize("n_q,n_kv", [(8, 2), (2, 2), (4, 2), (16, 2), (32, 8)])
def test_groups_of_every_shape(n_q, n_kv):
    """Three groups (2, 5 and 40 members: the last needs several member tiles at every G), prefixes
    of 4, 37 and 130 blocks (not multiples of the 4-block step), loners in between, batch order
    interleaved; default plan and a plan forced into many parts."""
    rng = np.random.default_rng(n_q * 100 + n_kv)
    sizes, shared = [2, 5, 40], [4, 37, 130]
    group_of = np.concatenate([np.full(n, g) for g, n in enumerate(sizes)] + [np.full(6, -1)])
    group_of = group_of[rng.permutation(len(group_of))]
    lens = np.array([(shared[g] * 16 if g >= 0 else 0) + int(rng.integers(1, 700)) for g in group_of])
    c = shared_case(1, lens, group_of, shared, n_q, n_kv)
    print("groups", n_q, n_kv, "B", len(lens), flush=True)
    ref, ref_lse, spread = oracle_decode(c)
    for kw in (dict(), dict(n_cu=64, wg_per_cu=8, min_chunk_blk=1, tile_blk=1, max_split=64, group_wg_per_cu=8),
               dict(n_cu=8, wg_per_cu=1, min_chunk_blk=4, tile_blk=4, max_split=3)):
        dc = DeviceCase(c, **kw)
        plan = dc.ctx.plan_decode_shared(c["lens"], c["row_off"], c["block_ids"])
        # with 8 query heads per kv head and parts on the 4-block grid the private blocks go to the
        # matrix-core kernel, which starts at multiples of 64 keys: shared prefixes end there
        on_grid = n_q // n_kv == 8 and kw.get("tile_blk", 4) % 4 == 0
        want = [p // 4 * 4 for p in shared] if on_grid else shared
        assert plan["n_groups"] == 3 and sorted(plan["group_prefix"].tolist()) == want
        out, lse = run_shared(dc)
        assert_close(out, ref, f"shared {kw}", spread)
        assert_lse_close(lse, ref_lse, f"shared lse {kw}")


def test_without_sharing_equals_plain_decode_bit_for_bit():
    c = hw.build_case(entropy=[9, 2], lens=np.array([1, 17, 300, 5000, 64]), n_q_heads=8, n_kv_heads=2,
                      head_dim=128, threads=4)
    dc = DeviceCase(c)
    a_out, a_lse = dc.decode()
    b_out, b_lse = run_shared(dc)
    assert np.array_equal(a_out, b_out) and np.array_equal(a_lse, b_lse)


def test_groups_at_head_dim_64():
    group_of = [0, 0, 0, -1]
    c = shared_case(3, [400, 500, 330, 90], group_of, [20], n_q=8, n_kv=2, d=64)
    dc = DeviceCase(c)
    plan = dc.ctx.plan_decode_shared(c["lens"], c["row_off"], c["block_ids"])
    assert plan["n_groups"] == 1 and plan["group_prefix"][0] == 20
    out, lse = run_shared(dc)
    ref, ref_lse, spread = oracle_decode(c)
    assert_close(out, ref, "d64 shared", spread)
    assert_lse_close(lse, ref_lse, "d64 shared lse")


def test_new_rows_are_written_into_private_blocks():
    """The step's own K/V row arrives with the call; it lands in a block no other trajectory
    names, also when the prefix ends exactly one token before it."""
    group_of = [0, 0, 0, 0]
    shared = [10]
    lens = np.array([161, 162, 176, 177])        # own row at slot 0 / 1 / 15 of the first private block, and one later
    c = shared_case(4, lens, group_of, shared, n_q=8, n_kv=2, d=128)
    rng = np.random.default_rng(8)
    k_new = hw.f32_to_bf16_bits(rng.standard_normal((4, 2, 128), dtype=np.float32))
    v_new = hw.f32_to_bf16_bits(rng.standard_normal((4, 2, 128), dtype=np.float32))
    pool = c["pool"].copy()
    for b in range(4):                            # the caller has not stored the rows: poison them
        blk = c["block_ids"][c["row_off"][b] + (lens[b] - 1) // 16]
        hw.k_view(pool)[blk, :, (lens[b] - 1) % 16, :] = 0x7FC0
        hw.v_view(pool)[blk, :, :, (lens[b] - 1) % 16] = 0x7FC0
    ref_pool = pool.copy()
    for b in range(4):
        oa.write_kv(ref_pool, c["row_off"], c["block_ids"], [int(lens[b]) - 1], b, k_new[b:b + 1], v_new[b:b + 1])
    ref, ref_lse, spread = oracle_decode(c, pool=ref_pool)
    dc = DeviceCase({**c, "pool": pool})
    out, lse = run_shared(dc, to_dev_bf16(k_new), to_dev_bf16(v_new))
    assert_close(out, ref, "shared + new rows", spread)
    assert_lse_close(lse, ref_lse, "shared + new rows lse")
    assert np.array_equal(dc.pool_bits().reshape(ref_pool.shape), ref_pool)


def test_needle_in_shared_and_private_parts():
    """A dominant key with a marker value placed at the first and last shared position, the first
    private position and the last position: a dropped or doubled range changes the answer."""
    shared_blk = 9
    lens = np.array([shared_blk * 16 + 40, shared_blk * 16 + 1, shared_blk * 16 + 300])
    base = shared_case(5, lens, [0, 0, 0], [shared_blk], poison=False)
    for pos in (0, shared_blk * 16 - 1, shared_blk * 16, int(lens[0]) - 1):
        c = {**base, "pool": base["pool"].copy()}
        b = 0
        blk = c["block_ids"][c["row_off"][b] + pos // 16]
        qf = bits_to_f64(c["q"][b])                         # [n_q][d]
        for h in range(2):
            key = qf[h * 4] * 6.0                           # logit ~ 6 |q|^2 / sqrt(d): dominates
            hw.k_view(c["pool"])[blk, h, pos % 16, :] = hw.f32_to_bf16_bits(key.astype(np.float32))
            hw.v_view(c["pool"])[blk, h, :, pos % 16] = hw.f32_to_bf16_bits(np.full(128, 1000.0, np.float32))
        ref, ref_lse, spread = oracle_decode(c)
        assert abs(ref[0, 0]).max() > 900                   # the marker is what the row returns
        out, lse = run_shared(DeviceCase(c))
        assert_close(out, ref, f"needle at {pos}", spread)
        assert_lse_close(lse, ref_lse, f"needle lse at {pos}")


def test_grpo_workload_every_row():
    """Workload 6 at full size in the configuration the benchmark times: every (trajectory, query
    head) output row and LSE against the oracle, which reads each trajectory's own table row."""
    c = hw.make_workload(6, seed=0, threads=16)
    w = c["workload"]
    dc = DeviceCase(c)
    plan = dc.ctx.plan_decode_shared(c["lens"], c["row_off"], c["block_ids"])
    ref_plan = op.plan_decode_shared(c["lens"], c["row_off"], c["block_ids"], 8, 32)
    assert plan["n_groups"] == 8 and np.array_equal(plan["group_prefix"], ref_plan["group_prefix"])
    out, lse = run_shared(dc)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    print(f"workload 6: tokens {int(c['lens'].sum())}, {w.B * w.n_q_heads} rows", flush=True)
    ref, ref_lse, spread = oracle_decode(c)
    assert ref.shape == (w.B, w.n_q_heads, w.head_dim)
    print(f"workload 6: max |err| {np.abs(out - ref).max():.3e}, max |lse err| {np.abs(lse - ref_lse).max():.3e}",
          flush=True)
    assert_close(out, ref, "grpo workload", spread)
    assert_lse_close(lse, ref_lse, "grpo workload lse")
    # plain decode over the same tables: the same rows, under the plain path's own bound
    out2, lse2 = dc.decode()
    assert_close(out2, ref, "grpo workload, plain decode", spread)
    assert_lse_close(lse2, ref_lse, "grpo workload, plain decode lse")


@pytest.mark.parametrize("n_q,n_kv", [(6, 2), (10, 2), (40, 8), (14, 2), (12, 1)])
def test_groups_with_other_head_groups(n_q, n_kv):
    """3, 5, 6, 7 and 12 query heads per kv head (40/8: Qwen3-14B): the shared prefix runs on the 128-row
    matrix-core kernel, the private blocks on the one for short-row tiles, which starts at multiples of
    4 blocks: prefixes of 21 and 7 blocks are shared as 20 and 4."""
    lens = [16 * 21 + 5, 16 * 21 + 300, 16 * 40, 16 * 21 + 1, 2000,        # group 0: 21 common blocks
            16 * 7 + 9, 16 * 7 + 100, 16 * 9,                              # group 1: 7 common blocks
            700, 33]                                                        # nobody's
    group_of = [0] * 5 + [1] * 3 + [-1, -1]
    c = shared_case(22, lens, group_of, [21, 7], n_q=n_q, n_kv=n_kv)
    ref, ref_lse, spread = oracle_decode(c)
    for kw in (dict(), dict(n_cu=8, wg_per_cu=2, min_chunk_blk=4, group_wg_per_cu=2, max_split=8)):
        dc = DeviceCase(c, **kw)
        plan = dc.ctx.plan_decode_shared(c["lens"], c["row_off"], c["block_ids"])
        assert plan["n_groups"] == 2 and sorted(plan["group_prefix"].tolist()) == [4, 20]
        out, lse = run_shared(dc)
        assert_close(out, ref, f"shared, {n_q}/{n_kv} {kw}", spread)
        assert_lse_close(lse, ref_lse, f"shared lse, {n_q}/{n_kv} {kw}")
