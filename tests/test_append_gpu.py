"""Parity of heddle_attn_append with the float64 oracle, through the C ABI (needs the GPU)."""
import math

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, to_dev_bf16, bits_to_f64, torch_mod,
                            bf16_to_host_bits)

pytestmark = pytest.mark.gpu


def small(seed, L, C, n_q=8, n_kv=2, d=128, **kw):
    return hw.build_case(entropy=[0, seed], lens=L, chunk_lens=C, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d,
                         threads=4, **kw)


def oracle_append(c, rows=None):
    # the 128-row kernel divides by the unrounded weight sum, the kernel for short-row tiles by the
    # sum of the rounded weights; a batch may use both, so the bound is the one for either
    pool = c["pool"].copy()
    out, lse, spread = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"], c["k_new"],
                                 c["v_new"], c["n_kv_heads"], rows=rows, with_spread=True, centered=None)
    return pool, out, lse, spread


RAGGED_L = [0, 1, 15, 16, 17, 100, 0, 500, 33, 1000]
RAGGED_C = [1, 40, 1, 16, 33, 31, 130, 7, 64, 129]


@pytest.mark.parametrize("n_q,n_kv,d", [(8, 2, 128), (2, 2, 128), (4, 2, 128), (16, 2, 128), (32, 8, 128), (6, 2, 128),
                                        (10, 2, 128), (40, 8, 128), (12, 2, 128), (14, 2, 128), (24, 1, 128),
                                        (32, 1, 128), (8, 2, 64), (2, 2, 64), (4, 2, 64), (16, 2, 64), (32, 8, 64)])
def test_ragged_append_all_head_shapes(n_q, n_kv, d):
    c = small(40, RAGGED_L, RAGGED_C, n_q=n_q, n_kv=n_kv, d=d)
    print("append ragged", n_q, n_kv, d, flush=True)
    dc = DeviceCase(c)
    out, lse = dc.append()
    pool, ref, ref_lse, spread = oracle_append(c)
    assert np.array_equal(dc.pool_bits(), pool), "pool after append differs from the oracle's"
    assert_close(out, ref, "append out", spread)
    assert_lse_close(lse, ref_lse, "append lse")


def test_append_equals_token_by_token_decode_on_gpu():
    L, C = [0, 5, 16, 300], [3, 20, 1, 37]
    c = small(41, L, C)
    dc = DeviceCase(c)
    out, lse = dc.append()
    # the pool now holds the chunk: decode each chunk row's query at len = L + i + 1
    for b in range(4):
        for i in sorted(x for x in {0, 1, C[b] // 2, C[b] - 1} if 0 <= x < C[b]):
            r = int(c["cu_chunk"][b]) + i
            lens = np.maximum(np.array(L), 1)
            lens[b] = L[b] + i + 1
            qb = np.zeros((4,) + c["q"].shape[1:], dtype=np.uint16)
            qb[b] = c["q"][r]
            dc2_q = to_dev_bf16(qb)
            import torch
            o = torch.empty((4,) + c["q"].shape[1:], dtype=torch.bfloat16, device="cuda")
            ls = torch.empty((4, c["n_q_heads"]), dtype=torch.float32, device="cuda")
            dc.ctx.attn_decode(lens, c["row_off"], dc.row_off, dc.block_ids, dc2_q, o, ls)
            torch.cuda.synchronize()
            got = bits_to_f64(bf16_to_host_bits(o))[b]
            # both are bf16-rounded results of the same sum: allow two output ulps plus weight rounding
            assert np.allclose(got, out[r], rtol=2.0 ** -6, atol=2e-3), (b, i)
            assert np.abs(ls.cpu().numpy()[b] - lse[r]).max() < 1e-3, (b, i)


def test_append_in_two_pieces_equals_one_piece_on_gpu():
    L, C = [7, 400], [50, 90]
    c = small(42, L, C)
    one = DeviceCase(c)
    out1, lse1 = one.append()
    C1 = [20, 33]
    cu = c["cu_chunk"]
    rows1 = np.concatenate([np.arange(cu[b], cu[b] + C1[b]) for b in range(2)])
    rows2 = np.concatenate([np.arange(cu[b] + C1[b], cu[b + 1]) for b in range(2)])
    cA = dict(c, q=c["q"][rows1], k_new=c["k_new"][rows1], v_new=c["v_new"][rows1],
              cu_chunk=np.array([0, C1[0], C1[0] + C1[1]], dtype=np.int32))
    two = DeviceCase(cA)
    outA, lseA = two.append()
    cB = dict(c, q=c["q"][rows2], k_new=c["k_new"][rows2], v_new=c["v_new"][rows2],
              lens=np.array([L[0] + C1[0], L[1] + C1[1]], dtype=np.int32),
              cu_chunk=np.array([0, C[0] - C1[0], C[0] - C1[0] + C[1] - C1[1]], dtype=np.int32))
    import torch
    two.case = cB
    two.q = to_dev_bf16(cB["q"])
    two.out = torch.empty(cB["q"].shape, dtype=torch.bfloat16, device="cuda")
    two.lse = torch.empty(cB["q"].shape[:2], dtype=torch.float32, device="cuda")
    outB, lseB = two.append()
    assert np.array_equal(one.pool_bits(), two.pool_bits())
    assert np.allclose(out1[rows1], outA, rtol=2.0 ** -6, atol=2e-3)
    assert np.allclose(out1[rows2], outB, rtol=2.0 ** -6, atol=2e-3)
    assert np.abs(lse1[rows2] - lseB).max() < 1e-3


def test_append_needles():
    """Dominant keys with 1000-markers in V: every chunk row's own position (the causal edge),
    the last retained position, the first, and a block boundary inside the chunk."""
    n_q, n_kv, d = 8, 2, 128
    G = n_q // n_kv
    L, C = [50], [40]
    base = small(43, L, C, poison=True)
    for h in range(n_kv):
        base["q"][:, h * G:(h + 1) * G] = base["q"][:, h * G:h * G + 1]

    def key_for(qrow):
        qv = bits_to_f64(qrow)
        return hw.f32_to_bf16_bits((40.0 * math.sqrt(d) * qv / (qv @ qv)).astype(np.float32))

    # (a) every row finds its own key: logit 40 on the diagonal, later rows' keys are masked
    c = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in base.items()}
    for i in range(C[0]):
        for h in range(n_kv):
            c["k_new"][i, h] = key_for(c["q"][i, h * G])
            c["v_new"][i, h] = hw.f32_to_bf16_bits(np.full(d, 100.0 + i, dtype=np.float32))
    out, lse = DeviceCase(c).append()
    pool, ref, ref_lse, spread = oracle_append(c)
    assert_close(out, ref, "needle diagonal", spread)
    assert_lse_close(lse, ref_lse)
    # keys of earlier rows are random w.r.t. this row's q: its own key dominates
    for i in range(C[0]):
        assert np.abs(out[i] - (100.0 + i)).max() < 1.0, i

    # (b) needle in the retained context at position pos, seen by every row
    for pos in (0, 15, 16, L[0] - 1):
        c = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in base.items()}
        c["q"][:] = c["q"][0]                         # one query direction for all rows
        blk = c["block_ids"][pos // 16]
        for h in range(n_kv):
            hw.k_view(c["pool"])[blk, h, pos % 16] = key_for(c["q"][0, h * G])
            marker = np.zeros(d, dtype=np.float32)
            marker[(pos + h) % d] = 1000.0
            hw.v_view(c["pool"])[blk, h, :, pos % 16] = hw.f32_to_bf16_bits(marker)
        out, lse = DeviceCase(c).append()
        pool, ref, ref_lse, spread = oracle_append(c)
        assert_close(out, ref, f"needle at {pos}", spread)
        assert_lse_close(lse, ref_lse)
        for j in range(n_q):
            assert np.abs(out[:, j, (pos + j // G) % d] - 1000.0).max() < 8.0, (pos, j)


def test_append_of_rows_the_caller_has_stored():
    """k = v = NULL: the chunk's rows are in the pool already; the call attends and leaves the pool alone."""
    torch = torch_mod()
    c = small(47, [0, 10, 300, 31], [9, 1, 70, 33])
    dc = DeviceCase(c)
    out, lse = dc.append()                                   # stores the rows
    pool_after = dc.pool_bits().copy()
    out2 = torch.full(c["q"].shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse2 = torch.full(c["q"].shape[:2], float("nan"), dtype=torch.float32, device="cuda")
    dc.ctx.attn_append(c["lens"], c["cu_chunk"], c["row_off"], dc.row_off, dc.block_ids, dc.q, None, None, out2, lse2)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_to_host_bits(out2), bf16_to_host_bits(dc.out))        # same kernels, same inputs
    assert np.array_equal(lse2.cpu().numpy(), dc.lse.cpu().numpy())
    assert np.array_equal(dc.pool_bits(), pool_after)
    _, ref, ref_lse, spread = oracle_append(c)
    assert_close(bits_to_f64(bf16_to_host_bits(out2)), ref, "append of stored rows", spread)
    import paper_2603_28101_amd as heddle
    with pytest.raises(heddle.HeddleError) as e:             # only one of the two
        dc.ctx.attn_append(c["lens"], c["cu_chunk"], c["row_off"], dc.row_off, dc.block_ids, dc.q, dc.k_new, None,
                           out2, lse2)
    assert e.value.code == heddle.E_INVAL


def test_append_rejects_bad_arguments():
    import paper_2603_28101_amd as heddle
    c = small(44, [10, 20], [5, 6])
    dc = DeviceCase(c)
    before = dc.pool_bits().copy()
    good = dict(c)
    for bad in (dict(lens=np.array([-1, 20], dtype=np.int32)),
                dict(cu_chunk=np.array([0, 5, 5], dtype=np.int32)),
                dict(lens=np.array([10, 40], dtype=np.int32))):        # table too short for L + C
        dc.case = dict(good, **bad)
        with pytest.raises(heddle.HeddleError) as e:
            dc.append()
        assert e.value.code == heddle.E_INVAL
    assert np.array_equal(dc.pool_bits(), before)
    dc.case = good
    out, _ = dc.append()
    assert_close(out, oracle_append(c)[1])


_FULL_APPEND = {}


def full_size_append(seed):
    """Workload 5 of that seed appended on the GPU once (default plan, the launch configuration the
    benchmark times); the comparisons below share the result.  Only the latest seed is kept."""
    if seed not in _FULL_APPEND:
        _FULL_APPEND.clear()
        c = hw.make_workload(5, seed, threads=16)
        print(f"append workload seed {seed}: pool {c['pool'].nbytes / 1e9:.2f} GB, context {int(c['lens'].sum())}, "
              f"chunk rows {int(c['chunk_lens'].sum())}", flush=True)
        dc = DeviceCase(c)
        out, lse = dc.append()
        _FULL_APPEND[seed] = (c, out, lse, dc.pool_bits())
    return _FULL_APPEND[seed]


@pytest.mark.parametrize("seed,part", [(s, p) for s in (0, 1) for p in range(4)])
def test_full_size_append_workload_row_subset(seed, part):
    """The tool-output append workload at full size.  The whole oracle is minutes of float64 work,
    so it evaluates a fixed subset of chunk rows: rows 0, 1, C-2, C-1 and every 17th row of every
    trajectory, all query heads (every trajectory, every kv head, the causal edge at both ends of each
    chunk, rows of every 128-row tile).  The trajectories are spread over four test cases (b % 4) so
    that no case computes for minutes.  Every chunk of this workload has at least 64 rows, so all
    tiles run in the 128-row kernel, which divides by the unrounded weight sum: the derived bound is
    the one for weights perturbed in the numerator only."""
    c, out, lse, pool_after = full_size_append(seed)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    cu = c["cu_chunk"]
    assert int(c["chunk_lens"].min()) >= 64
    rows = []
    for b in range(part, len(c["lens"]), 4):
        C = int(cu[b + 1] - cu[b])
        rows += [int(cu[b]) + r for r in sorted({0, 1, C - 2, C - 1} | set(range(0, C, 17))) if 0 <= r < C]
    pool = c["pool"].copy()
    ref, ref_lse, spread = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"],
                                     c["k_new"], c["v_new"], c["n_kv_heads"], rows=rows, with_spread=True,
                                     centered=False)
    print(f"append workload seed {seed} part {part}: {len(rows)} rows x {c['n_q_heads']} heads compared, "
          f"max |err| {np.abs(out[rows] - ref[rows]).max():.3e}", flush=True)
    assert_close(out[rows], ref[rows], "append workload", spread[rows])
    assert_lse_close(lse[rows], ref_lse[rows], "append workload lse")
    if part == 0:
        # the whole chunk is in the pool, bit for bit, and nothing else changed
        assert np.array_equal(pool_after, pool)
    if part == 3:
        _FULL_APPEND.clear()


# ------------------------------------------------------------------ small batches: split-K over the keys

def test_single_long_trajectory_short_chunk_is_split_and_exact():
    """One trajectory of 40 000 tokens with an 8-token chunk: one tile, cut into many parts."""
    c = small(31, [40000], [8], 8, 2, 128)
    dc = DeviceCase(c)
    sp = dc.ctx.plan_append_split(c["lens"], c["cu_chunk"])
    assert sp["n_tiles"] == 1 and sp["tile_nsplit"][0] > 8
    out, lse = dc.append()
    _, ref, ref_lse, spread = oracle_append(c)
    assert_close(out, ref, "split append", spread)
    assert_lse_close(lse, ref_lse, "split append lse")


@pytest.mark.parametrize("n_q,n_kv,d", [(8, 2, 128), (2, 2, 128), (4, 2, 128), (16, 2, 128), (32, 8, 128), (6, 2, 128),
                                        (10, 2, 128), (40, 8, 128), (14, 2, 128), (32, 1, 128), (8, 2, 64), (16, 2, 64)])
def test_short_multi_token_decode(n_q, n_kv, d):
    """A verify step of speculative decoding: 2-8 new tokens on each of a few trajectories of very
    different lengths (ragged parts, L = 0 among them); default plan and one forced into many parts."""
    L = [0, 1, 63, 64, 65, 1000, 4097, 20000]
    C = [8, 2, 3, 5, 8, 4, 7, 6]
    c = small(32, L, C, n_q, n_kv, d)
    _, ref, ref_lse, spread = oracle_append(c)
    for kw in (dict(), dict(n_cu=1024, append_min_steps=1, max_split=64), dict(n_cu=16, max_split=3)):
        dc = DeviceCase(c, **kw)
        out, lse = dc.append()
        assert_close(out, ref, f"multi-token decode {kw}", spread)
        assert_lse_close(lse, ref_lse, f"multi-token decode lse {kw}")


def test_split_parts_meet_the_causal_edge():
    """Chunks long enough that the last part holds the whole causal triangle of a tile, with part
    boundaries right at and around the first row's position."""
    L = [64 * 7, 64 * 7 - 1, 64 * 7 + 1, 200]
    C = [40, 33, 64, 130]
    c = small(33, L, C, 8, 2, 128)
    _, ref, ref_lse, spread = oracle_append(c)
    dc = DeviceCase(c, n_cu=512, append_min_steps=1, max_split=64)
    sp = dc.ctx.plan_append_split(c["lens"], c["cu_chunk"])
    assert (sp["tile_nsplit"] > 1).any()
    out, lse = dc.append()
    assert_close(out, ref, "parts at the causal edge", spread)
    assert_lse_close(lse, ref_lse, "parts at the causal edge lse")


def _sampled_rows(c, trajectories):
    cu = c["cu_chunk"]
    rows = []
    for b in trajectories:
        C = int(cu[b + 1] - cu[b])
        rows += [int(cu[b]) + r for r in sorted({0, 1, C // 2, C - 1}) if 0 <= r < C]
    return sorted(set(rows))


def test_verify_workload_at_full_size_every_row():
    """The verify-4-tokens workload at full size, in the configuration the benchmark times: every
    chunk row and query head against the oracle, and the pool after the call bit for bit."""
    c = hw.make_workload(7, 0, threads=16)
    dc = DeviceCase(c)
    sp = dc.ctx.plan_append_split(c["lens"], c["cu_chunk"])
    assert sp["tile_nsplit"].max() > 1                      # the long ones are cut
    out, lse = dc.append()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    print(f"workload 7: {out.shape[0]} rows x {out.shape[1]} heads", flush=True)
    pool, ref, ref_lse, spread = oracle_append(c)
    print(f"workload 7: max |err| {np.abs(out - ref).max():.3e}, max |lse err| {np.abs(lse - ref_lse).max():.3e}",
          flush=True)
    assert_close(out, ref, "workload 7", spread)
    assert_lse_close(lse, ref_lse, "workload 7 lse")
    assert np.array_equal(dc.pool_bits(), pool)


def test_straggler_append_workload_at_full_size_every_row():
    """The single-straggler append workload at full size, in the configuration the benchmark times
    (both row tiles cut over the keys): every chunk row and query head against the oracle (a row
    of 114 000 keys takes the float64 oracle about a second), and the pool after the call bit for bit."""
    c = hw.make_workload(8, 0, threads=16)
    dc = DeviceCase(c)
    sp = dc.ctx.plan_append_split(c["lens"], c["cu_chunk"])
    assert sp["tile_nsplit"].min() > 1
    out, lse = dc.append()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    print(f"workload 8: {out.shape[0]} rows x {out.shape[1]} heads", flush=True)
    pool, ref, ref_lse, spread = oracle_append(c)
    print(f"workload 8: max |err| {np.abs(out - ref).max():.3e}, max |lse err| {np.abs(lse - ref_lse).max():.3e}",
          flush=True)
    assert_close(out, ref, "workload 8", spread)
    assert_lse_close(lse, ref_lse, "workload 8 lse")
    assert np.array_equal(dc.pool_bits(), pool)


@pytest.mark.parametrize("n_q,n_kv,d", [(2, 2, 128), (8, 2, 128), (10, 2, 128), (16, 2, 128), (2, 2, 64), (8, 2, 64)])
def test_tiles_of_at_most_64_rows(n_q, n_kv, d):
    """Tiles whose rows (chunk rows x query heads per kv head) number 64, one chunk row more, one
    chunk row less and a single row: half of the workgroup's row slots or fewer carry a row.  Over
    contexts in which the second half of the first 64-key step lies wholly, partly or not at all
    behind what the rows see, and over contexts long enough to be cut into parts."""
    G = n_q // n_kv
    h = 64 // G
    L = [0, 5, 31, 32, 33, 63, 64, 100, 1000, 3000, 0, 40]
    C = [h, h, 1, h, max(1, h - 1), h, h + 1, h, h, h, h + 1, 128 // G + h]
    c = small(42, L, C, n_q, n_kv, d)
    pool, ref, ref_lse, spread = oracle_append(c)
    for kw in ({}, dict(n_cu=64, append_wg_per_cu=4, append_min_steps=1)):
        dc = DeviceCase(c, **kw)
        out, lse = dc.append()
        assert_close(out, ref, f"tiles of at most 64 rows {kw}", spread)
        assert_lse_close(lse, ref_lse, f"tiles of at most 64 rows lse {kw}")
        assert np.array_equal(dc.pool_bits(), pool)


@pytest.mark.parametrize("n_q,n_kv,d", [(2, 2, 64), (2, 2, 128), (1, 1, 128)])
def test_tall_tiles_over_short_contexts_with_one_step_parts(n_q, n_kv, d):
    """One query head per kv head makes tiles of 128 chunk rows; with parts of a single 64-key step
    (append_min_steps = 1 on a large grid) several candidate parts of such a tile can lie behind
    what its first row sees.  They are all merged back (a row with an empty share of a part would
    be an empty softmax), and the result stays the oracle's."""
    c = small(41, [31, 7, 70, 0, 130, 64], [106, 75, 106, 128, 200, 127], n_q, n_kv, d)
    kw = dict(n_cu=256, append_wg_per_cu=4, append_min_steps=1)
    dc = DeviceCase(c, **kw)
    sp = dc.ctx.plan_append_split(c["lens"], c["cu_chunk"])
    first_tile = {int(b): int(n) for b, r0, n in zip(sp["tile_b"], sp["tile_row0"], sp["tile_nsplit"]) if r0 == 0}
    assert first_tile == {0: 1, 1: 1, 2: 2, 3: 1, 4: 3, 5: 2}
    pool, ref, ref_lse, spread = oracle_append(c)
    out, lse = dc.append()
    assert_close(out, ref, "tall tiles, one-step parts", spread)
    assert_lse_close(lse, ref_lse, "tall tiles, one-step parts lse")
    assert np.array_equal(dc.pool_bits(), pool)


def test_append_up_to_the_maximum_context():
    """Chunks that end exactly at the largest context the library accepts, one through the
    128-row kernel (40 rows), one through the short-row kernel (3 rows), both cut into parts."""
    top = 131072
    c = small(34, [top - 40, top - 3, 5], [40, 3, 2], 8, 2, 128)
    dc = DeviceCase(c)
    out, lse = dc.append()
    rows = _sampled_rows(c, [0, 1, 2])
    pool, ref, ref_lse, spread = oracle_append(c, rows=rows)
    assert_close(out[rows], ref[rows], "maximum context append", spread[rows])
    assert_lse_close(lse[rows], ref_lse[rows], "maximum context append lse")
    assert np.array_equal(dc.pool_bits(), pool)
    import paper_2603_28101_amd as heddle
    with pytest.raises(heddle.HeddleError):                 # one token more is refused before any device work
        over = small(35, [top - 2], [3], 8, 2, 128)
        DeviceCase(over).append()


def test_softmax_scale_of_the_context_is_used():
    """A scale other than 1/sqrt(d) in the 128-row kernel (chunks of 40 and 70 rows) and in the
    short-row kernel (chunks of 3 and 5 rows)."""
    for C in ([40, 70], [3, 5]):
        c = small(36, [100, 3000], C, 8, 2, 128)
        for scale in (0.03, 0.25):
            pool = c["pool"].copy()
            ref, ref_lse, spread = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"],
                                             c["k_new"], c["v_new"], 2, scale=scale, with_spread=True, centered=None)
            out, lse = DeviceCase(c, scale=scale).append()
            assert_close(out, ref, f"append scale {scale}", spread)
            assert_lse_close(lse, ref_lse, f"append scale {scale} lse")
