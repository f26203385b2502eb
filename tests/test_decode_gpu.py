"""Parity of heddle_attn_decode with the float64 oracle, through the C ABI (needs the GPU)."""
import math

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from oracle import planner as op
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, to_dev_bf16, bits_to_f64, torch_mod,
                            bf16_to_host_bits)

pytestmark = pytest.mark.gpu


def oracle_decode(c, lens=None, pool=None):
    """(out, lse, spread) of the float64 oracle."""
    return oa.decode(c["pool"] if pool is None else pool, c["row_off"], c["block_ids"],
                     c["lens"] if lens is None else lens, c["q"], c["n_kv_heads"], with_spread=True)


def small(seed, lens, n_q, n_kv, d, **kw):
    return hw.build_case(entropy=[0, seed], lens=lens, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d, threads=4, **kw)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_workload(seed):
    c = hw.make_workload(1, seed)
    print("tiny decode seed", seed, "lens", c["lens"].tolist(), flush=True)
    out, lse = DeviceCase(c).decode()
    ref, ref_lse, spread = oracle_decode(c)
    assert_close(out, ref, "tiny out", spread)
    assert_lse_close(lse, ref_lse, "tiny lse")


RAGGED = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 255, 256, 257, 1000, 1024, 2049, 4097]


@pytest.mark.parametrize("n_q,n_kv,d", [(8, 2, 128), (8, 2, 64), (2, 2, 128), (4, 2, 128), (16, 2, 128),
                                        (16, 2, 64), (3, 3, 64), (32, 8, 128)])
def test_ragged_lengths_all_head_shapes(n_q, n_kv, d):
    c = small(10, RAGGED, n_q, n_kv, d)
    print("ragged", n_q, n_kv, d, flush=True)
    ref, ref_lse, spread = oracle_decode(c)
    # default plan (mostly unsplit) and a plan forced into many small splits
    for kw in (dict(), dict(n_cu=64, wg_per_cu=8, min_chunk_blk=1, tile_blk=1, max_split=64),
               dict(n_cu=8, wg_per_cu=1, min_chunk_blk=4, tile_blk=4, max_split=3)):
        out, lse = DeviceCase(c, **kw).decode()
        assert_close(out, ref, f"ragged {kw}", spread)
        assert_lse_close(lse, ref_lse, f"ragged lse {kw}")


def test_lse_output_is_optional():
    c = small(11, [100, 7], 8, 2, 128)
    dc = DeviceCase(c)
    out, lse = dc.decode(want_lse=False)
    assert np.isnan(lse).all()
    ref, _, spread = oracle_decode(c)
    assert_close(out, ref, "no lse", spread)


def test_needle_at_every_split_and_wave_boundary():
    """One key dominates the softmax by e^40 and carries a 1000-marker in V: dropping or
    double counting any token range, or an off-by-one at a boundary, changes the answer."""
    n_q, n_kv, d = 8, 2, 128
    L = 3000
    kw = dict(n_cu=4, wg_per_cu=2, min_chunk_blk=8, tile_blk=4, max_split=64)
    plan = op.plan_decode([L], n_kv, **kw)
    assert plan["n_items"] >= 4
    positions = {0, L - 1, L - 2, (L // 16) * 16 - 1, (L // 16) * 16}
    for lo, hi in zip(plan["item_blk_begin"], plan["item_blk_end"]):
        lo, hi = int(lo), int(hi)
        per_wave = -(-(hi - lo) // 4)
        for w in range(5):
            for blk in (lo + w * per_wave - 1, lo + w * per_wave):
                if lo <= blk < hi:
                    positions |= {blk * 16, min(blk * 16 + 15, L - 1)}
    positions = sorted(p for p in positions if 0 <= p < L)
    print("needle positions", len(positions), flush=True)
    base = small(12, [L], n_q, n_kv, d, poison=False)
    G = n_q // n_kv
    for h in range(n_kv):
        base["q"][0, h * G:(h + 1) * G] = base["q"][0, h * G]
    dc = DeviceCase(base, **kw)
    for pos in positions:
        c = dict(base)
        c["pool"] = base["pool"].copy()
        blk = base["block_ids"][pos // 16]
        for h in range(n_kv):
            qv = bits_to_f64(base["q"][0, h * G])
            hw.k_view(c["pool"])[blk, h, pos % 16] = hw.f32_to_bf16_bits((40.0 * math.sqrt(d) * qv / (qv @ qv)).astype(np.float32))
            marker = np.zeros(d, dtype=np.float32)
            marker[(pos + h) % d] = 1000.0
            hw.v_view(c["pool"])[blk, h, :, pos % 16] = hw.f32_to_bf16_bits(marker)
        dc.pool.copy_(to_dev_bf16(c["pool"]))
        out, lse = dc.decode()
        ref, ref_lse, spread = oracle_decode(c)
        assert_close(out, ref, f"needle at {pos}", spread)
        assert_lse_close(lse, ref_lse, f"needle lse at {pos}")
        for j in range(n_q):
            assert abs(out[0, j, (pos + j // G) % d] - 1000.0) < 8.0, (pos, j)


def test_physical_block_permutation_leaves_output_bits_unchanged():
    c = small(13, [700, 33, 16, 2500], 8, 2, 128)
    out1, lse1 = DeviceCase(c).decode()
    perm = np.random.default_rng(5).permutation(c["n_blocks"])
    c2 = dict(c)
    c2["pool"] = np.empty_like(c["pool"])
    c2["pool"][perm] = c["pool"]
    c2["block_ids"] = perm[c["block_ids"]].astype(np.int32)
    out2, lse2 = DeviceCase(c2).decode()
    assert np.array_equal(out1, out2) and np.array_equal(lse1, lse2)


def test_poisoned_tails_and_free_blocks_do_not_leak():
    lens = [5, 16, 17, 30, 1, 250]
    c = small(14, lens, 8, 2, 128, poison=True)
    out, lse = DeviceCase(c).decode()
    clean = small(14, lens, 8, 2, 128, poison=False)
    out2, lse2 = DeviceCase(clean).decode()
    assert np.isfinite(out).all()
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


def test_new_row_is_stored_then_attended():
    lens = [1, 16, 17, 300, 64]
    c = small(15, lens, 8, 2, 128)
    rng = np.random.default_rng(3)
    k_new = hw.f32_to_bf16_bits(rng.standard_normal((5, 2, 128), dtype=np.float32))
    v_new = hw.f32_to_bf16_bits(rng.standard_normal((5, 2, 128), dtype=np.float32))
    dc = DeviceCase(c)
    out, lse = dc.decode(k_new=to_dev_bf16(k_new), v_new=to_dev_bf16(v_new))
    pool = c["pool"].copy()
    for b in range(5):
        oa.write_kv(pool, c["row_off"], c["block_ids"], [lens[b] - 1], b, k_new[b:b + 1], v_new[b:b + 1])
    assert np.array_equal(dc.pool_bits(), pool)          # exactly those rows changed, bit for bit
    ref, ref_lse, spread = oracle_decode(c, pool=pool)
    assert_close(out, ref, "decode with new row", spread)
    assert_lse_close(lse, ref_lse)


def test_invalid_arguments_are_rejected_without_side_effects():
    import paper_2603_28101_amd as heddle
    c = small(16, [40, 9], 8, 2, 128)
    dc = DeviceCase(c)
    good, _ = dc.decode()
    before = bf16_to_host_bits(dc.out).copy()
    for lens in ([0, 9], [40, 17], [131073, 9]):        # zero length; table too short; too long
        with pytest.raises(heddle.HeddleError) as e:
            dc.decode(lens=lens)
        assert e.value.code == heddle.E_INVAL
    with pytest.raises(heddle.HeddleError):
        dc.decode(k_new=to_dev_bf16(c["q"][:, :2]))       # k_new without v_new
    assert np.array_equal(bf16_to_host_bits(dc.out), before)
    again, _ = dc.decode()
    assert np.array_equal(good, again)


def test_back_to_back_calls_share_scratch_safely():
    big = small(17, [5000, 4000, 3000, 100], 8, 2, 128)
    tiny = small(18, [3, 50], 8, 2, 128)
    d_big, d_tiny = DeviceCase(big), DeviceCase(tiny)
    ref_big, _, sp_big = oracle_decode(big)
    ref_tiny, _, sp_tiny = oracle_decode(tiny)
    for _ in range(3):
        assert_close(d_big.decode()[0], ref_big, "big", sp_big)
        assert_close(d_tiny.decode()[0], ref_tiny, "tiny", sp_tiny)
    # same context, shrinking then growing batch
    out_small, _ = d_big.decode(lens=[17, 1, 1, 1])
    ref_small, _, sp_small = oracle_decode(big, lens=[17, 1, 1, 1])
    assert_close(out_small, ref_small, "shrunk batch", sp_small)
    assert_close(d_big.decode()[0], ref_big, "big again", sp_big)


@pytest.mark.parametrize("cfg,seed", [(2, 0), (2, 1), (3, 0), (4, 0), (9, 0)])
def test_full_size_workloads_every_row(cfg, seed):
    """The named workloads at full size, in the launch configuration the benchmark times
    (default plan): every (trajectory, query head) output row and every LSE is compared with the
    oracle, so a wrong (item, kv head) anywhere in the plan of the full-size batch shows."""
    c = hw.make_workload(cfg, seed, threads=16)
    w = c["workload"]
    print(f"workload {cfg} seed {seed}: pool {c['pool'].nbytes / 1e9:.2f} GB, tokens {int(c['lens'].sum())}", flush=True)
    dc = DeviceCase(c)
    out, lse = dc.decode()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    ref, ref_lse, spread = oracle_decode(c)
    assert ref.shape == (w.B, w.n_q_heads, w.head_dim)
    print(f"workload {cfg} seed {seed}: {w.B * w.n_q_heads} rows compared, max |err| {np.abs(out - ref).max():.3e}, "
          f"max |lse err| {np.abs(lse - ref_lse).max():.3e}", flush=True)
    assert_close(out, ref, f"workload {cfg} seed {seed}", spread)
    assert_lse_close(lse, ref_lse, f"workload {cfg} seed {seed} lse")


def test_maximum_context_single_trajectory():
    """One trajectory at the supported maximum (131 072 tokens, 8 192 blocks) next to minimal ones:
    the plan cuts it into many items; sampled heads are compared with the oracle."""
    lens = [131072, 1, 16, 131071]
    c = small(19, lens, 8, 2, 128)
    dc = DeviceCase(c)
    out, lse = dc.decode()
    assert np.isfinite(out).all()
    pairs = [(0, 0), (0, 7), (1, 3), (2, 5), (3, 1), (3, 6)]
    ref, ref_lse, spread = oa.decode_rows(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"], 2, pairs,
                                          with_spread=True)
    assert_close(np.array([out[b, j] for b, j in pairs]), ref, "max context", spread)
    assert_lse_close(np.array([lse[b, j] for b, j in pairs]), ref_lse, "max context lse")


def test_many_short_trajectories():
    rng = np.random.default_rng(21)
    lens = rng.integers(1, 40, 700).tolist()
    c = small(20, lens, 4, 2, 64)
    out, lse = DeviceCase(c).decode()
    ref, ref_lse, spread = oracle_decode(c)
    assert_close(out, ref, "many short", spread)
    assert_lse_close(lse, ref_lse, "many short lse")


def test_dominant_logits_and_large_values():
    """Keys scaled so that logits span hundreds of units: the lazily moved maximum must keep
    every exponent in range, whatever block the largest logit sits in."""
    lens = [300, 77]
    c = small(22, lens, 8, 2, 128, poison=False)
    kf = bits_to_f64(hw.k_view(c["pool"])).astype(np.float32) * 16.0
    hw.k_view(c["pool"])[:] = hw.f32_to_bf16_bits(kf)
    out, lse = DeviceCase(c).decode()
    ref, ref_lse, spread = oracle_decode(c)
    assert_close(out, ref, "dominant logits", spread)
    assert np.abs(lse - ref_lse).max() < 1e-3 * np.maximum(1.0, np.abs(ref_lse)).max()


@pytest.mark.parametrize("n_q,n_kv", [(8, 2), (16, 2)])
def test_softmax_scale_of_the_context_is_used(n_q, n_kv):
    """A scale other than 1/sqrt(d), in the packed-dot kernel (G = 4) and in the matrix-core kernel
    that runs decode at G = 8."""
    c = small(21, [1, 40, 700, 5000], n_q, n_kv, 128)
    for scale in (0.03, 0.25):
        ref, ref_lse, spread = oa.decode(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"], n_kv, scale=scale,
                                         with_spread=True)
        out, lse = DeviceCase(c, scale=scale).decode()
        assert_close(out, ref, f"scale {scale}", spread)
        assert_lse_close(lse, ref_lse, f"scale {scale} lse")


def test_kernel_timers_count_and_time_the_launches():
    """The measurement aids: with recording on every launch, three decode calls leave three
    durations per launched kernel, the average is their mean, recording every 2nd launch keeps
    two of three, and turning recording off leaves the results unchanged."""
    c = small(31, [5000, 300, 17], 8, 2, 128)
    ref, _, spread = oracle_decode(c)
    dc = DeviceCase(c, n_cu=4, wg_per_cu=1, min_chunk_blk=16)      # the long trajectory is split: both kernels run
    dc.ctx.timing_enable(1)
    for _ in range(3):
        out, _ = dc.decode()
    assert_close(out, ref, "timed decode", spread)
    for which in (0, 1):                       # split-K kernel, combine kernel
        avg, n = dc.ctx.timing_read(which)
        samples = dc.ctx.timing_samples(which)
        assert n == 3 and samples.shape == (3,)
        assert (samples > 0).all() and (samples < 1e5).all()
        assert abs(avg - float(samples.astype(np.float64).mean())) <= 1e-3 * avg
    assert dc.ctx.timing_read(2)[1] == 0 and dc.ctx.timing_samples(2).shape == (0,)      # no append was launched
    dc.ctx.timing_enable(2)
    for _ in range(3):
        dc.decode()
    assert dc.ctx.timing_read(0)[1] == 2
    dc.ctx.timing_enable(0)
    out, _ = dc.decode()
    assert dc.ctx.timing_read(0)[1] == 2       # nothing recorded while off
    assert_close(out, ref, "untimed decode", spread)


@pytest.mark.parametrize("n_q,n_kv", [(6, 2), (10, 2), (40, 8), (12, 2), (14, 2), (24, 1), (32, 1)])
def test_ragged_lengths_other_head_groups(n_q, n_kv):
    """3, 5, 6, 7, 12, 24 and 32 query heads per kv head (40/8 is the Qwen3-14B shape): the step runs
    on the matrix-core kernel, default plan and one forced into many parts (parts start at
    multiples of 4 blocks there)."""
    c = small(12, RAGGED, n_q, n_kv, 128)
    print("ragged, other head groups", n_q, n_kv, flush=True)
    ref, ref_lse, spread = oa.decode(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"], n_kv, with_spread=True,
                                     centered=None)
    for kw in (dict(), dict(n_cu=64, wg_per_cu=8, min_chunk_blk=4, tile_blk=4, max_split=64),
               dict(n_cu=8, wg_per_cu=1, min_chunk_blk=8, tile_blk=8, max_split=3)):
        dc = DeviceCase(c, **kw)
        out, lse = dc.decode()
        assert_close(out, ref, f"ragged {kw}", spread)
        assert_lse_close(lse, ref_lse, f"ragged lse {kw}")
    # the step's new rows, then the pool bit for bit
    rng = np.random.default_rng(5)
    B = len(RAGGED)
    k_bits = hw.f32_to_bf16_bits(rng.standard_normal((B, n_kv, 128), dtype=np.float32))
    v_bits = hw.f32_to_bf16_bits(rng.standard_normal((B, n_kv, 128), dtype=np.float32))
    pool = c["pool"].copy()
    for b in range(B):
        oa.write_kv(pool, c["row_off"], c["block_ids"], [int(c["lens"][b]) - 1], b, k_bits[b:b + 1], v_bits[b:b + 1])
    out, lse = dc.decode(k_new=to_dev_bf16(k_bits), v_new=to_dev_bf16(v_bits))
    ref, ref_lse, spread = oa.decode(pool, c["row_off"], c["block_ids"], c["lens"], c["q"], n_kv, with_spread=True,
                                     centered=None)
    assert np.array_equal(dc.pool_bits(), pool)
    assert_close(out, ref, "with new rows", spread)


def test_head_shapes_no_kernel_is_built_for_are_refused():
    import paper_2603_28101_amd as heddle
    torch = __import__("torch")
    pool = torch.zeros((4, 2, 2, 16 * 128), dtype=torch.bfloat16, device="cuda")
    for n_q, n_kv, d, kw in ((6, 2, 64, {}),                    # 3 heads per kv head at d = 64
                             (10, 2, 128, dict(tile_blk=2)),    # parts that would not start at multiples of 64 keys
                             (66, 2, 128, {})):                 # 33 heads per kv head
        with pytest.raises(heddle.HeddleError) as e:
            heddle.Context(n_q, n_kv, d, 4, kv_pool=pool, device=0, **kw)
        assert e.value.code == heddle.E_UNSUPPORTED, (n_q, n_kv, d)


def test_binding_refuses_tensors_that_would_fault():
    """The C ABI sees plain pointers; the Python binding checks what is behind them before the call:
    a host tensor, a tensor of the wrong element size or one that is too short raises there."""
    torch = __import__("torch")
    c = small(33, [40, 9], 8, 2, 128)
    dc = DeviceCase(c)
    good, _ = dc.decode()
    cases = {
        "q on the host": dict(q=dc.q.cpu()),
        "out too short": dict(out=dc.out[:1]),
        "q in float32": dict(q=dc.q.float()),
        "lse too short": dict(lse=dc.lse[:1, :4].contiguous()),
        "block ids too short": dict(block_ids=dc.block_ids[:2]),
    }
    for what, kw in cases.items():
        a = dict(row_off=dc.row_off, block_ids=dc.block_ids, q=dc.q, out=dc.out, lse=dc.lse)
        a.update(kw)
        with pytest.raises(ValueError):
            dc.ctx.attn_decode(c["lens"], c["row_off"], a["row_off"], a["block_ids"], a["q"], a["out"], a["lse"])
    with pytest.raises(ValueError):
        import paper_2603_28101_amd as heddle
        heddle.Context(8, 2, 128, c["n_blocks"] + 1, kv_pool=dc.pool, device=0)      # pool smaller than n_blocks says
    again, _ = dc.decode()
    assert np.array_equal(good, again)


def test_many_queued_calls_with_different_plans():
    """Forty decode calls with forty different batches are issued behind several milliseconds of other work on
    the same stream, so that the host runs far ahead of the device and goes round the ring of pinned
    plan buffers five times; every call must still run with its own plan (a buffer handed out again
    before its copy kernel has read it would show as a wrong result)."""
    import paper_2603_28101_amd as heddle
    torch = __import__("torch")
    rng = np.random.default_rng(77)
    lens_all = [np.concatenate([rng.integers(1, 600, int(rng.integers(2, 9))), [int(rng.integers(1500, 5000))]])
                for _ in range(40)]
    B_max, longest = 9, 5000
    # one pool and table for all calls: every call uses the first B trajectories at its own lengths
    c = small(34, [longest] * B_max, 8, 2, 128)
    dc = DeviceCase(c)
    outs = [torch.full((B_max, 8, 128), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in lens_all]
    lses = [torch.full((B_max, 8), float("nan"), dtype=torch.float32, device="cuda") for _ in lens_all]
    busy = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    dc.decode()                                    # scratch of the largest size first
    torch.cuda.synchronize()
    for _ in range(200):                           # ~8 ms of reads in front of the calls
        heddle.stream_read(busy, busy.numel(), sink)
    for lens, out, lse in zip(lens_all, outs, lses):
        B = len(lens)
        dc.ctx.attn_decode(lens, c["row_off"][: B + 1], dc.row_off, dc.block_ids, dc.q, out, lse)
    torch.cuda.synchronize()
    for i, (lens, out, lse) in enumerate(zip(lens_all, outs, lses)):
        B = len(lens)
        ref, ref_lse, spread = oa.decode(c["pool"], c["row_off"][: B + 1], c["block_ids"], lens, c["q"][:B], 2,
                                         with_spread=True)
        assert_close(bits_to_f64(bf16_to_host_bits(out))[:B], ref, f"queued call {i}", spread)
        assert_lse_close(lse.cpu().numpy()[:B], ref_lse, f"queued call {i} lse")


def test_one_context_serves_a_pool_per_layer():
    """The layers of a model share block table, lengths and block manager and keep a pool each.  Three
    decode steps, each storing a new row, are queued without a wait in between, the context pointed at
    layer 0, layer 1 and layer 0 again: every call reads and writes the pool it was issued with."""
    torch = torch_mod()
    lens = [1, 16, 17, 300, 64, 2100]
    c = small(21, lens, 8, 2, 128)
    host_pools = [c["pool"].copy(), c["pool"] ^ np.uint16(0x8000)]       # layer 1: every value negated
    dc = DeviceCase(c)
    dev_pools = [dc.pool, to_dev_bf16(host_pools[1])]
    rng = np.random.default_rng(8)
    calls = []
    for layer in (0, 1, 0):
        k_new = hw.f32_to_bf16_bits(rng.standard_normal((6, 2, 128), dtype=np.float32))
        v_new = hw.f32_to_bf16_bits(rng.standard_normal((6, 2, 128), dtype=np.float32))
        out = torch.full(c["q"].shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full(c["q"].shape[:2], float("nan"), dtype=torch.float32, device="cuda")
        k_dev, v_dev = to_dev_bf16(k_new), to_dev_bf16(v_new)
        dc.ctx.set_kv_pool(dev_pools[layer])
        dc.ctx.attn_decode(c["lens"], c["row_off"], dc.row_off, dc.block_ids, dc.q, out, lse, k_dev, v_dev)
        for b in range(6):
            oa.write_kv(host_pools[layer], c["row_off"], c["block_ids"], [lens[b] - 1], b, k_new[b:b + 1],
                        v_new[b:b + 1])
        calls.append((layer, out, lse, k_dev, v_dev, oracle_decode(c, pool=host_pools[layer])))
    torch.cuda.synchronize()
    for i, (layer, out, lse, _, _, (ref, ref_lse, spread)) in enumerate(calls):
        assert_close(bits_to_f64(bf16_to_host_bits(out)), ref, f"call {i} on layer {layer}", spread)
        assert_lse_close(lse.cpu().numpy().astype(np.float64), ref_lse)
    for layer in (0, 1):
        assert np.array_equal(bf16_to_host_bits(dev_pools[layer]), host_pools[layer]), f"pool of layer {layer}"
    with pytest.raises(Exception):
        dc.ctx.set_kv_pool(torch.empty(16, dtype=torch.bfloat16, device="cuda"))       # too small for the context


def test_table_entries_past_the_needed_blocks_are_never_read():
    """A table row may be longer than its trajectory needs (blocks reserved ahead, or stale entries):
    what stands behind the needed blocks is never used as an address.  The padding names blocks of
    the pool that no trajectory owns and that are filled with NaN and Inf patterns: a stray read of
    one shows as a bit difference in the output, a stray write as a difference in the pool.  Decode,
    shared-prefix decode and append give the bits of the exact table.  (That ids outside the pool
    behind the needed blocks never reach a work item is checked on the host, without a GPU.)"""
    torch = torch_mod()
    group_of = [0, 0, 0, -1, -1]
    lens = np.array([330, 500, 421, 17, 2100], dtype=np.int32)
    c = hw.build_case(entropy=[0, 61], lens=lens, n_q_heads=8, n_kv_heads=2, head_dim=128, threads=4,
                      group_of=np.asarray(group_of), shared_blocks=np.asarray([20]))
    owned = set(int(x) for x in c["block_ids"])
    junk = [i for i in range(c["n_blocks"]) if i not in owned][:4]       # poisoned by the generator
    assert len(junk) == 4 and not np.isfinite(bits_to_f64(c["pool"][junk])).any()
    rows = [list(c["block_ids"][c["row_off"][b]:c["row_off"][b + 1]]) for b in range(5)]
    need = [-(-int(n) // 16) for n in lens]
    padded = [r[:n] + junk[: 1 + b % 4] for b, (r, n) in enumerate(zip(rows, need))]
    p_off = np.concatenate([[0], np.cumsum([len(r) for r in padded])]).astype(np.int32)
    p_ids = np.asarray([x for r in padded for x in r], dtype=np.int64).astype(np.int32)
    exact = DeviceCase(c)
    dirty = DeviceCase(dict(c, row_off=p_off, block_ids=p_ids))
    rng = np.random.default_rng(4)
    k_new = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((5, 2, 128), dtype=np.float32)))
    v_new = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((5, 2, 128), dtype=np.float32)))
    for dc in (exact, dirty):
        dc.decode(k_new=k_new, v_new=v_new)
    assert np.array_equal(bf16_to_host_bits(dirty.out), bf16_to_host_bits(exact.out))
    assert np.array_equal(dirty.lse.cpu().numpy(), exact.lse.cpu().numpy())
    for dc in (exact, dirty):
        cc = dc.case
        assert dc.ctx.plan_decode_shared(cc["lens"], cc["row_off"], cc["block_ids"])["n_groups"] == 1
        dc.out.fill_(float("nan"))
        dc.ctx.attn_decode_shared(cc["lens"], cc["row_off"], cc["block_ids"], dc.row_off, dc.block_ids, dc.q, dc.out,
                                  dc.lse)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_to_host_bits(dirty.out), bf16_to_host_bits(exact.out))
    assert np.array_equal(dirty.pool_bits(), exact.pool_bits())
    ref, ref_lse, spread = oa.decode(exact.pool_bits(), c["row_off"], c["block_ids"], lens, c["q"], 2, with_spread=True,
                                     centered=None)
    assert_close(bits_to_f64(bf16_to_host_bits(dirty.out)), ref, "shared decode over a padded table", spread)
    # append of 3 tokens onto contexts shortened by 3: the rows written and attended lie inside the needed blocks
    chunk = np.full(5, 3, dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
    q3 = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((15, 8, 128), dtype=np.float32)))
    k3 = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((15, 2, 128), dtype=np.float32)))
    v3 = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((15, 2, 128), dtype=np.float32)))
    outs = []
    for dc in (exact, dirty):
        cc = dc.case
        o = torch.full((15, 8, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
        dc.ctx.attn_append(lens - 3, cu, cc["row_off"], dc.row_off, dc.block_ids, q3, k3, v3, o, None)
        outs.append(o)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_to_host_bits(outs[1]), bf16_to_host_bits(outs[0]))
    assert np.isfinite(bits_to_f64(bf16_to_host_bits(outs[1]))).all()
    assert np.array_equal(dirty.pool_bits(), exact.pool_bits())
