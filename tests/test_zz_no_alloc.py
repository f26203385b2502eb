"""GPU test of heddle_attn_decode_static: the decode entry point whose scratch (plan image,
split-K partials) is a static device array of the library, for callers that cannot allocate.
Its output is compared with heddle_attn_decode's on the same inputs (same kernels, same plan:
bit for bit) and with the float64 oracle, on two calls in a row, the second with a smaller batch,
so that what the first call left in the shared array is there when the second runs."""
from __future__ import annotations

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, bf16_to_host_bits, bits_to_f64, torch_mod)

pytestmark = pytest.mark.gpu


def _both_entry_points(dc, lens, B):
    """(bits, lse) of heddle_attn_decode_static and of heddle_attn_decode for the first B trajectories."""
    torch = torch_mod()
    c = dc.case
    res = []
    for call in (dc.ctx.attn_decode_static, dc.ctx.attn_decode):
        dc.out.fill_(float("nan"))
        dc.lse.fill_(float("nan"))
        call(lens[:B], c["row_off"][: B + 1], dc.row_off, dc.block_ids, dc.q, dc.out, dc.lse)
        torch.cuda.synchronize()
        res.append((bf16_to_host_bits(dc.out)[:B].copy(), dc.lse.cpu().numpy()[:B].copy()))
    return res


def test_static_scratch_decode_two_calls_second_smaller():
    # long-tailed lengths: the long ones are split over several items (partials + combine pass),
    # the short ones finish in one item
    lens = np.array([9000, 300, 17, 4100, 1, 2500, 12000, 640, 33, 7000, 5000, 128], dtype=np.int32)
    case = hw.build_case(entropy=[0x5C, 1], lens=lens, n_q_heads=32, n_kv_heads=8, head_dim=128, threads=4)
    # few compute units in the plan: the batch is cut into parts as a full-size batch is on the real chip
    dc = DeviceCase(case, n_cu=32)
    plan = dc.ctx.plan_decode(lens)
    assert plan["nsplit"].max() > 1 and (plan["nsplit"] == 1).any()
    ref, ref_lse, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], lens, case["q"],
                                     case["n_kv_heads"], with_spread=True)
    for B in (len(lens), 5):                      # the second call is the smaller one
        (bits_s, lse_s), (bits_h, lse_h) = _both_entry_points(dc, lens, B)
        assert np.array_equal(bits_s, bits_h), f"B={B}: static-scratch output differs from heddle_attn_decode's"
        assert np.array_equal(lse_s, lse_h), f"B={B}: static-scratch LSE differs from heddle_attn_decode's"
        # the first B trajectories of the batch under a plan of their own: compare with the oracle as well
        if B == len(lens):
            assert_close(bits_to_f64(bits_s), ref, "static decode", spread)
            assert_lse_close(lse_s.astype(np.float64), ref_lse, "static decode lse")
        else:
            r, rl, sp = oa.decode(case["pool"], case["row_off"][: B + 1], case["block_ids"], lens[:B], case["q"][:B],
                                  case["n_kv_heads"], with_spread=True)
            assert_close(bits_to_f64(bits_s), r, "static decode, smaller batch", sp)
            assert_lse_close(lse_s.astype(np.float64), rl, "static decode lse, smaller batch")


def test_static_scratch_stores_new_rows_like_the_heap_variant():
    torch = torch_mod()
    lens = np.array([700, 49, 16, 3000], dtype=np.int32)
    case = hw.build_case(entropy=[0x5C, 2], lens=lens, n_q_heads=16, n_kv_heads=2, head_dim=128, threads=2)
    rng = np.random.default_rng(5)
    rows = hw.f32_to_bf16_bits(rng.standard_normal((2, len(lens), 2, 128), dtype=np.float32))
    pools, outs = [], []
    for name in ("attn_decode_static", "attn_decode"):
        dc = DeviceCase(case, n_cu=16)
        from tests.gpu_util import to_dev_bf16
        k_new, v_new = to_dev_bf16(rows[0]), to_dev_bf16(rows[1])
        getattr(dc.ctx, name)(lens, case["row_off"], dc.row_off, dc.block_ids, dc.q, dc.out, dc.lse, k_new, v_new)
        torch.cuda.synchronize()
        pools.append(dc.pool_bits().copy())
        outs.append(bf16_to_host_bits(dc.out).copy())
    assert np.array_equal(pools[0], pools[1]) and np.array_equal(outs[0], outs[1])
    pool = case["pool"].copy()
    for b in range(len(lens)):
        oa.write_kv(pool, case["row_off"], case["block_ids"], [int(lens[b]) - 1], b, rows[0][b:b + 1], rows[1][b:b + 1])
    assert np.array_equal(pools[0], pool)


def test_static_scratch_rejects_what_does_not_fit():
    import paper_2603_28101_amd as heddle
    torch = torch_mod()
    # 1000 trajectories of one block each = 1000 partial slots: 1000 * 32 * 132 * 4 bytes > 16 MiB
    B = 1000
    lens = np.full(B, 16, dtype=np.int32)
    case = hw.build_case(entropy=[0x5C, 3], lens=lens, n_q_heads=32, n_kv_heads=8, head_dim=128, threads=4,
                         poison=False)
    dc = DeviceCase(case)
    dc.out.fill_(7.0)
    with pytest.raises(heddle.HeddleError) as e:
        dc.ctx.attn_decode_static(lens, case["row_off"], dc.row_off, dc.block_ids, dc.q, dc.out, dc.lse)
    assert e.value.code == heddle.E_NOMEM and "static scratch too small" in str(e.value)
    torch.cuda.synchronize()
    assert bool((dc.out == 7.0).all()), "a refused call must not touch its output"
    # the same batch fits the heap variant, and a batch under the limit still runs afterwards
    out, lse = dc.decode()
    ref, ref_lse, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], lens, case["q"],
                                     case["n_kv_heads"], with_spread=True)
    assert_close(out, ref, "heap decode of the large batch", spread)
    n = 900
    dc.ctx.attn_decode_static(lens[:n], case["row_off"][: n + 1], dc.row_off, dc.block_ids, dc.q, dc.out, dc.lse)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(bf16_to_host_bits(dc.out))[:n], ref[:n], "static decode under the limit", spread[:n])
