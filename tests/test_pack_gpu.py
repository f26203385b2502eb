"""GPU parity of heddle_kv_pack / heddle_kv_unpack with the oracle's pack / unpack: byte work,
so every comparison is bit-exact.  (Staging form of a trajectory's cache, Sec. 4.2 / Sec. 5.3.)"""
import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from tests.gpu_util import DeviceCase, bf16_to_host_bits, torch_mod

pytestmark = pytest.mark.gpu


def _case(seed=3, lens=(700, 1, 16, 17, 4095, 33), n_q=8, n_kv=2, d=128):
    return hw.build_case(entropy=[7, seed], lens=np.asarray(lens, dtype=np.int32), n_q_heads=n_q,
                         n_kv_heads=n_kv, head_dim=d, threads=4)


def _staging(n_blocks, case):
    torch = torch_mod()
    per_block = case["n_kv_heads"] * 2 * 16 * case["head_dim"]
    return torch.full((max(n_blocks, 1), per_block), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)


@pytest.mark.parametrize("n_kv,d", [(2, 128), (1, 64), (8, 128), (4, 64)])
def test_pack_matches_oracle(n_kv, d):
    case = _case(seed=5 + n_kv, n_q=n_kv * 2, n_kv=n_kv, d=d)
    dc = DeviceCase(case)
    for b, L in enumerate(case["lens"]):
        ref = oa.pack(case["pool"], case["row_off"], case["block_ids"], b, int(L))
        ids = case["block_ids"][case["row_off"][b]:case["row_off"][b + 1]][: ref.shape[0]]
        st = _staging(ref.shape[0], case)
        dc.ctx.kv_pack(ids, st)
        torch_mod().cuda.synchronize()
        got = bf16_to_host_bits(st)[: ref.shape[0]].reshape(ref.shape)
        assert np.array_equal(got, ref), f"trajectory {b} (length {L})"


def test_unpack_under_other_blocks_then_decode():
    """Pack every trajectory, unpack under a fresh random assignment of blocks into a second
    pool, and the pool bytes equal the oracle's unpack; decoding over the moved caches gives the
    same bits as over the originals."""
    case = _case(seed=11)
    dc = DeviceCase(case)
    out0, lse0 = dc.decode()
    rng = np.random.default_rng(2)
    nb = case["n_blocks"]
    ref_pool = np.full_like(case["pool"], 0x7FC0)            # destination pool starts as NaN patterns
    torch = torch_mod()
    moved = DeviceCase({**case, "pool": ref_pool.copy()})
    perm = rng.permutation(nb).astype(np.int32)
    new_ids, cursor = np.empty_like(case["block_ids"]), 0
    for b, L in enumerate(case["lens"]):
        lo, hi = int(case["row_off"][b]), int(case["row_off"][b + 1])
        staged_ref = oa.pack(case["pool"], case["row_off"], case["block_ids"], b, int(L))
        n = staged_ref.shape[0]
        dst = perm[cursor:cursor + (hi - lo)]
        cursor += hi - lo
        new_ids[lo:hi] = dst
        oa.unpack(ref_pool, dst[:n], staged_ref)
        st = _staging(n, case)
        dc.ctx.kv_pack(case["block_ids"][lo:lo + n], st)
        moved.ctx.kv_unpack(dst[:n], st)
    torch.cuda.synchronize()
    got_pool = bf16_to_host_bits(moved.pool).reshape(ref_pool.shape)
    assert np.array_equal(got_pool, ref_pool)
    from tests.gpu_util import to_dev_i32
    moved.block_ids = to_dev_i32(new_ids)
    out1, lse1 = moved.decode()
    assert np.array_equal(out0, out1) and np.array_equal(lse0, lse1)


def test_roundtrip_whole_workload_shape():
    """All blocks of the small long-tail workload in one call each way."""
    case = hw.make_workload(1, seed=0)
    dc = DeviceCase(case)
    used = np.concatenate([case["block_ids"][case["row_off"][b]:case["row_off"][b + 1]]
                           for b in range(len(case["lens"]))]).astype(np.int32)
    st = _staging(len(used), case)
    dc.ctx.kv_pack(used, st)
    torch = torch_mod()
    torch.cuda.synchronize()
    got = bf16_to_host_bits(st).reshape((len(used),) + case["pool"].shape[1:])
    assert np.array_equal(got, case["pool"][used])
    dc.pool.view(torch.int16).zero_()
    dc.ctx.kv_unpack(used, st)
    torch.cuda.synchronize()
    back = bf16_to_host_bits(dc.pool).reshape(case["pool"].shape)
    assert np.array_equal(back[used], case["pool"][used])
    untouched = np.setdiff1d(np.arange(case["n_blocks"]), used)
    assert not back[untouched].any()


def test_empty_and_errors():
    import paper_2603_28101_amd as heddle
    case = _case(seed=1, lens=(40,))
    dc = DeviceCase(case)
    st = _staging(4, case)
    before = bf16_to_host_bits(st).copy()
    dc.ctx.kv_pack(np.zeros(0, dtype=np.int32), st)
    dc.ctx.kv_unpack(np.zeros(0, dtype=np.int32), st)
    torch_mod().cuda.synchronize()
    assert np.array_equal(bf16_to_host_bits(st), before)
    with pytest.raises(heddle.HeddleError):
        dc.ctx.kv_pack(np.array([case["n_blocks"]], dtype=np.int32), st)
    with pytest.raises(heddle.HeddleError):
        dc.ctx.kv_pack(np.array([-1], dtype=np.int32), st)
    with pytest.raises(heddle.HeddleError):
        dc.ctx.kv_unpack(np.array([1, 1], dtype=np.int32), st)


@pytest.mark.parametrize("n_kv,d", [(2, 128), (8, 128), (2, 64), (1, 128)])
def test_copy_blocks_matches_oracle(n_kv, d):
    """heddle_kv_copy: forks of blocks inside the pool, bit for bit, nothing else touched; then a
    trajectory that names the copies decodes like the one that names the originals."""
    import paper_2603_28101_amd as heddle
    torch = torch_mod()
    case = _case(seed=5, lens=(700, 1, 16, 17, 33), n_q=n_kv * 4, n_kv=n_kv, d=d)
    dc = DeviceCase(case)
    used = set(int(x) for x in case["block_ids"])
    free = [i for i in range(case["n_blocks"]) if i not in used]
    row0 = case["block_ids"][case["row_off"][0]:case["row_off"][1]]
    n = min(len(free), len(row0))
    assert n >= 5
    src, dst = np.asarray(row0[:n], dtype=np.int32), np.asarray(free[:n], dtype=np.int32)
    pool = case["pool"].copy()
    oa.copy_blocks(pool, src, dst)
    dc.ctx.kv_copy(src, dst)
    torch.cuda.synchronize()
    assert np.array_equal(dc.pool_bits(), pool)
    dc.ctx.kv_copy(np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int32))      # nothing to do
    for bad_src, bad_dst in (([int(src[0])], [case["n_blocks"]]), ([-1], [int(dst[0])]),
                             ([int(src[0]), int(src[1])], [int(dst[0]), int(dst[0])]),     # a destination twice
                             ([int(src[0]), int(dst[1])], [int(dst[1]), int(dst[2])])):    # a destination is a source
        with pytest.raises(heddle.HeddleError) as e:
            dc.ctx.kv_copy(np.asarray(bad_src, dtype=np.int32), np.asarray(bad_dst, dtype=np.int32))
        assert e.value.code == heddle.E_INVAL
    torch.cuda.synchronize()
    assert np.array_equal(dc.pool_bits(), pool)


def test_pack_of_the_benchmark_workload_at_full_size():
    """The launch `bench.py --op pack` times: every block of the Qwen3-8B decode workload (1.77 GB)
    gathered in one call; all bytes compared, then scattered back into a cleared pool."""
    torch = torch_mod()
    case = hw.make_workload(2, 0, threads=16)
    dc = DeviceCase(case)
    used = np.concatenate([case["block_ids"][case["row_off"][b]:case["row_off"][b + 1]]
                           for b in range(len(case["lens"]))]).astype(np.int32)
    print("pack full size:", len(used), "blocks", flush=True)
    st = _staging(len(used), case)
    dc.ctx.kv_pack(used, st)
    torch.cuda.synchronize()
    got = bf16_to_host_bits(st).reshape((len(used),) + case["pool"].shape[1:])
    assert np.array_equal(got, case["pool"][used])
    del got
    dc.pool.view(torch.int16).zero_()
    dc.ctx.kv_unpack(used, st)
    torch.cuda.synchronize()
    back = bf16_to_host_bits(dc.pool).reshape(case["pool"].shape)
    assert np.array_equal(back[used], case["pool"][used])
    mask = np.ones(case["n_blocks"], dtype=bool)
    mask[used] = False
    assert not back[mask].any()
