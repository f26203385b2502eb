"""Stream behaviour of the C ABI (needs the GPU): a context whose scratch was reserved never
synchronises inside an attention call, and calls of one context on different streams are ordered by
the library because they share its scratch."""
from __future__ import annotations

import numpy as np
import pytest

import heddle_workloads as hw
import paper_2603_28101_amd as heddle
from oracle import attention as oa
from tests.gpu_util import (DeviceCase, assert_close, assert_lse_close, bf16_to_host_bits, bits_to_f64, to_dev_bf16,
                            torch_mod)

pytestmark = pytest.mark.gpu


def _queue_reads(torch, stream, buf, sink, ms):
    """Enqueues about `ms` milliseconds of streaming reads of buf (at no more than 8 TB/s)."""
    reps = int(ms * 1e-3 * 8e12 / (buf.numel() * buf.element_size())) + 1
    for _ in range(reps):
        heddle.stream_read(buf, buf.numel() * buf.element_size(), sink, stream)
    return reps


def test_reserved_context_never_synchronises_in_attention_calls():
    torch = torch_mod()
    lens = np.array([3000, 900, 8000, 15, 2200, 5000, 77, 4500], dtype=np.int32)
    chunk = np.array([12, 7, 40, 1, 16, 33, 5, 2], dtype=np.int32)
    case = hw.build_case(entropy=[0x57, 1], lens=lens, chunk_lens=chunk, n_q_heads=32, n_kv_heads=8, head_dim=128,
                         threads=8)
    # every kernel has run once in this process (code objects loaded) before the context under test exists
    warm = hw.build_case(entropy=[0x57, 2], lens=[40, 3], chunk_lens=[5, 2], n_q_heads=32, n_kv_heads=8, head_dim=128,
                         threads=1)
    wd = DeviceCase(warm)
    wd.append()
    wd.ctx.attn_decode(warm["lens"], warm["row_off"], wd.row_off, wd.block_ids, wd.q[:2].contiguous(),
                       wd.out[:2].contiguous())
    filler = torch.empty(1 << 30, dtype=torch.int32, device="cuda")         # 4 GiB
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    stream = torch.cuda.Stream()
    heddle.stream_read(filler, filler.numel() * 4, sink, stream)
    torch.cuda.synchronize()

    dc = DeviceCase(case)
    dc.ctx.reserve(len(lens), int(chunk.sum()))
    dq = to_dev_bf16(case["q"][: len(lens)])                               # decode queries: one row per trajectory
    dout = torch.full((len(lens), 32, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    dlse = torch.full((len(lens), 32), float("nan"), dtype=torch.float32, device="cuda")
    k_new, v_new = to_dev_bf16(case["k_new"]), to_dev_bf16(case["v_new"])
    torch.cuda.synchronize()

    _queue_reads(torch, stream, filler, sink, 25.0)
    # the context's first decode and first append, behind 25 ms of queued work: a call that
    # synchronised (to grow its scratch) would return only when the stream has drained
    dc.ctx.attn_decode(lens, case["row_off"], dc.row_off, dc.block_ids, dq, dout, dlse, stream=stream)
    busy_after_decode = not stream.query()
    dc.ctx.attn_append(lens, case["cu_chunk"], case["row_off"], dc.row_off, dc.block_ids, dc.q, k_new, v_new,
                       dc.out, dc.lse, stream=stream)
    busy_after_append = not stream.query()
    torch.cuda.synchronize()
    assert busy_after_decode, "the first decode call of a reserved context waited for the stream"
    assert busy_after_append, "the first append call of a reserved context waited for the stream"

    ref, ref_lse, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], lens, case["q"][: len(lens)], 8,
                                     with_spread=True)
    assert_close(bits_to_f64(bf16_to_host_bits(dout)), ref, "decode behind queued work", spread)
    assert_lse_close(dlse.cpu().numpy().astype(np.float64), ref_lse)
    pool = case["pool"].copy()
    aref, aref_lse, aspread = oa.append(pool, case["row_off"], case["block_ids"], lens, case["cu_chunk"], case["q"],
                                        case["k_new"], case["v_new"], 8, with_spread=True, centered=None)
    assert_close(bits_to_f64(bf16_to_host_bits(dc.out)), aref, "append behind queued work", aspread)
    assert np.array_equal(dc.pool_bits(), pool)
    with pytest.raises(heddle.HeddleError):
        dc.ctx.reserve(0)


def test_calls_of_one_context_on_two_streams_are_ordered():
    """Decode on one stream, pack of a trajectory's blocks on another straight after it, decode
    again on the first: all three use the context's plan buffer and staging ring.  Behind 10 ms of
    queued work on the first stream the pack is issued long before the first decode has run."""
    torch = torch_mod()
    lens = np.array([9000, 300, 4100, 2500, 12000, 640], dtype=np.int32)
    case = hw.build_case(entropy=[0x57, 3], lens=lens, n_q_heads=8, n_kv_heads=2, head_dim=128, threads=4)
    dc = DeviceCase(case, n_cu=32)
    dc.ctx.reserve(len(lens))
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    filler = torch.empty(1 << 28, dtype=torch.int32, device="cuda")         # 1 GiB
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    out1 = torch.full_like(dc.out, float("nan"))
    out2 = torch.full_like(dc.out, float("nan"))
    ids = case["block_ids"][case["row_off"][4]:case["row_off"][5]]           # the 12 000-token trajectory
    staging = torch.zeros((len(ids), 2 * 2 * 16 * 128), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    _queue_reads(torch, a, filler, sink, 10.0)
    dc.ctx.attn_decode(lens, case["row_off"], dc.row_off, dc.block_ids, dc.q, out1, dc.lse, stream=a)
    dc.ctx.kv_pack(ids, staging, stream=b)
    lens2 = lens.copy()
    lens2[[0, 4]] = [5000, 3333]
    dc.ctx.attn_decode(lens2, case["row_off"], dc.row_off, dc.block_ids, dc.q, out2, None, stream=a)
    torch.cuda.synchronize()
    ref, _, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], lens, case["q"], 2, with_spread=True)
    assert_close(bits_to_f64(bf16_to_host_bits(out1)), ref, "decode on stream a", spread)
    ref2, _, spread2 = oa.decode(case["pool"], case["row_off"], case["block_ids"], lens2, case["q"], 2, with_spread=True)
    assert_close(bits_to_f64(bf16_to_host_bits(out2)), ref2, "second decode on stream a", spread2)
    packed = oa.pack(case["pool"], case["row_off"], case["block_ids"], 4, 12000)
    assert np.array_equal(bf16_to_host_bits(staging).reshape(packed.shape), packed)


def test_two_contexts_over_one_pool_overlap_on_two_streams():
    """The documented way to stage a cache while decode runs: a second context over the same pool
    on a second stream.  Nothing orders the two contexts against each other (each has its own plan
    buffer and staging ring), both only read the pool: eight decode steps on one stream interleaved
    with eight packs on the other, no synchronisation in between, every result as if issued alone."""
    torch = torch_mod()
    lens = np.array([9000, 300, 4100, 2500, 12000, 640], dtype=np.int32)
    case = hw.build_case(entropy=[0x57, 4], lens=lens, n_q_heads=8, n_kv_heads=2, head_dim=128, threads=4)
    dc = DeviceCase(case)
    side = heddle.Context(8, 2, 128, case["n_blocks"], kv_pool=dc.pool, device=0)
    dc.ctx.reserve(len(lens))
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [torch.full_like(dc.out, float("nan")) for _ in range(8)]
    stagings, packed_ref = [], []
    for i in range(8):
        t = i % len(lens)
        ids = case["block_ids"][case["row_off"][t]:case["row_off"][t + 1]]
        stagings.append((ids, torch.zeros((len(ids), 2 * 2 * 16 * 128), dtype=torch.bfloat16, device="cuda")))
        packed_ref.append(oa.pack(case["pool"], case["row_off"], case["block_ids"], t, int(lens[t])))
    step_lens = [np.maximum(1, lens - 37 * i).astype(np.int32) for i in range(8)]
    torch.cuda.synchronize()
    for i in range(8):
        dc.ctx.attn_decode(step_lens[i], case["row_off"], dc.row_off, dc.block_ids, dc.q, outs[i], None, stream=a)
        side.kv_pack(stagings[i][0], stagings[i][1], stream=b)
    torch.cuda.synchronize()
    for i in range(8):
        ref, _, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], step_lens[i], case["q"], 2,
                                   with_spread=True)
        assert_close(bits_to_f64(bf16_to_host_bits(outs[i])), ref, f"decode {i} beside a pack", spread)
        got = bf16_to_host_bits(stagings[i][1]).reshape(packed_ref[i].shape)
        assert np.array_equal(got, packed_ref[i]), f"pack {i} beside a decode"


def test_misaligned_pointers_are_refused():
    torch = torch_mod()
    case = hw.build_case(entropy=[0x57, 4], lens=[50, 9], n_q_heads=8, n_kv_heads=2, head_dim=128, threads=1)
    dc = DeviceCase(case)
    flat = torch.zeros(2 * 8 * 128 + 8, dtype=torch.bfloat16, device="cuda")
    for off in (1, 4):                                                      # 2 and 8 bytes off a 16-byte boundary
        with pytest.raises(heddle.HeddleError) as e:
            dc.ctx.attn_decode(case["lens"], case["row_off"], dc.row_off, dc.block_ids, dc.q,
                               flat.data_ptr() + 2 * off)
        assert e.value.code == heddle.E_INVAL
    bad_ids = case["block_ids"].copy()
    bad_ids[0] = case["n_blocks"]
    with pytest.raises(heddle.HeddleError) as e:
        dc.ctx.attn_decode_shared(case["lens"], case["row_off"], bad_ids, dc.row_off, dc.block_ids, dc.q, dc.out)
    assert e.value.code == heddle.E_INVAL
    out, lse = dc.decode()
    ref, ref_lse, spread = oa.decode(case["pool"], case["row_off"], case["block_ids"], case["lens"], case["q"], 2,
                                     with_spread=True)
    assert_close(out, ref, "after refused calls", spread)


def test_reserved_sizes_hold_for_random_batches_within_the_limits():
    """heddle_ctx_reserve sizes the scratch from upper bounds of the plan rules.  Random decode,
    shared-prefix decode and append batches within the reserved limits, under the default plan and
    under plans forced into many parts, must leave the allocated sizes as reserve made them."""
    torch = torch_mod()
    rng = np.random.default_rng(77)
    max_B, max_rows = 48, 2000
    for kw in (dict(), dict(n_cu=64, wg_per_cu=8, min_chunk_blk=1, tile_blk=4, max_split=64, group_wg_per_cu=4,
                            append_wg_per_cu=4, append_min_steps=1), dict(n_cu=8, max_split=3)):
        for n_q, n_kv in ((32, 8), (16, 2), (10, 2)):
            # one pool for all batches of this shape: 48 trajectories of up to 6000 + 300 tokens
            # the first 40 trajectories are four groups whose members share 8, 20, 50 and 100 leading blocks
            lens_max = np.full(max_B, 6400, dtype=np.int32)
            group_of = np.array([b % 4 if b < 40 else -1 for b in range(max_B)])
            shared = np.array([8, 20, 50, 100])
            pool_case = hw.build_case(entropy=[0x58, n_q], lens=lens_max, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=128,
                                      threads=8, poison=False, group_of=group_of, shared_blocks=shared)
            dc = DeviceCase(pool_case, **kw)
            dc.ctx.reserve(max_B, max_rows, with_shared_prefix=True)
            sizes = dc.ctx.scratch_bytes()
            qbuf = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((max_rows, n_q, 128), dtype=np.float32)))
            kbuf = to_dev_bf16(hw.f32_to_bf16_bits(rng.standard_normal((max_rows, n_kv, 128), dtype=np.float32)))
            obuf = torch.empty_like(qbuf)
            for trial in range(12):
                B = int(rng.integers(1, max_B + 1))
                kind = trial % 3
                if kind == 2:                                   # append: long-tailed contexts, chunks that sum to <= max_rows
                    L = np.minimum(rng.lognormal(np.log(800), 1.2, B).astype(np.int32) + 1, 6000)
                    C = rng.integers(1, max(2, max_rows // B), B).astype(np.int32)
                    cu = np.concatenate([[0], np.cumsum(C)]).astype(np.int32)
                    dc.ctx.attn_append(L, cu, pool_case["row_off"][: B + 1], dc.row_off, dc.block_ids, qbuf, kbuf, kbuf,
                                       obuf, None)
                else:
                    lens = np.minimum(rng.lognormal(np.log(600), 1.5, B).astype(np.int32) + 1, 6400)
                    if trial % 2:
                        lens[:] = int(rng.integers(1, 6400))    # equal lengths: the most items for a given total
                    if kind == 1:                               # long enough to use the shared blocks
                        lens = np.maximum(lens, np.where(group_of[:B] >= 0, shared[group_of[:B]] * 16 + 1, 1)).astype(np.int32)
                    if kind == 0:
                        dc.ctx.attn_decode(lens, pool_case["row_off"][: B + 1], dc.row_off, dc.block_ids, qbuf, obuf)
                    else:
                        dc.ctx.attn_decode_shared(lens, pool_case["row_off"][: B + 1], pool_case["block_ids"], dc.row_off,
                                                  dc.block_ids, qbuf, obuf)
                assert dc.ctx.scratch_bytes() == sizes, (kw, n_q, n_kv, trial, kind, B)
            torch.cuda.synchronize()
            dc.ctx.close()
