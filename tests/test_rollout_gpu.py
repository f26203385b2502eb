"""A small rollout through every entry point in the order a worker would call them (paper
Sec. 2.1: a trajectory alternates generation with tool calls and keeps its context; Sec. 4.2: a
preempted trajectory keeps its cache; Sec. 7: the samples of a prompt share its tokens):

  prompt prefill (append with L = 0) -> decode steps that store their own K/V row -> a tool-output
  chunk (append) -> more decode -> one trajectory is packed, its blocks freed and handed to
  another, later it is unpacked under new blocks -> decode with shared prompt blocks.

The library's block manager hands out the blocks; the float64 oracle mirrors every call on its own
copy of the pool, and outputs and the pool are compared after each call.  A second test draws
such rollouts at random: head shape, prompts and samples, and a sequence of decode steps, tool
outputs, preemptions, resumptions, departures and arrivals.  Needs the GPU."""
import os

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from oracle.kv_manager import KVManager
from tests.gpu_util import (assert_close, assert_lse_close, bf16_to_host_bits, bits_to_f64, to_dev_bf16, to_dev_i32,
                            torch_mod)

pytestmark = pytest.mark.gpu

N_Q, N_KV, D = 8, 2, 128
N_BLOCKS = 400


def bf16(rng, shape):
    return hw.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


class Worker:
    """Library context and oracle state side by side."""

    def __init__(self, seed, n_q=N_Q, n_kv=N_KV, d=D, n_blocks=N_BLOCKS):
        import paper_2603_28101_amd as heddle
        torch = torch_mod()
        self.rng = np.random.default_rng(seed)
        self.n_q, self.n_kv, self.d = n_q, n_kv, d
        pool = np.full((n_blocks, n_kv, 2, 16 * d), 0x7FC0, dtype=np.uint16)       # everything starts as NaN
        self.ref_pool = pool.copy()
        self.pool = to_dev_bf16(pool)
        self.ctx = heddle.Context(n_q, n_kv, d, n_blocks, kv_pool=self.pool, device=0)
        self.ref_blocks = KVManager(n_blocks)
        self.tables = []          # per trajectory: list of physical blocks
        self.lens = []            # tokens stored
        self.torch = torch

    # -- blocks: the library's manager and the oracle's must hand out the same ids
    def grow(self, b, tokens):
        need = -(-tokens // 16) - len(self.tables[b])
        if need > 0:
            got = self.ctx.kv_alloc(need)
            code, ref = self.ref_blocks.alloc(need)
            assert code == 0 and got.tolist() == ref
            self.tables[b] += got.tolist()

    def csr(self, order):
        row_off = np.concatenate([[0], np.cumsum([len(self.tables[b]) for b in order])]).astype(np.int32)
        ids = np.asarray([x for b in order for x in self.tables[b]], dtype=np.int32)
        return row_off, ids

    def check_pool(self, what):
        got = bf16_to_host_bits(self.pool).reshape(self.ref_pool.shape)
        assert np.array_equal(got, self.ref_pool), f"pool differs after {what}"

    # -- calls
    def append(self, order, chunk_lens, what):
        rng, torch = self.rng, self.torch
        for b, c in zip(order, chunk_lens):
            self.grow(b, self.lens[b] + c)
        row_off, ids = self.csr(order)
        n_rows = int(sum(chunk_lens))
        q = bf16(rng, (n_rows, self.n_q, self.d))
        k, v = bf16(rng, (n_rows, self.n_kv, self.d)), bf16(rng, (n_rows, self.n_kv, self.d))
        L = np.asarray([self.lens[b] for b in order], dtype=np.int32)
        cu = np.concatenate([[0], np.cumsum(chunk_lens)]).astype(np.int32)
        out = torch.full((n_rows, self.n_q, self.d), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((n_rows, self.n_q), float("nan"), dtype=torch.float32, device="cuda")
        self.ctx.attn_append(L, cu, row_off, to_dev_i32(row_off), to_dev_i32(ids), to_dev_bf16(q), to_dev_bf16(k),
                             to_dev_bf16(v), out, lse)
        torch.cuda.synchronize()
        ref, ref_lse, spread = oa.append(self.ref_pool, row_off, ids, L, cu, q, k, v, self.n_kv, with_spread=True,
                                         centered=None)
        assert_close(bits_to_f64(bf16_to_host_bits(out)), ref, what, spread)
        assert_lse_close(lse.cpu().numpy(), ref_lse, what)
        for b, c in zip(order, chunk_lens):
            self.lens[b] += c
        self.check_pool(what)

    def decode(self, order, what, shared=False, expect_groups=True):
        rng, torch = self.rng, self.torch
        for b in order:
            self.grow(b, self.lens[b] + 1)
        row_off, ids = self.csr(order)
        B = len(order)
        q = bf16(rng, (B, self.n_q, self.d))
        k, v = bf16(rng, (B, self.n_kv, self.d)), bf16(rng, (B, self.n_kv, self.d))
        lens = np.asarray([self.lens[b] + 1 for b in order], dtype=np.int32)      # the new row included
        out = torch.full((B, self.n_q, self.d), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, self.n_q), float("nan"), dtype=torch.float32, device="cuda")
        args = (to_dev_i32(row_off), to_dev_i32(ids), to_dev_bf16(q), out, lse, to_dev_bf16(k), to_dev_bf16(v))
        if shared:
            plan = self.ctx.plan_decode_shared(lens, row_off, ids)
            assert plan["n_groups"] >= 1 or not expect_groups, "the samples of a prompt were expected to share its blocks"
            self.ctx.attn_decode_shared(lens, row_off, ids, *args)
        else:
            self.ctx.attn_decode(lens, row_off, *args)
        torch.cuda.synchronize()
        for i in range(B):
            oa.write_kv(self.ref_pool, row_off, ids, [int(lens[i]) - 1], i, k[i:i + 1], v[i:i + 1])
        ref, ref_lse, spread = oa.decode(self.ref_pool, row_off, ids, lens, q, self.n_kv, with_spread=True,
                                         centered=None if shared else True)
        assert_close(bits_to_f64(bf16_to_host_bits(out)), ref, what, spread)
        assert_lse_close(lse.cpu().numpy(), ref_lse, what)
        for b in order:
            self.lens[b] += 1
        self.check_pool(what)


    def fork(self, leader, members):
        """The members start from the leader's whole blocks (one more holder each) and from a copy of
        its partly filled last block in a block of their own."""
        whole = self.lens[leader] // 16
        for b in members:
            self.tables[b] = list(self.tables[leader][:whole])
            if whole:
                self.ctx.kv_retain(np.asarray(self.tables[b], dtype=np.int32))
                assert self.ref_blocks.retain(self.tables[b]) == 0
            self.lens[b] = whole * 16
            self.grow(b, self.lens[leader])
            self.lens[b] = self.lens[leader]
        if self.lens[leader] % 16 and members:
            src = [self.tables[leader][whole]] * len(members)
            dst = [self.tables[b][whole] for b in members]
            self.ctx.kv_copy(np.asarray(src, dtype=np.int32), np.asarray(dst, dtype=np.int32))
            oa.copy_blocks(self.ref_pool, src, dst)
            self.torch.cuda.synchronize()
        self.check_pool("fork")

    def release(self, b):
        self.ctx.kv_free(np.asarray(self.tables[b], dtype=np.int32))
        assert self.ref_blocks.free(self.tables[b]) == 0
        assert self.ctx.kv_num_free() == self.ref_blocks.num_free()
        self.tables[b] = []

    def preempt(self, b):
        """Packs the trajectory's whole cache (shared blocks included) and frees its table."""
        torch = self.torch
        n_blk = -(-self.lens[b] // 16)
        blocks = self.tables[b][:n_blk]
        staging = torch.empty((n_blk, self.n_kv * 2 * 16 * self.d), dtype=torch.bfloat16, device="cuda")
        self.ctx.kv_pack(np.asarray(blocks, dtype=np.int32), staging)
        torch.cuda.synchronize()
        row_off, ids = self.csr([b])
        staged_ref = oa.pack(self.ref_pool, row_off, ids, 0, self.lens[b])
        assert np.array_equal(bf16_to_host_bits(staging).reshape(staged_ref.shape), staged_ref)
        self.release(b)
        return staging, staged_ref

    def resume(self, b, staging, staged_ref):
        """The trajectory comes back under whatever blocks are free now (all its own from here on)."""
        n_blk = staged_ref.shape[0]
        got = self.ctx.kv_alloc(n_blk)
        code, ref_ids = self.ref_blocks.alloc(n_blk)
        assert code == 0 and got.tolist() == ref_ids
        self.ctx.kv_unpack(got, staging)
        self.torch.cuda.synchronize()
        oa.unpack(self.ref_pool, got, staged_ref)
        self.tables[b] = got.tolist()
        self.check_pool("unpack")


def test_rollout_of_six_trajectories():
    torch = torch_mod()
    w = Worker(2026)
    # two prompts; samples 0-2 belong to the first, 3-5 to the second
    prompts = [200, 75]
    w.tables = [[] for _ in range(6)]
    w.lens = [0] * 6

    # 1. prefill the two prompts once each (trajectories 0 and 3)
    w.append([0, 3], prompts, "prompt prefill")
    # the other samples of a prompt start from its whole blocks (shared physically: one more holder
    # each) and from a copy of its partly filled last block (8 and 11 tokens) in a block of their own
    for leader, members in ((0, (1, 2)), (3, (4, 5))):
        whole = w.lens[leader] // 16
        assert w.lens[leader] % 16 != 0
        for b in members:
            w.tables[b] = list(w.tables[leader][:whole])
            w.ctx.kv_retain(np.asarray(w.tables[b], dtype=np.int32))
            assert w.ref_blocks.retain(w.tables[b]) == 0
            w.lens[b] = whole * 16
            w.grow(b, w.lens[leader])                                     # the block for the copy
            w.lens[b] = w.lens[leader]
        src = [w.tables[leader][whole]] * len(members)
        dst = [w.tables[b][whole] for b in members]
        w.ctx.kv_copy(np.asarray(src, dtype=np.int32), np.asarray(dst, dtype=np.int32))
        oa.copy_blocks(w.ref_pool, src, dst)
    torch.cuda.synchronize()
    w.check_pool("forks of the prompts' last blocks")
    assert w.lens == [200, 200, 200, 75, 75, 75]

    # 2. a few decode steps for everybody, shared-prefix path (12 and 4 whole prompt blocks)
    for step in range(3):
        w.decode([0, 1, 2, 3, 4, 5], f"shared decode step {step}", shared=True)
    # 3. tool outputs of very different sizes for some, a verify-like 3-token chunk for one
    w.append([1, 4, 5], [150, 33, 3], "tool outputs")
    # 4. plain decode in a different batch order, twice
    for step in range(2):
        w.decode([5, 2, 0, 4], f"decode step {step}")

    # 5. trajectory 1 is preempted: its private blocks packed, its whole table freed; the prompt's
    #    blocks stay allocated, samples 0 and 2 still hold them ...
    b = 1
    n_blk = -(-w.lens[b] // 16)
    shared_blk = prompts[0] // 16
    private = w.tables[b][shared_blk:n_blk]
    staging = torch.empty((len(private), N_KV * 2 * 16 * D), dtype=torch.bfloat16, device="cuda")
    w.ctx.kv_pack(np.asarray(private, dtype=np.int32), staging)
    torch.cuda.synchronize()
    row_off, ids = w.csr([b])
    staged_ref = oa.pack(w.ref_pool, row_off, ids, 0, w.lens[b])[shared_blk:]
    assert np.array_equal(bf16_to_host_bits(staging).reshape(staged_ref.shape), staged_ref)
    free_before = w.ctx.kv_num_free()
    w.ctx.kv_free(np.asarray(w.tables[b], dtype=np.int32))
    assert w.ref_blocks.free(w.tables[b]) == 0
    assert w.ctx.kv_num_free() == free_before + len(w.tables[b]) - shared_blk
    prompt_blocks = w.tables[b][:shared_blk]
    w.tables[b] = []
    # ... which the next tool output of trajectory 3 takes (most recently freed first)
    w.append([3], [300], "tool output into recycled blocks")
    # 6. trajectory 1 comes back: it holds the prompt's blocks again and gets new private ones
    w.ctx.kv_retain(np.asarray(prompt_blocks, dtype=np.int32))
    assert w.ref_blocks.retain(prompt_blocks) == 0
    got = w.ctx.kv_alloc(len(private))
    code, ref_ids = w.ref_blocks.alloc(len(private))
    assert code == 0 and got.tolist() == ref_ids
    w.ctx.kv_unpack(got, staging)
    torch.cuda.synchronize()
    oa.unpack(w.ref_pool, got, staged_ref)
    w.tables[b] = prompt_blocks + got.tolist()
    w.check_pool("unpack")
    # 7. everybody decodes again, shared path, then plain
    w.decode([0, 1, 2, 3, 4, 5], "shared decode after resume", shared=True)
    w.decode([0, 1, 2, 3, 4, 5], "decode after resume")
    assert w.ctx.kv_num_free() == w.ref_blocks.num_free()
    # 8. everybody finishes: each frees its whole table, shared blocks return with their last holder
    for b in range(6):
        w.ctx.kv_free(np.asarray(w.tables[b], dtype=np.int32))
        assert w.ref_blocks.free(w.tables[b]) == 0
    assert w.ctx.kv_num_free() == N_BLOCKS == w.ref_blocks.num_free()


SEEDS = range(int(os.environ.get("HEDDLE_RANDOM_FIRST", "0")),
              int(os.environ.get("HEDDLE_RANDOM_FIRST", "0")) + max(6, int(os.environ.get("HEDDLE_RANDOM_CASES", "0"))))


@pytest.mark.parametrize("seed", SEEDS)
def test_random_rollout(seed):
    """A rollout drawn at random: a head shape, one to three prompts with one to four samples each,
    then a dozen steps, each a decode step (plain or shared-prefix) of a random subset in random
    order, tool outputs of random sizes, a preemption (pack, free), a resumption (alloc, unpack), a
    departure (free) or an arrival (a new prompt into recycled blocks).  The oracle mirrors every
    call; outputs, block ids and the whole pool are compared after each."""
    rng = np.random.default_rng([104, seed])
    n_q, n_kv, d = [(8, 2, 128), (4, 1, 128), (16, 2, 128), (2, 2, 128), (10, 2, 128), (8, 2, 64), (32, 8, 128)][
        int(rng.integers(0, 7))]
    n_blocks = 700
    w = Worker([104, seed, 1], n_q, n_kv, d, n_blocks)
    n_prompts = int(rng.integers(1, 4))
    groups = [int(rng.integers(1, 5)) for _ in range(n_prompts)]
    n_traj = sum(groups)
    w.tables = [[] for _ in range(n_traj)]
    w.lens = [0] * n_traj
    leaders, b = [], 0
    for g in groups:
        leaders.append(b)
        b += g
    prompt_len = [int(rng.choice([5, 16, 40, 75, 128, 200, 333])) for _ in range(n_prompts)]
    print(f"random rollout {seed}: heads {n_q}/{n_kv} d {d} prompts {prompt_len} samples {groups}", flush=True)
    w.append(leaders, prompt_len, "prompt prefill")
    for leader, g in zip(leaders, groups):
        w.fork(leader, list(range(leader + 1, leader + g)))
    live, away = set(range(n_traj)), {}
    for step in range(12):
        op = str(rng.choice(["decode", "decode", "shared", "shared", "append", "append", "preempt", "resume", "leave",
                             "arrive"]))
        room = w.ctx.kv_num_free()
        members = sorted(live)
        what = f"rollout {seed} step {step} {op}"
        if op in ("decode", "shared") and members:
            order = [int(x) for x in rng.permutation(members)[:int(rng.integers(1, len(members) + 1))]]
            if room < len(order):
                continue
            print(what, order, flush=True)
            w.decode(order, what, shared=op == "shared", expect_groups=False)
        elif op == "append" and members:
            order = [int(x) for x in rng.permutation(members)[:int(rng.integers(1, len(members) + 1))]]
            chunk = [int(rng.choice([1, 3, 8, 17, 40, 90, 160])) for _ in order]
            if room < sum(-(-c // 16) + 1 for c in chunk):
                continue
            print(what, order, chunk, flush=True)
            w.append(order, chunk, what)
        elif op == "preempt" and len(members) > 1:
            b = int(rng.choice(members))
            print(what, b, flush=True)
            away[b] = w.preempt(b)
            live.discard(b)
        elif op == "resume" and away:
            b = int(rng.choice(sorted(away)))
            if room < away[b][1].shape[0]:
                continue
            print(what, b, flush=True)
            w.resume(b, *away.pop(b))
            live.add(b)
        elif op == "leave" and len(members) > 1:
            b = int(rng.choice(members))
            print(what, b, flush=True)
            w.release(b)
            live.discard(b)
        elif op == "arrive" and room > 40:
            w.tables.append([])
            w.lens.append(0)
            b = len(w.lens) - 1
            n = int(rng.choice([1, 16, 50, 129, 300]))
            print(what, b, n, flush=True)
            w.append([b], [n], what)
            live.add(b)
    for b in sorted(live):
        w.release(b)
    # trajectories still away hold no blocks: everything is free again
    assert w.ctx.kv_num_free() == n_blocks == w.ref_blocks.num_free()
