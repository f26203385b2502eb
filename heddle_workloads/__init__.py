"""Seeded synthetic inputs for paged-KV trajectory attention.

This module only *draws inputs* (context lengths, block tables, bf16 bit
patterns for Q / K / V).  It holds none of the attention arithmetic, none of
the split-K planning and none of the block-manager logic, so that the CPU
oracle and the HIP library can both be fed from it without sharing any code of
the method itself.

The shapes follow the rollout setting of the paper: batches of multi-step
trajectories (Sec. 2.1) whose lengths are long-tailed (Sec. 2.2: the slowest
trajectory takes more than four times the median), on Qwen3-8B/32B-shaped
attention heads (Sec. 7, workloads), with per-worker batches of the order of
one hundred trajectories (Sec. 7.1).  The paper's datasets are replaced by
lognormal length draws.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BLOCK_TOKENS = 16

# bf16 bit patterns used to poison memory no kernel may read into a result
POISON_NAN = np.uint16(0x7FC1)
POISON_INF = np.uint16(0x7F80)


@dataclass(frozen=True)
class Workload:
    cfg_id: int
    name: str
    kind: str  # "decode" | "append"
    B: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int


WORKLOADS = {
    1: Workload(1, "tiny-decode", "decode", 8, 8, 2, 64),
    2: Workload(2, "qwen3-8b-decode", "decode", 64, 32, 8, 128),
    3: Workload(3, "qwen3-32b-tp4-decode", "decode", 128, 16, 2, 128),
    4: Workload(4, "straggler-decode", "decode", 256, 32, 8, 128),
    5: Workload(5, "tool-append", "append", 32, 32, 8, 128),
    6: Workload(6, "grpo-group-decode", "decode", 128, 32, 8, 128),
    7: Workload(7, "verify-4-tokens", "append", 64, 32, 8, 128),
    8: Workload(8, "straggler-append", "append", 1, 32, 8, 128),
    9: Workload(9, "qwen3-14b-decode", "decode", 64, 40, 8, 128),
}

GROUP_SAMPLES = 16   # samples per prompt (Sec. 7, Workloads)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def k_view(pool: np.ndarray) -> np.ndarray:
    """K tiles of a pool as [n_blocks][n_kv][16 tokens][d] (a view)."""
    nb, nkv, _, n = pool.shape
    return pool[:, :, 0, :].reshape(nb, nkv, BLOCK_TOKENS, n // BLOCK_TOKENS)


def v_view(pool: np.ndarray) -> np.ndarray:
    """V tiles of a pool as [n_blocks][n_kv][d][16 tokens] (a view): V is stored transposed,
    the 16 tokens of one head-dim element are contiguous."""
    nb, nkv, _, n = pool.shape
    return pool[:, :, 1, :].reshape(nb, nkv, n // BLOCK_TOKENS, BLOCK_TOKENS)


def _lognormal_lengths(rng, n, median, sigma, lo, hi):
    x = np.exp(rng.normal(math.log(median), sigma, n))
    return np.clip(np.rint(x), lo, hi).astype(np.int64)


def draw_lengths(cfg_id: int, rng: np.random.Generator):
    """First draws of a workload's generator: context lengths (and chunk
    lengths for the append workload).  Returns (lens, chunk_lens or None)."""
    if cfg_id == 1:
        return rng.integers(1, 513, 8).astype(np.int64), None
    if cfg_id == 2:
        return _lognormal_lengths(rng, 64, 4096, 1.0, 256, 32768), None
    if cfg_id == 3:
        return _lognormal_lengths(rng, 128, 8192, 1.2, 512, 65536), None
    if cfg_id == 4:
        body = _lognormal_lengths(rng, 243, 2048, 0.8, 16, 65535)
        tail = rng.integers(65536, 131073, 13).astype(np.int64)
        return np.concatenate([body, tail]), None
    if cfg_id == 5:
        L = _lognormal_lengths(rng, 32, 8192, 1.0, 1024, 65536)
        C = rng.integers(64, 1025, 32).astype(np.int64)
        return L, C
    if cfg_id == 6:
        return draw_group_lengths(rng)[0], None
    if cfg_id == 7:   # the lengths of workload 2, four new tokens each (a speculative-decoding verify step)
        return _lognormal_lengths(rng, 64, 4096, 1.0, 256, 32768), np.full(64, 4, dtype=np.int64)
    if cfg_id == 8:   # one long-tail trajectory alone on the GPU receives a short tool output
        return rng.integers(100000, 120001, 1).astype(np.int64), rng.integers(32, 65, 1).astype(np.int64)
    if cfg_id == 9:   # the length law of workload 2 under the Qwen3-14B head shape (5 query heads per kv head)
        return _lognormal_lengths(rng, 64, 4096, 1.0, 256, 32768), None
    raise ValueError(f"unknown workload {cfg_id}")


def draw_group_lengths(rng: np.random.Generator):
    """Workload 6: 8 prompts x 16 samples.  Every sample of a prompt starts with the prompt's
    tokens (whole blocks of them are shared physically), then continues on its own.
    Returns (lens[128], group_of[128], prompt_tokens[8]); the batch order is a random
    interleaving of the samples."""
    n_prompts = 8
    prompt = _lognormal_lengths(rng, n_prompts, 2048, 0.6, 256, 8192)
    own = _lognormal_lengths(rng, n_prompts * GROUP_SAMPLES, 4096, 1.0, 17, 32768)
    group_of = np.repeat(np.arange(n_prompts), GROUP_SAMPLES)
    order = rng.permutation(n_prompts * GROUP_SAMPLES)
    group_of = group_of[order]
    lens = prompt[group_of] + own[order]
    return lens.astype(np.int64), group_of.astype(np.int64), prompt


def _bf16_normal(rng, shape):
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


_SLAB_BLOCKS = 512


def _fill_pool(pool: np.ndarray, entropy, threads: int) -> None:
    """Fill every physical block with N(0,1) bf16 values, slab by slab; each
    slab has its own child generator so the result does not depend on the
    number of threads."""
    n_blocks = pool.shape[0]
    n_slabs = (n_blocks + _SLAB_BLOCKS - 1) // _SLAB_BLOCKS
    children = np.random.SeedSequence(entropy).spawn(max(n_slabs, 1))

    def work(i):
        lo = i * _SLAB_BLOCKS
        hi = min(lo + _SLAB_BLOCKS, n_blocks)
        g = np.random.default_rng(children[i])
        pool[lo:hi] = _bf16_normal(g, pool[lo:hi].shape)

    if threads <= 1 or n_slabs <= 1:
        for i in range(n_slabs):
            work(i)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, range(n_slabs)))


def build_case(
    *,
    entropy,
    lens,
    n_q_heads: int,
    n_kv_heads: int,
    head_dim: int,
    chunk_lens=None,
    overprovision: float = 1.25,
    poison: bool = True,
    permute: bool = True,
    rng: np.random.Generator | None = None,
    threads: int = 8,
    group_of=None,
    shared_blocks=None,
):
    """Assemble one batch.

    group_of, shared_blocks  optional prefix sharing: trajectory b belongs to group group_of[b]
                (-1: none) and the first shared_blocks[g] entries of the block-table rows of
                all members of group g name the same physical blocks.  A shared block must lie
                wholly below every member's retained length.

    lens        tokens already held in the paged pool per trajectory.
    chunk_lens  if given, tokens to be appended per trajectory; the block
                table then covers lens + chunk_lens tokens and the slots of
                the chunk are left poisoned in the pool.

    Returns a dict of numpy arrays:
      pool       uint16 [n_blocks][n_kv][2][16*d]    (bf16 bits; index 2 = 0: K tile, token-major
                 [16][d]; index 2 = 1: V tile, transposed [d][16]; see k_view / v_view)
      row_off    int32  [B+1]   CSR offsets into block_ids
      block_ids  int32  [row_off[B]]
      lens       int32  [B]
      q          uint16 [n_rows][n_q][d]   n_rows = B (decode) or sum(chunk_lens)
      k_new, v_new  uint16 [n_rows][n_kv][d]  (append only)
      chunk_lens int32 [B], cu_chunk int32 [B+1]  (append only)
    Draw order: block permutation, Q, chunk K/V, then the pool slabs.
    """
    lens = np.asarray(lens, dtype=np.int64)
    B = lens.shape[0]
    if rng is None:
        rng = np.random.default_rng(entropy)
    total = lens.copy()
    if chunk_lens is not None:
        chunk_lens = np.asarray(chunk_lens, dtype=np.int64)
        total = total + chunk_lens
    nblk = (total + BLOCK_TOKENS - 1) // BLOCK_TOKENS
    row_off = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(nblk, out=row_off[1:])
    n_ref = int(row_off[-1])
    n_blocks = max(int(math.ceil(n_ref * overprovision)), n_ref, 1)

    if group_of is None:
        if permute:
            block_ids = rng.permutation(n_blocks)[:n_ref].astype(np.int32)
        else:
            block_ids = np.arange(n_ref, dtype=np.int32)
    else:
        group_of = np.asarray(group_of, dtype=np.int64)
        shared_blocks = np.asarray(shared_blocks, dtype=np.int64)
        own_blk = nblk.copy()
        for b in range(B):
            if group_of[b] >= 0:
                p = int(shared_blocks[group_of[b]])
                if p * BLOCK_TOKENS > lens[b]:
                    raise ValueError("a shared block must lie below the retained length")
                own_blk[b] -= p
        n_unique = int(shared_blocks.sum() + own_blk.sum())
        n_blocks = max(int(math.ceil(n_unique * overprovision)), n_unique, 1)
        phys = rng.permutation(n_blocks)[:n_unique] if permute else np.arange(n_unique)
        g_off = np.concatenate([[0], np.cumsum(shared_blocks)])
        cursor = int(g_off[-1])
        block_ids = np.empty(n_ref, dtype=np.int32)
        for b in range(B):
            lo = int(row_off[b])
            p = 0
            if group_of[b] >= 0:
                g = int(group_of[b])
                p = int(shared_blocks[g])
                block_ids[lo:lo + p] = phys[g_off[g]:g_off[g] + p]
            block_ids[lo + p:lo + int(nblk[b])] = phys[cursor:cursor + int(own_blk[b])]
            cursor += int(own_blk[b])

    n_rows = B if chunk_lens is None else int(chunk_lens.sum())
    q = _bf16_normal(rng, (n_rows, n_q_heads, head_dim))
    out = {}
    if chunk_lens is not None:
        out["k_new"] = _bf16_normal(rng, (n_rows, n_kv_heads, head_dim))
        out["v_new"] = _bf16_normal(rng, (n_rows, n_kv_heads, head_dim))
        cu = np.zeros(B + 1, dtype=np.int64)
        np.cumsum(chunk_lens, out=cu[1:])
        out["chunk_lens"] = chunk_lens.astype(np.int32)
        out["cu_chunk"] = cu.astype(np.int32)

    pool = np.empty((n_blocks, n_kv_heads, 2, BLOCK_TOKENS * head_dim), dtype=np.uint16)
    ent = list(entropy) if isinstance(entropy, (list, tuple)) else [int(entropy)]
    _fill_pool(pool, ent + [0x6B76], threads)

    if poison:
        referenced = np.zeros(n_blocks, dtype=bool)
        referenced[block_ids] = True
        free_blocks = np.nonzero(~referenced)[0]
        pool[free_blocks[0::2]] = POISON_NAN
        pool[free_blocks[1::2]] = POISON_INF
        # slots at or beyond the retained length inside referenced blocks
        for b in range(B):
            first = int(lens[b])
            row = block_ids[row_off[b]:row_off[b + 1]]
            blk, slot = divmod(first, BLOCK_TOKENS)
            if blk < len(row):
                if slot:
                    k_view(pool)[row[blk], :, slot:, :] = POISON_NAN
                    v_view(pool)[row[blk], :, :, slot:] = POISON_NAN
                    blk += 1
                if blk < len(row):
                    pool[row[blk:]] = POISON_NAN

    out.update(
        pool=pool,
        row_off=row_off.astype(np.int32),
        block_ids=block_ids,
        lens=lens.astype(np.int32),
        q=q,
        n_q_heads=n_q_heads,
        n_kv_heads=n_kv_heads,
        head_dim=head_dim,
        n_blocks=n_blocks,
    )
    return out


def make_workload(cfg_id: int, seed: int = 0, *, threads: int = 8, **kw):
    """One of the named workloads, generator = default_rng([cfg_id, seed]);
    draw order: lengths, chunk lengths, block permutation, Q, chunk K/V, pool."""
    w = WORKLOADS[cfg_id]
    rng = np.random.default_rng([cfg_id, seed])
    if cfg_id == 6:
        lens, group_of, prompt = draw_group_lengths(rng)
        chunk = None
        # whole prompt blocks are shared; a prompt's last, partly filled block is private
        kw = dict(kw, group_of=group_of, shared_blocks=prompt // BLOCK_TOKENS)
    else:
        lens, chunk = draw_lengths(cfg_id, rng)
    case = build_case(
        entropy=[cfg_id, seed],
        lens=lens,
        chunk_lens=chunk,
        n_q_heads=w.n_q_heads,
        n_kv_heads=w.n_kv_heads,
        head_dim=w.head_dim,
        rng=rng,
        threads=threads,
        **kw,
    )
    case["workload"] = w
    if cfg_id == 6:
        case["group_of"] = group_of.astype(np.int32)
        case["shared_blocks"] = (prompt // BLOCK_TOKENS).astype(np.int32)
    return case


def workload_lengths(cfg_id: int, seed: int = 0):
    """Only the length draws of a named workload (cheap; no pool)."""
    rng = np.random.default_rng([cfg_id, seed])
    return draw_lengths(cfg_id, rng)


def unique_kv_tokens(case) -> int:
    """Tokens of context held in distinct physical blocks: a block that several block-table
    rows name is counted once (tokens of its first owner)."""
    seen = set()
    total = 0
    for b in range(len(case["lens"])):
        row = case["block_ids"][case["row_off"][b]:case["row_off"][b + 1]]
        n = int(case["lens"][b])
        for i, blk in enumerate(row):
            t = min(BLOCK_TOKENS, n - i * BLOCK_TOKENS)
            if t <= 0:
                break
            if int(blk) not in seen:
                seen.add(int(blk))
                total += t
    return total


def kv_bytes(lens, n_kv_heads: int, head_dim: int) -> int:
    """Bytes of K and V (bf16) that one decode step over these contexts has to
    read: every live token once per kv head."""
    return int(np.asarray(lens, dtype=np.int64).sum()) * 2 * n_kv_heads * head_dim * 2
