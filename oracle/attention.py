"""Float64 definition of decode and append attention over a paged KV pool.
TEST INFRASTRUCTURE ONLY (see package docstring).

Conventions (the paper fixes none of these; it delegates generation to an
inference engine, Sec. 7 "Implementation", and cites paged attention, Sec. 9):

  pool       uint16 [n_blocks][n_kv][2][16*d]  bf16 bit patterns; [..][0] is the K tile,
             token-major [16][d]; [..][1] is the V tile stored transposed, [d][16]
  table      CSR: block_ids[row_off[b] + p // 16] is the physical block that
             holds token position p of trajectory b, slot p % 16
  heads      query head j reads kv head j // (n_q / n_kv)
  scale      1 / sqrt(d)
  len[b]     number of KV rows the query sees, its own row included
  append     chunk row i of trajectory b sits at position L_b + i and sees
             positions 0 .. L_b + i inclusive
"""
from __future__ import annotations

import math

import numpy as np

BLOCK_TOKENS = 16


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening: a bf16 is the upper half of a float32."""
    u32 = bits.astype(np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def gather(pool_bits, row_off, block_ids, b: int, length: int):
    """K, V of trajectory b as float64 [n_kv][length][d], read through the
    block table (definition of the paged layout)."""
    nblk = (length + BLOCK_TOKENS - 1) // BLOCK_TOKENS
    row = np.asarray(block_ids[row_off[b]:row_off[b + 1]])
    if nblk > row.shape[0]:
        raise ValueError("block table row shorter than the context")
    blocks = pool_bits[row[:nblk]]                       # [nblk][n_kv][2][16*d]
    n_kv = blocks.shape[1]
    d = blocks.shape[3] // BLOCK_TOKENS
    k_tiles = blocks[:, :, 0, :].reshape(nblk, n_kv, BLOCK_TOKENS, d)
    v_tiles = blocks[:, :, 1, :].reshape(nblk, n_kv, d, BLOCK_TOKENS).transpose(0, 1, 3, 2)
    kv = np.stack([k_tiles, v_tiles])                    # [2][nblk][n_kv][16][d]
    kv = kv.transpose(0, 2, 1, 3, 4).reshape(2, n_kv, nblk * BLOCK_TOKENS, d)
    kv = bf16_bits_to_f64(kv[:, :, :length, :])
    return kv[0], kv[1]


def attend(q, K, V, scale):
    """softmax(scale * K q) V for one query vector; also the log-sum-exp and
    the weights."""
    z = scale * (K @ q)
    m = z.max()
    e = np.exp(z - m)
    denom = e.sum()
    w = e / denom
    return w @ V, m + math.log(denom), w


def weight_spread(w, V, out, centered=True):
    """Standard deviation of the output under independent unit-variance relative
    perturbations of the weights, to first order.  centered: numerator and denominator are
    perturbed alike, sqrt(sum_t w_t^2 (V[t] - out)^2); otherwise only the numerator is,
    sqrt(sum_t w_t^2 V[t]^2); centered=None: some keys one way and the rest the other way,
    bounded by the root of the sum of both squares.  The tests use it to bound what rounding
    the weights to bf16 may do to a result."""
    if centered is None:
        return np.sqrt((w * w) @ ((V - out) ** 2) + (w * w) @ (V ** 2))
    dev = V - out if centered else V
    return np.sqrt((w * w) @ (dev ** 2))


def decode(pool_bits, row_off, block_ids, lens, q_bits, n_kv_heads: int, scale=None, with_spread=False,
           centered=True):
    """One new token per trajectory.  q_bits uint16 [B][n_q][d].
    Returns out float64 [B][n_q][d], lse float64 [B][n_q] (and weight_spread [B][n_q][d])."""
    B, n_q, d = q_bits.shape
    G = n_q // n_kv_heads
    s = 1.0 / math.sqrt(d) if scale is None else float(scale)
    q = bf16_bits_to_f64(q_bits)
    out = np.zeros((B, n_q, d))
    lse = np.zeros((B, n_q))
    spread = np.zeros((B, n_q, d))
    for b in range(B):
        if lens[b] < 1:
            raise ValueError("decode needs len >= 1")
        K, V = gather(pool_bits, row_off, block_ids, b, int(lens[b]))
        for j in range(n_q):
            out[b, j], lse[b, j], w = attend(q[b, j], K[j // G], V[j // G], s)
            if with_spread:
                spread[b, j] = weight_spread(w, V[j // G], out[b, j], centered)
    return (out, lse, spread) if with_spread else (out, lse)


def decode_rows(pool_bits, row_off, block_ids, lens, q_bits, n_kv_heads, pairs, scale=None, with_spread=False,
                centered=True):
    """decode() restricted to a list of (b, j) pairs; for sampled checks on
    batches too large to evaluate in full."""
    _, n_q, d = q_bits.shape
    G = n_q // n_kv_heads
    s = 1.0 / math.sqrt(d) if scale is None else float(scale)
    outs, lses, spreads = [], [], []
    cache = {}
    for b, j in pairs:
        if b not in cache:
            cache = {b: gather(pool_bits, row_off, block_ids, b, int(lens[b]))}
        K, V = cache[b]
        o, l, w = attend(bf16_bits_to_f64(q_bits[b, j]), K[j // G], V[j // G], s)
        outs.append(o)
        lses.append(l)
        if with_spread:
            spreads.append(weight_spread(w, V[j // G], o, centered))
    if with_spread:
        return np.array(outs), np.array(lses), np.array(spreads)
    return np.array(outs), np.array(lses)


def decode_split(pool_bits, row_off, block_ids, lens, q_bits, n_kv_heads, plan, scale=None):
    """The same result reached the split-K way, in float64: every planned item
    yields (m, l, acc) over its token range; the parts of a trajectory are
    merged with M = max m, out = sum e^(m-M) acc / sum e^(m-M) l.  Exists to
    show that the merge formula is exact, not to be fast."""
    B, n_q, d = q_bits.shape
    G = n_q // n_kv_heads
    s = 1.0 / math.sqrt(d) if scale is None else float(scale)
    q = bf16_bits_to_f64(q_bits)
    n_parts = int(plan["part_off"][B])
    pm = np.full((n_parts, n_q), -np.inf)
    pl = np.zeros((n_parts, n_q))
    pacc = np.zeros((n_parts, n_q, d))
    for it in range(len(plan["item_b"])):
        b, k = int(plan["item_b"][it]), int(plan["item_s"][it])
        t0 = int(plan["item_blk_begin"][it]) * BLOCK_TOKENS
        t1 = min(int(plan["item_blk_end"][it]) * BLOCK_TOKENS, int(lens[b]))
        K, V = gather(pool_bits, row_off, block_ids, b, int(lens[b]))
        slot = int(plan["part_off"][b]) + k
        for j in range(n_q):
            z = s * (K[j // G][t0:t1] @ q[b, j])
            m = z.max()
            e = np.exp(z - m)
            pm[slot, j], pl[slot, j], pacc[slot, j] = m, e.sum(), e @ V[j // G][t0:t1]
    out = np.zeros((B, n_q, d))
    lse = np.zeros((B, n_q))
    for b in range(B):
        sl = slice(int(plan["part_off"][b]), int(plan["part_off"][b + 1]))
        for j in range(n_q):
            M = pm[sl, j].max()
            f = np.exp(pm[sl, j] - M)
            denom = (f * pl[sl, j]).sum()
            out[b, j] = (f[:, None] * pacc[sl, j]).sum(axis=0) / denom
            lse[b, j] = M + math.log(denom)
    return out, lse


def write_kv(pool_bits, row_off, block_ids, positions, b: int, k_bits, v_bits):
    """Bit-for-bit copy of rows k_bits/v_bits [n][n_kv][d] into the slots of
    trajectory b at the given token positions (in place)."""
    row = np.asarray(block_ids[row_off[b]:row_off[b + 1]])
    for i, p in enumerate(positions):
        blk, slot = divmod(int(p), BLOCK_TOKENS)
        if blk >= row.shape[0]:
            raise ValueError("block table row too short for the appended token")
        n_kv, d = k_bits.shape[1], k_bits.shape[2]
        pool_bits[row[blk], :, 0, :].reshape(n_kv, BLOCK_TOKENS, d)[:, slot, :] = k_bits[i]
        pool_bits[row[blk], :, 1, :].reshape(n_kv, d, BLOCK_TOKENS)[:, :, slot] = v_bits[i]


def append(pool_bits, row_off, block_ids, ctx_lens, cu_chunk, q_bits, k_bits, v_bits,
           n_kv_heads: int, scale=None, rows=None, with_spread=False, centered=False):
    """Append a chunk per trajectory: first store the chunk's K/V rows at
    positions L_b .. L_b + C_b - 1 (pool_bits is modified in place), then each
    chunk row attends causally: row i of trajectory b sees L_b + i + 1 keys.

    q_bits uint16 [sum C][n_q][d]; k_bits, v_bits uint16 [sum C][n_kv][d].
    rows: optional iterable of flat row indices to evaluate (others stay 0).
    Returns out float64 [sum C][n_q][d], lse float64 [sum C][n_q]."""
    n_rows, n_q, d = q_bits.shape
    G = n_q // n_kv_heads
    s = 1.0 / math.sqrt(d) if scale is None else float(scale)
    B = len(ctx_lens)
    for b in range(B):
        lo, hi = int(cu_chunk[b]), int(cu_chunk[b + 1])
        if hi - lo < 1 or ctx_lens[b] < 0:
            raise ValueError("append needs C >= 1 and L >= 0")
        L = int(ctx_lens[b])
        write_kv(pool_bits, row_off, block_ids, range(L, L + hi - lo), b,
                 k_bits[lo:hi], v_bits[lo:hi])
    want = None if rows is None else set(int(r) for r in rows)
    out = np.zeros((n_rows, n_q, d))
    lse = np.zeros((n_rows, n_q))
    spread = np.zeros((n_rows, n_q, d)) if with_spread else None
    for b in range(B):
        lo, hi = int(cu_chunk[b]), int(cu_chunk[b + 1])
        L = int(ctx_lens[b])
        todo = [r for r in range(lo, hi) if want is None or r in want]
        if not todo:
            continue
        K, V = gather(pool_bits, row_off, block_ids, b, L + hi - lo)
        for r in todo:
            n_keys = L + (r - lo) + 1
            qr = bf16_bits_to_f64(q_bits[r])
            for j in range(n_q):
                out[r, j], lse[r, j], w = attend(qr[j], K[j // G][:n_keys], V[j // G][:n_keys], s)
                if with_spread:
                    spread[r, j] = weight_spread(w, V[j // G][:n_keys], out[r, j], centered)
    return (out, lse, spread) if with_spread else (out, lse)


def pack(pool_bits, row_off, block_ids, b: int, length: int):
    """Contiguous copy of trajectory b's first ceil(length/16) blocks, in table
    order: uint16 [nblk][n_kv][2][16*d].  (Staging form of a trajectory's
    cache for eviction or migration, Sec. 4.2 / Sec. 5.3.)"""
    nblk = (length + BLOCK_TOKENS - 1) // BLOCK_TOKENS
    row = np.asarray(block_ids[row_off[b]:row_off[b + 1]])[:nblk]
    return pool_bits[row].copy()


def unpack(pool_bits, dst_blocks, staged):
    """Inverse of pack under a (possibly different) list of physical blocks."""
    for i, blk in enumerate(dst_blocks):
        pool_bits[int(blk)] = staged[i]


def copy_blocks(pool_bits, src_blocks, dst_blocks):
    """Block dst[i] becomes a bit-for-bit copy of block src[i] (all kv heads, K and V, all 16 slots).
    A sample that continues a shared prompt (16 samples per prompt, Sec. 7) names the prompt's whole
    blocks in its own table and takes a copy of the partly filled last one, which it will write to."""
    for s, d in zip(src_blocks, dst_blocks):
        pool_bits[int(d)] = pool_bits[int(s)]
