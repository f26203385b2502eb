"""Pure-Python attention on dense lists: the pin the numpy oracle is held to.

No numpy arithmetic, no block table: K and V arrive as plain nested lists in
token order, sums use math.fsum, exponentials math.exp."""
import math


def bf16_to_float(bits: int) -> float:
    import struct
    return struct.unpack("<f", struct.pack("<I", (int(bits) & 0xFFFF) << 16))[0]


def softmax_attention(q, K, V, scale):
    """q: list[d]; K, V: list[n][d].  Returns (out list[d], lse, weights)."""
    n, d = len(K), len(q)
    z = [scale * math.fsum(q[c] * K[t][c] for c in range(d)) for t in range(n)]
    zmax = max(z)
    e = [math.exp(zt - zmax) for zt in z]
    denom = math.fsum(e)
    w = [et / denom for et in e]
    out = [math.fsum(w[t] * V[t][c] for t in range(n)) for c in range(len(V[0]))]
    return out, zmax + math.log(denom), w


def dense_from_pool(pool, row_off, block_ids, b, length, h):
    """Token-ordered K, V lists of kv head h, element by element with flat offsets (no
    reshapes): position p lives in block block_ids[row_off[b] + p // 16], slot p % 16;
    element c of its K row is at [blk][h][0][slot*d + c], of its V row at [blk][h][1][c*16 + slot]
    (the V tile is stored transposed)."""
    d = pool.shape[3] // 16
    K, V = [], []
    for p in range(length):
        blk = int(block_ids[int(row_off[b]) + p // 16])
        slot = p % 16
        K.append([bf16_to_float(pool[blk, h, 0, slot * d + c]) for c in range(d)])
        V.append([bf16_to_float(pool[blk, h, 1, c * 16 + slot]) for c in range(d)])
    return K, V
