"""Pins of the float64 attention oracle (no GPU).

Each test holds the oracle to something it does not compute itself: a
pure-Python brute force, a closed form, or an invariant of softmax attention."""
import math

import numpy as np
import pytest

import heddle_workloads as hw
from oracle import attention as oa
from oracle import planner as op
from tests import brute


def small_case(seed, lens, n_q=4, n_kv=2, d=8, chunk=None, **kw):
    return hw.build_case(entropy=[0, seed], lens=lens, chunk_lens=chunk, n_q_heads=n_q,
                         n_kv_heads=n_kv, head_dim=d, threads=1, **kw)


def run_decode(c, lens=None, scale=None):
    return oa.decode(c["pool"], c["row_off"], c["block_ids"], c["lens"] if lens is None else lens,
                     c["q"], c["n_kv_heads"], scale)


def bits(x):
    return hw.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_bf16_widening_exact():
    vals = np.array([0.0, 1.0, -2.5, 3.140625, 2.0 ** -126, -65280.0], dtype=np.float32)
    b = bits(vals)
    assert np.array_equal(oa.bf16_bits_to_f64(b), vals.astype(np.float64))
    for x, y in zip(b, vals):
        assert brute.bf16_to_float(x) == float(y)


def test_bf16_rounding_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: goes to 1 + 2^-6.
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = oa.bf16_bits_to_f64(bits(x))
    assert list(got) == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_decode_matches_pure_python_brute_force(seed):
    lens = [1, 17, 40][: 3]
    c = small_case(seed, lens)
    out, lse = run_decode(c)
    G = c["n_q_heads"] // c["n_kv_heads"]
    s = 1 / math.sqrt(c["head_dim"])
    for b in range(len(lens)):
        for j in range(c["n_q_heads"]):
            K, V = brute.dense_from_pool(c["pool"], c["row_off"], c["block_ids"], b, lens[b], j // G)
            q = [brute.bf16_to_float(x) for x in c["q"][b, j]]
            ref, ref_lse, w = brute.softmax_attention(q, K, V, s)
            assert abs(math.fsum(w) - 1) < 1e-12
            assert np.allclose(out[b, j], ref, rtol=1e-12, atol=1e-13)
            assert abs(lse[b, j] - ref_lse) < 1e-12


def test_gqa_mapping_is_contiguous_groups():
    # make kv head 1 all zeros in K and a marker in V: exactly q heads 2,3 (G=2) must see it
    c = small_case(3, [20], poison=False)
    pool = c["pool"]
    pool[:, 1, 0] = 0
    pool[:, 1, 1] = bits(7.0)      # every V element of kv head 1
    out, lse = run_decode(c)
    assert np.allclose(out[0, 2:], 7.0) and np.allclose(lse[0, 2:], math.log(20))
    assert not np.allclose(out[0, :2], 7.0)


def test_len_one_returns_v_and_logit():
    c = small_case(4, [1, 1, 1])
    out, lse = run_decode(c)
    s = 1 / math.sqrt(c["head_dim"])
    for b in range(3):
        blk = c["block_ids"][c["row_off"][b]]
        for j in range(4):
            v0 = oa.bf16_bits_to_f64(hw.v_view(c["pool"])[blk, j // 2, :, 0])
            k0 = oa.bf16_bits_to_f64(hw.k_view(c["pool"])[blk, j // 2, 0])
            assert np.array_equal(out[b, j], v0)
            assert abs(lse[b, j] - s * float(oa.bf16_bits_to_f64(c["q"][b, j]) @ k0)) < 1e-13


def test_identical_keys_give_mean_of_values():
    n = 37
    c = small_case(5, [n], poison=False)
    row = c["block_ids"][: c["row_off"][1]]
    key = hw.k_view(c["pool"])[row[0], :, 0].copy()         # [n_kv][d]
    hw.k_view(c["pool"])[row] = key[None, :, None, :]
    out, lse = run_decode(c)
    K, V = oa.gather(c["pool"], c["row_off"], c["block_ids"], 0, n)
    s = 1 / math.sqrt(c["head_dim"])
    for j in range(4):
        assert np.allclose(out[0, j], V[j // 2].mean(axis=0), rtol=1e-13, atol=1e-14)
        z = s * float(oa.bf16_bits_to_f64(c["q"][0, j]) @ oa.bf16_bits_to_f64(key[j // 2]))
        assert abs(lse[0, j] - (z + math.log(n))) < 1e-12


def test_constant_values_are_returned():
    c = small_case(6, [50, 3], poison=False)
    const = bits(np.linspace(-2, 2, 8))
    hw.v_view(c["pool"])[:] = const[None, None, :, None]
    out, _ = run_decode(c)
    assert np.allclose(out, oa.bf16_bits_to_f64(const), rtol=1e-14, atol=1e-15)


def test_physical_block_permutation_is_invisible():
    c = small_case(7, [100, 33, 16])
    out, lse = run_decode(c)
    perm = np.random.default_rng(99).permutation(c["n_blocks"])
    pool2 = np.empty_like(c["pool"])
    pool2[perm] = c["pool"]                 # block i moves to perm[i]
    out2, lse2 = oa.decode(pool2, c["row_off"], perm[c["block_ids"]].astype(np.int32), c["lens"],
                           c["q"], c["n_kv_heads"])
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


def test_poison_outside_context_never_leaks():
    c = small_case(8, [5, 16, 31], poison=True)
    out, lse = run_decode(c)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    clean = small_case(8, [5, 16, 31], poison=False)
    out2, _ = run_decode(clean)
    assert np.array_equal(out, out2)


def needle_case(seed, lens, b, pos, n_q=4, n_kv=2, d=8):
    """Key at (b, pos) is made to dominate every head's softmax; its value row
    is a one-hot marker times 1000."""
    c = small_case(seed, lens, n_q=n_q, n_kv=n_kv, d=d)
    G = n_q // n_kv
    blk = c["block_ids"][c["row_off"][b] + pos // 16]
    for h in range(n_kv):
        # all q heads of the group must agree: make them identical first
        c["q"][b, h * G:(h + 1) * G] = c["q"][b, h * G]
        qv = oa.bf16_bits_to_f64(c["q"][b, h * G])
        hw.k_view(c["pool"])[blk, h, pos % 16] = bits(40.0 * math.sqrt(d) * qv / (qv @ qv))   # logit = 40
        marker = np.zeros(d, dtype=np.float32)
        marker[(pos + h) % d] = 1000.0
        hw.v_view(c["pool"])[blk, h, :, pos % 16] = bits(marker)
    return c


@pytest.mark.parametrize("pos", [0, 15, 16, 31, 32, 36])
def test_needle_is_found_at_every_kind_of_position(pos):
    lens = [9, 37]
    c = needle_case(11, lens, 1, pos)
    out, _ = run_decode(c)
    for j in range(4):
        expect = np.zeros(8)
        expect[(pos + j // 2) % 8] = 1000.0
        assert np.allclose(out[1, j], expect, atol=1e-6), (pos, j)


def test_logit_shift_moves_only_lse():
    # scaling q by a changes logits; instead shift all logits by a constant: add c*q/|q|^2/s to
    # every key of one head => every logit grows by c exactly in real arithmetic
    c = small_case(12, [29], n_q=2, n_kv=2, poison=False)
    out, lse = run_decode(c)
    # use the float64 path directly to avoid re-rounding keys to bf16
    K, V = oa.gather(c["pool"], c["row_off"], c["block_ids"], 0, 29)
    s = 1 / math.sqrt(8)
    for j in range(2):
        q = oa.bf16_bits_to_f64(c["q"][0, j])
        shift = 3.25
        K2 = K[j] + (shift / s) * q / (q @ q)
        o2, l2, _ = oa.attend(q, K2, V[j], s)
        assert np.allclose(o2, out[0, j], rtol=1e-11, atol=1e-12)
        assert abs(l2 - lse[0, j] - shift) < 1e-11


@pytest.mark.parametrize("seed", [0, 1])
def test_split_k_merge_equals_definition(seed):
    lens = [1, 16, 17, 100, 333, 64]
    c = small_case(20 + seed, lens)
    out, lse = run_decode(c)
    for kw in (dict(n_cu=2, wg_per_cu=2, min_chunk_blk=1, tile_blk=1, max_split=64),
               dict(n_cu=4, wg_per_cu=4, min_chunk_blk=2, tile_blk=2, max_split=3),
               op.DEFAULTS):
        plan = op.plan_decode(lens, c["n_kv_heads"], **kw)
        out2, lse2 = oa.decode_split(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"],
                                     c["n_kv_heads"], plan)
        assert np.allclose(out, out2, rtol=1e-12, atol=1e-13)
        assert np.allclose(lse, lse2, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- append

def run_append(c, rows=None):
    pool = c["pool"].copy()
    out, lse = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"],
                         c["k_new"], c["v_new"], c["n_kv_heads"], rows=rows)
    return pool, out, lse


def test_append_equals_token_by_token_decode():
    L, C = [0, 5, 16, 30], [3, 20, 1, 17]
    c = small_case(30, L, chunk=C)
    pool_after, out, lse = run_append(c)
    # replay: write one row, decode at len = L+i+1, for every trajectory separately
    pool = c["pool"].copy()
    for b in range(4):
        for i in range(C[b]):
            r = int(c["cu_chunk"][b]) + i
            oa.write_kv(pool, c["row_off"], c["block_ids"], [L[b] + i], b,
                        c["k_new"][r:r + 1], c["v_new"][r:r + 1])
            lens = np.array(L) + 0
            lens[b] = L[b] + i + 1
            lens = np.maximum(lens, 1)
            qb = np.zeros((4,) + c["q"].shape[1:], dtype=np.uint16)
            qb[b] = c["q"][r]
            # other trajectories may have poison at len 1 when L=0; evaluate only b
            o, l = oa.decode_rows(pool, c["row_off"], c["block_ids"], lens, qb, c["n_kv_heads"],
                                  [(b, j) for j in range(c["n_q_heads"])])
            assert np.allclose(o, out[r], rtol=1e-12, atol=1e-13)
            assert np.allclose(l, lse[r], rtol=0, atol=1e-12)
    assert np.array_equal(pool, pool_after)


def test_append_from_empty_context_is_dense_causal_attention():
    C = [11]
    c = small_case(31, [0], chunk=C, n_q=2, n_kv=1, d=4)
    _, out, lse = run_append(c)
    K = [[brute.bf16_to_float(x) for x in c["k_new"][i, 0]] for i in range(11)]
    V = [[brute.bf16_to_float(x) for x in c["v_new"][i, 0]] for i in range(11)]
    for i in range(11):
        for j in range(2):
            q = [brute.bf16_to_float(x) for x in c["q"][i, j]]
            ref, ref_lse, _ = brute.softmax_attention(q, K[: i + 1], V[: i + 1], 0.5)
            assert np.allclose(out[i, j], ref, rtol=1e-12, atol=1e-13)
            assert abs(lse[i, j] - ref_lse) < 1e-12


def test_append_in_two_pieces_equals_one_piece():
    L, C = [7, 40], [25, 9]
    c = small_case(32, L, chunk=C)
    pool1, out1, lse1 = run_append(c)
    C1 = [10, 4]
    C2 = [C[i] - C1[i] for i in range(2)]
    cu = c["cu_chunk"]
    rows1 = np.concatenate([np.arange(cu[b], cu[b] + C1[b]) for b in range(2)])
    rows2 = np.concatenate([np.arange(cu[b] + C1[b], cu[b + 1]) for b in range(2)])
    pool = c["pool"].copy()
    cu1 = np.array([0, C1[0], C1[0] + C1[1]])
    cu2 = np.array([0, C2[0], C2[0] + C2[1]])
    oA, lA = oa.append(pool, c["row_off"], c["block_ids"], L, cu1, c["q"][rows1],
                       c["k_new"][rows1], c["v_new"][rows1], c["n_kv_heads"])
    oB, lB = oa.append(pool, c["row_off"], c["block_ids"], [L[0] + C1[0], L[1] + C1[1]], cu2,
                       c["q"][rows2], c["k_new"][rows2], c["v_new"][rows2], c["n_kv_heads"])
    assert np.array_equal(pool, pool1)
    assert np.allclose(out1[rows1], oA, rtol=1e-13, atol=1e-14)
    assert np.allclose(out1[rows2], oB, rtol=1e-13, atol=1e-14)
    assert np.allclose(lse1[rows2], lB, rtol=0, atol=1e-13)


def test_append_writes_exactly_the_chunk_slots():
    L, C = [3, 16, 0], [14, 16, 33]
    c = small_case(33, L, chunk=C)
    pool_after, _, _ = run_append(c)
    expect = c["pool"].copy()
    for b in range(3):
        for i in range(C[b]):
            p = L[b] + i
            blk = c["block_ids"][c["row_off"][b] + p // 16]
            r = c["cu_chunk"][b] + i
            for h in range(2):
                d = c["head_dim"]
                for e in range(d):
                    expect[blk, h, 0, (p % 16) * d + e] = c["k_new"][r, h, e]
                    expect[blk, h, 1, e * 16 + p % 16] = c["v_new"][r, h, e]
    assert np.array_equal(pool_after, expect)
    changed = np.nonzero((pool_after != c["pool"]).any(axis=(1, 2, 3)))[0]
    referenced = set(int(x) for x in c["block_ids"])
    assert set(int(x) for x in changed) <= referenced


def test_append_row_subset_matches_full():
    c = small_case(34, [20, 5], chunk=[9, 12])
    _, out, lse = run_append(c)
    rows = [0, 8, 9, 20]
    _, out_s, lse_s = run_append(c, rows=rows)
    assert np.array_equal(out[rows], out_s[rows]) and np.array_equal(lse[rows], lse_s[rows])
    assert not out_s[1].any()


def test_needle_in_append_sees_own_row_and_last_context_row():
    # the row's own key dominates: out = own V (causal mask includes self)
    L, C = [18], [6]
    c = small_case(35, L, chunk=C, n_q=2, n_kv=2)
    for i in range(6):
        for h in range(2):
            qv = oa.bf16_bits_to_f64(c["q"][i, h])
            c["k_new"][i, h] = bits(60.0 * math.sqrt(8) * qv / (qv @ qv))
            c["v_new"][i, h] = bits(np.full(8, 100.0 + i))
    _, out, _ = run_append(c)
    for i in range(6):
        # a later row's key would dominate even more if it leaked: check exact own marker
        assert np.allclose(out[i], 100.0 + i, atol=1e-6), i


def test_pack_unpack_round_trip():
    c = small_case(36, [40, 7])
    staged = oa.pack(c["pool"], c["row_off"], c["block_ids"], 0, 40)
    row = c["block_ids"][: c["row_off"][1]]
    assert staged.shape[0] == 3 and np.array_equal(staged[1], c["pool"][row[1]])
    pool2 = c["pool"].copy()
    free = [i for i in range(c["n_blocks"]) if i not in set(int(x) for x in c["block_ids"])]
    dst = free[:3] if len(free) >= 3 else list(row)
    oa.unpack(pool2, dst, staged)
    K1, V1 = oa.gather(c["pool"], c["row_off"], c["block_ids"], 0, 40)
    ids2 = c["block_ids"].copy()
    ids2[:3] = dst
    K2, V2 = oa.gather(pool2, c["row_off"], ids2, 0, 40)
    assert np.array_equal(K1, K2) and np.array_equal(V1, V2)


def test_copy_blocks_forks_a_trajectory():
    """A fork: trajectory 1 names the whole blocks of trajectory 0 and a copy of its partly filled last
    block.  Its gathered K/V (the gather is pinned by the flat-offset brute force) equals trajectory 0's,
    the copy equals what pack and unpack would have moved, and no other block changes."""
    c = small_case(37, [40, 7])
    pool = c["pool"].copy()
    row0 = [int(x) for x in c["block_ids"][: c["row_off"][1]]]            # 3 blocks, the last holds 8 tokens
    free = [i for i in range(c["n_blocks"]) if i not in set(int(x) for x in c["block_ids"])]
    assert free, "the generator over-provisions the pool"
    fork_blk = free[0]
    oa.copy_blocks(pool, [row0[2]], [fork_blk])
    ids = np.concatenate([c["block_ids"], np.asarray(row0[:2] + [fork_blk], dtype=c["block_ids"].dtype)])
    row_off = np.concatenate([c["row_off"], [len(ids)]]).astype(c["row_off"].dtype)
    K0, V0 = oa.gather(pool, row_off, ids, 0, 40)
    K2, V2 = oa.gather(pool, row_off, ids, 2, 40)
    assert np.array_equal(K0, K2) and np.array_equal(V0, V2)
    via_staging = c["pool"].copy()
    oa.unpack(via_staging, [fork_blk], oa.pack(c["pool"], c["row_off"], c["block_ids"], 0, 40)[2:3])
    assert np.array_equal(pool, via_staging)
    untouched = [i for i in range(c["n_blocks"]) if i != fork_blk]
    assert np.array_equal(pool[untouched], c["pool"][untouched])
    assert not np.array_equal(pool[fork_blk], c["pool"][fork_blk])       # the free block held poison before


def test_weight_spread_matches_direct_perturbation():
    """weight_spread is the first-order standard deviation of the output under independent
    relative perturbations of the weights; check it against an explicit finite perturbation."""
    rng = np.random.default_rng(0)
    n, d = 23, 5
    w = rng.random(n)
    w /= w.sum()
    V = rng.standard_normal((n, d))
    out = w @ V
    eps = 1e-6
    # exact derivative of out wrt delta_t at 0: w_t (V_t - out); spread = sqrt(sum of squares)
    J = np.zeros((n, d))
    for t in range(n):
        w2 = w.copy()
        w2[t] *= 1 + eps
        J[t] = ((w2 @ V) / w2.sum() - out) / eps
    assert np.allclose(oa.weight_spread(w, V, out), np.sqrt((J ** 2).sum(axis=0)), rtol=1e-4)
    # a single dominant token: the output cannot move
    w1 = np.zeros(n)
    w1[3] = 1.0
    assert np.allclose(oa.weight_spread(w1, V, V[3]), 0.0)


def _finite_difference_std(w, V, in_denominator, eps=1e-6):
    """Root of the summed squares of d out / d delta_t at delta = 0, by finite differences, where the
    output is sum_t w_t (1 + delta_t) V_t over a denominator that carries the perturbation of the
    keys flagged in `in_denominator` only (the others enter it unperturbed)."""
    n, d = V.shape
    base = (w @ V) / w.sum()
    J = np.zeros((n, d))
    for t in range(n):
        num = w.copy()
        num[t] *= 1 + eps
        den = w.sum() + (w[t] * eps if in_denominator[t] else 0.0)
        J[t] = ((num @ V) / den - base) / eps
    return np.sqrt((J ** 2).sum(axis=0))


def test_weight_spread_numerator_only_and_mixed_modes():
    """centered=False is the first-order standard deviation when only the numerator carries the
    perturbed weights (the 128-row append kernel divides by the unrounded sum); centered=None bounds
    every mixture in which some keys' perturbations reach the denominator and the others' do not
    (a batch served by two kernels, a shared prefix next to private blocks).  Both against explicit
    finite perturbations; the derivative of out wrt delta_t is w_t V_t without the denominator and
    w_t (V_t - out) with it."""
    rng = np.random.default_rng(1)
    n, d = 29, 6
    w = rng.random(n) ** 3           # a few large weights, many small ones
    w /= w.sum()
    V = rng.standard_normal((n, d)) + 0.7          # a mean away from zero separates the two modes
    out = w @ V
    none_in = np.zeros(n, dtype=bool)
    all_in = np.ones(n, dtype=bool)
    unc = oa.weight_spread(w, V, out, centered=False)
    cen = oa.weight_spread(w, V, out, centered=True)
    both = oa.weight_spread(w, V, out, centered=None)
    assert np.allclose(unc, _finite_difference_std(w, V, none_in), rtol=1e-4)
    assert np.allclose(cen, _finite_difference_std(w, V, all_in), rtol=1e-4)
    assert not np.allclose(unc, cen, rtol=5e-2), "the two modes must differ on this input"
    # the bound for mixtures: never below either pure mode, equal to the root of both squares, and
    # above every mixture of keys
    assert np.allclose(both, np.sqrt(unc ** 2 + cen ** 2), rtol=1e-12)
    for trial in range(20):
        mask = rng.random(n) < rng.random()
        mixed = _finite_difference_std(w, V, mask)
        assert (mixed <= both * (1 + 1e-4)).all(), trial
    # the halves of a mixture add in squares: keys [0, k) with the denominator, the rest without
    k = 11
    mask = np.arange(n) < k
    expect = np.sqrt((w[:k] ** 2) @ ((V[:k] - out) ** 2) + (w[k:] ** 2) @ (V[k:] ** 2))
    assert np.allclose(_finite_difference_std(w, V, mask), expect, rtol=1e-4)
    # a single dominant key: with the denominator the output cannot move, without it it moves by V_t
    w1 = np.zeros(n)
    w1[4] = 1.0
    assert np.allclose(oa.weight_spread(w1, V, V[4], centered=False), np.abs(V[4]))
    assert np.allclose(oa.weight_spread(w1, V, V[4], centered=None), np.abs(V[4]))


def test_spread_reported_by_decode_and_append_is_weight_spread_of_their_weights():
    """decode(with_spread) and append(with_spread, centered=...) hand the mode through: recompute the
    spread of one row from attend()'s weights."""
    c = small_case(41, [37, 5], chunk=[6, 3])
    for centered in (True, False, None):
        _, _, sp = oa.decode(c["pool"], c["row_off"], c["block_ids"], c["lens"], c["q"][:2], c["n_kv_heads"],
                             with_spread=True, centered=centered)
        K, V = oa.gather(c["pool"], c["row_off"], c["block_ids"], 0, 37)
        G = c["n_q_heads"] // c["n_kv_heads"]
        j = c["n_q_heads"] - 1
        o, _, w = oa.attend(oa.bf16_bits_to_f64(c["q"][0, j]), K[j // G], V[j // G], 1.0 / np.sqrt(c["head_dim"]))
        assert np.allclose(sp[0, j], oa.weight_spread(w, V[j // G], o, centered), rtol=1e-12)
        pool = c["pool"].copy()
        _, _, spa = oa.append(pool, c["row_off"], c["block_ids"], c["lens"], c["cu_chunk"], c["q"], c["k_new"],
                              c["v_new"], c["n_kv_heads"], with_spread=True, centered=centered)
        K, V = oa.gather(pool, c["row_off"], c["block_ids"], 1, 5 + 3)
        r = int(c["cu_chunk"][1]) + 1                      # second chunk row of trajectory 1: sees 5 + 2 keys
        o, _, w = oa.attend(oa.bf16_bits_to_f64(c["q"][r, j]), K[j // G][:7], V[j // G][:7],
                            1.0 / np.sqrt(c["head_dim"]))
        assert np.allclose(spa[r, j], oa.weight_spread(w, V[j // G][:7], o, centered), rtol=1e-12)
