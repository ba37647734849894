"""Pins for the K/V append oracle (CPU only).

The synthetic batches are generated with this step's K/V rows already in the
cache, so the cache itself is the expected value: read the new rows out of it
position by position, wipe their slots, append, and the original bits must come
back -- with every other byte untouched.
"""
import numpy as np
import pytest

from oracle import attention as A
from oracle import kv_append as KA
from paper_2412_18106_amd import workloads as W

P, D_, V = W.PREFILL, W.DECODE, W.VERIFY


def new_rows(b):
    """K_new / V_new [sum q, Hkv, D] (bit patterns) read back, position by position, from a cache that
    already holds them."""
    k_new = np.zeros((b.total_q, b.num_kv_heads, b.head_dim), np.uint16)
    v_new = np.zeros_like(k_new)
    t = 0
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        for r in range(ql):
            blk, slot = b.block_table[i, (c + r) // b.block_size], (c + r) % b.block_size
            k_new[t + r] = b.k_cache[blk, :, slot, :]
            v_new[t + r] = b.v_cache[blk, :, slot, :]
        t += ql
    return k_new, v_new


def new_slot_mask(b):
    """Boolean [num_blocks, B]: slots that belong to this step's tokens."""
    m = np.zeros((b.k_cache.shape[0], b.block_size), bool)
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        for j in range(c, c + ql):
            m[b.block_table[i, j // b.block_size], j % b.block_size] = True
    return m


def wipe(cache, m, fill):
    out = cache.copy()
    blocks, slots = np.nonzero(m)
    out[blocks, :, slots, :] = fill
    return out


SPECS = [W.SeqSpec(9, 0, P), W.SeqSpec(1, 7, D_), W.SeqSpec(5, 3, P), W.SeqSpec(1, 0, D_),
         W.SeqSpec(3, 6, V, W.MASK_TREE, parents=[-1, 0, 0]), W.SeqSpec(4, 4, P)]


@pytest.mark.parametrize("bs", [4, 16])
def test_round_trip_restores_the_cache_bit_for_bit(bs):
    b = W.make_custom(SPECS, 4, 2, seed=11, head_dim=8, block_size=bs)
    k_new, v_new = new_rows(b)
    m = new_slot_mask(b)
    assert m.sum() == b.total_q                      # every new token has its own slot
    k0, v0 = wipe(b.k_cache, m, 0x7FC0), wipe(b.v_cache, m, 0x7FC0)   # NaN patterns in the new slots
    assert not np.array_equal(k0, b.k_cache)
    k1, v1 = KA.append_kv_oracle(b.seqs, k_new, v_new, k0, v0, b.block_table, bs)
    assert np.array_equal(k1, b.k_cache) and np.array_equal(v1, b.v_cache)


def test_nothing_else_is_written_and_inputs_are_not_modified():
    b = W.make_custom(SPECS, 4, 2, seed=12, head_dim=8, block_size=4)
    rng = np.random.default_rng(0)
    k_new = rng.integers(0, 2 ** 15, (b.total_q, 2, 8)).astype(np.uint16)
    v_new = rng.integers(0, 2 ** 15, (b.total_q, 2, 8)).astype(np.uint16)
    k_before, v_before = b.k_cache.copy(), b.v_cache.copy()
    k1, v1 = KA.append_kv_oracle(b.seqs, k_new, v_new, b.k_cache, b.v_cache, b.block_table, 4)
    assert np.array_equal(b.k_cache, k_before) and np.array_equal(b.v_cache, v_before)
    m = new_slot_mask(b)
    blocks, slots = np.nonzero(~m)
    assert np.array_equal(k1[blocks, :, slots, :], k_before[blocks, :, slots, :])   # block tails, spare blocks, history
    assert np.array_equal(v1[blocks, :, slots, :], v_before[blocks, :, slots, :])
    # and the new slots hold exactly the new rows, in token order (brute force over tokens)
    t = 0
    for i, (ql, c, *_rest) in enumerate(b.seqs):
        for r in range(ql):
            j = c + r
            blk, slot = b.block_table[i, j // 4], j % 4
            for g in range(2):
                assert k1[blk, g, slot].tolist() == k_new[t + r, g].tolist()
                assert v1[blk, g, slot].tolist() == v_new[t + r, g].tolist()
        t += ql


def test_k_and_v_are_not_swapped_and_heads_keep_their_order():
    b = W.make_custom([W.SeqSpec(3, 2, P)], 2, 2, seed=3, head_dim=4, block_size=4)
    k_new = np.zeros((3, 2, 4), np.uint16)
    v_new = np.zeros((3, 2, 4), np.uint16)
    for r in range(3):
        for g in range(2):
            k_new[r, g] = 1000 + 100 * r + 10 * g + np.arange(4)
            v_new[r, g] = 2000 + 100 * r + 10 * g + np.arange(4)
    k1, v1 = KA.append_kv_oracle(b.seqs, k_new, v_new, b.k_cache, b.v_cache, b.block_table, 4)
    # positions 2, 3 are in logical block 0, position 4 in logical block 1
    assert k1[b.block_table[0, 0], 1, 2].tolist() == [1010, 1011, 1012, 1013]
    assert v1[b.block_table[0, 0], 0, 3].tolist() == [2100, 2101, 2102, 2103]
    assert k1[b.block_table[0, 1], 0, 0].tolist() == [1200, 1201, 1202, 1203]
    assert v1[b.block_table[0, 1], 1, 0].tolist() == [2210, 2211, 2212, 2213]


def test_attention_after_append_equals_attention_on_the_prefilled_cache():
    b = W.make_custom(SPECS, 4, 2, seed=13, head_dim=8, block_size=4)
    k_new, v_new = new_rows(b)
    m = new_slot_mask(b)
    k1, v1 = KA.append_kv_oracle(b.seqs, k_new, v_new, wipe(b.k_cache, m, 0), wipe(b.v_cache, m, 0),
                                 b.block_table, 4)
    kw = dict(num_q_heads=4, num_kv_heads=2, block_size=4, scale=b.scale)
    o_ref = A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks, **kw)
    o_app = A.attention_oracle(b.seqs, b.q, k1, v1, b.block_table, b.tree_masks, **kw)
    assert np.array_equal(o_ref, o_app)


def test_shared_prefix_blocks_are_never_written():
    specs = [W.SeqSpec(6, 10, P), W.SeqSpec(6, 10, P, share_prefix_with=0)]
    b = W.make_custom(specs, 2, 1, seed=5, head_dim=4, block_size=4)
    shared = set(b.block_table[0, :2].tolist()) & set(b.block_table[1, :2].tolist())
    assert len(shared) == 2                       # the two full prefix blocks are shared
    rng = np.random.default_rng(1)
    k_new = rng.integers(1, 2 ** 15, (12, 1, 4)).astype(np.uint16)
    k1, v1 = KA.append_kv_oracle(b.seqs, k_new, k_new, b.k_cache, b.v_cache, b.block_table, 4)
    for blk in shared:
        assert np.array_equal(k1[blk], b.k_cache[blk]) and np.array_equal(v1[blk], b.v_cache[blk])
    # the partial prefix block is private to each sequence: both receive their own rows
    assert not np.array_equal(k1[b.block_table[0, 2]], k1[b.block_table[1, 2]])


def test_fused_qkv_views():
    hq, hkv, d = 4, 2, 8
    qkv = np.arange(5 * (hq + 2 * hkv) * d, dtype=np.uint16).reshape(5, hq + 2 * hkv, d)
    q, k, v = KA.split_fused_qkv(qkv, hq, hkv)
    assert q.shape == (5, 4, 8) and k.shape == (5, 2, 8) and v.shape == (5, 2, 8)
    assert q.base is not None and k[2, 1, 3] == qkv[2, 5, 3] and v[4, 0, 7] == qkv[4, 6, 7]
    with pytest.raises(ValueError):
        KA.split_fused_qkv(qkv, 4, 1)


def test_position_beyond_the_table_is_an_error():
    b = W.make_custom([W.SeqSpec(2, 2, P)], 2, 1, seed=1, head_dim=4, block_size=4)
    k_new = np.zeros((2, 1, 4), np.uint16)
    with pytest.raises(ValueError):
        KA.append_kv_oracle([(2, 100, P, 0, 0)], k_new, k_new, b.k_cache, b.v_cache, b.block_table, 4)


def test_empty_batch():
    b = W.make_custom([W.SeqSpec(2, 2, P)], 2, 1, seed=1, head_dim=4, block_size=4)
    k1, v1 = KA.append_kv_oracle([], np.zeros((0, 1, 4), np.uint16), np.zeros((0, 1, 4), np.uint16),
                                 b.k_cache, b.v_cache, b.block_table, 4)
    assert np.array_equal(k1, b.k_cache) and np.array_equal(v1, b.v_cache)
