"""Pins for the fp64 attention oracle (CPU only).

Each test ties the oracle to something it does not compute itself: a pure-Python
triple loop, a closed form, a library dense attention, or an identity the paper
states (exactness of padding, prefix reuse, chunking, causal speculation).
"""
import math

import numpy as np
import pytest

from oracle import attention as A
from paper_2412_18106_amd import workloads as W

P, D_, V = W.PREFILL, W.DECODE, W.VERIFY


def run(b, **kw):
    return A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks,
                              num_q_heads=b.num_q_heads, num_kv_heads=b.num_kv_heads,
                              block_size=b.block_size, scale=b.scale, **kw)


def tiny(specs, seed, hq=2, hkv=1, d=4, bs=4, scale=None):
    return W.make_custom(specs, hq, hkv, seed, head_dim=d, block_size=bs, scale=scale)


def bf(x):
    return W.bf16_bits_to_f32(x).astype(np.float64)


def brute_force(b):
    """Pure-Python floats, independent of numpy linear algebra and of the oracle's helpers."""
    hq, hkv, d, bs = b.num_q_heads, b.num_kv_heads, b.head_dim, b.block_size
    g = hq // hkv
    q, kc, vc = bf(b.q).tolist(), bf(b.k_cache).tolist(), bf(b.v_cache).tolist()
    out = [[[0.0] * d for _ in range(hq)] for _ in range(b.total_q)]
    t0 = 0
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        wpr = (ql + 31) // 32
        for r in range(ql):
            for h in range(hq):
                keys = []
                for j in range(c + ql):
                    if mk == W.MASK_CAUSAL:
                        ok = j <= c + r
                    else:
                        ok = j < c or ((int(b.tree_masks[off + r * wpr + (j - c) // 32]) >> ((j - c) % 32)) & 1) == 1
                    if ok:
                        keys.append(j)
                if not keys:
                    continue
                sc = []
                for j in keys:
                    blk = int(b.block_table[i][j // bs])
                    krow = kc[blk][h // g][j % bs]
                    sc.append(b.scale * sum(q[t0 + r][h][x] * krow[x] for x in range(d)))
                mx = max(sc)
                ex = [math.exp(s - mx) for s in sc]
                den = sum(ex)
                for e, j in zip(ex, keys):
                    blk = int(b.block_table[i][j // bs])
                    vrow = vc[blk][h // g][j % bs]
                    for x in range(d):
                        out[t0 + r][h][x] += e / den * vrow[x]
        t0 += ql
    return np.array(out)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_brute_force_tiny_mixed(seed):
    rng = np.random.default_rng(100 + seed)
    specs = [W.SeqSpec(int(rng.integers(1, 7)), int(rng.integers(0, 7)), P),
             W.SeqSpec(1, int(rng.integers(0, 7)), D_),
             W.SeqSpec(5, int(rng.integers(0, 7)), V, W.MASK_TREE, W.random_tree(rng, 5)),
             W.SeqSpec(3, 6, V, W.MASK_CAUSAL)]
    b = tiny(specs, seed, hq=4, hkv=2, scale=0.9)
    np.testing.assert_allclose(run(b), brute_force(b), rtol=0, atol=1e-13)


def test_brute_force_wide_tree_two_mask_words():
    rng = np.random.default_rng(7)
    b = tiny([W.SeqSpec(40, 3, V, W.MASK_TREE, W.random_tree(rng, 40))], 9, scale=1.3)
    np.testing.assert_allclose(run(b), brute_force(b), rtol=0, atol=1e-13)


def test_weights_sum_to_one_and_pair_counts():
    rng = np.random.default_rng(5)
    tree = W.random_tree(rng, 6)
    b = tiny([W.SeqSpec(5, 3, P), W.SeqSpec(1, 9, D_), W.SeqSpec(6, 2, V, W.MASK_TREE, tree)], 11, hq=4, hkv=2)
    _, wts = run(b, return_weights=True)
    pop = int(sum(bin(int(w)).count("1") for w in b.tree_masks))
    closed = {0: 5 * 3 + 5 * 6 // 2, 1: 1 * 9 + 1, 2: 6 * 2 + pop}
    for (i, h), p in wts.items():
        np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
        assert int((p > 0).sum()) == closed[i]
    assert A.allowed_pairs(b.seqs, b.tree_masks) == [closed[0], closed[1], closed[2]]


def test_constant_v_gives_that_v():
    b = tiny([W.SeqSpec(4, 5, P), W.SeqSpec(1, 7, D_)], 3)
    row = bf(b.v_cache)[0, 0, 0].copy()
    b.v_cache[:] = b.v_cache[0, 0, 0]
    o = run(b)
    np.testing.assert_allclose(o, np.broadcast_to(row, o.shape), atol=1e-14)


def test_single_visible_key_returns_its_v_exactly():
    b = tiny([W.SeqSpec(3, 0, P)], 4)
    o = run(b)
    v0 = bf(b.v_cache)[b.block_table[0, 0], 0, 0]
    assert np.array_equal(o[0, 0], v0) and np.array_equal(o[0, 1], v0)   # row 0 sees key 0 only


def test_zero_query_gives_mean_of_visible_v():
    b = tiny([W.SeqSpec(4, 6, P)], 5)
    b.q[:] = 0
    o = run(b)
    vals = np.concatenate([bf(b.v_cache)[b.block_table[0, k], 0] for k in range(3)])[:10]
    for r in range(4):
        np.testing.assert_allclose(o[r, 0], vals[: 6 + r + 1].mean(axis=0), atol=1e-14)


def test_large_scale_selects_argmax_key():
    b = tiny([W.SeqSpec(1, 9, D_)], 6, scale=4000.0)
    o = run(b)
    q = bf(b.q)[0]
    keys = np.concatenate([bf(b.k_cache)[b.block_table[0, k], 0] for k in range(3)])[:10]
    vals = np.concatenate([bf(b.v_cache)[b.block_table[0, k], 0] for k in range(3)])[:10]
    for h in range(2):
        np.testing.assert_allclose(o[0, h], vals[int(np.argmax(keys @ q[h]))], atol=1e-9)


def test_against_library_dense_attention():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(8)
    tree = W.random_tree(rng, 7)
    b = W.make_custom([W.SeqSpec(9, 21, P), W.SeqSpec(7, 13, V, W.MASK_TREE, tree)], 4, 2, 21,
                      head_dim=16, block_size=8)
    o = run(b)
    t0 = 0
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        n = c + ql
        nb = -(-n // 8)
        kk = np.concatenate([bf(b.k_cache)[b.block_table[i, k]] for k in range(nb)], axis=1)[:, :n]
        vv = np.concatenate([bf(b.v_cache)[b.block_table[i, k]] for k in range(nb)], axis=1)[:, :n]
        mask = np.zeros((ql, n), dtype=bool)
        for r in range(ql):
            if mk == W.MASK_CAUSAL:
                mask[r, : c + r + 1] = True
            else:
                mask[r, :c] = True
                s = r
                while s >= 0:
                    mask[r, c + s] = True
                    s = b.parents[i][s]
        qt = torch.from_numpy(bf(b.q)[t0 : t0 + ql].transpose(1, 0, 2).copy())      # [Hq, q, D]
        kt = torch.from_numpy(np.repeat(kk, 2, axis=0))
        vt = torch.from_numpy(np.repeat(vv, 2, axis=0))
        ref = torch.nn.functional.scaled_dot_product_attention(
            qt[None], kt[None], vt[None], attn_mask=torch.from_numpy(mask)[None, None], scale=b.scale)
        np.testing.assert_allclose(o[t0 : t0 + ql], ref[0].numpy().transpose(1, 0, 2), atol=1e-12)
        t0 += ql


def _invisible_slots(b):
    """Boolean array over [block, slot]: True where no sequence may ever read a visible key."""
    touched = np.zeros(b.k_cache.shape[0::2][:2], dtype=bool)  # [blocks, B]
    vis_any = np.zeros_like(touched)
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        vis = A.visible_keys(ql, c, mk, b.tree_masks, off).any(axis=0)
        for j in range(c + ql):
            if vis[j]:
                vis_any[b.block_table[i, j // b.block_size], j % b.block_size] = True
    return ~vis_any


def test_invisible_slots_do_not_matter_bitwise():
    rng = np.random.default_rng(12)
    # a tree where node 2 is nobody's ancestor except its own row -> partially invisible corner
    b = tiny([W.SeqSpec(3, 6, P), W.SeqSpec(4, 5, V, W.MASK_TREE, [-1, 0, 0, 1]), W.SeqSpec(1, 2, D_)], 13)
    o1 = run(b)
    inv = _invisible_slots(b)
    assert inv.any()
    big = W.f32_to_bf16_bits(np.float32(3.0e4))
    for blk, slot in zip(*np.nonzero(inv)):
        b.k_cache[blk, :, slot, :] = big
        b.v_cache[blk, :, slot, :] = big
    assert np.array_equal(run(b), o1)


def _needle(b, seq, row, head, key_pos, alpha=200.0):
    """Put a key aligned with the query row (score ~ alpha*|q|*scale) and a marker V at key_pos."""
    t0 = sum(s[0] for s in b.seqs[:seq])
    g = b.num_q_heads // b.num_kv_heads
    qv = bf(b.q)[t0 + row, head]
    blk = b.block_table[seq, key_pos // b.block_size]
    b.k_cache[blk, head // g, key_pos % b.block_size] = W.f32_to_bf16_bits((alpha * qv / np.linalg.norm(qv)).astype(np.float32))
    b.v_cache[blk, head // g, key_pos % b.block_size] = W.f32_to_bf16_bits(np.full(b.head_dim, 7.0, dtype=np.float32))


@pytest.mark.parametrize("c", [0, 1, 3, 4, 7])
def test_needle_at_last_visible_and_first_invisible(c):
    specs = [W.SeqSpec(6, c, P)]
    for row in (0, 2, 5):
        b = tiny(specs, 30 + c, hq=2, hkv=2, d=8)
        base = run(b)
        _needle(b, 0, row, 1, c + row)               # last visible key of that row
        hit = run(b)
        np.testing.assert_allclose(hit[row, 1], 7.0, atol=1e-6)
        if row > 0:
            assert np.array_equal(hit[row - 1, 1], base[row - 1, 1])   # previous row must not see it
        # the other KV head is untouched
        assert np.array_equal(hit[:, 0], base[:, 0])
    b = tiny([W.SeqSpec(6, c, P)], 30 + c, hq=2, hkv=2, d=8)
    base = run(b)
    n = c + 6
    if n % 4:                                        # block-tail slot >= n
        _needle(b, 0, 5, 1, n)
        assert np.array_equal(run(b), base)


def test_needle_at_non_ancestor_tree_node():
    parents = [-1, 0, 0, 2]            # node 1 is not an ancestor of node 3
    b = tiny([W.SeqSpec(4, 5, V, W.MASK_TREE, parents)], 41, hq=2, hkv=2, d=8)
    base = run(b)
    _needle(b, 0, 3, 0, 5 + 1)
    assert np.array_equal(run(b)[3], base[3])
    b2 = tiny([W.SeqSpec(4, 5, V, W.MASK_TREE, parents)], 41, hq=2, hkv=2, d=8)
    _needle(b2, 0, 3, 0, 5 + 2)        # node 2 is an ancestor
    np.testing.assert_allclose(run(b2)[3, 0], 7.0, atol=1e-6)


def test_tree_mask_bits_are_ancestor_sets():
    rng = np.random.default_rng(3)
    for n in (1, 2, 9, 33, 64):
        par = W.random_tree(rng, n)
        words = W.pack_tree_mask(par)
        vis = A.visible_keys(n, 0, W.MASK_TREE, words, 0)
        for r in range(n):
            anc, s = set(), r
            while s >= 0:
                anc.add(s)
                s = par[s]
            assert set(np.nonzero(vis[r])[0].tolist()) == anc


def _copy_logical(dst, di, src, si, n_keys, dst_off=0):
    """Copy logical key positions 0..n_keys-1 of sequence si in src to dst sequence di."""
    for j in range(n_keys):
        sb, ss = src.block_table[si, j // src.block_size], j % src.block_size
        db, ds = dst.block_table[di, (j + dst_off) // dst.block_size], (j + dst_off) % dst.block_size
        dst.k_cache[db, :, ds] = src.k_cache[sb, :, ss]
        dst.v_cache[db, :, ds] = src.v_cache[sb, :, ss]


def test_chain_verify_equals_causal_equals_sequential_decodes():
    c, q = 6, 5
    full = tiny([W.SeqSpec(q, c, V, W.MASK_CAUSAL)], 50, hq=4, hkv=2)
    chain = tiny([W.SeqSpec(q, c, V, W.MASK_TREE, W.chain_tree(q))], 51, hq=4, hkv=2)
    chain.q[:] = full.q
    _copy_logical(chain, 0, full, 0, c + q)
    o_full = run(full)
    np.testing.assert_allclose(run(chain), o_full, atol=1e-14)
    dec = tiny([W.SeqSpec(1, c + r, D_) for r in range(q)], 52, hq=4, hkv=2)
    for r in range(q):
        dec.q[r] = full.q[r]
        _copy_logical(dec, r, full, 0, c + r + 1)
    np.testing.assert_allclose(run(dec), o_full, atol=1e-14)


def test_prefix_cached_prefill_equals_rows_of_full_prefill_and_chunking():
    p, n = 7, 6
    full = tiny([W.SeqSpec(p + n, 0, P)], 60, hq=4, hkv=2)
    o_full = run(full)
    apc = tiny([W.SeqSpec(n, p, P)], 61, hq=4, hkv=2)
    apc.q[:] = full.q[p:]
    _copy_logical(apc, 0, full, 0, p + n)
    np.testing.assert_allclose(run(apc), o_full[p:], atol=1e-14)
    # two chunks of one prompt scheduled in the same step: (q=5,c=0) and (q=8,c=5)
    ch = tiny([W.SeqSpec(5, 0, P), W.SeqSpec(8, 5, P)], 62, hq=4, hkv=2)
    ch.q[:] = full.q
    _copy_logical(ch, 0, full, 0, 5)
    _copy_logical(ch, 1, full, 0, 13)
    np.testing.assert_allclose(run(ch), o_full, atol=1e-14)


def test_block_permutation_sharing_and_block_size_invariance():
    a = tiny([W.SeqSpec(4, 9, P), W.SeqSpec(1, 9, D_)], 70, hq=4, hkv=2)
    o = run(a)
    # permute physical blocks together with the table
    perm = np.random.default_rng(1).permutation(a.k_cache.shape[0])
    inv = np.argsort(perm)
    a2_k, a2_v = a.k_cache[perm], a.v_cache[perm]
    tab = inv[a.block_table].astype(np.int32)
    o2 = A.attention_oracle(a.seqs, a.q, a2_k, a2_v, tab, a.tree_masks, num_q_heads=4, num_kv_heads=2,
                            block_size=4, scale=a.scale)
    assert np.array_equal(o, o2)
    # shared prefix blocks == private copies
    sh = tiny([W.SeqSpec(4, 9, P), W.SeqSpec(3, 9, P, share_prefix_with=0)], 71, hq=4, hkv=2)
    assert (sh.block_table[0, :2] == sh.block_table[1, :2]).all() and sh.block_table[0, 2] != sh.block_table[1, 2]
    pr = tiny([W.SeqSpec(4, 9, P), W.SeqSpec(3, 9, P)], 72, hq=4, hkv=2)
    pr.q[:] = sh.q
    _copy_logical(pr, 0, sh, 0, 13)
    _copy_logical(pr, 1, sh, 1, 12)
    assert np.array_equal(run(sh), run(pr))
    # same logical K/V on pages of 4 and of 16
    b4 = tiny([W.SeqSpec(5, 14, P)], 73, hq=4, hkv=2, bs=4)
    b16 = tiny([W.SeqSpec(5, 14, P)], 74, hq=4, hkv=2, bs=16)
    b16.q[:] = b4.q
    _copy_logical(b16, 0, b4, 0, 19)
    assert np.array_equal(run(b4), run(b16))


def test_gqa_equals_expanded_mha():
    a = tiny([W.SeqSpec(3, 6, P), W.SeqSpec(1, 4, D_)], 80, hq=4, hkv=2)
    o = run(a)
    k2, v2 = np.repeat(a.k_cache, 2, axis=1), np.repeat(a.v_cache, 2, axis=1)
    o2 = A.attention_oracle(a.seqs, a.q, k2, v2, a.block_table, a.tree_masks, num_q_heads=4,
                            num_kv_heads=4, block_size=4, scale=a.scale)
    assert np.array_equal(o, o2)


def test_row_subset_entry_point_matches_full():
    rng = np.random.default_rng(4)
    b = tiny([W.SeqSpec(5, 3, P), W.SeqSpec(4, 6, V, W.MASK_TREE, W.random_tree(rng, 4))], 90, hq=4, hkv=2)
    o = run(b)
    rows = [(0, 0, 0), (0, 4, 3), (1, 2, 1), (1, 3, 2)]
    sub = A.attention_oracle_rows(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks, rows,
                                  num_q_heads=4, num_kv_heads=2, block_size=4, scale=b.scale)
    starts = [0, 5]
    for (i, r, h), got in zip(rows, sub):
        np.testing.assert_allclose(got, o[starts[i] + r, h], rtol=0, atol=1e-14)


def test_split_merge_equals_whole_row_and_empty_partition_has_zero_weight():
    rng = np.random.default_rng(17)
    n, rows, d = 23, 5, 6
    sc = rng.normal(size=(rows, n)) * 3
    vals = rng.normal(size=(n, d))
    vis = rng.random((rows, n)) < 0.7
    vis[:, 0] = True
    vis[2, 8:15] = False                      # partition [8,15) has no visible key for row 2
    whole = A.masked_softmax_rows(sc, vis) @ vals
    cuts = [0, 8, 15, 16, 23]
    parts = [A.partial_attention(sc[:, a:b], vis[:, a:b], vals[a:b]) for a, b in zip(cuts, cuts[1:])]
    assert not np.isfinite(parts[1][0][2])
    got = A.merge_partials(parts)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, whole, atol=1e-12)
    # closed form for two partitions of one row, written out by hand
    s = np.array([[0.3, -1.2, 2.0]])
    v = np.array([[1.0], [2.0], [4.0]])
    e = np.exp(s[0])
    expect = (e * v[:, 0]).sum() / e.sum()
    got = A.merge_partials([A.partial_attention(s[:, :1], np.ones((1, 1), bool), v[:1]),
                            A.partial_attention(s[:, 1:], np.ones((1, 2), bool), v[1:])])
    assert abs(got[0, 0] - expect) < 1e-14


def test_row_without_visible_key_is_zero_not_nan():
    words = np.zeros(2, dtype=np.uint32)      # empty 2x2 corner, no cached context
    b = tiny([W.SeqSpec(2, 0, V, W.MASK_TREE, [-1, 0])], 95)
    o = A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, words, num_q_heads=2,
                           num_kv_heads=1, block_size=4, scale=1.0)
    assert np.array_equal(o, np.zeros_like(o))
