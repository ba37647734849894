"""K/V append and the fused-QKV run on the GPU (through the C ABI) against the oracles.

The append is byte work: the caches must match the oracle bit for bit.  Every
synthetic batch is generated with this step's rows already in its cache, so the
test reads them out, overwrites their slots (NaN patterns), appends through the
library and compares whole caches -- new slots, history, block tails and spare
blocks alike.
"""
import numpy as np
import pytest

from oracle import attention as A
from oracle import kv_append as KA
from paper_2412_18106_amd import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
P, D_, V = W.PREFILL, W.DECODE, W.VERIFY
NAN_BITS = 0x7FC0


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2412_18106_amd import runner
    return runner


def new_rows_and_wiped_caches(b):
    """(k_new, v_new [tokens, Hkv, D] bits, caches with the new slots overwritten by NaN patterns)."""
    k_new = np.zeros((b.total_q, b.num_kv_heads, b.head_dim), np.uint16)
    v_new = np.zeros_like(k_new)
    k0, v0 = b.k_cache.copy(), b.v_cache.copy()
    t = 0
    for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
        pos = np.arange(c, c + ql)
        blk, slot = b.block_table[i, pos // b.block_size], pos % b.block_size
        k_new[t:t + ql] = b.k_cache[blk, :, slot, :]
        v_new[t:t + ql] = b.v_cache[blk, :, slot, :]
        k0[blk, :, slot, :] = NAN_BITS
        v0[blk, :, slot, :] = NAN_BITS
        t += ql
    return k_new, v_new, k0, v0


def to_dev(torch, bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def run_append(gpu, b, fused_layout):
    """Append through the C ABI; returns the two caches as bit patterns."""
    import torch
    from paper_2412_18106_amd import binding as X
    k_new, v_new, k0, v0 = new_rows_and_wiped_caches(b)
    db = gpu.DeviceBatch(b)
    try:
        db.k_cache.copy_(to_dev(torch, k0))
        db.v_cache.copy_(to_dev(torch, v0))
        if fused_layout:
            hq, hkv = b.num_q_heads, b.num_kv_heads
            fused = torch.zeros(b.total_q, hq + 2 * hkv, b.head_dim, dtype=torch.bfloat16, device="cuda")
            fused[:, hq:hq + hkv] = to_dev(torch, k_new)
            fused[:, hq + hkv:] = to_dev(torch, v_new)
            X.xy_attn_append_kv(db.plan, fused[:, hq:hq + hkv], fused[:, hq + hkv:], db.k_cache, db.v_cache,
                                db.block_table)
        else:
            X.xy_attn_append_kv(db.plan, to_dev(torch, k_new), to_dev(torch, v_new), db.k_cache, db.v_cache,
                                db.block_table)
        torch.cuda.synchronize()
        return (db.k_cache.view(torch.int16).cpu().numpy().view(np.uint16),
                db.v_cache.view(torch.int16).cpu().numpy().view(np.uint16), k_new, v_new, k0, v0)
    finally:
        db.close()


@pytest.mark.parametrize("index", [1, 2, 4])
def test_append_restores_config_caches_bit_for_bit(gpu, index):
    b = W.make_config(index)
    k1, v1, k_new, v_new, k0, v0 = run_append(gpu, b, fused_layout=(index != 2))
    k_ref, v_ref = KA.append_kv_oracle(b.seqs, k_new, v_new, k0, v0, b.block_table, b.block_size)
    assert np.array_equal(k_ref, b.k_cache) and np.array_equal(v_ref, b.v_cache)   # the oracle's own round trip
    assert np.array_equal(k1, k_ref), "K cache differs from the oracle"
    assert np.array_equal(v1, v_ref), "V cache differs from the oracle"


def test_append_ragged_positions_block_boundaries_and_shared_prefixes(gpu):
    specs = [W.SeqSpec(1, 127, D_), W.SeqSpec(1, 128, D_), W.SeqSpec(130, 126, P), W.SeqSpec(7, 0, P),
             W.SeqSpec(5, 255, V, W.MASK_TREE, parents=[-1, 0, 0, 1, 2]),
             W.SeqSpec(40, 300, P), W.SeqSpec(40, 300, P, share_prefix_with=5), W.SeqSpec(1, 0, D_)]
    b = W.make_custom(specs, 8, 2, 77)
    k1, v1, k_new, v_new, k0, v0 = run_append(gpu, b, fused_layout=True)
    k_ref, v_ref = KA.append_kv_oracle(b.seqs, k_new, v_new, k0, v0, b.block_table, b.block_size)
    assert np.array_equal(k1, k_ref) and np.array_equal(v1, v_ref)


@pytest.mark.parametrize("bs", [16, 64])
def test_append_small_pages(gpu, bs):
    specs = [W.SeqSpec(1, bs - 1, D_), W.SeqSpec(1, bs, D_), W.SeqSpec(3 * bs + 5, bs + 3, P), W.SeqSpec(7, 0, P),
             W.SeqSpec(40, 300, P), W.SeqSpec(40, 300, P, share_prefix_with=4)]
    b = W.make_custom(specs, 8, 2, 78 + bs, block_size=bs)
    k1, v1, k_new, v_new, k0, v0 = run_append(gpu, b, fused_layout=True)
    k_ref, v_ref = KA.append_kv_oracle(b.seqs, k_new, v_new, k0, v0, b.block_table, b.block_size)
    assert np.array_equal(k1, k_ref) and np.array_equal(v1, v_ref)


def test_append_config5_sampled_tokens_and_untouched_bytes(gpu):
    # full size (7.8 GB of cache): compare the new slots of sampled sequences and whole sampled blocks
    b = W.make_config(5)
    k1, v1, k_new, v_new, k0, v0 = run_append(gpu, b, fused_layout=True)
    rng = np.random.default_rng(5)
    starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])
    for i in list(rng.integers(0, len(b.seqs), 24)) + [0, 1, len(b.seqs) - 1]:
        ql, c = b.seqs[i][0], b.seqs[i][1]
        for r in {0, ql - 1, int(rng.integers(0, ql))}:
            blk, slot = b.block_table[i, (c + r) // 128], (c + r) % 128
            assert np.array_equal(k1[blk, :, slot], k_new[starts[i] + r])
            assert np.array_equal(v1[blk, :, slot], v_new[starts[i] + r])
    for blk in rng.integers(0, b.k_cache.shape[0], 64):          # whole blocks against the generated cache
        assert np.array_equal(k1[blk], b.k_cache[blk]) and np.array_equal(v1[blk], b.v_cache[blk])


def test_fused_qkv_run_matches_the_attention_oracle(gpu):
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_config(1)
    k_new, v_new, k0, v0 = new_rows_and_wiped_caches(b)
    hq, hkv = b.num_q_heads, b.num_kv_heads
    db = gpu.DeviceBatch(b)
    try:
        db.k_cache.copy_(to_dev(torch, k0))
        db.v_cache.copy_(to_dev(torch, v0))
        fused = torch.zeros(b.total_q, hq + 2 * hkv, b.head_dim, dtype=torch.bfloat16, device="cuda")
        fused[:, :hq] = db.q
        fused[:, hq:hq + hkv] = to_dev(torch, k_new)
        fused[:, hq + hkv:] = to_dev(torch, v_new)
        db.out.fill_(float("nan"))
        X.xy_attn_run_fused_qkv(db.plan, fused, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out,
                                db.workspace, b.scale)
        torch.cuda.synchronize()
        got = db.out.float().cpu().numpy()
        assert np.array_equal(db.k_cache.view(torch.int16).cpu().numpy().view(np.uint16), b.k_cache)
    finally:
        db.close()
    ref = A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks,
                             num_q_heads=hq, num_kv_heads=hkv, block_size=b.block_size, scale=b.scale)
    assert not np.isnan(got).any()
    err = np.abs(got.astype(np.float64) - ref)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


def test_append_errors_and_empty_plan(gpu):
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_config(1)
    db = gpu.DeviceBatch(b)
    try:
        k_new = torch.zeros(b.total_q, b.num_kv_heads, 128, dtype=torch.bfloat16, device="cuda")
        rc = X._lib.xy_attn_append_kv(db.plan, None, None, 0, 0, None, None, 0, 0, 0, None, None)
        assert rc == X.XY_ERR_ARG
        rc = X._lib.xy_attn_append_kv(db.plan, k_new.data_ptr() + 2, k_new.data_ptr(), k_new.stride(0), k_new.stride(1),
                                      db.k_cache.data_ptr(), db.v_cache.data_ptr(), db.k_cache.stride(0),
                                      db.k_cache.stride(1), db.k_cache.stride(2), db.block_table.data_ptr(), None)
        assert rc == X.XY_ERR_ARG                      # misaligned base
        rc = X._lib.xy_attn_append_kv(db.plan, k_new.data_ptr(), k_new.data_ptr(), k_new.stride(0) + 4, k_new.stride(1),
                                      db.k_cache.data_ptr(), db.v_cache.data_ptr(), db.k_cache.stride(0),
                                      db.k_cache.stride(1), db.k_cache.stride(2), db.block_table.data_ptr(), None)
        assert rc == X.XY_ERR_ARG                      # stride not a multiple of 8 elements
    finally:
        db.close()
    plan = X.xy_attn_plan_create(X.xy_attn_default_config(8, 2, 4), [])
    assert X._lib.xy_attn_append_kv(plan, None, None, 0, 0, None, None, 0, 0, 0, None, None) == 0
    X.xy_attn_plan_destroy(plan)
    torch.cuda.synchronize()
