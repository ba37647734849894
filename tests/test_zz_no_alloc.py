"""xy_attn_run_static (the entry point that allocates nothing: K/V-split partial results in the library's fixed
device array) against xy_attn_run with a caller's workspace, bit for bit, on two calls in a row, the second with
a smaller input; and its refusals."""
import numpy as np
import pytest

from paper_2412_18106_amd import workloads as W

pytestmark = pytest.mark.gpu
P, D_, V = W.PREFILL, W.DECODE, W.VERIFY


def _both_ways(b, **cfg):
    import torch
    from paper_2412_18106_amd import binding as X
    from paper_2412_18106_amd.runner import DeviceBatch
    db = DeviceBatch(b, **cfg)              # uploads the plan
    try:
        assert 0 < X.xy_attn_plan_workspace_bytes(db.plan) <= X.XY_STATIC_WORKSPACE_BYTES
        want = db.run_numpy()               # xy_attn_run, workspace from the caller
        db.out.fill_(float("nan"))
        before = torch.cuda.memory_allocated()
        X.xy_attn_run_static(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out,
                             b.scale)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        got = db.out.float().cpu().numpy()
    finally:
        db.close()
    assert not np.isnan(got).any()
    assert np.array_equal(got, want)


def test_static_workspace_run_equals_run_twice_in_a_row_second_smaller():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    rng = np.random.default_rng(77)
    # first call: split decodes, split tree verifies of both unit shapes, a prefill chunk beside them
    specs = [W.SeqSpec(1, int(c), D_) for c in rng.integers(600, 5000, size=24)]
    specs += [W.SeqSpec(int(n), int(c), V, W.MASK_TREE, W.random_tree(rng, int(n)))
              for n, c in zip(rng.integers(2, 9, size=12), rng.integers(700, 4000, size=12))]
    specs += [W.SeqSpec(40, 5000, V, W.MASK_TREE, W.random_tree(rng, 40)), W.SeqSpec(300, 900, P)]
    _both_ways(W.make_custom(specs, 32, 8, 4242))
    # second call, smaller: the array still holds the first call's partial results
    _both_ways(W.make_config(1), split_kv_blocks=1)
    _both_ways(W.make_custom([W.SeqSpec(1, 700, D_)], 8, 2, 4243), split_kv_blocks=2)


def test_static_workspace_run_refusals():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    from paper_2412_18106_amd import binding as X
    from paper_2412_18106_amd.runner import DeviceBatch
    b = W.make_config(1)
    db = DeviceBatch(b, split_kv_blocks=1)
    try:
        # a plan that has not been copied to the GPU: that copy would allocate
        fresh = X.xy_attn_plan_create(db.cfg, b.seqs)
        with pytest.raises(X.XyError) as e:
            X.xy_attn_run_static(fresh, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, b.scale)
        assert e.value.status == X.XY_ERR_ARG
        X.xy_attn_plan_destroy(fresh)
        # a plan whose partial results do not fit the fixed array: 512 decodes on 32768 tokens, 64 / 8 heads
        cfg = X.xy_attn_default_config(64, 8, 257, split_kv_blocks=8)
        big = X.xy_attn_plan_create(cfg, [(1, 32768, D_, 0, 0)] * 512)
        assert X.xy_attn_plan_workspace_bytes(big) > X.XY_STATIC_WORKSPACE_BYTES
        X.xy_attn_plan_upload(big)
        db.out.fill_(float("nan"))
        with pytest.raises(X.XyError) as e:
            X.xy_attn_run_static(big, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, b.scale)
        assert e.value.status == X.XY_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert torch.isnan(db.out.float()).all()          # nothing was enqueued
        X.xy_attn_plan_destroy(big)
    finally:
        db.close()
