"""Move a synthetic Batch to the GPU and run it through the C-ABI library (marshalling only)."""
from __future__ import annotations

import numpy as np

from . import binding as X


class DeviceBatch:
    """Device-resident tensors of a workloads.Batch plus a plan for them."""

    def __init__(self, batch, device="cuda:0", _resident=None, **cfg_overrides):
        import torch

        self.batch = batch
        self.torch = torch
        dev = torch.device(device)

        def bf16(a):
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

        if _resident is None:
            self.q = bf16(batch.q)
            self.k_cache = bf16(batch.k_cache)
            self.v_cache = bf16(batch.v_cache)
            self.tree_masks = torch.from_numpy(batch.tree_masks.view(np.int32)).to(dev)
        else:       # tensors that already sit on the GPU (see subset)
            self.q, self.k_cache, self.v_cache, self.tree_masks = _resident
        self.block_table = torch.from_numpy(np.ascontiguousarray(batch.block_table, dtype=np.int32)).to(dev)
        self.out = torch.empty_like(self.q)
        cfg_overrides.setdefault("block_size", batch.block_size)
        self.cfg = X.xy_attn_default_config(batch.num_q_heads, batch.num_kv_heads, batch.max_blocks_per_seq,
                                            **cfg_overrides)
        import time
        t0 = time.perf_counter()
        self.plan = X.xy_attn_plan_create(self.cfg, batch.seqs)
        X.xy_attn_plan_upload(self.plan)
        self.plan_first_ms = (time.perf_counter() - t0) * 1e3     # first plan of an object: allocates its arena on the GPU
        nbytes = X.xy_attn_plan_workspace_bytes(self.plan)
        self.workspace = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=dev)

    def replan_ms(self, repeats=20):
        """Host time of planning a step in a serving loop: the same batch planned again in the existing plan object
        (xy_attn_plan_rebuild) and its tables sent to the GPU with one asynchronous copy; median of repeats."""
        import time
        descs = X.make_descs(self.batch.seqs)
        times = []
        for _ in range(repeats):
            self.torch.cuda.synchronize()
            t0 = time.perf_counter()
            X.xy_attn_plan_rebuild(self.plan, self.cfg, descs)
            X.xy_attn_plan_upload_async(self.plan)
            times.append((time.perf_counter() - t0) * 1e3)
        self.torch.cuda.synchronize()
        return float(np.median(times))

    def run(self, stream=None):
        X.xy_attn_run(self.plan, self.q, self.k_cache, self.v_cache, self.block_table, self.tree_masks,
                      self.out, self.workspace, self.batch.scale, stream)
        return self.out

    def run_numpy(self):
        """Run once, synchronise, return O as float32 numpy [tokens, Hq, D]."""
        self.out.fill_(float("nan"))
        self.run()
        self.torch.cuda.synchronize()
        return self.out.float().cpu().numpy()

    def subset(self, keep, **cfg_overrides):
        """The sequences listed in keep (ascending indices) as a batch of their own: same K/V caches and mask words
        on the GPU (shared, not copied), their rows of Q and of the block table, a plan of its own."""
        from .workloads import Batch
        b = self.batch
        starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])
        rows = np.concatenate([np.arange(starts[i], starts[i + 1]) for i in keep]) if len(keep) else np.zeros(0, np.int64)
        sub = Batch(name=b.name + "_subset", num_q_heads=b.num_q_heads, num_kv_heads=b.num_kv_heads,
                    head_dim=b.head_dim, block_size=b.block_size, scale=b.scale, seqs=[b.seqs[i] for i in keep],
                    q=b.q[rows], k_cache=b.k_cache, v_cache=b.v_cache, block_table=b.block_table[list(keep)],
                    tree_masks=b.tree_masks, parents=[b.parents[i] for i in keep] if b.parents else [])
        q = self.q[self.torch.from_numpy(rows).to(self.q.device)].contiguous()
        cfg_overrides.setdefault("block_size", int(self.cfg.block_size))
        return DeviceBatch(sub, device=str(self.q.device), _resident=(q, self.k_cache, self.v_cache, self.tree_masks),
                           **cfg_overrides)

    def close(self):
        if self.plan is not None:
            X.xy_attn_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
