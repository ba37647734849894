"""A synthetic serving trace driven through the library end to end (one MI355X).

Every step: the token-budget scheduler composes a chunk from the waiting prefill
and decode tokens (paper section 3.1), the radix-tree block manager places the
chunk's tokens -- reusing cached prefixes token by token, copy-on-write for a
block that matches in part, evicting least recently used leaves (section 4.1.1)
-- the descriptors and block-table rows become a plan, and one fused-QKV run
appends the new K/V rows and computes attention.  Nothing is computed here: this
module only moves the integers from one C call to the next and keeps the books
of the trace.

    python -m paper_2412_18106_amd.serving [--requests N] [--budget T] [--reserved R] ...

prints one JSON line: steps, tokens, reuse, host and GPU time per step.

The trace is synthetic (no tokenizer, no model): prompts are integer sequences
that share a few long "system prompt" prefixes, output lengths are drawn, the
"generated" token ids are a hash of (request, position), and the QKV projection
output of a step is seeded noise.  Speculative (verify) segments are not part of
the trace; they are covered by the fixed configurations and the sweeps.
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass, field

import numpy as np

from . import binding as X

PREFILL, DECODE = X.XY_PREFILL, X.XY_DECODE


@dataclass
class Request:
    rid: int
    arrival: int
    prompt: list
    output_len: int
    seq: int = -1               # handle of the block manager
    computed: int = 0           # tokens whose K/V are in the cache
    generated: int = 0
    tokens: list = field(default_factory=list)   # prompt + generated so far
    cached: int = 0             # prompt tokens reused from the cache at admission


def synthetic_requests(n, seed, prefix_lens=(1500, 1000, 500), suffix=(64, 1024), outputs=(16, 128), vocab=32000,
                       arrivals_per_step=2):
    """n requests; each prompt = one of a few shared prefixes (or none) + a private suffix."""
    rng = np.random.default_rng(seed)
    prefixes = [list(map(int, rng.integers(0, vocab, size=pl))) for pl in prefix_lens]
    reqs = []
    for i in range(n):
        k = int(rng.integers(0, len(prefixes) + 1))
        head = prefixes[k] if k < len(prefixes) else []
        tail = list(map(int, rng.integers(0, vocab, size=int(rng.integers(suffix[0], suffix[1] + 1)))))
        reqs.append(Request(i, i // arrivals_per_step, head + tail, int(rng.integers(outputs[0], outputs[1] + 1))))
    return reqs


def generated_token(rid, index, vocab=32000):
    return (rid * 1000003 + index * 7919 + 12345) % vocab


def run_trace(requests, *, num_q_heads, num_kv_heads, num_blocks, block_size=128, token_budget=2048,
              reserved_decode_slots=256, max_steps=100000, fused_fn=None, on_step=None, device="cuda:0"):
    """Run the trace to completion.  fused_fn(step, tokens) -> bf16 tensor [tokens, Hq + 2 Hkv, 128] on the
    device (default: seeded noise made on the device); on_step(info) receives the integers and tensors of
    every step (for tests).  Returns a summary dict."""
    import torch
    dev = torch.device(device)
    hq, hkv, d = num_q_heads, num_kv_heads, 128
    k_cache = torch.zeros(num_blocks, hkv, block_size, d, dtype=torch.bfloat16, device=dev)
    v_cache = torch.zeros_like(k_cache)
    mgr = X.KvManager(num_blocks, block_size)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    if fused_fn is None:
        def fused_fn(step, tokens):
            return (torch.randn(tokens, hq + 2 * hkv, d, generator=gen, device=dev, dtype=torch.float32) * 0.5).to(torch.bfloat16)
    pending = sorted(requests, key=lambda r: (r.arrival, r.rid))
    active, finished = [], 0
    stats = {"steps": 0, "tokens": 0, "prefill_tokens": 0, "decode_tokens": 0, "prompt_tokens": 0, "reused_tokens": 0,
             "cow_copies": 0, "deferred": 0, "host_sched_ms": 0.0, "host_plan_ms": 0.0, "gpu_ms": 0.0}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    step, stalled = 0, 0
    scale = 1.0 / np.sqrt(d)
    while (pending or active) and step < max_steps:
        t0 = time.perf_counter()
        copies = []
        while pending and pending[0].arrival <= step:           # admission: match the prompt against the cache
            r = pending[0]
            try:
                r.seq, r.cached, cp = mgr.open(r.prompt)
            except X.XyError:
                break                                           # no block for the copy-on-write: try again next step
            pending.pop(0)
            r.computed, r.tokens = r.cached, list(r.prompt)
            copies += cp
            stats["prompt_tokens"] += len(r.prompt)
            stats["reused_tokens"] += r.cached
            active.append(r)
        queue = []
        for r in active:
            if r.computed < len(r.prompt):
                queue.append((r.rid, PREFILL, len(r.prompt) - r.computed, r.computed))
            else:
                queue.append((r.rid, DECODE, 1, r.computed))
        chunk = X.xy_serve_schedule_chunk(token_budget, reserved_decode_slots, queue)
        by_id = {r.rid: r for r in active}
        placed = []
        for rid, kind, ql, ctx in chunk:                        # place the chunk's tokens in the cache
            r = by_id[rid]
            try:
                mgr.extend(r.seq, r.tokens[r.computed:r.computed + ql])
            except X.XyError:
                stats["deferred"] += 1                          # no room this step: the entry waits
                continue
            placed.append((r, kind, ql, ctx))
        if not placed:
            step += 1
            stalled = stalled + 1 if (chunk or not pending or pending[0].arrival < step) else 0
            if stalled > 3:
                raise RuntimeError("the trace cannot make progress: every block is pinned or private "
                                   "(num_blocks is too small for the requests in flight)")
            continue
        stalled = 0
        seqs = [(ql, ctx, kind, 0, 0) for (_r, kind, ql, ctx) in placed]
        rows = [mgr.block_row(r.seq) for (r, _k, _q, _c) in placed]
        max_blocks = max(len(x) for x in rows)
        table = np.zeros((len(rows), max_blocks), dtype=np.int32)
        for i, x in enumerate(rows):
            table[i, :len(x)] = x
            table[i, len(x):] = x[-1]
        t1 = time.perf_counter()
        cfg = X.xy_attn_default_config(hq, hkv, max_blocks, block_size=block_size)
        plan = X.xy_attn_plan_create(cfg, seqs)
        X.xy_attn_plan_upload(plan)
        ws = torch.empty(max(X.xy_attn_plan_workspace_bytes(plan), 16) // 4, dtype=torch.float32, device=dev)
        t2 = time.perf_counter()
        n_tok = sum(s[0] for s in seqs)
        fused = fused_fn(step, n_tok)
        out = torch.empty(n_tok, hq, d, dtype=torch.bfloat16, device=dev)
        table_dev = torch.from_numpy(table).to(dev)
        ev[0].record()
        X.xy_attn_copy_block_rows(copies, hkv, k_cache, v_cache)
        X.xy_attn_run_fused_qkv(plan, fused, k_cache, v_cache, table_dev, None, out, ws, scale)
        ev[1].record()
        torch.cuda.synchronize()
        stats["gpu_ms"] += ev[0].elapsed_time(ev[1])
        X.xy_attn_plan_destroy(plan)
        if on_step is not None:
            on_step({"step": step, "seqs": seqs, "block_table": table, "copies": list(copies), "fused": fused,
                     "out": out, "k_cache": k_cache, "v_cache": v_cache, "requests": [p[0].rid for p in placed]})
        for r, kind, ql, _ctx in placed:                        # book-keeping of the trace
            r.computed += ql
            if kind == PREFILL:
                stats["prefill_tokens"] += ql
                if r.computed == len(r.prompt):                 # the prompt's last token produced the first output
                    r.tokens.append(generated_token(r.rid, 0))
                    r.generated = 1
            else:
                stats["decode_tokens"] += 1
                r.tokens.append(generated_token(r.rid, r.generated))
                r.generated += 1
            if r.generated >= r.output_len and r.computed >= len(r.prompt):
                mgr.close(r.seq)
                active.remove(r)
                finished += 1
        stats["steps"] += 1
        stats["tokens"] += n_tok
        stats["cow_copies"] += len(copies)
        stats["host_sched_ms"] += (t1 - t0) * 1e3
        stats["host_plan_ms"] += (t2 - t1) * 1e3
        step += 1
    stats.update(mgr.stats())
    stats["finished"] = finished
    mgr.destroy()
    return stats


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--requests", type=int, default=96)
    ap.add_argument("--budget", type=int, default=2048)
    ap.add_argument("--reserved", type=int, default=256)
    ap.add_argument("--blocks", type=int, default=640, help="physical K/V blocks (the cache limit)")
    ap.add_argument("--block-size", type=int, default=128)
    ap.add_argument("--heads", type=int, nargs=2, default=(32, 8), metavar=("HQ", "HKV"))
    ap.add_argument("--seed", type=int, default=7)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("the trace needs a GPU", file=sys.stderr)
        return 2
    reqs = synthetic_requests(args.requests, args.seed)
    t0 = time.perf_counter()
    st = run_trace(reqs, num_q_heads=args.heads[0], num_kv_heads=args.heads[1], num_blocks=args.blocks,
                   block_size=args.block_size, token_budget=args.budget, reserved_decode_slots=args.reserved)
    wall = time.perf_counter() - t0
    n = max(st["steps"], 1)
    line = {"workload": "synthetic_serving_trace", "requests": args.requests, "token_budget": args.budget,
            "reserved_decode_slots": args.reserved, "num_blocks": args.blocks, "block_size": args.block_size,
            "num_q_heads": args.heads[0], "num_kv_heads": args.heads[1], **st,
            "prefix_reuse_fraction": st["reused_tokens"] / max(st["prompt_tokens"], 1),
            "gpu_ms_per_step": st["gpu_ms"] / n, "host_sched_ms_per_step": st["host_sched_ms"] / n,
            "host_plan_ms_per_step": st["host_plan_ms"] / n, "tokens_per_s_gpu_time": st["tokens"] / (st["gpu_ms"] * 1e-3 + 1e-12),
            "wall_s": wall}
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
