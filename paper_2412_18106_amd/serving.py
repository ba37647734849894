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
output of a step is seeded noise.

Speculative decoding (sections 3.1 and 4.1.2): a request may be marked speculative;
once its prompt is in the cache, each of its steps is a VERIFY segment -- a drawn
draft of up to 31 tokens, a chain (causal corner) or a token tree (packed corner
mask) whose first tokens form the path that will be accepted -- instead of a one
token decode.  The K/V rows of a draft are written behind the sequence's cached
tokens: into the free rows of its private tail block and, past that, into blocks
of a small draft pool the driver keeps outside the block manager.  After the step
the accepted tokens are appended for real (xy_kv_extend); accepted rows that sat
in a pool block are copied into the block the manager allocated for them
(xy_attn_copy_block_rows, enqueued in front of the next step); the rest of the
draft is simply left behind the sequence's end, where nothing looks.
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass, field

import numpy as np

from . import binding as X
from .workloads import pack_tree_mask

PREFILL, DECODE, VERIFY = X.XY_PREFILL, X.XY_DECODE, X.XY_VERIFY
MAX_DRAFT = 31


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
    speculative: bool = False   # its decode steps are verify segments
    prompt_ids: object = None   # the prompt as an int32 array, made at admission


def synthetic_requests(n, seed, prefix_lens=(1500, 1000, 500), suffix=(64, 1024), outputs=(16, 128), vocab=32000,
                       arrivals_per_step=2, speculative_fraction=0.0):
    """n requests; each prompt = one of a few shared prefixes (or none) + a private suffix; a fraction of them
    decode speculatively (verify segments)."""
    rng = np.random.default_rng(seed)
    prefixes = [list(map(int, rng.integers(0, vocab, size=pl))) for pl in prefix_lens]
    reqs = []
    for i in range(n):
        k = int(rng.integers(0, len(prefixes) + 1))
        head = prefixes[k] if k < len(prefixes) else []
        tail = list(map(int, rng.integers(0, vocab, size=int(rng.integers(suffix[0], suffix[1] + 1)))))
        reqs.append(Request(i, i // arrivals_per_step, head + tail, int(rng.integers(outputs[0], outputs[1] + 1))))
    if speculative_fraction > 0:
        for r in reqs:                                  # drawn last: the prompts do not depend on the fraction
            r.speculative = bool(rng.random() < speculative_fraction)
    return reqs


def draft_for(rid, index, remaining, max_draft=MAX_DRAFT):
    """The synthetic draft of a speculative request at its index-th generated token: (parents, accepted, tree).
    parents: token tree in an order that puts the accepted path first (node i < accepted hangs below node i - 1);
    accepted: how many tokens the verification keeps (at least 1, at most what the request still has to
    generate); tree: whether the corner mask is passed explicitly (a pure chain may use the causal corner)."""
    rng = np.random.default_rng([977, int(rid), int(index)])
    n = int(rng.integers(2, max_draft + 1))
    chain = n if rng.random() < 0.35 else int(rng.integers(1, n + 1))      # length of the principal path; a third are pure chains
    parents = [i - 1 for i in range(chain)] + [int(rng.integers(0, i)) for i in range(chain, n)]
    accepted = max(1, min(int(rng.integers(1, chain + 1)), int(remaining)))
    tree = chain < n or bool(rng.random() < 0.3)
    return parents, accepted, tree


def generated_token(rid, index, vocab=32000):
    return (rid * 1000003 + index * 7919 + 12345) % vocab


def run_trace(requests, *, num_q_heads, num_kv_heads, num_blocks, block_size=128, token_budget=2048,
              reserved_decode_slots=256, max_steps=100000, fused_fn=None, on_step=None, device="cuda:0",
              sync_before_timing=True, draft_pool_blocks=0):
    """Run the trace to completion.  fused_fn(step, tokens) -> bf16 tensor [tokens, Hq + 2 Hkv, 128] on the
    device (default: seeded noise made on the device); on_step(info) receives the integers and tensors of
    every step (for tests).  Returns a summary dict."""
    import torch
    dev = torch.device(device)
    hq, hkv, d = num_q_heads, num_kv_heads, 128
    k_cache = torch.zeros(num_blocks, hkv, block_size, d, dtype=torch.bfloat16, device=dev)
    v_cache = torch.zeros_like(k_cache)
    # the last draft_pool_blocks physical blocks are the driver's: rows of draft tokens that do not fit a sequence's
    # tail block live there for one step
    assert 0 <= draft_pool_blocks < num_blocks
    managed = num_blocks - draft_pool_blocks
    mgr = X.KvManager(managed, block_size)
    commit_copies = []          # accepted draft rows to move out of the pool before the next step runs
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    if fused_fn is None:
        def fused_fn(step, tokens):
            return (torch.randn(tokens, hq + 2 * hkv, d, generator=gen, device=dev, dtype=torch.float32) * 0.5).to(torch.bfloat16)
    # one plan object and one workspace for the whole trace: every step plans in place (no allocation per step
    # unless a step's plan or partial results are larger than any before)
    plan = X.xy_attn_plan_create(X.xy_attn_default_config(hq, hkv, 1, block_size=block_size), [])
    ws = torch.empty(1 << 20, dtype=torch.float32, device=dev)
    pending = sorted(requests, key=lambda r: (r.arrival, r.rid))
    active, finished = [], 0
    stats = {"steps": 0, "tokens": 0, "prefill_tokens": 0, "decode_tokens": 0, "verify_tokens": 0, "verify_segments": 0,
             "accepted_tokens": 0, "commit_copies": 0, "lost_verify_segments": 0, "prompt_tokens": 0, "reused_tokens": 0,
             "cow_copies": 0, "deferred": 0, "host_sched_ms": 0.0, "host_plan_ms": 0.0, "gpu_ms": 0.0}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    step, stalled = 0, 0
    idle_steps, last_done = 0, -1
    scale = 1.0 / np.sqrt(d)
    while (pending or active) and step < max_steps:
        t0 = time.perf_counter()
        copies = commit_copies                                  # first: what the last step's verification kept
        commit_copies = []
        carried = len(copies)
        while pending and pending[0].arrival <= step:           # admission: match the prompt against the cache
            r = pending[0]
            if r.prompt_ids is None:
                r.prompt_ids = np.ascontiguousarray(r.prompt, dtype=np.int32)   # chunks of it go to the manager as views
            try:
                r.seq, r.cached, cp = mgr.open(r.prompt_ids)
            except X.XyError:
                break                                           # no block for the copy-on-write: try again next step
            pending.pop(0)
            r.computed, r.tokens = r.cached, list(r.prompt)
            copies += cp
            stats["prompt_tokens"] += len(r.prompt)
            stats["reused_tokens"] += r.cached
            active.append(r)
        queue, drafts = [], {}
        for r in active:
            if r.computed < len(r.prompt):
                queue.append((r.rid, PREFILL, len(r.prompt) - r.computed, r.computed))
            elif r.speculative and draft_pool_blocks:
                drafts[r.rid] = draft_for(r.rid, r.generated, r.output_len - r.generated)
                queue.append((r.rid, VERIFY, len(drafts[r.rid][0]), r.computed))
            else:
                queue.append((r.rid, DECODE, 1, r.computed))
        chunk = X.xy_serve_schedule_chunk(token_budget, reserved_decode_slots, queue)
        by_id = {r.rid: r for r in active}
        placed = []
        pool_next = managed                                     # the draft pool is handed out anew every step
        for rid, kind, ql, ctx in chunk:                        # place the chunk's tokens in the cache
            r = by_id[rid]
            if kind == VERIFY:
                # the draft's rows go behind the cached tokens: free rows of the private tail block, then pool blocks
                have = len(mgr.block_row(r.seq))
                extra = -(-(ctx + ql) // block_size) - have
                if pool_next + extra > num_blocks:              # pool exhausted: a plain decode this step
                    kind, ql = DECODE, 1
                else:
                    placed.append((r, kind, ql, ctx, list(range(pool_next, pool_next + extra))))
                    pool_next += extra
                    continue
            try:
                end_tok = r.computed + ql
                mgr.extend(r.seq, r.prompt_ids[r.computed:end_tok] if end_tok <= len(r.prompt_ids)
                           else r.tokens[r.computed:end_tok])
            except X.XyError:
                stats["deferred"] += 1                          # no room this step: the entry waits
                continue
            placed.append((r, kind, ql, ctx, []))
        if not placed:
            step += 1
            stalled = stalled + 1 if (chunk or not pending or pending[0].arrival < step) else 0
            if stalled > 3:
                raise RuntimeError("the trace cannot make progress: every block is pinned or private "
                                   "(num_blocks is too small for the requests in flight)")
            continue
        stalled = 0
        seqs, words = [], []
        for (r, kind, ql, ctx, _pool) in placed:
            if kind == VERIFY and drafts[r.rid][2]:
                seqs.append((ql, ctx, kind, X.XY_MASK_TREE, sum(len(w) for w in words)))
                words.append(pack_tree_mask(drafts[r.rid][0]))
            else:
                seqs.append((ql, ctx, kind, 0, 0))
        tree_words = np.concatenate(words) if words else np.zeros(1, dtype=np.uint32)
        # block-table rows: the manager writes a sequence's blocks straight into its row, pool blocks follow, the
        # rest of the row repeats the last entry (any valid block: nobody may see those slots)
        max_blocks = max(-(-(ctx + ql) // block_size) for (_r, _k, ql, ctx, _p) in placed)
        table = np.zeros((len(placed), max_blocks), dtype=np.int32)
        for i, (r, _k, _q, _c, pool) in enumerate(placed):
            n = mgr.block_row_into(r.seq, table[i])
            if pool:
                table[i, n:n + len(pool)] = pool
                n += len(pool)
            table[i, n:] = table[i, n - 1]
        t1 = time.perf_counter()
        cfg = X.xy_attn_default_config(hq, hkv, max_blocks, block_size=block_size)
        X.xy_attn_plan_rebuild(plan, cfg, seqs)
        X.xy_attn_plan_upload_async(plan)
        need = X.xy_attn_plan_workspace_bytes(plan)
        if need > ws.numel() * 4:
            ws = torch.empty(need // 4 * 2, dtype=torch.float32, device=dev)
        t2 = time.perf_counter()
        n_tok = sum(s[0] for s in seqs)
        fused = fused_fn(step, n_tok)
        out = torch.empty(n_tok, hq, d, dtype=torch.bfloat16, device=dev)
        table_dev = torch.from_numpy(table).to(dev)
        masks_dev = torch.from_numpy(tree_words.view(np.int32)).to(dev)
        if sync_before_timing:
            torch.cuda.synchronize()
        ev[0].record()
        # two launches: a prompt admitted this step may copy-on-write from a block that an accepted draft has just
        # filled, and the copies of one launch run side by side
        X.xy_attn_copy_block_rows(copies[:carried], hkv, k_cache, v_cache)
        X.xy_attn_copy_block_rows(copies[carried:], hkv, k_cache, v_cache)
        X.xy_attn_run_fused_qkv(plan, fused, k_cache, v_cache, table_dev, masks_dev, out, ws, scale)
        ev[1].record()
        torch.cuda.synchronize()
        stats["gpu_ms"] += ev[0].elapsed_time(ev[1])
        if on_step is not None:
            on_step({"step": step, "seqs": seqs, "block_table": table, "copies": list(copies), "fused": fused,
                     "tree_masks": tree_words, "out": out, "k_cache": k_cache, "v_cache": v_cache,
                     "requests": [p[0].rid for p in placed]})
        for r, kind, ql, ctx, pool in placed:                   # book-keeping of the trace
            if kind == VERIFY:
                # the verification keeps the first `accepted` tokens of the draft: they join the sequence for real
                accepted = drafts[r.rid][1]
                new_tokens = [generated_token(r.rid, r.generated + i) for i in range(accepted)]
                had = len(mgr.block_row(r.seq))
                stats["verify_tokens"] += ql
                stats["verify_segments"] += 1
                try:
                    mgr.extend(r.seq, r.tokens[r.computed:r.computed + 1] + new_tokens[:accepted - 1])
                except X.XyError:
                    stats["lost_verify_segments"] += 1          # no block for the accepted tokens: the step is lost
                    continue
                row = mgr.block_row(r.seq)
                mine = [(pool[q - had], row[q], min(block_size, ctx + accepted - q * block_size))
                        for q in range(had, len(row))]          # accepted rows that sat in a pool block
                r.tokens += new_tokens
                r.computed += accepted
                r.generated += accepted
                stats["accepted_tokens"] += accepted
                if r.generated >= r.output_len:
                    mgr.close(r.seq)                            # (its rows need not be moved: its blocks are free again)
                    active.remove(r)
                    finished += 1
                else:
                    commit_copies += mine
                    stats["commit_copies"] += len(mine)
                continue
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
        # over-admission can leave every open sequence waiting for a block another one holds: give up, do not spin
        total_done = finished * 10 ** 9 + sum(r.computed for r in active)
        idle_steps = idle_steps + 1 if total_done == last_done else 0
        last_done = total_done
        if idle_steps > 50:
            raise RuntimeError("the trace makes no progress: the open sequences hold every block and none can grow "
                               "(num_blocks is too small for the requests in flight)")
        stats["steps"] += 1
        stats["tokens"] += n_tok
        stats["cow_copies"] += len(copies) - carried
        stats["host_sched_ms"] += (t1 - t0) * 1e3
        if stats["steps"] == 1:
            stats["host_plan_first_ms"] = (t2 - t1) * 1e3      # the library's first launch loads its code object (tens of ms)
        else:
            stats["host_plan_ms"] += (t2 - t1) * 1e3
        step += 1
    stats.update(mgr.stats())
    stats["finished"] = finished
    X.xy_attn_plan_destroy(plan)
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
    ap.add_argument("--speculative", type=float, default=0.0, metavar="FRACTION",
                    help="fraction of the requests that decode speculatively (verify segments of up to 31 draft tokens)")
    ap.add_argument("--draft-pool", type=int, default=64, help="blocks of the cache set aside for draft rows (used with --speculative)")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("the trace needs a GPU", file=sys.stderr)
        return 2
    reqs = synthetic_requests(args.requests, args.seed, speculative_fraction=args.speculative)
    t0 = time.perf_counter()
    st = run_trace(reqs, num_q_heads=args.heads[0], num_kv_heads=args.heads[1], num_blocks=args.blocks,
                   block_size=args.block_size, token_budget=args.budget, reserved_decode_slots=args.reserved,
                   draft_pool_blocks=args.draft_pool if args.speculative > 0 else 0)
    wall = time.perf_counter() - t0
    n = max(st["steps"], 1)
    line = {"workload": "synthetic_serving_trace", "requests": args.requests, "token_budget": args.budget,
            "reserved_decode_slots": args.reserved, "num_blocks": args.blocks, "block_size": args.block_size,
            "speculative_fraction": args.speculative,
            "num_q_heads": args.heads[0], "num_kv_heads": args.heads[1], **st,
            "prefix_reuse_fraction": st["reused_tokens"] / max(st["prompt_tokens"], 1),
            "gpu_ms_per_step": st["gpu_ms"] / n, "host_sched_ms_per_step": st["host_sched_ms"] / n,
            "host_plan_ms_per_step": st["host_plan_ms"] / max(n - 1, 1), "tokens_per_s_gpu_time": st["tokens"] / (st["gpu_ms"] * 1e-3 + 1e-12),
            "wall_s": wall}
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
