#!/usr/bin/env python3
"""Benchmark of the attention meta-kernel path on one MI355X.

A step is one xy_attn_run over one synthetic mixed batch that already sits in
HBM (plan built and uploaded beforehand; its host time is reported separately).

The default run times the four single-GPU workloads the metric is quoted on, in
one process: the SplitFuse step (2) and the verify-heavy step (4), both bounded
by HBM bandwidth; the prefix-cached prefill batch (3), bounded by the bf16 MFMA
rate; and the long mixed batch (5: two 2048-token prefill chunks on 32768 cached
tokens next to 16 verify segments and 256 decodes at 64 / 8 heads), the largest
of them, whose figures are the headline of the line.  ``per_config`` carries
the same figures for each of the four.  ``--config N`` times one workload only.

Prints ONE JSON line.  A workload's ``value`` is the algorithmic HBM rate (every
sequence's K and V read once per KV head, Q in, O out, block table) over the
step time when it is HBM-bound, or the mask-aware TFLOP/s (4*D*Hq*visible pairs)
when it is MFMA-bound.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "mixed-batch attention TFLOP/s (mask-aware) + decode HBM GB/s, % of roofline"
from paper_2412_18106_amd.metrics import PEAK_BF16_TFLOPS, PEAK_HBM_GBS, work_counts  # noqa: E402  (no GPU needed)

BOUND = {1: "hbm", 2: "hbm", 3: "mfma", 4: "hbm", 5: "mfma"}
WORKLOAD = {1: "config1_tiny_hybrid", 2: "config2_splitfuse_llama3_8b_512prefill_64decodes",
            3: "config3_apc_prefill_8x1024_on_4k-16k_prefix", 4: "config4_verify_heavy_128_trees",
            5: "config5_long_mixed_qwen2_72b"}
DEFAULT_SET = (2, 3, 4, 5)
HEADLINE = 5
# HBM bytes per launch of the unit kernel with the default plan: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of
# `bench.py --config N` (one run per counter), each scaled by what the same counter reads for a plain 1 GiB device
# copy in the same run (fetch x2.0, write x1.0).  They belong to one version of the kernel and planner sources:
# when those differ from the version named here the line says null instead of a stale figure.
TRAFFIC = {"sources_sha256_16": "23cb2771df9b9a00", "bytes": {2: 1279255478, 3: 339915441, 4: 1229376021, 5: 8480453414}}


def sources_digest():
    h = hashlib.sha256()
    for rel in ("paper_2412_18106_amd/csrc/attn_kernels.hip", "paper_2412_18106_amd/csrc/plan.cpp"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def time_steps(db, steps, warmup):
    import torch
    for _ in range(warmup):
        db.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        db.run()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_kernels(db, steps):
    """Average duration of the persistent unit kernel and of the merge kernel, by HIP events on the launch stream."""
    import torch
    from paper_2412_18106_amd import binding as X
    s = torch.cuda.current_stream()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    args = (db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, db.workspace,
            db.batch.scale, s)
    for e in evs:
        e[0].record(s)
        X.xy_attn_run_phase(X.XY_PHASE_UNITS, *args)
        e[1].record(s)
        X.xy_attn_run_phase(X.XY_PHASE_MERGE, *args)
        e[2].record(s)
    torch.cuda.synchronize()
    units = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    merge = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    return units, merge


def time_fused_steps(db, fused, steps, warmup):
    """Steps that start from the fused projection output: K/V append, then attention with Q read in place."""
    import torch
    from paper_2412_18106_amd import binding as X
    args = (db.plan, fused, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, db.workspace,
            db.batch.scale)
    for _ in range(warmup):
        X.xy_attn_run_fused_qkv(*args)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        X.xy_attn_run_fused_qkv(*args)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    s = torch.cuda.current_stream()
    hq, hkv = db.batch.num_q_heads, db.batch.num_kv_heads
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    for e in evs:
        e[0].record(s)
        X.xy_attn_append_kv(db.plan, fused[:, hq:hq + hkv], fused[:, hq + hkv:], db.k_cache, db.v_cache,
                            db.block_table)
        e[1].record(s)
    torch.cuda.synchronize()
    return sec, float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))


def time_cold_steps(db, steps):
    """Step time with the caches evicted before every step, by events around the run.

    The eviction is a streaming READ of 1 GiB of other memory: it leaves the caches full of clean lines.  (A fill
    would leave them full of dirty lines, and the step would be charged their write-back, about 50 us.)"""
    import torch
    from paper_2412_18106_amd import binding as X
    scrub = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    s = torch.cuda.current_stream()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    for e in evs:
        X.xy_probe_stream_read(scrub, sink)
        e[0].record(s)
        db.run()
        e[1].record(s)
    torch.cuda.synchronize()
    return float(np.mean([e[0].elapsed_time(e[1]) for e in evs])) * 1e-3


def measured_peaks():
    """What this GPU reaches on a plain streaming read and on back-to-back bf16 MFMAs, and what other instructions
    between the MFMAs of a lone wavefront cost (probe kernels of the library)."""
    import torch
    from paper_2412_18106_amd import binding as X
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    buf = torch.ones(1 << 32, dtype=torch.uint8, device="cuda")      # 4 GiB: far beyond the last-level cache
    s = torch.cuda.current_stream()
    out = {}
    for name, launch, work in (("stream_read_GBps", lambda: X.xy_probe_stream_read(buf, sink), float(buf.numel()) / 1e9),
                               ("stream_read_once_GBps", lambda: X.xy_probe_stream_read_once(buf, sink), float(buf.numel()) / 1e9),
                               ("mfma_bf16_TFLOPs", lambda: X.xy_probe_mfma(4000, sink), 2048 * 4000 * 16 * 32768 / 1e12)):
        launch()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(5)]
        for e in ev:
            e[0].record(s)
            launch()
            e[1].record(s)
        torch.cuda.synchronize()
        out[name] = work / (min(e[0].elapsed_time(e[1]) for e in ev) * 1e-3)
    del buf
    # what the instructions between the MFMAs of a lone wavefront cost: cycles per 32 MFMAs (1024 alone)
    cycles = torch.zeros(1024, dtype=torch.int64, device="cuda")
    iters = 2000
    mix = {}
    for name, code in X.XY_MIX.items():
        X.xy_probe_issue_mix(code, iters, cycles, sink)
        X.xy_probe_issue_mix(code, iters, cycles, sink)
        torch.cuda.synchronize()
        mix[name] = float(cycles.max().item()) / iters
    out["lone_wavefront_cycles_per_32_mfma"] = mix
    return out


def attribution(db, overrides, steps, warmup):
    """The prefill part and the decode / verify part of a mixed batch timed as batches of their own (the same
    sequences, K/V caches and queries, each part with a plan of its own)."""
    from paper_2412_18106_amd import workloads as W
    out = {}
    for name, kinds in (("prefill_only", (W.PREFILL,)), ("decode_verify_only", (W.DECODE, W.VERIFY))):
        keep = [i for i, s in enumerate(db.batch.seqs) if s[2] in kinds]
        if not keep:
            continue
        sub = db.subset(keep, **{k: v for k, v in overrides.items() if k != "block_size"})
        pairs, flops, nbytes = work_counts(sub.batch)
        sec = time_steps(sub, steps, warmup)
        sub.close()
        out[name] = {"ms_per_step": sec * 1e3, "tflops_mask_aware": flops / sec / 1e12,
                     "gbps_algorithmic": nbytes / sec / 1e9, "num_seqs": len(keep),
                     "roofline_frac": max(flops / (PEAK_BF16_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)) / sec}
        del sub
    return out


def cpu_baseline(b, bound, budget_s=15.0):
    """The fp64 oracle as it stands, timed on the host on a bounded sample of the same batch: (sequence, KV head)
    slices in batch order -- the query heads of one KV head with that head's K/V -- until budget_s of wall time
    have been spent (at least one slice)."""
    from oracle import attention as A
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    group = b.num_q_heads // b.num_kv_heads
    sub_flops = sub_bytes = 0.0
    done, seqs_done = 0, set()
    t0 = time.perf_counter()
    for i, seq in enumerate(b.seqs):
        one = type("B", (), {"seqs": [seq], "tree_masks": b.tree_masks, "head_dim": b.head_dim, "num_q_heads": group,
                             "num_kv_heads": 1, "block_size": b.block_size, "total_q": seq[0]})
        _, fl, by = work_counts(one)          # of one (sequence, KV head) slice
        for g in range(b.num_kv_heads):
            if done and time.perf_counter() - t0 > budget_s:
                break
            A.attention_oracle(b.seqs, b.q[:, g * group:(g + 1) * group], b.k_cache[:, g:g + 1], b.v_cache[:, g:g + 1],
                               b.block_table, b.tree_masks, num_q_heads=group, num_kv_heads=1,
                               block_size=b.block_size, scale=b.scale, only_seqs=[i])
            sub_flops += fl
            sub_bytes += by
            done += 1
            seqs_done.add(i)
        else:
            continue
        break
    dt = time.perf_counter() - t0
    if bound == "hbm":
        val, unit = sub_bytes / dt / 1e9, "GB/s"
    else:
        val, unit = sub_flops / dt / 1e12, "TFLOP/s"
    return {"value": val, "unit": unit, "cores": int(cores), "kind": "oracle",
            "sample": f"the first {done} (sequence, KV head) slices of the same batch in batch order "
                      f"({len(seqs_done)} of {len(b.seqs)} sequences; each slice = the {group} query heads "
                      f"of one KV head, all rows), {dt:.2f} s wall (numpy fp64, BLAS threads = cores)",
            "seconds": dt}


def measure(index, args, overrides, extras):
    """Times one workload; returns (record, batch).  extras: also the cold-cache run and the prefill / decode split."""
    import torch
    from paper_2412_18106_amd import binding as X
    from paper_2412_18106_amd import workloads as W
    from paper_2412_18106_amd.runner import DeviceBatch
    b = W.make_config(index)
    pairs, flops, nbytes = work_counts(b)
    db = DeviceBatch(b, **overrides)
    units, _, merges = X.plan_arrays(db.plan, db.cfg.num_workers)
    append_ms = None
    if args.fused_qkv:
        hq, hkv = b.num_q_heads, b.num_kv_heads
        fused = torch.zeros(b.total_q, hq + 2 * hkv, b.head_dim, dtype=torch.bfloat16, device="cuda")
        fused[:, :hq] = db.q
        pos = 0                              # this step's rows, read back from the generated cache
        for i, (ql, c, kind, mk, off) in enumerate(b.seqs):
            p_ = np.arange(c, c + ql)
            blk = torch.from_numpy(b.block_table[i, p_ // b.block_size].astype(np.int64)).cuda()
            slot = torch.from_numpy((p_ % b.block_size).astype(np.int64)).cuda()
            fused[pos:pos + ql, hq:hq + hkv] = db.k_cache[blk, :, slot, :]
            fused[pos:pos + ql, hq + hkv:] = db.v_cache[blk, :, slot, :]
            pos += ql
        sec, append_ms = time_fused_steps(db, fused, args.steps, args.warmup)
    else:
        sec = time_steps(db, args.steps, args.warmup)
    k_units_ms, k_merge_ms = time_kernels(db, args.steps)
    bound = BOUND[index]
    gbs, tflops = nbytes / sec / 1e9, flops / sec / 1e12
    if bound == "hbm":
        value, unit = gbs, "GB/s"
        roof = {"bound": "hbm", "achieved": nbytes / (k_units_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        value, unit = tflops, "TFLOP/s"
        roof = {"bound": "mfma", "achieved": flops / (k_units_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    fresh = not overrides and TRAFFIC["sources_sha256_16"] == sources_digest()
    roof["traffic"] = TRAFFIC["bytes"].get(index) if fresh else None
    roof["kernel"] = "xy_attn_units_kernel"
    roof["kernel_ms"] = k_units_ms
    roof["merge_kernel_ms"] = k_merge_ms
    rec = {
        "workload": WORKLOAD[index], "value": value, "unit": unit, "ms_per_step": sec * 1e3, "bound": bound,
        "gbps_algorithmic": gbs, "tflops_mask_aware": tflops,
        "roofline_frac_step": max(flops / (PEAK_BF16_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)) / sec,
        "visible_pairs": pairs, "flops": flops, "algorithmic_bytes": nbytes,
        # host time of planning this step in a serving loop (rebuild in the existing plan object + one asynchronous
        # copy of its tables), and of the very first plan of the object (allocates its memory on the GPU)
        "plan_and_upload_ms": db.replan_ms(), "plan_first_ms": db.plan_first_ms,
        "roofline": roof,
        "shape": {"num_q_heads": b.num_q_heads, "num_kv_heads": b.num_kv_heads, "head_dim": b.head_dim,
                  "block_size": b.block_size, "num_seqs": len(b.seqs), "query_tokens": b.total_q,
                  "units": int(len(units)), "split_families": int(len(merges)), "plan": db.cfg.as_dict()},
    }
    if append_ms is not None:
        app_bytes = 2 * 2 * b.total_q * b.num_kv_heads * b.head_dim * 2      # K and V rows, read and written
        rec["step"] = "fused_qkv: kv_append + attention"
        rec["kv_append"] = {"kernel": "xy_attn_append_kernel", "kernel_ms": append_ms, "bytes": app_bytes,
                            "GBps": app_bytes / (append_ms * 1e-3) / 1e9}
    if extras:
        if not args.no_cold:
            rec["ms_per_step_cold_caches"] = time_cold_steps(db, min(args.steps, 30)) * 1e3
        if not args.no_attribution and index in (2, 5) and not args.fused_qkv:
            rec["attribution"] = attribution(db, overrides, max(10, args.steps // 4), 5)
    db.close()
    del db
    torch.cuda.empty_cache()
    return rec, b


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=0,
                    help="time one workload 1..5 only (default 0: workloads 2, 3, 4 and 5, headline = 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plan", type=str, default="", help="comma separated plan overrides, e.g. split_kv_blocks=8")
    ap.add_argument("--fused-qkv", action="store_true",
                    help="a step starts from the fused projection output: K/V rows are appended to the cache "
                         "(xy_attn_run_fused_qkv) before attention; the append kernel is also timed alone")
    ap.add_argument("--no-attribution", action="store_true",
                    help="skip timing the prefill-only and decode/verify-only sub-batches of a mixed workload")
    ap.add_argument("--no-cold", action="store_true", help="skip the run with caches evicted before every step")
    ap.add_argument("--no-peaks", action="store_true", help="skip the stream-read and MFMA probe kernels")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one plain device copy of this many MiB (a known-size kernel to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters with)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)

    overrides = {}
    for kv in filter(None, args.plan.split(",")):
        k, v = kv.split("=")
        overrides[k] = int(v)
    indices = DEFAULT_SET if args.config == 0 else (args.config,)
    head_index = HEADLINE if args.config == 0 else args.config
    per_config, head_batch = {}, None
    for index in indices:
        rec, b = measure(index, args, overrides, extras=(index == head_index))
        per_config[str(index)] = rec
        if index == head_index:
            head_batch = b
        del b
    head = per_config[str(head_index)]
    line = {
        "metric": METRIC, "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": dict({"workload": head["workload"]}, **head["shape"]),
    }
    for k in ("gbps_algorithmic", "tflops_mask_aware", "roofline_frac_step", "visible_pairs", "flops",
              "algorithmic_bytes", "plan_and_upload_ms", "plan_first_ms", "roofline", "ms_per_step_cold_caches", "attribution",
              "kv_append"):
        if k in head:
            line[k] = head[k]
    if args.fused_qkv:
        line["config"]["step"] = head["step"]
    if len(per_config) > 1:
        line["per_config"] = {k: {kk: vv for kk, vv in v.items() if kk not in ("attribution",)}
                              for k, v in per_config.items()}
    if not args.no_peaks:
        line["measured_peaks"] = measured_peaks()
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        line["copy_calibration_bytes"] = n
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(head_batch, head["bound"])
    print(json.dumps(line))


if __name__ == "__main__":
    main()
