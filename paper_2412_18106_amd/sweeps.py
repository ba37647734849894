"""Paper-shaped sweeps of the attention path on one MI355X (a second, synthetic workload).

The paper evaluates its attention kernel on four families of shapes (section 6.2:
prefix-cached prefill over the cached-prefix length, chunked prefill of long
prompts, speculative verification at batch 4 / length 31 and batch 8 / length 15,
decode over batch size and context length) and discusses the page size of the
K/V cache (section 4.1.1).  This module rebuilds those shapes
with seeded synthetic tensors, runs each through the library and prints one JSON
line per case: step time, mask-aware TFLOP/s, algorithmic GB/s and the fraction
of the roofline max(FLOPs / MFMA peak, bytes / HBM peak).  The numbers of the
paper itself are speedups over vendor kernels on another machine and are not
comparable; these lines only show how the path behaves over the same axes.

    python -m paper_2412_18106_amd.sweeps [--family prefix|chunked|verify|decode|pages|all] [--steps K]

Parity of these shapes against the fp64 oracle is covered by the GPU tests, which
take their cases from the generators below.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from . import workloads as W
from .metrics import roofline_fraction, work_counts

SEED = 241218106 + 100


def prefix_cases():
    """A prompt of 4k / 8k tokens whose first p tokens are already cached (p = 0 .. 4k): the prefill
    computes the other tokens on top of the cached prefix (Llama-3-8B head shape, batch 4)."""
    for prompt in (4096, 8192):
        for p in (0, 1024, 2048, 3072, 4096):
            if p >= prompt:
                continue
            yield (f"prefix_prompt{prompt}_cached{p}", 32, 8, [W.SeqSpec(prompt - p, p, W.PREFILL)] * 4, {})


def chunked_cases():
    """One prompt prefilled in chunks of 4k / 8k: the chunk that ends at 16k, 32k and 64k tokens."""
    for chunk in (4096, 8192):
        for end in (16384, 32768, 65536):
            yield (f"chunked_chunk{chunk}_end{end}", 32, 8, [W.SeqSpec(chunk, end - chunk, W.PREFILL)], {})


def verify_cases():
    """Tree verification at (batch 4, 31 draft tokens) and (batch 8, 15 draft tokens) over the context;
    once with the default 32-row units, once with the whole tree in one unit (K/V read once)."""
    rng = np.random.default_rng(SEED)
    for batch, spec in ((4, 31), (8, 15)):
        for ctx in (1024, 4096, 16384):
            specs = [W.SeqSpec(spec, ctx, W.VERIFY, W.MASK_TREE, W.random_tree(rng, spec)) for _ in range(batch)]
            yield (f"verify_b{batch}_spec{spec}_ctx{ctx}", 32, 8, specs, {})
            yield (f"verify_b{batch}_spec{spec}_ctx{ctx}_one_unit_per_tree", 32, 8, specs, {"verify_tile_tokens": spec})


def decode_cases():
    """Decode over batch size x context length at a multi-head shape (32 query heads, 32 KV heads: no
    K/V sharing between heads) and at the grouped shape (32 / 8)."""
    for hq, hkv in ((32, 32), (32, 8)):
        for batch in (8, 32, 128):
            for ctx in (1024, 4096, 16384):
                if hkv == 32 and batch * ctx > 128 * 4096:      # keep the cache of the multi-head shape below 10 GB
                    continue
                yield (f"decode_h{hq}_{hkv}_b{batch}_ctx{ctx}", hq, hkv, [W.SeqSpec(1, ctx, W.DECODE)] * batch, {})


def page_cases():
    """Decode and one prefill chunk over the page size (16 / 32 / 64 / 128 tokens per block-table entry):
    smaller pages fragment the K/V reads into smaller contiguous pieces (section 4.1.1)."""
    for bs in (16, 32, 64, 128):
        yield (f"pages_decode_h32_8_b128_ctx4096_page{bs}", 32, 8, [W.SeqSpec(1, 4096, W.DECODE)] * 128, {"block_size": bs})
    for bs in (16, 32, 64, 128):
        yield (f"pages_prefill_chunk2048_end16384_page{bs}", 32, 8, [W.SeqSpec(2048, 14336, W.PREFILL)] * 2, {"block_size": bs})


FAMILIES = {"prefix": prefix_cases, "chunked": chunked_cases, "verify": verify_cases, "decode": decode_cases,
            "pages": page_cases}


def build_case(name, hq, hkv, specs, overrides):
    """The seeded synthetic batch of one case."""
    return W.make_custom(list(specs), hq, hkv, SEED, name=name, block_size=overrides.get("block_size", 128))


def run_case(name, hq, hkv, specs, overrides, steps):
    import torch
    from .runner import DeviceBatch
    b = build_case(name, hq, hkv, specs, overrides)
    pairs, flops, nbytes = work_counts(b)
    db = DeviceBatch(b, **overrides)
    try:
        for _ in range(3):
            db.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            db.run()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        line = {"case": name, "num_q_heads": hq, "num_kv_heads": hkv, "num_seqs": len(b.seqs),
                "query_tokens": b.total_q, "plan_overrides": overrides, "ms_per_step": sec * 1e3,
                "tflops_mask_aware": flops / sec / 1e12, "gbps_algorithmic": nbytes / sec / 1e9,
                "roofline_frac": roofline_fraction(flops, nbytes, sec)}
        return line
    finally:
        db.close()


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--family", default="all", choices=list(FAMILIES) + ["all"])
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("the sweeps need a GPU", file=sys.stderr)
        return 2
    for fam in (FAMILIES if args.family == "all" else [args.family]):
        for case in FAMILIES[fam]():
            line = run_case(*case, steps=args.steps)
            line["family"] = fam
            print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
