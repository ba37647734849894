"""Work counts of a batch for the throughput figures (no GPU, no oracle).

Mask-aware FLOPs: 4 * D * Hq per visible (row, key) pair -- QK^T and PV, two
FLOPs per multiply-add -- with the pairs counted in closed form: q*c + q(q+1)/2
for a causal sequence, q*c + popcount(corner mask) for a tree (the paper's
section 4.2.2: invalid regions are skipped in every stage).  Algorithmic bytes:
every sequence's K and V read once per KV head, Q in, O out, 4 bytes per block
table entry.
"""
from __future__ import annotations

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published


def work_counts(b):
    """(visible pairs, mask-aware FLOPs, algorithmic bytes) from the drawn lengths of a workloads.Batch."""
    pairs = 0
    kv_tokens = 0
    blocks = 0
    for (ql, c, kind, mk, off) in b.seqs:
        if mk == 1:
            wpr = (ql + 31) // 32
            pop = sum(bin(int(w)).count("1") for w in b.tree_masks[off: off + ql * wpr])
            pairs += ql * c + pop
        else:
            pairs += ql * c + ql * (ql + 1) // 2
        kv_tokens += c + ql
        blocks += -(-(c + ql) // b.block_size)
    flops = 4 * b.head_dim * b.num_q_heads * pairs
    kv_bytes = kv_tokens * 2 * b.num_kv_heads * b.head_dim * 2
    qo_bytes = 2 * b.total_q * b.num_q_heads * b.head_dim * 2
    return pairs, flops, kv_bytes + qo_bytes + 4 * blocks


def roofline_fraction(flops, nbytes, seconds):
    """Fraction of the roofline time max(FLOPs / MFMA peak, bytes / HBM peak) over the measured time."""
    return max(flops / (PEAK_BF16_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)) / seconds
