"""Shared helpers of the GPU parity tests: the fp64 oracle over whole batches, spread over the host cores.

The oracle is called as it stands, once per (sequence, KV head): the query heads of one KV head and that KV
head's slice of the caches are handed to it as a batch with one KV head (the definition is per head, so the
slices change no arithmetic).  The calls run in a thread pool with one BLAS thread each, which is what makes
every output row of the two large configurations affordable inside a test.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import attention as A

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def host_workers():
    return max(1, min(16, os.cpu_count() or 1))


def oracle_sequences(b, seq_indices=None, workers=None):
    """fp64 O[t, h, :] of the listed sequences of batch b (all by default); other rows stay zero."""
    from threadpoolctl import threadpool_limits
    hq, hkv = b.num_q_heads, b.num_kv_heads
    group = hq // hkv
    seq_indices = list(range(len(b.seqs))) if seq_indices is None else [int(i) for i in seq_indices]
    out = np.zeros((b.total_q, hq, b.head_dim), dtype=np.float64)
    starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])

    def job(args):
        i, g = args
        o = A.attention_oracle(b.seqs, b.q[:, g * group:(g + 1) * group], b.k_cache[:, g:g + 1], b.v_cache[:, g:g + 1],
                               b.block_table, b.tree_masks, num_q_heads=group, num_kv_heads=1,
                               block_size=b.block_size, scale=b.scale, only_seqs=[i])
        out[starts[i]:starts[i + 1], g * group:(g + 1) * group] = o[starts[i]:starts[i + 1]]

    # heaviest jobs first so the pool drains evenly
    jobs = sorted(((i, g) for i in seq_indices for g in range(hkv)),
                  key=lambda a: -b.seqs[a[0]][0] * (b.seqs[a[0]][1] + b.seqs[a[0]][0]))
    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(max_workers=workers or host_workers()) as ex:
            list(ex.map(job, jobs))
    return out


def check_sequences(got, ref, b, seq_indices, what=""):
    """Every (token, head, d) element of the listed sequences: max-abs and mean-abs per sequence.
    Returns (sum of abs errors, number of elements, max) so that callers can add up an overall mean."""
    starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])
    total, count, worst = 0.0, 0, 0.0
    for i in seq_indices:
        g = got[starts[i]:starts[i + 1]]
        assert not np.isnan(g).any(), f"{what}: NaN in the output of sequence {i} (row never written?)"
        err = np.abs(g.astype(np.float64) - ref[starts[i]:starts[i + 1]])
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, \
            f"{what}: sequence {i} {b.seqs[i][:3]}: max {err.max():.3e} mean {err.mean():.3e}"
        total += float(err.sum())
        count += err.size
        worst = max(worst, float(err.max()))
    return total, count, worst
