"""The helper that spreads the oracle over the host cores returns exactly what one oracle call returns."""
import numpy as np

from oracle import attention as A
from paper_2412_18106_amd import workloads as W

import parity_util as PU


def test_oracle_per_sequence_and_kv_head_equals_one_call():
    b = W.make_config(1)
    whole = A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks,
                               num_q_heads=b.num_q_heads, num_kv_heads=b.num_kv_heads, block_size=b.block_size,
                               scale=b.scale)
    assert np.array_equal(PU.oracle_sequences(b, workers=3), whole)
    part = PU.oracle_sequences(b, [1, 3])
    starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])
    for i in range(len(b.seqs)):
        rows = slice(starts[i], starts[i + 1])
        assert np.array_equal(part[rows], whole[rows] if i in (1, 3) else np.zeros_like(whole[rows]))
    total, count, worst = PU.check_sequences(whole.astype(np.float32), whole, b, [0, 2], "self")
    assert count == (b.seqs[0][0] + b.seqs[2][0]) * b.num_q_heads * b.head_dim and worst < 1e-6
