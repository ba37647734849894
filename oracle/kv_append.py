"""Writing a step's new K/V rows into the paged cache: the definition the HIP path must match.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper's kernel reads a cache that holds "both historical and newly generated"
tokens (section 4.1.1): before attention runs, the K and V rows that the QKV
projection produced for this step's tokens have to land in their slots.  The
projection output is one fused tensor ``[tokens, Hq + 2 Hkv, headSize]`` that is
read in place by stride instead of being split and permuted first (section 5).

Definition.  Sequence ``i`` has ``c_i`` cached tokens and ``q_i`` new ones, its
packed tokens start at ``t_i`` (running sum of ``q``).  New token ``r`` is key
position ``j = c_i + r``; it goes to physical block ``block_table[i, j // B]``,
slot ``j % B`` (section 4.1.1), for every KV head:

    k_cache[block, g, slot, :] = k_new[t_i + r, g, :]      (same for V)

Nothing else in the cache changes.  Byte work: the stored bit patterns are
copied, never converted.
"""
from __future__ import annotations

import numpy as np


def split_fused_qkv(qkv, num_q_heads, num_kv_heads):
    """Views (no copies) of Q, K_new, V_new inside a fused ``[tokens, Hq + 2 Hkv, D]`` tensor:
    heads ``0 .. Hq-1`` are Q, the next ``Hkv`` are K, the last ``Hkv`` are V (section 5)."""
    qkv = np.asarray(qkv)
    if qkv.ndim != 3 or qkv.shape[1] != num_q_heads + 2 * num_kv_heads:
        raise ValueError("fused tensor must be [tokens, Hq + 2 Hkv, D]")
    return (qkv[:, :num_q_heads], qkv[:, num_q_heads:num_q_heads + num_kv_heads],
            qkv[:, num_q_heads + num_kv_heads:])


def append_kv_oracle(seqs, k_new, v_new, k_cache, v_cache, block_table, block_size):
    """Return copies of ``k_cache`` / ``v_cache`` (``[num_blocks, Hkv, B, D]``) with the rows of
    ``k_new`` / ``v_new`` (``[sum q, Hkv, D]``) written to their slots.

    ``seqs``: 5-tuples ``(query_len, context_len, kind, mask_kind, mask_word_offset)``.
    Raises ValueError when a token falls outside its row of the block table.
    """
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    k_new, v_new = np.asarray(k_new), np.asarray(v_new)
    block_table = np.asarray(block_table)
    t = 0
    for i, s in enumerate(seqs):
        q, c = int(s[0]), int(s[1])
        for r in range(q):
            j = c + r
            if j // block_size >= block_table.shape[1]:
                raise ValueError(f"sequence {i}: position {j} is beyond its block table row")
            block, slot = int(block_table[i, j // block_size]), j % block_size
            k_out[block, :, slot, :] = k_new[t + r]
            v_out[block, :, slot, :] = v_new[t + r]
        t += q
    return k_out, v_out
