"""Whole-row fp64 attention over a paged K/V cache: the definition the HIP path must match.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Nothing here tiles,
fuses or reorders: every query row gets its full score vector, one masked
softmax over it, and one weighted sum of V rows — the short-sequence three-stage
form QK -> Softmax -> SV of the paper's section 4.2.1, which never needs the
Update stage.

Conventions (paper section 3.2.1 for the Token-Table fields, 4.1.1 for paging,
4.1.2 for the speculative mask, 4.2.2 for the causal bound):

* a sequence is ``(query_len q, context_len c, kind, mask_kind, mask_word_offset)``;
  ``c`` is the *historical* kvLen, i.e. the tokens cached before this step's
  queries, so the sequence holds ``n = c + q`` keys and this step's own K/V are
  already in the cache at positions ``c .. c+q-1``;
* key position ``j`` of sequence ``i`` lives in physical block
  ``block_table[i, j // B]`` at slot ``j % B`` (section 4.1.1);
* query head ``h`` reads KV head ``h // (Hq // Hkv)``;
* row ``r`` of a PREFILL / DECODE / causal VERIFY sequence may see keys
  ``0 .. c + r`` (section 4.2.2: everything after is invalid);
* row ``r`` of a tree VERIFY sequence sees every cached key ``j < c`` and key
  ``c + s`` exactly when bit ``s`` of its packed mask row is set (section 4.1.2:
  only the specLen x specLen corner is materialised).  A mask row is
  ``ceil(q / 32)`` little-endian uint32 words, rows contiguous, the sequence's
  first word at ``mask_word_offset``;
* a row with no visible key is defined as all zeros.
"""
from __future__ import annotations

import numpy as np

PREFILL, DECODE, VERIFY = 0, 1, 2
MASK_CAUSAL, MASK_TREE = 0, 1


def widen(x):
    """Exact widening to fp64; uint16 arrays are taken as bf16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        x = (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return x.astype(np.float64)


def _seq_fields(s):
    """Accept a 5-tuple or any object with the five named attributes."""
    if isinstance(s, (tuple, list)):
        q, c, kind, mk, off = s
    else:
        q, c, kind, mk, off = (s.query_len, s.context_len, s.kind, s.mask_kind,
                               s.mask_word_offset)
    return int(q), int(c), int(kind), int(mk), int(off)


def visible_keys(q, c, mask_kind, tree_words, mask_word_offset):
    """Boolean matrix [q, c + q]: which key positions each query row may see."""
    n = c + q
    vis = np.zeros((q, n), dtype=bool)
    if mask_kind == MASK_CAUSAL:
        for r in range(q):
            vis[r, : c + r + 1] = True
    else:
        words_per_row = (q + 31) // 32
        vis[:, :c] = True
        for r in range(q):
            for s in range(q):
                w = int(tree_words[mask_word_offset + r * words_per_row + s // 32])
                if (w >> (s % 32)) & 1:
                    vis[r, c + s] = True
    return vis


def gather_kv(cache, block_row, n, kv_head, block_size):
    """Rows 0..n-1 of one sequence for one KV head, read through its block-table row.

    ``cache`` is indexed ``[physical_block, kv_head, slot, d]``.
    """
    out = np.empty((n, cache.shape[-1]), dtype=np.float64)
    for j0 in range(0, n, block_size):
        m = min(block_size, n - j0)
        out[j0 : j0 + m] = widen(cache[int(block_row[j0 // block_size]), kv_head, :m, :])
    return out


def masked_softmax_rows(scores, vis):
    """Row softmax over the visible entries only; invisible entries get weight 0.

    A row with nothing visible gets all-zero weights.
    """
    neg = np.where(vis, scores, -np.inf)
    mx = neg.max(axis=1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.where(vis, np.exp(neg - mx), 0.0)
    den = e.sum(axis=1, keepdims=True)
    return np.divide(e, den, out=np.zeros_like(e), where=den > 0)


def attention_oracle(seqs, q, k_cache, v_cache, block_table, tree_masks, *,
                     num_q_heads, num_kv_heads, block_size, scale,
                     only_seqs=None, return_weights=False, row_chunk=256):
    """O[t, h, :] for every scheduled token t and head h, in fp64.

    q            [sum(query_len), Hq, D]   (float dtype, or uint16 = bf16 bits; widened exactly)
    k_cache      [num_blocks, Hkv, B, D]   likewise for v_cache
    block_table  [num_seqs, max_blocks]    integer physical block ids
    tree_masks   1-D uint32 words, or None when no sequence uses a tree mask
    only_seqs    optional iterable of sequence indices; other rows stay 0
    return_weights   also return {(seq, head): [q, n] weight matrix}

    Rows are processed ``row_chunk`` at a time purely to bound memory; rows are
    independent, so this changes no arithmetic.
    """
    hq, hkv = int(num_q_heads), int(num_kv_heads)
    group = hq // hkv
    d = q.shape[-1]
    total_q = sum(_seq_fields(s)[0] for s in seqs)
    assert q.shape[0] == total_q and q.shape[1] == hq
    out = np.zeros((total_q, hq, d), dtype=np.float64)
    weights = {}
    wanted = None if only_seqs is None else set(int(x) for x in only_seqs)
    t0 = 0
    for i, s in enumerate(seqs):
        ql, c, _kind, mk, off = _seq_fields(s)
        if wanted is not None and i not in wanted:
            t0 += ql
            continue
        n = c + ql
        vis = visible_keys(ql, c, mk, tree_masks, off)
        for g in range(hkv):
            kk = gather_kv(k_cache, block_table[i], n, g, block_size)
            vv = gather_kv(v_cache, block_table[i], n, g, block_size)
            for h in range(g * group, (g + 1) * group):
                for r0 in range(0, ql, row_chunk):
                    r1 = min(ql, r0 + row_chunk)
                    qq = widen(q[t0 + r0 : t0 + r1, h, :])
                    sc = scale * (qq @ kk.T)
                    p = masked_softmax_rows(sc, vis[r0:r1])
                    out[t0 + r0 : t0 + r1, h, :] = p @ vv
                    if return_weights:
                        weights.setdefault((i, h), np.zeros((ql, n)))[r0:r1] = p
        t0 += ql
    return (out, weights) if return_weights else out


def attention_oracle_rows(seqs, q, k_cache, v_cache, block_table, tree_masks, rows, *,
                          num_q_heads, num_kv_heads, block_size, scale):
    """The same definition for a hand-picked list of ``(seq, row, head)`` triples.

    Returns an array [len(rows), D].  Used where the full batch is too large to
    evaluate on the host in seconds.
    """
    group = int(num_q_heads) // int(num_kv_heads)
    starts = np.concatenate([[0], np.cumsum([_seq_fields(s)[0] for s in seqs])])
    d = q.shape[-1]
    res = np.zeros((len(rows), d), dtype=np.float64)
    for idx, (i, r, h) in enumerate(rows):
        ql, c, _kind, mk, off = _seq_fields(seqs[i])
        n = c + ql
        vis = visible_keys(ql, c, mk, tree_masks, off)[r : r + 1]
        g = h // group
        kk = gather_kv(k_cache, block_table[i], n, g, block_size)
        vv = gather_kv(v_cache, block_table[i], n, g, block_size)
        qq = widen(q[starts[i] + r, h, :])[None, :]
        p = masked_softmax_rows(scale * (qq @ kk.T), vis)
        res[idx] = (p @ vv)[0]
    return res


def partial_attention(scores, vis, values):
    """Un-normalised softmax state of one key partition: (m, l, acc).

    m = max visible score (-inf if none), l = sum exp(s - m), acc = sum exp(s - m) v.
    This is what a K/V-split work unit hands to the merge (section 4.2.1, the
    Update stage's running quantities).
    """
    neg = np.where(vis, scores, -np.inf)
    m = neg.max(axis=1)
    safe = np.where(np.isfinite(m), m, 0.0)
    e = np.where(vis, np.exp(neg - safe[:, None]), 0.0)
    return m, e.sum(axis=1), e @ values


def merge_partials(parts):
    """Merge per-partition (m, l, acc) triples into normalised output rows.

    O = sum_p exp(m_p - m*) acc_p / sum_p exp(m_p - m*) l_p with m* = max_p m_p;
    a partition with no visible key (m_p = -inf) has weight 0; a row with no
    visible key anywhere is zeros.
    """
    ms = np.stack([p[0] for p in parts])
    mstar = ms.max(axis=0)
    safe = np.where(np.isfinite(mstar), mstar, 0.0)
    num = 0.0
    den = 0.0
    for m, l, acc in parts:
        w = np.where(np.isfinite(m), np.exp(np.where(np.isfinite(m), m, 0.0) - safe), 0.0)
        num = num + w[:, None] * acc
        den = den + w * l
    den = np.asarray(den)
    return np.divide(num, den[:, None], out=np.zeros_like(num), where=den[:, None] > 0)


def allowed_pairs(seqs, tree_masks):
    """Number of visible (row, key) pairs per sequence — the mask-aware work count."""
    counts = []
    for s in seqs:
        ql, c, _kind, mk, off = _seq_fields(s)
        counts.append(int(visible_keys(ql, c, mk, tree_masks, off).sum()))
    return counts
