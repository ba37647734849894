"""Seeded synthetic mixed batches shaped like the paper's serving workloads.

This module only *draws inputs* (lengths, block tables, token trees, bf16 noise);
it contains none of the attention arithmetic and none of the planning rules, so
both the HIP path and the CPU oracle can be fed from it without sharing code.

The five named configurations stand in for the paper's evaluation workloads
(section 6.2: prefix-reuse prefill, chunked prefill, verify, paged decode), whose
own inputs are not available; lengths, head shapes and page size follow those
descriptions, values are N(0,1)*0.5 noise rounded to bf16.

Recipe (identical for every configuration):
  * ``rng = numpy.random.default_rng(241218106 + config_index)``;
  * all lengths are drawn first, then token trees, then the block table
    permutation, then one tensor seed; Q, the K pool and the V pool are drawn in
    fixed-size chunks from generators keyed by (tensor seed, tensor id, chunk);
  * the *whole* physical pool is noise, including tails of partially filled
    blocks and about 1/8 spare blocks, so a masking bug cannot hide behind zeros;
  * unused block-table entries point at spare blocks (valid memory, wrong data).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

PREFILL, DECODE, VERIFY = 0, 1, 2
MASK_CAUSAL, MASK_TREE = 0, 1
BASE_SEED = 241218106


@dataclass
class SeqSpec:
    query_len: int
    context_len: int
    kind: int
    mask_kind: int = MASK_CAUSAL
    parents: list | None = None     # token tree (VERIFY + MASK_TREE only)
    share_prefix_with: int | None = None   # index of an earlier sequence with equal context_len


@dataclass
class Batch:
    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    scale: float
    seqs: list            # [(query_len, context_len, kind, mask_kind, mask_word_offset)]
    q: np.ndarray         # uint16 bf16 bits [sum q, Hq, D]
    k_cache: np.ndarray   # uint16 bf16 bits [num_blocks, Hkv, B, D]
    v_cache: np.ndarray
    block_table: np.ndarray   # int32 [num_seqs, max_blocks]
    tree_masks: np.ndarray    # uint32 words (length >= 1)
    parents: list = field(default_factory=list)

    @property
    def total_q(self):
        return int(sum(s[0] for s in self.seqs))

    @property
    def max_blocks_per_seq(self):
        return int(self.block_table.shape[1])


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _noise_chunk(args):
    key, idx, out, lo, hi = args
    rng = np.random.default_rng(list(key) + [idx])
    out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(0.5))


def noise_bf16(key, shape, chunk=1 << 22, threads=8):
    """N(0,1)*0.5 noise as bf16 bits.

    ``key`` is a list of integers; chunk ``i`` of the flat tensor is drawn from
    ``default_rng(key + [i])``, so the result does not depend on the thread count.
    """
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.uint16)
    jobs = [(key, i, out, lo, min(total, lo + chunk)) for i, lo in enumerate(range(0, total, chunk))]
    if len(jobs) <= 1:
        for j in jobs:
            _noise_chunk(j)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(_noise_chunk, jobs))
    return out.reshape(shape)


def random_tree(rng, n):
    """parent[0] = -1, parent[r] uniform in {-1, ..., r-1}."""
    return [-1] + [int(rng.integers(-1, r)) for r in range(1, n)]


def chain_tree(n):
    return [r - 1 for r in range(n)]


def pack_tree_mask(parents):
    """Rows of ceil(n/32) little-endian uint32 words; bit s of row r set iff s is r or an ancestor of r."""
    n = len(parents)
    wpr = (n + 31) // 32
    words = np.zeros(n * wpr, dtype=np.uint32)
    for r in range(n):
        s = r
        while s >= 0:
            words[r * wpr + s // 32] |= np.uint32(1 << (s % 32))
            s = parents[s]
    return words


def build_batch(name, specs, num_q_heads, num_kv_heads, rng, head_dim=128, block_size=128,
                scale=None, spare_fraction=0.125):
    """Lay a list of SeqSpec out on a shuffled physical pool and draw Q / K / V."""
    b = block_size
    need = [-(-(s.context_len + s.query_len) // b) for s in specs]
    max_blocks = max(need) if need else 1
    # logical -> how many private blocks each sequence consumes
    private = []
    for i, s in enumerate(specs):
        if s.share_prefix_with is not None:
            assert specs[s.share_prefix_with].context_len == s.context_len
            private.append(need[i] - s.context_len // b)
        else:
            private.append(need[i])
    used = int(sum(private))
    spare = max(2, int(np.ceil(used * spare_fraction)))
    num_blocks = used + spare
    perm = rng.permutation(num_blocks).astype(np.int32)
    table = np.empty((len(specs), max_blocks), dtype=np.int32)
    spare_ids = perm[used:]
    cursor = 0
    copies = []   # (dst_block, src_block, rows) for private partial prefix blocks
    for i, s in enumerate(specs):
        shared_full = 0
        if s.share_prefix_with is not None:
            shared_full = s.context_len // b
            table[i, :shared_full] = table[s.share_prefix_with, :shared_full]
        cnt = need[i] - shared_full
        table[i, shared_full:need[i]] = perm[cursor:cursor + cnt]
        cursor += cnt
        if s.share_prefix_with is not None and s.context_len % b:
            copies.append((int(table[i, shared_full]), int(table[s.share_prefix_with, shared_full]),
                           s.context_len % b))
        # unused entries: valid memory holding unrelated noise
        for k in range(need[i], max_blocks):
            table[i, k] = spare_ids[(i + k) % len(spare_ids)]
    total_q = sum(s.query_len for s in specs)
    tensor_seed = int(rng.integers(0, 2 ** 31))
    q = noise_bf16([tensor_seed, 0], (total_q, num_q_heads, head_dim))
    k_cache = noise_bf16([tensor_seed, 1], (num_blocks, num_kv_heads, b, head_dim))
    v_cache = noise_bf16([tensor_seed, 2], (num_blocks, num_kv_heads, b, head_dim))
    for dst, src, rows in copies:
        k_cache[dst, :, :rows, :] = k_cache[src, :, :rows, :]
        v_cache[dst, :, :rows, :] = v_cache[src, :, :rows, :]
    seqs, tree_masks = specs_to_seqs(specs)
    parents = [s.parents for s in specs]
    return Batch(name=name, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, head_dim=head_dim,
                 block_size=b, scale=float(scale if scale is not None else 1.0 / np.sqrt(head_dim)),
                 seqs=seqs, q=q, k_cache=k_cache, v_cache=v_cache, block_table=table,
                 tree_masks=tree_masks, parents=parents)


def _log_uniform(rng, lo, hi, n):
    return [int(np.floor(np.exp(rng.uniform(np.log(lo), np.log(hi))))) for _ in range(n)]


def config_specs(index, rng):
    """(name, Hq, Hkv, [SeqSpec]) of configuration ``index`` in 1..5; lengths drawn from rng."""
    if index == 1:
        tree = random_tree(rng, 4)
        specs = [SeqSpec(128, 0, PREFILL), SeqSpec(1, 256, DECODE), SeqSpec(1, 256, DECODE),
                 SeqSpec(4, 192, VERIFY, MASK_TREE, tree)]
        return "tiny_hybrid", 8, 2, specs
    if index == 2:
        ctx = rng.integers(1024, 8193, size=64)
        specs = [SeqSpec(512, 2048, PREFILL)] + [SeqSpec(1, int(c), DECODE) for c in ctx]
        return "splitfuse_llama3_8b", 32, 8, specs
    if index == 3:
        ctx = rng.integers(4096, 16385, size=4)
        specs = []
        for k in range(4):
            specs.append(SeqSpec(1024, int(ctx[k]), PREFILL))
            specs.append(SeqSpec(1024, int(ctx[k]), PREFILL, share_prefix_with=2 * k))
        return "apc_prefill", 32, 8, specs
    if index == 4:
        lens = rng.integers(1, 9, size=128)
        ctx = rng.integers(512, 4097, size=128)
        specs = [SeqSpec(int(l), int(c), VERIFY, MASK_TREE, random_tree(rng, int(l)))
                 for l, c in zip(lens, ctx)]
        return "verify_heavy", 32, 8, specs
    if index == 5:
        vctx = _log_uniform(rng, 256, 32768, 16)
        dctx = _log_uniform(rng, 256, 32768, 256)
        specs = [SeqSpec(2048, 32768, PREFILL), SeqSpec(2048, 32768, PREFILL)]
        specs += [SeqSpec(4, c, VERIFY, MASK_CAUSAL, chain_tree(4)) for c in vctx]
        specs += [SeqSpec(1, c, DECODE) for c in dctx]
        return "long_mixed_qwen2_72b", 64, 8, specs
    raise ValueError("config index must be 1..5")


def specs_to_seqs(specs):
    """Descriptor tuples (query_len, context_len, kind, mask_kind, mask_word_offset) and the mask words."""
    seqs, words, off = [], [], 0
    for s in specs:
        if s.mask_kind == MASK_TREE:
            wds = pack_tree_mask(s.parents)
            seqs.append((s.query_len, s.context_len, s.kind, MASK_TREE, off))
            words.append(wds)
            off += len(wds)
        else:
            seqs.append((s.query_len, s.context_len, s.kind, MASK_CAUSAL, 0))
    tree_masks = np.concatenate(words) if words else np.zeros(1, dtype=np.uint32)
    return seqs, tree_masks


def make_config_descs(index):
    """Only the descriptors of configuration ``index`` (same lengths and trees as make_config)."""
    rng = np.random.default_rng(BASE_SEED + index)
    name, hq, hkv, specs = config_specs(index, rng)
    seqs, tree_masks = specs_to_seqs(specs)
    max_blocks = max(-(-(s.context_len + s.query_len) // 128) for s in specs)
    return name, hq, hkv, seqs, tree_masks, max_blocks


def make_config(index):
    rng = np.random.default_rng(BASE_SEED + index)
    name, hq, hkv, specs = config_specs(index, rng)
    return build_batch(name, specs, hq, hkv, rng)


def make_config_subset(index, kinds):
    """Configuration ``index`` with the same drawn lengths and trees, restricted to the sequences whose
    kind is in ``kinds`` (to time the prefill part and the decode / verify part of a mixed batch apart)."""
    rng = np.random.default_rng(BASE_SEED + index)
    name, hq, hkv, specs = config_specs(index, rng)
    keep = [i for i, s in enumerate(specs) if s.kind in kinds]
    remap = {old: new for new, old in enumerate(keep)}
    sub = []
    for i in keep:
        s = specs[i]
        share = remap.get(s.share_prefix_with) if s.share_prefix_with is not None else None
        sub.append(SeqSpec(s.query_len, s.context_len, s.kind, s.mask_kind, s.parents, share))
    return build_batch(name + "_subset", sub, hq, hkv, rng)


def make_custom(specs, num_q_heads, num_kv_heads, seed, head_dim=128, block_size=128, name="custom",
                scale=None):
    return build_batch(name, specs, num_q_heads, num_kv_heads, np.random.default_rng(seed),
                       head_dim=head_dim, block_size=block_size, scale=scale)
