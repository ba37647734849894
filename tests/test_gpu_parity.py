"""HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs.

Tolerance (bf16 inputs and outputs, fp32 accumulation, P rounded to bf16 before PV):
max-abs <= 2e-2 and mean-abs <= 2e-3 against the fp64 oracle.
"""
import numpy as np
import pytest

from oracle import attention as A
from paper_2412_18106_amd import workloads as W

import parity_util as PU

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
P, D_, V = W.PREFILL, W.DECODE, W.VERIFY


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2412_18106_amd import runner
    return runner


def oracle(b, **kw):
    return A.attention_oracle(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks,
                              num_q_heads=b.num_q_heads, num_kv_heads=b.num_kv_heads,
                              block_size=b.block_size, scale=b.scale, **kw)


def hip(gpu, b, **cfg):
    db = gpu.DeviceBatch(b, **cfg)
    try:
        return db.run_numpy()
    finally:
        db.close()


def check(got, ref, what=""):
    assert not np.isnan(got).any(), f"{what}: NaN in output (row never written?)"
    err = np.abs(got.astype(np.float64) - ref)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, f"{what}: max {err.max():.3e} mean {err.mean():.3e}"


# ---- the five configurations -------------------------------------------------------------

@pytest.mark.parametrize("index", [1, 2, 4])
def test_config_full_compare(gpu, index):
    b = W.make_config(index)
    check(hip(gpu, b), oracle(b), f"config {index}")


# Configurations 3 and 5 in full: every (token, head, d) element against the oracle, per sequence and overall.
# The batch is generated and run once per module; the oracle passes are split into several tests so that each
# finishes well inside a minute on the host cores.

class _BigConfig:
    def __init__(self, gpu, index):
        self.b = W.make_config(index)
        self.got = hip(gpu, self.b)
        self.abs_sum, self.count, self.worst = 0.0, 0, 0.0
        self.done = set()

    def compare(self, seq_indices, what):
        ref = PU.oracle_sequences(self.b, seq_indices)
        t, n, w = PU.check_sequences(self.got, ref, self.b, seq_indices, what)
        self.abs_sum += t
        self.count += n
        self.worst = max(self.worst, w)
        self.done.update(seq_indices)


@pytest.fixture(scope="module")
def config3(gpu):
    return _BigConfig(gpu, 3)


@pytest.fixture(scope="module")
def config5(gpu):
    return _BigConfig(gpu, 5)


@pytest.mark.parametrize("pair", range(4))
def test_config3_apc_every_row(config3, pair):
    """Each pair (2k, 2k + 1) shares its cached prefix blocks; all 1024 x 32 rows of both against the oracle."""
    b = config3.b
    c = b.seqs[2 * pair][1]
    assert (b.block_table[2 * pair, : c // 128] == b.block_table[2 * pair + 1, : c // 128]).all()
    config3.compare([2 * pair, 2 * pair + 1], "config 3")
    t0 = 2048 * pair       # each sequence of a pair has its own queries: the outputs differ
    assert np.abs(config3.got[t0:t0 + 1024] - config3.got[t0 + 1024:t0 + 2048]).max() > 1e-3


def test_config3_apc_overall(config3):
    missing = sorted(set(range(8)) - config3.done)       # when this test is run on its own
    if missing:
        config3.compare(missing, "config 3")
    assert config3.count == config3.got.size
    assert config3.worst <= MAX_ABS and config3.abs_sum / config3.count <= MEAN_ABS


@pytest.mark.parametrize("part", ["decode_and_verify", "prefill_0", "prefill_1"])
def test_config5_long_mixed_every_row(config5, part):
    """All 272 decode / verify sequences, then each 2048-token prefill on 32768 cached tokens (64 heads), row by row."""
    b = config5.b
    if part == "decode_and_verify":
        idx = [i for i, s in enumerate(b.seqs) if s[2] != P]
    else:
        idx = [[i for i, s in enumerate(b.seqs) if s[2] == P][int(part[-1])]]
    config5.compare(idx, f"config 5 {part}")


def test_config5_long_mixed_overall(config5):
    missing = sorted(set(range(len(config5.b.seqs))) - config5.done)
    if missing:
        config5.compare(missing, "config 5")
    assert config5.count == config5.got.size
    assert config5.worst <= MAX_ABS and config5.abs_sum / config5.count <= MEAN_ABS


# ---- plan parameters must not change the numbers beyond tolerance --------------------------

@pytest.mark.parametrize("cfg", [
    dict(prefill_heads_per_unit=1, prefill_tile_tokens=128),
    dict(prefill_heads_per_unit=2, prefill_tile_tokens=100, verify_tile_tokens=3),
    dict(split_kv_blocks=1, num_workers=7),
    dict(split_kv_blocks=0, num_workers=1, cost_row_floor=1),
    dict(split_kv_blocks=2, num_workers=512, verify_tile_tokens=1),
    dict(assign_policy=2),
    dict(assign_policy=2, split_kv_blocks=1, num_workers=5),
])
def test_plan_parameter_variants(gpu, cfg):
    rng = np.random.default_rng(11)
    specs = [W.SeqSpec(300, 77, P), W.SeqSpec(1, 700, D_), W.SeqSpec(7, 515, V, W.MASK_TREE, W.random_tree(rng, 7)),
             W.SeqSpec(5, 130, V), W.SeqSpec(1, 0, D_), W.SeqSpec(130, 0, P)]
    b = W.make_custom(specs, 8, 2, 123)
    check(hip(gpu, b, **cfg), oracle(b), str(cfg))


@pytest.mark.parametrize("seed", range(12))
def test_random_mixed_batches(gpu, seed):
    """Random small batches of all kinds and head shapes, every output element compared."""
    rng = np.random.default_rng(7000 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 8]))
    specs = []
    for _ in range(int(rng.integers(3, 10))):
        kind = int(rng.integers(0, 4))
        c = int(rng.integers(0, 900))
        if kind == 0:
            specs.append(W.SeqSpec(int(rng.integers(1, 400)), c, P))
        elif kind == 1:
            specs.append(W.SeqSpec(1, c, D_))
        elif kind == 2:
            n = int(rng.integers(1, 20))
            specs.append(W.SeqSpec(n, c, V, W.MASK_TREE, W.random_tree(rng, n)))
        else:
            specs.append(W.SeqSpec(int(rng.integers(1, 20)), c, V))
    b = W.make_custom(specs, hkv * group, hkv, 8000 + seed)
    cfg = dict(split_kv_blocks=int(rng.choice([-1, 0, 1, 2, 16])), num_workers=int(rng.choice([3, 64, 256])),
               assign_policy=int(rng.integers(0, 3)))
    check(hip(gpu, b, **cfg), oracle(b), f"seed {seed} {cfg}")


# ---- edge cases -----------------------------------------------------------------------------

@pytest.mark.parametrize("c", [0, 1, 127, 128, 129, 255])
def test_context_alignment_and_ragged_tiles(gpu, c):
    specs = [W.SeqSpec(67, c, P), W.SeqSpec(1, c, D_), W.SeqSpec(3, c, V), W.SeqSpec(129, c, P)]
    b = W.make_custom(specs, 4, 1, 200 + c)
    check(hip(gpu, b), oracle(b), f"c={c}")


@pytest.mark.parametrize("scale", [0.15, 0.2, 1.0])
def test_wide_units_on_both_sides_of_the_scale_fold(gpu, scale):
    """Wide units fold c = scale * log2(e) into Q up to c = 0.25 and keep it in fp32 above: 0.216 | 0.289, 1.44."""
    rng = np.random.default_rng(9)
    specs = [W.SeqSpec(200, 300, P), W.SeqSpec(70, 0, P), W.SeqSpec(40, 130, V, W.MASK_TREE, W.random_tree(rng, 40))]
    b = W.make_custom(specs, 8, 2, 77, scale=scale)
    check(hip(gpu, b, verify_tile_tokens=40), oracle(b), f"scale {scale}")


def test_wide_rows_that_meet_their_first_key_late_and_references_that_jump(gpu):
    """Exact softmax prefix of the wide path: a forest verify whose later trees see nothing of the first 32
    tree positions (no reference after the first step when the context is empty), and scores that outgrow
    the running reference by far more than the lazy margin in later blocks."""
    parents = [-1] + list(range(0, 39)) + [-1] + list(range(40, 59))     # two chains: 40 and 20 tokens
    b = W.make_custom([W.SeqSpec(60, 0, V, W.MASK_TREE, parents), W.SeqSpec(60, 5, V, W.MASK_TREE, parents)], 4, 1, 31)
    check(hip(gpu, b, verify_tile_tokens=64), oracle(b), "forest")       # 60 tokens x 4 heads: one wide unit each
    b = W.make_custom([W.SeqSpec(96, 700, P)], 4, 1, 32)
    blocks = b.block_table[0]
    k = W.bf16_bits_to_f32(b.k_cache)
    for n, pos in enumerate(range(100, 700, 100)):          # keys of growing magnitude deeper into the context
        k[blocks[pos // 128], :, pos % 128] *= 3.0 + 2.0 * n
    b.k_cache[:] = W.f32_to_bf16_bits(k)
    check(hip(gpu, b), oracle(b), "growing keys")


@pytest.mark.parametrize("jump", [20.0, 45.0, 90.0, 300.0])
def test_wide_scores_far_above_the_first_reference(gpu, jump):
    """A wide unit keeps the reference of a row's first step and is checked for overflow once, at its end
    (row sums below 2^64), then repeated with exact references if need be.  Keys deep in the context are
    scaled so that some scores lie about `jump` log2 units above everything seen before: 20 and 45 stay in the
    optimistic pass (probabilities up to 2^45), 90 and 300 leave it (finite beyond 2^64, and infinite)."""
    # scale 0.2: above the fold threshold, so the scores are exact products in fp32 (folding the scale into a
    # bf16 Q perturbs a score of hundreds of log2 units by more than one unit, which is not what is tested here)
    b = W.make_custom([W.SeqSpec(96, 900, P), W.SeqSpec(130, 400, P)], 4, 1, 33, scale=0.2)
    k = W.bf16_bits_to_f32(b.k_cache).astype(np.float64)
    qf = W.bf16_bits_to_f32(b.q).astype(np.float64)
    c = b.scale * np.log2(np.e)
    for seq, (t0, pos_list) in enumerate(((0, (300, 610, 899)), (96, (129, 395)))):
        blocks = b.block_table[seq]
        for n, pos in enumerate(pos_list):
            # make key `pos` point along one query row of head n, long enough for the wanted score
            qrow = qf[t0 + 5 + 20 * n, n]
            want = jump * (1.0 + 0.5 * n) / c                         # raw q.k
            k[blocks[pos // 128], 0, pos % 128] = qrow * (want / np.dot(qrow, qrow))
    b.k_cache[:] = W.f32_to_bf16_bits(k.astype(np.float32))
    check(hip(gpu, b), oracle(b), f"jump {jump}")


def test_head_shapes_mha_and_wide_groups(gpu):
    rng = np.random.default_rng(5)
    for hq, hkv in ((2, 2), (16, 1), (64, 8)):
        specs = [W.SeqSpec(70, 200, P), W.SeqSpec(1, 333, D_), W.SeqSpec(6, 250, V, W.MASK_TREE, W.random_tree(rng, 6))]
        b = W.make_custom(specs, hq, hkv, 300 + hq)
        check(hip(gpu, b), oracle(b), f"{hq}/{hkv}")


@pytest.mark.parametrize("hq,hkv", [(64, 1), (128, 2), (256, 1)])
def test_groups_up_to_the_largest_the_planner_accepts(gpu, hq, hkv):
    """64, 64 and 256 query heads per KV head: a single decode token is a wide unit of G rows, 256 rows at the limit
    (one token fills a unit), and a prefill tile holds 256 / G tokens."""
    rng = np.random.default_rng(50 + hq)
    specs = [W.SeqSpec(5, 200, P), W.SeqSpec(1, 333, D_), W.SeqSpec(1, 0, D_),
             W.SeqSpec(3, 250, V, W.MASK_TREE, W.random_tree(rng, 3)), W.SeqSpec(2, 127, V)]
    b = W.make_custom(specs, hq, hkv, 700 + hq)
    check(hip(gpu, b), oracle(b), f"{hq}/{hkv}")
    check(hip(gpu, b, split_kv_blocks=1), oracle(b), f"{hq}/{hkv} split")


def test_thousands_of_short_sequences(gpu):
    """2500 sequences (decodes, short chain and tree verifies, a few short prompts) on contexts of 0 .. 300 tokens:
    about twenty thousand units, most of them a single step long, all on the shared list."""
    rng = np.random.default_rng(77)
    specs = []
    for i in range(2500):
        kind = rng.integers(0, 10)
        ctx = int(rng.integers(0, 301))
        if kind == 0:
            specs.append(W.SeqSpec(int(rng.integers(1, 40)), ctx, P))
        elif kind == 1:
            n = int(rng.integers(2, 9))
            specs.append(W.SeqSpec(n, ctx, V, W.MASK_TREE, W.random_tree(rng, n)))
        elif kind == 2:
            specs.append(W.SeqSpec(int(rng.integers(2, 6)), ctx, V))
        else:
            specs.append(W.SeqSpec(1, ctx, D_))
    b = W.make_custom(specs, 32, 8, 900)
    check(hip(gpu, b), oracle(b), "short sequences")


def test_contexts_beyond_a_hundred_thousand_tokens(gpu):
    """A decode on 131072 cached tokens (1025 tiles, cut into pieces), a tree verify on 100000 and a short prefill
    chunk on 120000: block-table rows of more than a thousand entries, units of hundreds of K/V tiles."""
    rng = np.random.default_rng(9)
    specs = [W.SeqSpec(1, 131072, D_), W.SeqSpec(9, 100000, V, W.MASK_TREE, W.random_tree(rng, 9)),
             W.SeqSpec(70, 120000, P), W.SeqSpec(1, 17, D_)]
    b = W.make_custom(specs, 8, 2, 1234)
    got = hip(gpu, b)
    ref = PU.oracle_sequences(b)
    total, count, worst = PU.check_sequences(got, ref, b, range(len(specs)), "long contexts")
    assert total / count <= MEAN_ABS and worst <= MAX_ABS


def test_long_tree_verify_two_mask_words_and_many_rows(gpu):
    rng = np.random.default_rng(6)
    specs = [W.SeqSpec(40, 300, V, W.MASK_TREE, W.random_tree(rng, 40)),      # 40 x 4 = 160 rows, 2 words per row
             W.SeqSpec(31, 1000, V, W.MASK_TREE, W.random_tree(rng, 31)),
             W.SeqSpec(64, 90, V, W.MASK_TREE, W.random_tree(rng, 64)),
             W.SeqSpec(33, 129, V, W.MASK_TREE, W.chain_tree(33))]
    b = W.make_custom(specs, 8, 2, 400)
    check(hip(gpu, b), oracle(b))
    check(hip(gpu, b, verify_tile_tokens=16, split_kv_blocks=1), oracle(b))


def test_chain_tree_equals_causal_on_gpu(gpu):
    b1 = W.make_custom([W.SeqSpec(8, 777, V, W.MASK_TREE, W.chain_tree(8))], 8, 2, 500)
    b2 = W.make_custom([W.SeqSpec(8, 777, V, W.MASK_CAUSAL)], 8, 2, 500)
    assert np.array_equal(b1.q, b2.q) and np.array_equal(b1.k_cache, b2.k_cache)
    assert np.array_equal(hip(gpu, b1), hip(gpu, b2))


def _needle(b, seq, row, head, key_pos, value=2.0, alpha=150.0):
    t0 = sum(s[0] for s in b.seqs[:seq])
    g = b.num_q_heads // b.num_kv_heads
    qv = W.bf16_bits_to_f32(b.q[t0 + row, head]).astype(np.float64)
    blk = b.block_table[seq, key_pos // b.block_size]
    b.k_cache[blk, head // g, key_pos % b.block_size] = W.f32_to_bf16_bits((alpha * qv / np.linalg.norm(qv)).astype(np.float32))
    b.v_cache[blk, head // g, key_pos % b.block_size] = W.f32_to_bf16_bits(np.full(b.head_dim, value, dtype=np.float32))


@pytest.mark.parametrize("c", [0, 1, 126, 127, 128, 255, 256])
def test_needles_at_mask_boundaries(gpu, c):
    """A dominant key just inside / just outside the visible range must flip / not move the row."""
    q = 70
    for row in (0, 1, 63, 64, 69):
        b = W.make_custom([W.SeqSpec(q, c, P)], 4, 2, 600 + c, scale=1.0)
        base = hip(gpu, b)
        _needle(b, 0, row, 3, c + row)                 # last visible key of (row, head 3)
        hit = hip(gpu, b)
        assert np.abs(hit[row, 3] - 2.0).max() < 2e-2, (c, row)
        if row > 0:
            # a row's arithmetic does not depend on the keys only its neighbours see
            assert np.array_equal(hit[row - 1, 3], base[row - 1, 3])
        assert np.array_equal(hit[:, :2], base[:, :2])   # other KV head untouched
        check(hit, oracle(b), f"needle c={c} row={row}")
    # first invisible position after the last row, and a block-tail slot, when they exist in the block
    b = W.make_custom([W.SeqSpec(q, c, P)], 4, 2, 600 + c, scale=1.0)
    base = hip(gpu, b)
    n = c + q
    if n % 128:
        _needle(b, 0, q - 1, 3, n)
        assert np.array_equal(hip(gpu, b), base)


def test_needle_decode_split_boundary_and_spare_blocks(gpu):
    c = 128 * 5 + 17
    b = W.make_custom([W.SeqSpec(1, c, D_)], 8, 2, 700, scale=1.0)
    base = hip(gpu, b, split_kv_blocks=2)
    # garbage everywhere nobody may look: tail of the last block and all spare blocks
    used = set(b.block_table[0, : (c + 1 + 127) // 128].tolist())
    big = W.f32_to_bf16_bits(np.float32(1.0e4))
    for blk in range(b.k_cache.shape[0]):
        if blk not in used:
            b.k_cache[blk] = big
            b.v_cache[blk] = big
    last = b.block_table[0, (c + 1 - 1) // 128]
    b.k_cache[last, :, (c + 1) % 128:] = big
    b.v_cache[last, :, (c + 1) % 128:] = big
    assert np.array_equal(hip(gpu, b, split_kv_blocks=2), base)
    for pos in (0, 255, 256, 257, c):                  # both sides of a split boundary, and the own token
        bb = W.make_custom([W.SeqSpec(1, c, D_)], 8, 2, 700, scale=1.0)
        _needle(bb, 0, 0, 5, pos)
        hit = hip(gpu, bb, split_kv_blocks=2)
        assert np.abs(hit[0, 5] - 2.0).max() < 2e-2, pos
        check(hit, oracle(bb), f"pos {pos}")


@pytest.mark.parametrize("bs", [128, 16])
def test_nan_and_inf_bit_patterns_in_slots_nobody_may_see(gpu, bs):
    """A cache that was never initialised may hold any bit pattern behind a sequence's last token and in blocks no
    sequence owns: NaN and infinities there must not reach the output (a probability of zero does not cancel
    them: the kernel clears such V rows in LDS and overwrites such scores).  Every unit shape: wide prefill tiles,
    a wide tree, a K/V-split decode, narrow verifies; contexts that end inside a 32-key step and right at one."""
    tree40 = W.random_tree(np.random.default_rng(1), 40)
    tree5 = W.random_tree(np.random.default_rng(2), 5)
    specs = [W.SeqSpec(150, 333, P), W.SeqSpec(1, 700, D_), W.SeqSpec(40, 201, V, W.MASK_TREE, tree40),
             W.SeqSpec(5, 90, V, W.MASK_TREE, tree5), W.SeqSpec(3, 125, V), W.SeqSpec(1, 31, D_), W.SeqSpec(1, 0, D_),
             W.SeqSpec(64, 64, P), W.SeqSpec(70, 1, P)]
    b = W.make_custom(specs, 8, 2, 1234, block_size=bs)
    cfg = dict(split_kv_blocks=2)
    base = hip(gpu, b, **cfg)
    check(base, oracle(b), "finite garbage")
    used = set()
    patterns = np.array([0x7FC0, 0x7F80, 0xFF80, 0xFFC1], dtype=np.uint16)      # NaN, +Inf, -Inf, another NaN
    for i, (q, c, *_rest) in enumerate(b.seqs):
        n = c + q
        nblk = -(-n // bs)
        used.update(b.block_table[i, :nblk].tolist())
        if n % bs:
            last = b.block_table[i, nblk - 1]
            fill = patterns[np.arange((bs - n % bs) * 128) % 4].reshape(bs - n % bs, 128)
            b.k_cache[last, :, n % bs:] = fill
            b.v_cache[last, :, n % bs:] = fill[::-1]
    for blk in range(b.k_cache.shape[0]):
        if blk not in used:
            b.k_cache[blk] = patterns[blk % 4]
            b.v_cache[blk] = patterns[(blk + 1) % 4]
    got = hip(gpu, b, **cfg)
    assert not np.isnan(got).any() and np.array_equal(got, base)


def test_needle_tree_non_ancestor(gpu):
    parents = [-1, 0, 0, 2, 1]
    b = W.make_custom([W.SeqSpec(5, 300, V, W.MASK_TREE, parents)], 4, 2, 800, scale=1.0)
    base = hip(gpu, b)
    _needle(b, 0, 3, 0, 300 + 1)                       # node 1 is not an ancestor of node 3
    hit = hip(gpu, b)
    assert np.array_equal(hit[3, 0], base[3, 0])
    assert np.abs(hit[4, 0] - 2.0).max() < 0.7          # node 4 descends from node 1: it sees the needle
    _needle(b, 0, 3, 1, 300 + 2)                       # node 2 is an ancestor of node 3
    assert np.abs(hip(gpu, b)[3, 1] - 2.0).max() < 2e-2


def test_row_without_visible_key_is_zero(gpu):
    b = W.make_custom([W.SeqSpec(3, 0, V, W.MASK_TREE, [-1, 0, 1]), W.SeqSpec(1, 5, D_)], 4, 2, 900)
    b.tree_masks[:] = 0
    b.tree_masks[2] = 0b101
    got = hip(gpu, b)
    assert np.array_equal(got[:2], np.zeros_like(got[:2]))
    check(got, oracle(b))


def test_strided_q_and_out_views_of_a_fused_qkv_buffer(gpu):
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_custom([W.SeqSpec(50, 100, P), W.SeqSpec(1, 300, D_)], 8, 2, 1000)
    db = gpu.DeviceBatch(b)
    try:
        fused = torch.zeros(b.total_q, 8 + 2 * 2, 128, dtype=torch.bfloat16, device="cuda")
        fused[:, :8] = db.q
        out_wide = torch.full((b.total_q, 10, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
        X.xy_attn_run(db.plan, fused[:, :8], db.k_cache, db.v_cache, db.block_table, db.tree_masks,
                      out_wide[:, 1:9], db.workspace, b.scale)
        torch.cuda.synchronize()
        got = out_wide[:, 1:9].float().cpu().numpy()
        assert torch.isnan(out_wide[:, 0]).all() and torch.isnan(out_wide[:, 9]).all()
        check(got, oracle(b))
    finally:
        db.close()


@pytest.mark.parametrize("scale", [None, 1.0])
def test_k_v_caches_whose_rows_are_not_back_to_back(gpu, scale):
    """The cache strides are arguments: K and V as views with a token stride of 256 elements (rows padded,
    the other half filled with huge values) and a padded block stride.  The wide path then takes its
    general K/V loads instead of the ones for contiguous rows; the narrow path and the append kernel use the
    strides as well.  Both sides of the scale fold."""
    import torch
    from paper_2412_18106_amd import binding as X
    tree = W.random_tree(np.random.default_rng(3), 12)
    specs = [W.SeqSpec(200, 700, P), W.SeqSpec(1, 900, D_), W.SeqSpec(12, 333, V, W.MASK_TREE, tree),
             W.SeqSpec(64, 64, P), W.SeqSpec(1, 127, D_), W.SeqSpec(40, 1500, V)]
    kw = {} if scale is None else dict(scale=scale)
    b = W.make_custom(specs, 8, 2, 4321, **kw)
    db = gpu.DeviceBatch(b, verify_tile_tokens=16)          # 64-row verify units: wide, K/V-split
    try:
        nb, hkv, bs, d = db.k_cache.shape
        bufs = []
        for src in (db.k_cache, db.v_cache):
            big = torch.full((nb + 1, hkv, bs, 2 * d), 3.0e4, dtype=torch.bfloat16, device="cuda")
            view = big[:nb, :, :, :d]
            view.copy_(src)
            bufs.append(view)
        assert bufs[0].stride(2) == 2 * d and bufs[0].stride() == bufs[1].stride()
        X.xy_attn_run(db.plan, db.q, bufs[0], bufs[1], db.block_table, db.tree_masks, db.out, db.workspace, b.scale)
        torch.cuda.synchronize()
        check(db.out.float().cpu().numpy(), oracle(b), f"padded rows, scale {scale}")
    finally:
        db.close()


def test_deterministic_and_empty_batch_and_run_errors(gpu):
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_config(1)
    db = gpu.DeviceBatch(b, split_kv_blocks=1)
    try:
        a1 = db.run_numpy()
        a2 = db.run_numpy()
        assert np.array_equal(a1, a2)
        with pytest.raises(X.XyError) as e:
            X.xy_attn_run(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out,
                          db.workspace[:4], b.scale)
        assert e.value.status == X.XY_ERR_WORKSPACE
        with pytest.raises(X.XyError) as e:
            X.xy_attn_run(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out,
                          db.workspace, -1.0)
        assert e.value.status == X.XY_ERR_ARG
        with pytest.raises(X.XyError) as e:
            X.xy_attn_run(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, None, db.out,
                          db.workspace, b.scale)
        assert e.value.status == X.XY_ERR_ARG
    finally:
        db.close()
    cfg = X.xy_attn_default_config(8, 2, 4)
    plan = X.xy_attn_plan_create(cfg, [])
    assert X._lib.xy_attn_run(plan, None, 0, 0, None, None, 0, 0, 0, None, None, None, 0, 0, None, 0, 1.0, None) == 0
    X.xy_attn_plan_destroy(plan)
    torch.cuda.synchronize()


def test_one_plan_object_rebuilt_batch_after_batch(gpu):
    """A serving loop keeps one plan object: every batch is planned in place (xy_attn_plan_rebuild) and its tables
    reach the GPU with one asynchronous copy, either asked for or done by the run itself.  Each result is, bit for
    bit, what a fresh plan object gives; the run that allocates nothing refuses tables that are not current."""
    import torch
    from paper_2412_18106_amd import binding as X
    rng = np.random.default_rng(21)
    plan = X.xy_attn_plan_create(X.xy_attn_default_config(8, 2, 1), [])
    try:
        for step in range(6):
            specs = []
            for _ in range(int(rng.integers(1, 12)) if step != 3 else 40):          # step 3 outgrows the arena
                kind = int(rng.integers(0, 3))
                c = int(rng.integers(0, 3000))
                if kind == 0:
                    specs.append(W.SeqSpec(int(rng.integers(1, 300)), c, P))
                elif kind == 1:
                    specs.append(W.SeqSpec(1, c, D_))
                else:
                    n = int(rng.integers(1, 12))
                    specs.append(W.SeqSpec(n, c, V, W.MASK_TREE, W.random_tree(rng, n)))
            b = W.make_custom(specs, 8, 2, 5000 + step)
            db = gpu.DeviceBatch(b)
            try:
                want = db.run_numpy()                                  # a plan object of its own
                X.xy_attn_plan_rebuild(plan, db.cfg, b.seqs)
                ws = torch.empty(max(X.xy_attn_plan_workspace_bytes(plan), 16) // 4, dtype=torch.float32, device="cuda")
                if step % 2 == 0:
                    with pytest.raises(X.XyError) as e:                # rebuilt, not copied yet
                        X.xy_attn_run_static(plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks,
                                             db.out, b.scale)
                    assert e.value.status == X.XY_ERR_ARG
                    X.xy_attn_plan_upload_async(plan)
                db.out.fill_(float("nan"))
                X.xy_attn_run(plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, ws, b.scale)
                torch.cuda.synchronize()
                assert np.array_equal(db.out.float().cpu().numpy(), want), f"step {step}"
                db.out.fill_(float("nan"))
                X.xy_attn_run_static(plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out, b.scale)
                torch.cuda.synchronize()
                assert np.array_equal(db.out.float().cpu().numpy(), want), f"step {step}, static workspace"
            finally:
                db.close()
    finally:
        X.xy_attn_plan_destroy(plan)


@pytest.mark.parametrize("index", [2, 4])
def test_nothing_outside_the_workspace_and_the_output_is_written(gpu, index):
    """Canaries in front of and behind the K/V-split workspace, and around the output rows, survive a run; the
    inputs (Q, both caches, block table, mask words) are bit for bit what they were."""
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_config(index)
    db = gpu.DeviceBatch(b)
    try:
        want = db.run_numpy()
        need = X.xy_attn_plan_workspace_bytes(db.plan)
        assert need > 0 and need % 4 == 0
        guard = 4096                                         # bytes on either side, keeps the 16-byte alignment
        big = torch.full(((2 * guard + need) // 4,), -7, dtype=torch.int32, device="cuda")
        ws = big[guard // 4: (guard + need) // 4].view(torch.float32)
        out_big = torch.full((b.total_q + 2, b.num_q_heads, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
        out = out_big[1:-1]
        before = [t.clone() for t in (db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks)]
        for _ in range(3):
            X.xy_attn_run(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, out, ws, b.scale)
        torch.cuda.synchronize()
        assert (big[: guard // 4] == -7).all() and (big[(guard + need) // 4:] == -7).all()
        assert (ws.view(torch.int32) != -7).any()            # the workspace itself was used
        assert torch.isnan(out_big[0]).all() and torch.isnan(out_big[-1]).all()
        assert np.array_equal(out.float().cpu().numpy(), want)
        for t, t0 in zip((db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks), before):
            assert torch.equal(t.view(torch.int16) if t.dtype == torch.bfloat16 else t,
                               t0.view(torch.int16) if t0.dtype == torch.bfloat16 else t0)
    finally:
        db.close()


def test_two_plans_on_two_streams_do_not_disturb_each_other(gpu):
    """A plan with a shared list keeps its cursor and counters in its own device memory, a workspace belongs to one
    run at a time: two plans, each with its own workspace, may run at the same time on two streams."""
    import torch
    rng = np.random.default_rng(99)
    batches = []
    for n in range(2):
        specs = [W.SeqSpec(1, int(c), D_) for c in rng.integers(2000, 9000, size=48)]
        specs += [W.SeqSpec(300 + 50 * n, 1500, P)]
        specs += [W.SeqSpec(int(k), int(c), V, W.MASK_TREE, W.random_tree(rng, int(k)))
                  for k, c in zip(rng.integers(2, 9, size=16), rng.integers(800, 4000, size=16))]
        batches.append(W.make_custom(specs, 32, 8, 6100 + n))
    dbs = [gpu.DeviceBatch(b) for b in batches]
    try:
        from paper_2412_18106_amd import binding as X
        for db in dbs:          # both plans draw their narrow units from a shared list at run time
            units, offs, _ = X.plan_arrays(db.plan, db.cfg.num_workers)
            assert offs[-1] < len(units)
        alone = [db.run_numpy() for db in dbs]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for rep in range(5):
            for db in dbs:
                db.out.fill_(float("nan"))
            torch.cuda.synchronize()
            for _ in range(3):
                for db, st in zip(dbs, streams):
                    db.run(st)
            torch.cuda.synchronize()
            for db, want in zip(dbs, alone):
                assert np.array_equal(db.out.float().cpu().numpy(), want), f"repeat {rep}"
    finally:
        for db in dbs:
            db.close()


def test_run_can_be_captured_in_a_hip_graph_and_replayed(gpu):
    """A serving loop captures one step and replays it: the library enqueues kernels only (no allocation,
    no synchronisation, no memset) once the plan is uploaded.  Every replay is checked against the eager
    result, with eager work and synchronisations between replays."""
    import torch
    from paper_2412_18106_amd import binding as X
    b = W.make_config(1)
    db = gpu.DeviceBatch(b, split_kv_blocks=1)       # split families: unit kernel + merge kernel
    try:
        eager = db.run_numpy()
        q_alt = (db.q.float() * 0.5).to(torch.bfloat16)
        q_keep = db.q.clone()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            db.run()                                  # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            X.xy_attn_run(db.plan, db.q, db.k_cache, db.v_cache, db.block_table, db.tree_masks, db.out,
                          db.workspace, b.scale)
        for rep in range(4):
            db.out.fill_(float("nan"))
            if rep == 2:
                db.q.copy_(q_alt)                     # same buffers, new contents
            g.replay()
            torch.cuda.synchronize()
            got = db.out.float().cpu().numpy()
            if rep == 2:
                want = db.run_numpy()                 # eager run on the same contents
                db.q.copy_(q_keep)
            else:
                want = eager
            assert np.array_equal(got, want), f"replay {rep} differs from the eager run"
            _ = (db.k_cache.float().sum()).item()     # eager work and a synchronisation between replays
    finally:
        db.close()


@pytest.mark.parametrize("bs", [16, 32, 64])
def test_small_pages_mixed_batch(gpu, bs):
    """Pages of 16 / 32 / 64 tokens (section 4.1.1): a 128-key tile is gathered from several block-table
    entries; contexts straddle page and tile boundaries, the last page is partly filled, pairs share prefixes."""
    tree = W.random_tree(np.random.default_rng(bs), 9)
    specs = [W.SeqSpec(200, 300 + bs // 2, P), W.SeqSpec(1, 1000 + bs - 1, D_), W.SeqSpec(1, 127, D_), W.SeqSpec(1, 128, D_),
             W.SeqSpec(9, 500 + bs + 3, V, W.MASK_TREE, tree), W.SeqSpec(70, 0, P), W.SeqSpec(1, 2500, D_),
             W.SeqSpec(100, 3 * bs + 640, P), W.SeqSpec(100, 3 * bs + 640, P, share_prefix_with=7), W.SeqSpec(1, 0, D_)]
    b = W.make_custom(specs, 8, 2, 4000 + bs, block_size=bs)
    check(hip(gpu, b), oracle(b), f"block_size {bs}")
    check(hip(gpu, b, split_kv_blocks=2, prefill_tile_tokens=32), oracle(b), f"block_size {bs}, split")


def test_small_pages_needle_in_the_last_partial_page(gpu):
    # the last visible key sits in a partly filled 16-token page; the slots behind it hold large values
    c = 16 * 9 + 5
    b = W.make_custom([W.SeqSpec(1, c, D_)], 8, 2, 91, block_size=16)
    page, slot = b.block_table[0, c // 16], c % 16
    qrow = W.bf16_bits_to_f32(b.q[0, 0]).astype(np.float64)
    b.k_cache[page, 0, slot] = W.f32_to_bf16_bits((40.0 * qrow / np.linalg.norm(qrow)).astype(np.float32))
    b.v_cache[page, 0, slot] = W.f32_to_bf16_bits(np.full(128, 3.0, np.float32))
    b.k_cache[page, 0, slot + 1:] = W.f32_to_bf16_bits(np.float32(60.0))     # invisible: must not matter
    b.v_cache[page, 0, slot + 1:] = W.f32_to_bf16_bits(np.float32(-7.0))
    got, ref = hip(gpu, b), oracle(b)
    check(got, ref, "needle in a partial page")
    assert abs(got[0, 0].mean() - 3.0) < 0.1


@pytest.mark.parametrize("specs", [
    [W.SeqSpec(300, 2000, P)],                                              # one chunk: 40 wide families for 256 workers
    [W.SeqSpec(130, 5000, P), W.SeqSpec(1, 700, D_)],                       # with a decode that weighs little
    [W.SeqSpec(64, 1300, V, W.MASK_TREE, W.random_tree(np.random.default_rng(8), 64))],   # a 64-token tree
])
def test_wide_families_alone_are_cut_along_kv_and_merged(gpu, specs):
    """Fewer families of more than 32 rows than workers and little else to do: prefill families are cut along K/V
    as well (256-row partial results through the merge pass), tiles that end before a piece begins included."""
    from paper_2412_18106_amd import binding as X
    b = W.make_custom(specs, 8, 2, 606)
    db = gpu.DeviceBatch(b, verify_tile_tokens=64)
    try:
        units, _, merges = X.xy_attn_plan_get(db.plan)[:3]
        wide = units[units["q_count"] * units["head_count"] > 32]
        assert len(merges) > 0 and (wide["num_splits"] > 1).any()
        check(db.run_numpy(), oracle(b))
    finally:
        db.close()


def test_issue_mix_probe_runs_and_counts_cycles(gpu):
    """The measurement helper behind the instruction placement of the wide path: every mix runs, MFMAs alone take
    32 cycles each, and no mix is faster than that.  (How much slower each mix is belongs to bench.py's output.)"""
    import torch
    from paper_2412_18106_amd import binding as X
    cycles = torch.zeros(1024, dtype=torch.int64, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    iters = 200
    got = {}
    for name, code in X.XY_MIX.items():
        cycles.zero_()
        X.xy_probe_issue_mix(code, iters, cycles, sink)
        torch.cuda.synchronize()
        assert (cycles > 0).all(), name
        got[name] = float(cycles.max().item()) / iters
    assert 1000 <= got["none"] <= 1150, got
    assert all(v >= 0.98 * got["none"] for v in got.values()), got
    with pytest.raises(X.XyError):
        X.xy_probe_issue_mix(99, iters, cycles, sink)
