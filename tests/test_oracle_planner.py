"""Pins for the oracle planner: the paper's two worked examples and structural invariants."""
import os

import numpy as np
import pytest

from oracle import planner as PL

P, D_, V = 0, 1, 2
HERE = os.path.dirname(os.path.abspath(__file__))


def cfg(**kw):
    c = dict(num_q_heads=8, num_kv_heads=2, head_dim=128, block_size=128, max_blocks_per_seq=64,
             num_workers=4, prefill_tile_tokens=128, prefill_heads_per_unit=1, verify_tile_tokens=64,
             split_kv_blocks=0, cost_row_floor=1, assign_policy=0)
    c.update(kw)
    return c


def golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "planner_worked_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or ":" not in line:
                continue
            k, v = line.split(":")
            vals[k.strip()] = [int(x) for x in v.split()]
    return vals


def test_paper_example_six_times_headnum_units():
    g = golden()
    blocks = g["tiling_blocks_per_stage"]          # P, D, V, D in the paper's figure
    c = cfg(num_kv_heads=8)                        # MHA: every tiling block is headNum units
    seqs = [(blocks[0] * 128 - 5, 0, P, 0, 0), (1, 300, D_, 0, 0), (4, 200, V, 0, 0), (1, 77, D_, 0, 0)]
    units, offs, merges, ws = PL.plan_oracle(c, seqs)
    assert len(units) == g["total_units_over_headnum"][0] * c["num_q_heads"]
    per_stage = [len({(u["q_begin"]) for u in units if u["seq"] == i}) for i in range(4)]
    assert per_stage == blocks
    assert ws == 0 and len(merges) == 0


def test_paper_example_symmetric_round_robin():
    g = golden()
    w = g["cores"][0]
    c = cfg(num_q_heads=1, num_kv_heads=1, num_workers=w)
    # eight single-head decodes with strictly decreasing cost
    seqs = [(1, (20 - k) * 128 - 1, D_, 0, 0) for k in range(8)]
    units, offs, _, _ = PL.plan_oracle(c, seqs)
    worker_of_seq = {}
    for wk in range(w):
        for u in units[offs[wk]:offs[wk + 1]]:
            worker_of_seq[int(u["seq"])] = wk + 1
    assert [worker_of_seq[k] for k in range(8)] == g["core_sequence_one_based"]


def random_seqs(rng, n):
    out = []
    for _ in range(n):
        kind = int(rng.integers(0, 3))
        if kind == P:
            out.append((int(rng.integers(1, 700)), int(rng.integers(0, 5000)), P, 0, 0))
        elif kind == D_:
            out.append((1, int(rng.integers(0, 9000)), D_, 0, 0))
        else:
            out.append((int(rng.integers(1, 40)), int(rng.integers(0, 6000)), V, int(rng.integers(0, 2)), 0))
    return out


@pytest.mark.parametrize("seed", range(6))
def test_invariants(seed):
    rng = np.random.default_rng(seed)
    c = cfg(num_q_heads=8, num_kv_heads=2, num_workers=int(rng.integers(1, 40)),
            prefill_tile_tokens=int(rng.choice([32, 64, 128])), prefill_heads_per_unit=int(rng.choice([1, 2, 4])),
            verify_tile_tokens=int(rng.choice([8, 16, 64])), split_kv_blocks=int(rng.choice([0, 3, 16])),
            cost_row_floor=int(rng.choice([1, 64, 256])))
    seqs = random_seqs(rng, int(rng.integers(1, 30)))
    units, offs, merges, ws = PL.plan_oracle(c, seqs)
    b, d = c["block_size"], c["head_dim"]
    assert offs[0] == 0 and offs[-1] == len(units) and (np.diff(offs) >= 0).all()
    # every (seq, head, token) covered by exactly one family; splits partition [0, kv_block_end)
    cover = {}
    fam = {}
    for u in units:
        key = (int(u["seq"]), int(u["head_begin"]), int(u["q_begin"]))
        fam.setdefault(key, []).append(u)
    for (i, hb, qb), us in fam.items():
        ql, ctx, kind, mk, _ = seqs[i]
        us = sorted(us, key=lambda u: u["split_index"])
        u0 = us[0]
        assert [int(u["split_index"]) for u in us] == list(range(int(u0["num_splits"])))
        end = -(-(ctx + ql) // b) if mk == 1 else -(-(ctx + qb + int(u0["q_count"])) // b)
        assert us[0]["kv_block_begin"] == 0 and us[-1]["kv_block_end"] == end
        for a, nx in zip(us, us[1:]):
            assert a["kv_block_end"] == nx["kv_block_begin"] and a["kv_block_end"] > a["kv_block_begin"]
        if kind == P:
            assert len(us) == 1
        if c["split_kv_blocks"] and kind != P:
            assert all(u["kv_block_end"] - u["kv_block_begin"] <= c["split_kv_blocks"] for u in us)
        assert (u0["kind_flags"] & 3) == kind and (u0["kind_flags"] >> 2) == mk
        for h in range(hb, hb + int(u0["head_count"])):
            for t in range(qb, qb + int(u0["q_count"])):
                cover[(i, h, t)] = cover.get((i, h, t), 0) + 1
    want = {(i, h, t) for i, s in enumerate(seqs) for h in range(c["num_q_heads"]) for t in range(s[0])}
    assert set(cover) == want and set(cover.values()) == {1}
    # cost formula, and the sort order recovered from the snake assignment
    for u in units:
        rows = int(u["q_count"]) * int(u["head_count"])
        assert u["cost"] == max(rows, c["cost_row_floor"]) * (u["kv_block_end"] - u["kv_block_begin"])
    w = c["num_workers"]
    sorted_costs = []
    rounds = max(int(np.diff(offs).max()), 0)
    for r in range(rounds):
        lanes = range(w) if r % 2 == 0 else range(w - 1, -1, -1)
        for wk in lanes:
            if offs[wk] + r < offs[wk + 1]:
                sorted_costs.append(int(units[offs[wk] + r]["cost"]))
    assert sorted_costs == sorted(sorted_costs, reverse=True) and len(sorted_costs) == len(units)
    loads = [int(units[offs[k]:offs[k + 1]]["cost"].sum()) for k in range(w)]
    if len(units):
        assert max(loads) - min(loads) <= int(units["cost"].max())
    # workspace regions are disjoint, consecutive and hold rows*(D+2) floats (rounded up to 4) per split
    pos = 0
    for m in merges:
        assert m["ws_offset"] == pos
        pos += int(m["num_splits"]) * (-(-int(m["q_count"]) * int(m["head_count"]) * (d + 2) // 4) * 4)
    assert pos == ws
    for u in units:
        if u["num_splits"] == 1:
            assert u["ws_offset"] == -1
    # pure function
    again = PL.plan_oracle(c, seqs)
    assert units.tobytes() == again[0].tobytes() and (offs == again[1]).all()


@pytest.mark.parametrize("seed", range(4))
def test_least_loaded_assignment(seed):
    rng = np.random.default_rng(50 + seed)
    c = cfg(num_workers=int(rng.integers(2, 30)), assign_policy=1, split_kv_blocks=8, cost_row_floor=64)
    seqs = random_seqs(rng, 25)
    units, offs, _, _ = PL.plan_oracle(c, seqs)
    snake_units, snake_offs, _, _ = PL.plan_oracle(dict(c, assign_policy=0), seqs)
    assert sorted(units.tolist()) == sorted(snake_units.tolist())      # same units, other placement
    w = c["num_workers"]
    loads = np.array([int(units[offs[k]:offs[k + 1]]["cost"].sum()) for k in range(w)])
    snake = np.array([int(snake_units[snake_offs[k]:snake_offs[k + 1]]["cost"].sum()) for k in range(w)])
    # greedy list scheduling: every worker's load minus its last unit is at most the smallest final load
    for k in range(w):
        if offs[k + 1] > offs[k]:
            assert loads[k] - int(units[offs[k + 1] - 1]["cost"]) <= loads.min()
        assert (np.diff(units[offs[k]:offs[k + 1]]["cost"]) <= 0).all()     # assignment order = sorted order
    assert loads.sum() == snake.sum()


def test_least_loaded_tie_goes_to_lowest_index():
    c = cfg(num_q_heads=1, num_kv_heads=1, num_workers=3, assign_policy=1)
    seqs = [(1, 127, D_, 0, 0)] * 4            # four equal units
    units, offs, _, _ = PL.plan_oracle(c, seqs)
    assert np.diff(offs).tolist() == [2, 1, 1]
    assert [int(x) for x in units["seq"]] == [0, 3, 1, 2]


def test_dynamic_assignment_keeps_static_lists_for_units_of_at_most_two_tiles():
    """Policy 2 without a wide unit: a shared list only when the costs differ AND some unit visits more than two
    K/V tiles.  Decodes of one and two tiles: every unit on a worker's own list.  One of three tiles among them:
    all narrow units on the shared list behind worker_offsets[W]."""
    c = cfg(num_q_heads=4, num_kv_heads=1, num_workers=4, verify_tile_tokens=1, split_kv_blocks=0, cost_row_floor=1,
            assign_policy=2)
    short = [(1, 100, D_, 0, 0), (1, 200, D_, 0, 0), (1, 255, D_, 0, 0), (1, 5, D_, 0, 0), (1, 130, D_, 0, 0)]
    units, offs, _, _ = PL.plan_oracle(c, short)
    assert len(units) == 5 and offs[4] == 5                      # nothing behind the workers' lists
    assert np.diff(offs).tolist() == [1, 1, 1, 2]                 # least-loaded: loads 8, 8, 8 and 4 + 4
    units, offs, _, _ = PL.plan_oracle(c, short + [(1, 256, D_, 0, 0)])
    assert len(units) == 6 and offs[4] == 0                      # all six on the shared list, largest first
    assert [int(x) for x in units["seq"]] == [5, 1, 2, 4, 0, 3]


def test_empty_batch():
    units, offs, merges, ws = PL.plan_oracle(cfg(), [])
    assert len(units) == 0 and (offs == 0).all() and ws == 0


def test_cost_floor_one_is_tilesize_times_kvlen_in_blocks():
    c = cfg(num_q_heads=2, num_kv_heads=2, num_workers=1)
    units, _, _, _ = PL.plan_oracle(c, [(128, 128 * 7, P, 0, 0)])
    assert set(int(x) for x in units["cost"]) == {128 * 8}


def test_automatic_split_size_worked_examples():
    """split_kv_blocks = -1: equal narrow families are cut into the number of pieces that minimises
    (rounds of the 4 W wavefront slots) x (tiles per piece + 1), unequal ones at a size that follows a wavefront's
    share ceil(B / (4 W)) of the tiles (the share, at most 16 while small, two fifths of it beyond, at most 64);
    values worked out by hand."""
    base = dict(num_q_heads=32, num_kv_heads=8, num_workers=256, verify_tile_tokens=8, prefill_tile_tokens=64,
                prefill_heads_per_unit=4, split_kv_blocks=-1, cost_row_floor=128, assign_policy=1)
    # four 31-token causal verify segments on 16384 tokens: 4 token tiles each, every tile ends inside tile
    # 129 of 128 keys -> F = 16 x 8 = 128 families of 129 tiles for 1024 slots: 8 pieces fill the slots once
    # with 17 tiles each (cost 18; 7 pieces: 1 x 20, 9 pieces: 2 x 16) -> 4 x 4 x 8 x 8 = 1024 units
    units, _, merges, _ = PL.plan_oracle(cfg(**base), [(31, 16384, V, 0, 0)] * 4)
    assert len(units) == 1024 and set(units["num_splits"].tolist()) == {8}
    assert sorted(set((units["kv_block_end"] - units["kv_block_begin"]).tolist())) == [16, 17]
    assert len(merges) == 128
    # eight decodes on 1023 tokens: F = 64 families of 8 tiles: 8 pieces of one tile still fit the slots once
    # (512 units, cost 1 x 2; 4 pieces 1 x 3, 2 pieces 1 x 5, unsplit 1 x 9)
    units, _, _, _ = PL.plan_oracle(cfg(**base), [(1, 1023, D_, 0, 0)] * 8)
    assert len(units) == 8 * 8 * 8 and set((units["kv_block_end"] - units["kv_block_begin"]).tolist()) == {1}
    # unequal lengths: 300 decodes on 8191 and one on 127 tokens: (300 x 64 + 1) x 8 tiles / 1024 = 150.01 ->
    # share 151, two fifths of it 60 (between 16 and 64) -> 64 tiles in 2 pieces, the short one unsplit
    units, _, _, _ = PL.plan_oracle(cfg(**base), [(1, 8191, D_, 0, 0)] * 300 + [(1, 127, D_, 0, 0)])
    assert len(units) == 300 * 8 * 2 + 8
    # a tenth of them: share 16 (15.01 rounded up) -> 64 tiles in 4 pieces
    units, _, _, _ = PL.plan_oracle(cfg(**base), [(1, 8191, D_, 0, 0)] * 30 + [(1, 127, D_, 0, 0)])
    assert len(units) == 30 * 8 * 4 + 8
    # the same lengths throughout: F = 2400 families of 64 tiles; cost(k) = ceil(2400 k / 1024) x (ceil(64 / k) + 1):
    # k = 1: 3 x 65 = 195, 2: 5 x 33 = 165, 3: 8 x 23 = 184, 4: 10 x 17 = 170, 5: 12 x 14 = 168, 8: 19 x 9 = 171,
    # 16: 38 x 5 = 190 -> k = 2
    units, _, _, _ = PL.plan_oracle(cfg(**base), [(1, 8191, D_, 0, 0)] * 300)
    assert len(units) == 300 * 8 * 2 and set((units["kv_block_end"] - units["kv_block_begin"]).tolist()) == {32}
    # a verify tile of more than 32 rows is not counted among the narrow ones and is cut at 16 tiles, prefill is
    # never cut - as long as the wide families (8 per verify tile, 8 per prefill tile here) number at least W:
    # 16 such pairs of sequences give 256 wide families for 256 workers
    wide = dict(base, verify_tile_tokens=16)            # 16 tokens x 4 heads = 64 rows
    pair = [(16, 4096 - 16, V, 0, 0), (64, 8192, P, 0, 0)]
    units, _, _, _ = PL.plan_oracle(cfg(**wide), pair * 16)
    ver = units[units["seq"] == 0]
    assert len(ver) == 8 * 2 and set((ver["kv_block_end"] - ver["kv_block_begin"]).tolist()) == {16}
    assert set(units[units["seq"] == 1]["num_splits"].tolist()) == {1}
    # one such pair alone: 16 wide families for 256 workers, up to 16 pieces each but none shorter than 8 tiles:
    # the verify tile (32 tiles) in 4 pieces of 8, the prefill tile (65 tiles) in ceil(65 / 8) = 9 pieces of 7 or 8
    units, _, merges, _ = PL.plan_oracle(cfg(**wide), pair)
    ver, pre = units[units["seq"] == 0], units[units["seq"] == 1]
    assert len(ver) == 8 * 4 and set((ver["kv_block_end"] - ver["kv_block_begin"]).tolist()) == {8}
    assert len(pre) == 8 * 9 and set((pre["kv_block_end"] - pre["kv_block_begin"]).tolist()) == {7, 8}
    assert len(merges) == 16
    # a long prompt chunk alone: 512 tokens on 16384 -> 8 tiles x 8 head groups = 64 families, 4 pieces each
    units, _, _, _ = PL.plan_oracle(cfg(**base), [(512, 16384, P, 0, 0)])
    assert len(units) == 64 * 4 and set(units["num_splits"].tolist()) == {4}
    assert set((units["kv_block_end"] - units["kv_block_begin"]).tolist()) <= {32, 33, 34}
    # a fixed size still means what it meant
    fixed = dict(base, split_kv_blocks=16)
    units, _, _, _ = PL.plan_oracle(cfg(**fixed), [(31, 16384, V, 0, 0)] * 4)
    assert len(units) == 4 * 4 * 8 * 9


def test_dynamic_assignment_keeps_narrow_units_on_one_shared_sorted_list():
    rng = np.random.default_rng(5)
    seqs = random_seqs(rng, 30)
    c = cfg(num_q_heads=8, num_kv_heads=2, num_workers=6, prefill_tile_tokens=32, prefill_heads_per_unit=4,
            verify_tile_tokens=8, split_kv_blocks=4, cost_row_floor=16, assign_policy=2)
    units, offs, merges, ws = PL.plan_oracle(c, seqs)
    ref_units, ref_offs, ref_merges, ref_ws = PL.plan_oracle(dict(c, assign_policy=1), seqs)
    rows = units["q_count"] * units["head_count"]
    shared = units[offs[-1]:]
    assert offs[0] == 0 and (rows[:offs[-1]] > 32).all() and (shared["q_count"] * shared["head_count"] <= 32).all()
    assert len(shared) > 0 and offs[-1] > 0
    # the same units as the static plan, each exactly once
    key = lambda a: sorted(map(tuple, a[["seq", "head_begin", "q_begin", "split_index", "kv_block_begin",
                                         "kv_block_end", "ws_offset"]].tolist()))
    assert key(units) == key(ref_units) and ws == ref_ws and merges.tobytes() == ref_merges.tobytes()
    # shared list: cost descending, ties by (seq, head_begin, q_begin, split_index)
    order = [(-int(u["cost"]), int(u["seq"]), int(u["head_begin"]), int(u["q_begin"]), int(u["split_index"]))
             for u in shared]
    assert order == sorted(order)
    # wide units: least-loaded among themselves (summed cost per worker within one largest unit of the mean)
    loads = [int(units[offs[w]:offs[w + 1]]["cost"].sum()) for w in range(6)]
    assert max(loads) - min(loads) <= int(units[:offs[-1]]["cost"].max())


def test_dynamic_assignment_without_anything_to_even_out_is_the_least_loaded_plan():
    # decodes of one length: all narrow, all costs equal -> no shared list
    c = cfg(num_q_heads=8, num_kv_heads=2, num_workers=6, verify_tile_tokens=8, split_kv_blocks=4,
            cost_row_floor=16, assign_policy=2)
    seqs = [(1, 1000, D_, 0, 0)] * 7
    units, offs, _, _ = PL.plan_oracle(c, seqs)
    ref_units, ref_offs, _, _ = PL.plan_oracle(dict(c, assign_policy=1), seqs)
    assert offs[-1] == len(units) and units.tobytes() == ref_units.tobytes() and (offs == ref_offs).all()
    # one longer decode among them: costs differ -> everything narrow is shared
    units, offs, _, _ = PL.plan_oracle(c, seqs + [(1, 1300, D_, 0, 0)])
    assert offs[-1] == 0 and len(units) > 0
    # equal decodes next to one wide unit: shared as well, the wide unit on a worker
    units, offs, _, _ = PL.plan_oracle(dict(c, prefill_tile_tokens=32, prefill_heads_per_unit=4),
                                       seqs + [(32, 32, P, 0, 0)])
    assert offs[-1] == 2 and (units[offs[-1]:]["q_count"] * units[offs[-1]:]["head_count"] <= 32).all()


def test_chiplet_aware_placement_of_wide_units_worked_example():
    """Rule 5a by hand: W = 16 (two workers per chiplet), one KV head pair, 128-token prefill tiles of one head.
    Sequence 0: 1024 new tokens on nothing (tiles of 1..8 blocks), sequence 1: 256 tokens on 1024 (9 and 10
    blocks): groups (seq, KV head) cost 36, 36 (sequence 0, two KV heads) and 19, 19, in units of 128 rows.  Placed heaviest first on
    the least-loaded chiplet: chiplets 0, 1, 2, 3 -> heaviest 36 against a mean of 110 / 8: far more than 3 %
    above it, so the groups are dropped and the plan is the plain least-loaded one.  With eight such sequence
    pairs of equal length the 16 + 16 groups spread evenly (two heavy ones and two light ones per chiplet)
    and every group stays on the two workers of its chiplet."""
    c = cfg(num_q_heads=2, num_kv_heads=2, num_workers=16, prefill_tile_tokens=128, prefill_heads_per_unit=1,
            cost_row_floor=1, assign_policy=1)
    few = [(1024, 0, P, 0, 0), (256, 1024, P, 0, 0)]
    units, offs, _, _ = PL.plan_oracle(c, few)
    # plain least-loaded: the 16 heaviest units land on 16 different workers
    first = [int(units[offs[w]]["cost"]) for w in range(16)]
    assert sorted(first, reverse=True) == sorted([int(x) for x in np.sort(units["cost"])[::-1][:16]], reverse=True)
    many = few * 8
    units, offs, _, _ = PL.plan_oracle(c, many)
    chip_of = {}
    for w in range(16):
        for u in units[offs[w]:offs[w + 1]]:
            chip_of.setdefault((int(u["seq"]), int(u["head_begin"])), set()).add(w // 2)
    assert len(chip_of) == 32 and all(len(v) == 1 for v in chip_of.values())
    per_chip = [sum(int(units[offs[w]:offs[w + 1]]["cost"].sum()) for w in (2 * x, 2 * x + 1)) for x in range(8)]
    assert per_chip == [110 * 128] * 8            # cost = 128 rows x blocks
    # inside a chiplet the two workers are balanced by least-loaded placement
    loads = [int(units[offs[w]:offs[w + 1]]["cost"].sum()) for w in range(16)]
    assert max(loads) - min(loads) <= 10 * 128
    # W not a multiple of eight: no chiplets, nothing changes against the plain rule
    odd = dict(c, num_workers=12)
    units12, offs12, _, _ = PL.plan_oracle(odd, many)
    seen = {}
    for w in range(12):
        for u in units12[offs12[w]:offs12[w + 1]]:
            seen.setdefault((int(u["seq"]), int(u["head_begin"])), set()).add(w)
    assert any(len(v) > 2 for v in seen.values())


def test_automatic_verify_tile_worked_examples():
    """verify_tile_tokens = -1 with G = 4: narrow tiles of 8 tokens, except a segment of more than 8 tokens on at
    least 32 K/V tiles, which is one tile of up to 64 tokens."""
    c = cfg(num_q_heads=8, num_kv_heads=2, num_workers=4, verify_tile_tokens=-1, split_kv_blocks=0)
    def tiles(seq):
        units, _, _, _ = PL.plan_oracle(c, [seq])
        return sorted(set(zip(units["q_begin"].tolist(), units["q_count"].tolist())))
    assert tiles((1, 100000, D_, 0, 0)) == [(0, 1)]                           # a decode stays a decode
    assert tiles((8, 100000, V, 0, 0)) == [(0, 8)]                            # one narrow tile already
    assert tiles((31, 3968 - 31, V, 0, 0)) == [(0, 8), (8, 8), (16, 8), (24, 7)]     # 3968 keys = 31 tiles: narrow tiles
    assert tiles((31, 3969 - 31, V, 0, 0)) == [(0, 31)]                       # one key more, 32 tiles: the whole draft
    assert tiles((31, 4096, V, 0, 0)) == [(0, 31)]
    assert tiles((100, 9000, V, 0, 0)) == [(0, 64), (64, 36)]                 # at most 256 / G tokens per unit
    # a fixed tile still means what it meant
    fixed = dict(c, verify_tile_tokens=8)
    units, _, _, _ = PL.plan_oracle(fixed, [(31, 4096, V, 0, 0)])
    assert sorted(set(units["q_count"].tolist())) == [7, 8]


def threshold_cases():
    """Batches that sit exactly on, and one step beyond, the two thresholds of the plan rules; worked out by hand.
    Returns [(name, config, sequences, expectation)]; used here for the oracle and by the parity test for C++."""
    cases = []
    # Chiplet groups are dropped when the heaviest chiplet is MORE than 3 % above the mean: max * 800 > total * 103.
    # One head, 128-token prefill tiles (one unit = one group), loads 128 x tiles.  Seven groups of 697 tiles and
    # one of 721: 721 * 800 = 576800 = (721 + 7 * 697) * 103 -> kept: every group on the first worker of a chiplet
    # of its own (W = 16: workers 0, 2, .. 14).  One tile more on the heavy one: 722 * 800 = 577600 > 5601 * 103 =
    # 576903 -> dropped: plain least-loaded, the eight units on workers 0 .. 7.
    c = cfg(num_q_heads=1, num_kv_heads=1, num_workers=16, prefill_tile_tokens=128, prefill_heads_per_unit=1,
            cost_row_floor=1, assign_policy=1, max_blocks_per_seq=1024)
    light = (128, 696 * 128, P, 0, 0)
    cases.append(("chiplets_at_3_percent", c, [(128, 720 * 128, P, 0, 0)] + [light] * 7, [0, 2, 4, 6, 8, 10, 12, 14]))
    cases.append(("chiplets_beyond_3_percent", c, [(128, 721 * 128, P, 0, 0)] + [light] * 7, list(range(8))))
    # Wide families are cut to fill idle workers only while 2 N < M (W - U).  One 64-token prefill tile on 32 K/V
    # tiles (U = 1, M = 64 * 32 = 2048, W = 16: M (W - U) = 30720) next to decodes of 128 tiles each (load 128):
    # 120 of them give 2 N = 30720, not less -> the prefill unit stays whole; with one of them a tile shorter
    # 2 N = 30718 -> cut at max(8, ceil(32 / 16)) = 8 tiles: four pieces.
    c2 = cfg(num_q_heads=1, num_kv_heads=1, num_workers=16, prefill_tile_tokens=64, prefill_heads_per_unit=1,
             verify_tile_tokens=1, split_kv_blocks=-1, cost_row_floor=1, assign_policy=1, max_blocks_per_seq=128)
    pre = (64, 32 * 128 - 64, P, 0, 0)
    dec = (1, 128 * 128 - 1, D_, 0, 0)
    cases.append(("wide_cut_at_equality", c2, [pre] + [dec] * 120, 1))
    cases.append(("wide_cut_below", c2, [pre] + [dec] * 119 + [(1, 127 * 128 - 1, D_, 0, 0)], 4))
    # Unequal narrow families are cut at min(max(s, 2), max(16, min(64, floor(2 s / 5)))) tiles, s = ceil(B / L) a
    # wavefront's share.  One worker (L = 4), one head, two decodes of a and b tiles (B = a + b); expectation =
    # the pieces of the two.  s = 10: cut at 10 -> 3 + 1.  s = 42: floor(84 / 5) = 16 -> still 16: 7 + 5.
    # s = 43: floor(86 / 5) = 17: 6 + 5.  s = 160: 64: 7 + 4.  s = 165: floor(330 / 5) = 66 -> capped at 64: 7 + 5.
    c3 = cfg(num_q_heads=1, num_kv_heads=1, num_workers=1, verify_tile_tokens=1, split_kv_blocks=-1,
             cost_row_floor=1, assign_policy=1, max_blocks_per_seq=512)

    def two(a, b):
        return [(1, a * 128 - 1, D_, 0, 0), (1, b * 128 - 1, D_, 0, 0)]
    cases.append(("split_share_10", c3, two(30, 10), (3, 1)))
    cases.append(("split_share_42", c3, two(100, 68), (7, 5)))
    cases.append(("split_share_43", c3, two(100, 72), (6, 5)))
    cases.append(("split_share_160", c3, two(400, 240), (7, 4)))
    cases.append(("split_share_165", c3, two(400, 260), (7, 5)))
    return cases


@pytest.mark.parametrize("case", threshold_cases(), ids=[c[0] for c in threshold_cases()])
def test_both_sides_of_the_plan_thresholds(case):
    name, c, seqs, want = case
    units, offs, merges, _ = PL.plan_oracle(c, seqs)
    if name.startswith("chiplets"):
        assert len(units) == 8
        assert [w for w in range(16) if offs[w + 1] > offs[w]] == want
    elif name.startswith("split_share"):
        assert (int((units["seq"] == 0).sum()), int((units["seq"] == 1).sum())) == want
    else:
        pre = units[units["seq"] == 0]
        assert sorted(set(pre["num_splits"].tolist())) == [want] and len(pre) == want
        if want > 1:
            assert sorted((pre["kv_block_end"] - pre["kv_block_begin"]).tolist()) == [8, 8, 8, 8]
