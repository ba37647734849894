"""C++ planner (through the C ABI) against the oracle planner: exact integer match. CPU only."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import planner as PL
from paper_2412_18106_amd import binding as X
from paper_2412_18106_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def compare(cfg, seqs):
    plan = X.xy_attn_plan_create(cfg, seqs)
    try:
        units, offs, merges = X.plan_arrays(plan, cfg.num_workers)
        ws = X.xy_attn_plan_workspace_bytes(plan)
    finally:
        X.xy_attn_plan_destroy(plan)
    ou, oo, om, ows = PL.plan_oracle(cfg.as_dict(), seqs)
    assert units.dtype.itemsize == PL.UNIT_DTYPE.itemsize and merges.dtype.itemsize == PL.MERGE_DTYPE.itemsize
    assert units.tobytes() == ou.tobytes()
    assert offs.tolist() == oo.tolist()
    assert merges.tobytes() == om.tobytes()
    assert ws == 4 * ows
    return units


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_five_configs_default_parameters(index):
    _, hq, hkv, seqs, _, max_blocks = W.make_config_descs(index)
    cfg = X.xy_attn_default_config(hq, hkv, max_blocks)
    units = compare(cfg, seqs)
    assert len(units) > 0


@pytest.mark.parametrize("index", [2, 5])
def test_configs_paper_cost_and_single_head_units(index):
    _, hq, hkv, seqs, _, max_blocks = W.make_config_descs(index)
    cfg = X.xy_attn_default_config(hq, hkv, max_blocks, cost_row_floor=1, prefill_heads_per_unit=1,
                                   prefill_tile_tokens=128, num_workers=304, split_kv_blocks=0, assign_policy=0)
    compare(cfg, seqs)


@pytest.mark.parametrize("seed", range(20))
def test_fuzz(seed):
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 8]))
    group = int(rng.choice([1, 2, 4, 8]))
    hpu = int(rng.choice([g for g in (1, 2, 4, 8) if group % g == 0]))
    seqs = []
    for _ in range(int(rng.integers(0, 40))):
        kind = int(rng.integers(0, 3))
        if kind == 0:
            seqs.append((int(rng.integers(1, 1500)), int(rng.integers(0, 20000)), 0, 0, 0))
        elif kind == 1:
            seqs.append((1, int(rng.integers(0, 40000)), 1, 0, 0))
        else:
            ql = int(rng.integers(1, 70))
            seqs.append((ql, int(rng.integers(0, 9000)), 2, int(rng.integers(0, 2)) if ql <= 64 else 0,
                         int(rng.integers(0, 100))))
    cfg = X.xy_attn_default_config(
        hkv * group, hkv, 400, num_workers=int(rng.integers(1, 600)),
        prefill_heads_per_unit=hpu, prefill_tile_tokens=int(rng.integers(1, 256 // hpu + 1)),
        verify_tile_tokens=int(rng.integers(1, 256 // group + 1)) if rng.integers(0, 3) else -1,
        split_kv_blocks=int(rng.choice([-1, -1, 0, 1, 5, 16, 64])), cost_row_floor=int(rng.choice([1, 32, 128, 256])),
        assign_policy=int(rng.integers(0, 3)))
    compare(cfg, seqs)


@pytest.mark.parametrize("floor", [2 ** 24 - 1, 2 ** 24, 2 ** 25, 2 ** 30])
@pytest.mark.parametrize("policy", [0, 1, 2])
def test_costs_on_both_sides_of_32_bits_sort_alike(floor, policy):
    """The C++ planner sorts with a 64-bit (cost, place) key while every cost fits 32 bits and with a wider key
    beyond: a 256-tile unit costs floor x 256, which crosses 2^32 at floor = 2^24."""
    seqs = [(1, 32767, 1, 0, 0), (700, 12000, 0, 0, 0), (1, 5000, 1, 0, 0), (9, 300, 2, 0, 0), (40, 0, 0, 0, 0),
            (1, 32767, 1, 0, 0), (3, 70, 2, 1, 7)]
    cfg = X.xy_attn_default_config(8, 2, 400, num_workers=24, cost_row_floor=floor, assign_policy=policy,
                                   split_kv_blocks=0)
    units = compare(cfg, seqs)
    assert (int(units["cost"].max()) >= 2 ** 32) == (floor >= 2 ** 24)
    compare(X.xy_attn_default_config(8, 2, 400, num_workers=24, cost_row_floor=floor, assign_policy=policy), seqs)


@pytest.mark.parametrize("longest", [100, 255, 256, 700])
@pytest.mark.parametrize("workers", [4, 16])
def test_batches_of_short_decodes_on_both_sides_of_the_shared_list_rule(longest, workers):
    """Dynamic assignment without wide units: static lists while no unit visits more than two K/V tiles (up to 256
    keys, the decode token included), a shared list beyond."""
    rng = np.random.default_rng(longest + workers)
    seqs = [(1, int(c), 1, 0, 0) for c in rng.integers(0, longest, 60)] + [(1, longest - 1, 1, 0, 0), (1, longest, 1, 0, 0)]
    cfg = X.xy_attn_default_config(8, 2, 16, num_workers=workers)
    units = compare(cfg, seqs)
    plan = X.xy_attn_plan_create(cfg, seqs)
    _, offs, _ = X.plan_arrays(plan, workers)
    X.xy_attn_plan_destroy(plan)
    assert (offs[workers] == len(units)) == (longest <= 255)


@pytest.mark.parametrize("seed", range(16))
def test_fuzz_with_chiplet_aware_placement(seed):
    """Worker counts that are multiples of eight (wide units are then placed chiplet by chiplet), batches with
    many prefill and long verify sequences, policies 1 and 2."""
    rng = np.random.default_rng(5000 + seed)
    hkv = int(rng.choice([1, 2, 8]))
    group = int(rng.choice([1, 4, 8]))
    seqs = []
    for _ in range(int(rng.integers(1, 24))):
        kind = int(rng.integers(0, 4))
        if kind <= 1:
            seqs.append((int(rng.integers(1, 3000)), int(rng.integers(0, 30000)), 0, 0, 0))
        elif kind == 2:
            seqs.append((1, int(rng.integers(0, 40000)), 1, 0, 0))
        else:
            seqs.append((int(rng.integers(1, 70)), int(rng.integers(0, 9000)), 2, 0, 0))
    cfg = X.xy_attn_default_config(
        hkv * group, hkv, 400, num_workers=int(rng.choice([8, 16, 64, 256, 304])),
        prefill_tile_tokens=int(rng.choice([max(1, 64 // group), 256 // group])),
        verify_tile_tokens=int(rng.choice([-1, max(1, 32 // group), 256 // group])),
        split_kv_blocks=int(rng.choice([-1, 0, 16])), cost_row_floor=int(rng.choice([1, 128])),
        assign_policy=int(rng.integers(1, 3)))
    compare(cfg, seqs)


@pytest.mark.parametrize("bs", [16, 32, 64])
def test_page_size_changes_capacity_only(bs):
    """Units visit K/V in 128-key tiles whatever the page size: the plan of a batch is the same for every
    block_size, only the capacity check counts pages."""
    _, hq, hkv, seqs, _, max_blocks = W.make_config_descs(2)
    per = 128 // bs
    ref = compare(X.xy_attn_default_config(hq, hkv, max_blocks), seqs)
    units = compare(X.xy_attn_default_config(hq, hkv, max_blocks * per, block_size=bs), seqs)
    assert units.tobytes() == ref.tobytes()
    cfg = X.xy_attn_default_config(8, 2, 4, block_size=bs)
    assert _status(cfg, [(1, 4 * bs, X.XY_DECODE, 0, 0)]) == X.XY_ERR_CAPACITY
    X.xy_attn_plan_destroy(X.xy_attn_plan_create(cfg, [(1, 4 * bs - 1, X.XY_DECODE, 0, 0)]))


def test_empty_plan():
    cfg = X.xy_attn_default_config(8, 2, 4)
    plan = X.xy_attn_plan_create(cfg, [])
    units, offs, merges = X.plan_arrays(plan, cfg.num_workers)
    assert len(units) == 0 and (offs == 0).all() and len(merges) == 0
    assert X.xy_attn_plan_workspace_bytes(plan) == 0
    X.xy_attn_plan_destroy(plan)


def _status(cfg, seqs):
    with pytest.raises(X.XyError) as e:
        X.xy_attn_plan_create(cfg, seqs)
    return e.value.status


def test_error_paths():
    good = X.xy_attn_default_config(8, 2, 4)
    assert _status(good, [(2, 10, X.XY_DECODE, 0, 0)]) == X.XY_ERR_DESC          # decode must be one token
    assert _status(good, [(0, 10, X.XY_PREFILL, 0, 0)]) == X.XY_ERR_DESC
    assert _status(good, [(1, -1, X.XY_PREFILL, 0, 0)]) == X.XY_ERR_DESC
    assert _status(good, [(4, 10, X.XY_PREFILL, X.XY_MASK_TREE, 0)]) == X.XY_ERR_DESC   # tree only on verify
    assert _status(good, [(4, 10, 7, 0, 0)]) == X.XY_ERR_DESC
    assert _status(good, [(65, 10, X.XY_VERIFY, X.XY_MASK_TREE, 0)]) == X.XY_ERR_DESC   # tree corner is at most 64 x 64
    assert _status(good, [(1, 4 * 128, X.XY_DECODE, 0, 0)]) == X.XY_ERR_CAPACITY
    X.xy_attn_plan_destroy(X.xy_attn_plan_create(good, [(1, 4 * 128 - 1, X.XY_DECODE, 0, 0)]))
    for field, val in (("head_dim", 64), ("block_size", 48), ("num_workers", 0), ("num_kv_heads", 3),
                       ("prefill_tile_tokens", 128), ("verify_tile_tokens", 65), ("cost_row_floor", 0),
                       ("split_kv_blocks", -2), ("prefill_heads_per_unit", 3), ("assign_policy", 3),
                       ("verify_tile_tokens", -2), ("verify_tile_tokens", 0)):
        bad = X.xy_attn_default_config(8, 2, 4)
        setattr(bad, field, val)
        assert _status(bad, [(1, 5, X.XY_DECODE, 0, 0)]) == X.XY_ERR_ARG, field
    with pytest.raises(X.XyError):
        X.xy_attn_default_config(8, 3, 4)
    assert X.xy_attn_strerror(X.XY_ERR_CAPACITY) != X.xy_attn_strerror(X.XY_ERR_DESC)
    # run with a null plan is an argument error and touches no device
    assert X._lib.xy_attn_run(None, None, 0, 0, None, None, 0, 0, 0, None, None, None, 0, 0, None, 0, 1.0, None) == X.XY_ERR_ARG


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "xy_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(xy_attn_\w+)\s*\(", header))
    assert declared == set(X.EXPORTED)
    probe = open(os.path.join(ROOT, "include", "xy_probe.h")).read()
    probe = re.sub(r"/\*.*?\*/", "", probe, flags=re.S)
    declared_probe = set(re.findall(r"\b(xy_probe_\w+)\s*\(", probe))
    assert declared_probe == set(X.EXPORTED_PROBE)
    serve = open(os.path.join(ROOT, "include", "xy_serve.h")).read()
    serve = re.sub(r"/\*.*?\*/", "", serve, flags=re.S)
    declared_serve = set(re.findall(r"\b(xy_(?:serve|kv)_\w+)\s*\(", serve))
    assert declared_serve == set(X.EXPORTED_SERVE)
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2412_18106_amd", "libxyattn.so"))
    for name in declared | declared_serve | declared_probe:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header_sizes():
    assert ctypes.sizeof(X.xy_seq_desc) == 24
    assert ctypes.sizeof(X.xy_attn_config) == 48
    assert ctypes.sizeof(X.xy_work_unit) == 56 == PL.UNIT_DTYPE.itemsize
    assert ctypes.sizeof(X.xy_merge_item) == 32 == PL.MERGE_DTYPE.itemsize


def _plan_bytes(plan, workers):
    units, offs, merges = X.plan_arrays(plan, workers)
    return units.tobytes(), offs.tolist(), merges.tobytes(), X.xy_attn_plan_workspace_bytes(plan)


def test_rebuild_in_place_equals_a_fresh_plan_batch_after_batch():
    """A serving loop plans every step in one plan object: larger, smaller, empty and differently configured
    batches in turn give exactly the plan a fresh object gives, and a refused batch leaves the old plan alone."""
    rng = np.random.default_rng(42)
    plan = X.xy_attn_plan_create(X.xy_attn_default_config(8, 2, 4), [])
    try:
        last = None
        for step in range(14):
            index = int(rng.integers(1, 6))
            _, hq, hkv, seqs, _, max_blocks = W.make_config_descs(index)
            keep = sorted(rng.choice(len(seqs), size=int(rng.integers(0, len(seqs) + 1)), replace=False).tolist())
            seqs = [seqs[i] for i in keep]
            cfg = X.xy_attn_default_config(hq, hkv, max_blocks, num_workers=int(rng.choice([7, 64, 256])),
                                           assign_policy=int(rng.integers(0, 3)))
            X.xy_attn_plan_rebuild(plan, cfg, seqs)
            fresh = X.xy_attn_plan_create(cfg, seqs)
            last = _plan_bytes(fresh, cfg.num_workers)
            assert _plan_bytes(plan, cfg.num_workers) == last, step
            X.xy_attn_plan_destroy(fresh)
            workers = cfg.num_workers
        # refused batches: the plan is still the last good one
        for bad_seqs, status in (([(2, 10, X.XY_DECODE, 0, 0)], X.XY_ERR_DESC),
                                 ([(1, 10 ** 7, X.XY_DECODE, 0, 0)], X.XY_ERR_CAPACITY)):
            with pytest.raises(X.XyError) as e:
                X.xy_attn_plan_rebuild(plan, cfg, bad_seqs)
            assert e.value.status == status
            assert _plan_bytes(plan, workers) == last
        bad = X.xy_attn_default_config(8, 2, 4, head_dim=64)
        with pytest.raises(X.XyError):
            X.xy_attn_plan_rebuild(plan, bad, [(1, 5, X.XY_DECODE, 0, 0)])
        assert _plan_bytes(plan, workers) == last
        assert X._lib.xy_attn_plan_rebuild(None, None, None, 0) == X.XY_ERR_ARG
    finally:
        X.xy_attn_plan_destroy(plan)


def test_more_than_256_query_heads_per_kv_head_is_refused_by_the_planner_too():
    """xy_attn_default_config refuses the head shape; so does a configuration filled in by hand (with the tile
    chosen per sequence a unit would otherwise get more rows than the kernel covers)."""
    with pytest.raises(X.XyError):
        X.xy_attn_default_config(512, 1, 4)
    cfg = X.xy_attn_default_config(256, 1, 4)
    X.xy_attn_plan_destroy(X.xy_attn_plan_create(cfg, [(1, 5, X.XY_DECODE, 0, 0)]))
    cfg.num_q_heads = 512
    cfg.prefill_heads_per_unit = 1
    cfg.prefill_tile_tokens = 1
    assert _status(cfg, [(1, 5, X.XY_DECODE, 0, 0)]) == X.XY_ERR_ARG


def test_descriptor_marshalling_accepts_lists_and_record_arrays():
    seqs = [(3, 100, X.XY_VERIFY, X.XY_MASK_TREE, 5), (1, 7, X.XY_DECODE, 0, 0)]
    arr = X.make_descs(seqs)
    assert arr["query_len"].tolist() == [3, 1] and arr["mask_word_offset"].tolist() == [5, 0]
    assert X.make_descs(arr) is not None and X.make_descs([]).shape == (1,)
    cfg = X.xy_attn_default_config(8, 2, 4)
    a = X.xy_attn_plan_create(cfg, seqs)
    b = X.xy_attn_plan_create(cfg, arr)
    assert _plan_bytes(a, 256) == _plan_bytes(b, 256)
    X.xy_attn_plan_destroy(a)
    X.xy_attn_plan_destroy(b)


def test_thresholds_of_the_plan_rules_match_on_both_sides():
    """The hand-worked batches that sit on and just beyond the 3 % chiplet threshold and the 2 N < M (W - U) rule:
    the C++ planner and the oracle planner take the same side."""
    from test_oracle_planner import threshold_cases
    for name, c, seqs, _want in threshold_cases():
        cfgc = X.xy_attn_default_config(c["num_q_heads"], c["num_kv_heads"], c["max_blocks_per_seq"],
                                        **{k: v for k, v in c.items()
                                           if k not in ("num_q_heads", "num_kv_heads", "max_blocks_per_seq")})
        compare(cfgc, seqs)
