"""Integer work-unit plan, written out rule by rule (TEST INFRASTRUCTURE ONLY).

Follows the paper's section 3.2.1 (Token-Table -> tiling blocks x heads =
tiling units) and section 3.3.1 (load = tileSize x kvLen, sort descending,
symmetric round-robin onto cores -> Task-Table).  Where the paper leaves a
choice open (tile sizes, tie-breaks, blocks vs tokens in the load, K/V
splitting across cores) the rules below are the written contract that the
C++ planner must reproduce bit for bit.

Rules
-----
1. Sequences in input order; ``token_start`` is the running sum of query_len.
   PREFILL uses token tiles of ``prefill_tile_tokens`` and head groups of
   ``prefill_heads_per_unit``; DECODE and VERIFY use token tiles of
   ``verify_tile_tokens`` and head groups of ``G = Hq / Hkv`` (one unit per KV
   head).  Families are enumerated sequence-major, then token tile, then head
   group.  K/V is visited in tiles of ``T = 128`` keys whatever the page size
   (a tile is ``128 / block_size`` consecutive block-table entries; the unit
   fields called ``kv_block_*`` count these tiles).  A causal family visits
   tiles ``[0, ceil((c + q_begin + q_count) / T))`` (tiles wholly past the
   tile's last visible key are never visited, section 4.2.2); a tree-masked
   family visits ``[0, ceil((c + q) / T))``.
   1a. ``verify_tile_tokens = -1`` (automatic): a DECODE / VERIFY sequence is
   tiled in ``max(1, 32 // G)`` tokens unless ``q`` exceeds that and
   ``ceil((c + q) / 128) >= 32``: then in ``min(q, max(1, 256 // G))`` tokens.
2. A non-PREFILL family with ``nb`` blocks and ``split_kv_blocks = S > 0`` and
   ``nb > S`` is cut into ``k = ceil(nb / S)`` units, unit ``p`` covering blocks
   ``[floor(p nb / k), floor((p + 1) nb / k))``.
   ``split_kv_blocks = -1`` (automatic) sizes S to the batch.  Narrow
   families are the non-PREFILL families of at most 32 rows; ``F`` their
   number (token tiles times Hkv), ``L = 4 W`` the wavefront slots.  If all of
   them have the same ``nb``: ``S = ceil(nb / k)`` for the ``k`` that minimises
   ``ceil(F k / L) * (ceil(nb / k) + 1)`` over ``k = 1 .. nb``, smallest ``k``
   on ties (the ``+ 1`` is what a piece costs beyond its tiles).  Otherwise
   ``S = min(max(s, 2), max(16, min(64, floor(2 s / 5))))`` with
   ``s = ceil(B / L)`` and ``B`` the sum of their ``nb``.
   Non-PREFILL families of more than 32 rows use ``S = 16``.  When the batch
   has fewer families of more than 32 rows (PREFILL included) than workers,
   ``U < W``, and little else to do - ``2 N < M (W - U)`` with ``N`` the summed
   load ``max(rows, cost_row_floor) * nb`` of the families of at most 32 rows
   and ``M`` the largest such load of a wide family - each wide family, PREFILL
   too, is cut at ``S = max(8, ceil(nb / floor(W / U)))`` instead.
3. ``rows = q_count * head_count``; ``cost = max(rows, cost_row_floor) * blocks``
   (``cost_row_floor = 1`` is the paper's tileSize x kvLen in block units).
4. Stable sort by cost descending, ties by (seq, head_begin, q_begin,
   split_index) ascending.
5. ``assign_policy`` 0 (the paper's symmetric round-robin): sorted position
   ``p`` has round ``p // W`` and lane ``p % W``; worker = lane on even rounds,
   ``W - 1 - lane`` on odd rounds.  ``assign_policy`` 1 (least loaded): walking
   the same sorted list, each unit goes to the worker whose summed cost so far
   is smallest, the lowest index among equals.  Units are emitted grouped by
   worker in assignment order, with ``worker_offsets[W + 1]``.
   5a. With policies 1 and 2, when 8 divides W, units of more than 32 rows
   are placed chiplet by chiplet: those of one (sequence, KV head) form a
   group; the groups, by summed cost descending (ties by sequence, KV head),
   go to the chiplet whose load so far is smallest (lowest index among
   equals); a unit then goes to the least-loaded worker among the W / 8 of its
   group's chiplet.  If the heaviest chiplet exceeds 1.03 times the mean
   (``max * 8 * 100 > total * 103``), no grouping is used.
   ``assign_policy`` 2 (dynamic): units of more than 32 rows are assigned as
   with policy 1, counting only their own costs; units of at most 32 rows are
   emitted behind all workers' lists, in sorted order, as one shared list that
   starts at ``worker_offsets[W]``.  When no unit has more than 32 rows and
   either all costs are equal or no unit visits more than 2 K/V tiles, policy
   2 gives the plan of policy 1.
6. A partial result is ``slab = rows * (D + 2)`` fp32 elements rounded up to a
   multiple of 4.  Split families, in enumeration order, get consecutive
   workspace regions of ``num_splits * slab``; a unit's ``ws_offset`` is its
   family base plus ``split_index * slab``; unsplit units carry -1.  One merge
   item per split family.
"""
from __future__ import annotations

import numpy as np

PREFILL, DECODE, VERIFY = 0, 1, 2
MASK_CAUSAL, MASK_TREE = 0, 1
KV_TILE = 128
SPLIT_AUTO = -1          # split_kv_blocks value that sizes the K/V split to the batch
TILE_AUTO = -1           # verify_tile_tokens value that picks the token tile per sequence
NARROW_ROWS = 32         # units of at most this many rows are processed one per wavefront
CHIPLETS = 8             # L2 domains of the GPU: workers [x W / 8, (x + 1) W / 8) run on domain x when 8 divides W

UNIT_DTYPE = np.dtype([
    ("seq", "<i4"), ("head_begin", "<i4"), ("head_count", "<i4"),
    ("q_begin", "<i4"), ("q_count", "<i4"),
    ("kv_block_begin", "<i4"), ("kv_block_end", "<i4"),
    ("split_index", "<i4"), ("num_splits", "<i4"), ("kind_flags", "<i4"),
    ("cost", "<i8"), ("ws_offset", "<i8"),
])

MERGE_DTYPE = np.dtype([
    ("seq", "<i4"), ("head_begin", "<i4"), ("head_count", "<i4"),
    ("q_begin", "<i4"), ("q_count", "<i4"), ("num_splits", "<i4"),
    ("ws_offset", "<i8"),
])


def _verify_tile(cfg, ql, c, group):
    """Token tile of a DECODE / VERIFY sequence (rule 1a)."""
    t = cfg["verify_tile_tokens"]
    if t != TILE_AUTO:
        return t
    narrow = max(1, 32 // group)
    if ql <= narrow or _ceil_div(c + ql, KV_TILE) < 32:
        return narrow
    return min(ql, max(1, 256 // group))


def _ceil_div(a, b):
    return -(-a // b)


def plan_oracle(cfg, seqs):
    """cfg: dict with the plan parameters; seqs: list of
    (query_len, context_len, kind, mask_kind, mask_word_offset).

    Returns (units, worker_offsets, merges, workspace_floats) where units and
    merges are numpy structured arrays laid out like the C structs.
    """
    hq, hkv = cfg["num_q_heads"], cfg["num_kv_heads"]
    d = cfg["head_dim"]
    w = cfg["num_workers"]
    group = hq // hkv
    fam_units = []
    merges = []
    ws_floats = 0
    split_narrow = split_wide = cfg["split_kv_blocks"]
    wide_pieces = 1
    if cfg["split_kv_blocks"] == SPLIT_AUTO:
        wide_families = wide_max = narrow_total = 0
        for ql, c, kind, mk, _off in seqs:
            t = cfg["prefill_tile_tokens"] if kind == PREFILL else _verify_tile(cfg, ql, c, group)
            hc = cfg["prefill_heads_per_unit"] if kind == PREFILL else group
            for q_begin in range(0, ql, t):
                q_count = min(t, ql - q_begin)
                last = c + ql if mk == MASK_TREE else c + q_begin + q_count
                load = max(q_count * hc, cfg["cost_row_floor"]) * _ceil_div(last, KV_TILE)
                if q_count * hc > NARROW_ROWS:
                    wide_families += hq // hc
                    wide_max = max(wide_max, load)
                else:
                    narrow_total += load * (hq // hc)
        if 0 < wide_families < w and narrow_total * 2 < wide_max * (w - wide_families):
            wide_pieces = w // wide_families
        lengths = []            # nb of every narrow non-PREFILL token tile
        for ql, c, kind, mk, _off in seqs:
            if kind == PREFILL:
                continue
            tile = _verify_tile(cfg, ql, c, group)
            for q_begin in range(0, ql, tile):
                q_count = min(tile, ql - q_begin)
                if q_count * group > NARROW_ROWS:
                    continue
                last = c + ql if mk == MASK_TREE else c + q_begin + q_count
                lengths.append(_ceil_div(last, KV_TILE))
        slots = 4 * w
        if lengths and len(set(lengths)) == 1:
            nb, families = lengths[0], len(lengths) * hkv
            best_k = min(range(1, nb + 1), key=lambda k: (_ceil_div(families * k, slots) * (_ceil_div(nb, k) + 1), k))
            split_narrow = _ceil_div(nb, best_k)
        else:
            share = _ceil_div(sum(lengths) * hkv, slots)
            split_narrow = min(max(share, 2), max(16, min(64, 2 * share // 5)))
        split_wide = 16
    for i, (ql, c, kind, mk, _off) in enumerate(seqs):
        if kind == PREFILL:
            tile, hc = cfg["prefill_tile_tokens"], cfg["prefill_heads_per_unit"]
        else:
            tile, hc = _verify_tile(cfg, ql, c, group), group
        for q_begin in range(0, ql, tile):
            q_count = min(tile, ql - q_begin)
            last_key_excl = c + ql if mk == MASK_TREE else c + q_begin + q_count
            nb = _ceil_div(last_key_excl, KV_TILE)
            for head_begin in range(0, hq, hc):
                rows = q_count * hc
                s = split_narrow if rows <= NARROW_ROWS else split_wide
                may_split = kind != PREFILL
                if rows > NARROW_ROWS and wide_pieces > 1:
                    s = max(8, _ceil_div(nb, wide_pieces))
                    may_split = True
                k = _ceil_div(nb, s) if (may_split and s > 0 and nb > s) else 1
                slab = _ceil_div(rows * (d + 2), 4) * 4
                base = -1
                if k > 1:
                    base = ws_floats
                    ws_floats += k * slab
                    merges.append((i, head_begin, hc, q_begin, q_count, k, base))
                for p in range(k):
                    lo, hi = (p * nb) // k, ((p + 1) * nb) // k
                    cost = max(rows, cfg["cost_row_floor"]) * (hi - lo)
                    off = -1 if k == 1 else base + p * slab
                    fam_units.append((i, head_begin, hc, q_begin, q_count, lo, hi, p, k,
                                      kind | (mk << 2), cost, off))
    order = sorted(range(len(fam_units)),
                   key=lambda x: (-fam_units[x][10], fam_units[x][0], fam_units[x][1],
                                  fam_units[x][3], fam_units[x][7]))
    per_worker = [[] for _ in range(w)]
    shared = []                 # policy 2: the narrow units, for all workers
    if cfg.get("assign_policy", 0) == 0:
        for pos, x in enumerate(order):
            rnd, lane = divmod(pos, w)
            per_worker[lane if rnd % 2 == 0 else w - 1 - lane].append(fam_units[x])
    else:
        load = np.zeros(w, dtype=np.int64)
        narrow_costs = {u[10] for u in fam_units if u[2] * u[4] <= NARROW_ROWS}
        any_wide = any(u[2] * u[4] > NARROW_ROWS for u in fam_units)
        longest_narrow = max((u[6] - u[5] for u in fam_units if u[2] * u[4] <= NARROW_ROWS), default=0)
        share = cfg.get("assign_policy", 0) == 2 and (any_wide or (len(narrow_costs) > 1 and longest_narrow > 2))
        # chiplet-aware placement of the wide units (rule 5a)
        per_chip = w // CHIPLETS if w % CHIPLETS == 0 else 0
        chip_of_group = None
        if per_chip:
            group_cost = {}
            for u in fam_units:
                if u[2] * u[4] > NARROW_ROWS:
                    key = u[0] * hkv + u[1] // group
                    group_cost[key] = group_cost.get(key, 0) + u[10]
            chip_load = [0] * CHIPLETS
            chip_of_group = {}
            for key in sorted(group_cost, key=lambda g: (-group_cost[g], g)):
                x = chip_load.index(min(chip_load))
                chip_of_group[key] = x
                chip_load[x] += group_cost[key]
            if max(chip_load) * CHIPLETS * 100 > sum(chip_load) * 103:
                chip_of_group = None
        for x in order:
            u = fam_units[x]
            narrow = u[2] * u[4] <= NARROW_ROWS
            if share and narrow:
                shared.append(u)
                continue
            if not narrow and chip_of_group is not None:
                lo = chip_of_group[u[0] * hkv + u[1] // group] * per_chip
                k = lo + int(np.argmin(load[lo:lo + per_chip]))
            else:
                k = int(np.argmin(load))          # first index of the minimum
            per_worker[k].append(u)
            load[k] += u[10]
    flat = [u for lst in per_worker for u in lst] + shared
    offsets = np.zeros(w + 1, dtype=np.int32)
    offsets[1:] = np.cumsum([len(lst) for lst in per_worker])
    units = np.array(flat, dtype=UNIT_DTYPE) if flat else np.zeros(0, dtype=UNIT_DTYPE)
    marr = np.array(merges, dtype=MERGE_DTYPE) if merges else np.zeros(0, dtype=MERGE_DTYPE)
    return units, offsets, marr, ws_floats
