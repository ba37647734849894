"""Pins for the serving-side oracle (scheduler and radix-tree block manager; CPU only).

The block manager is pinned through what it is for: a shadow copy of the cache
content (token ids instead of K/V rows) is kept by the test itself -- copies and
writes applied exactly as a caller would issue them -- and after every operation
each open sequence, read back through its block row, must hold its own tokens
(the continuity of historical and new K/V that section 4.1.1 asks for).  Reuse
counts, copy-on-write and the eviction order are pinned on hand-built cases.
"""
import numpy as np
import pytest

from oracle import serving as S

P, D, V = S.PREFILL, S.DECODE, S.VERIFY


# ---- scheduler ------------------------------------------------------------------------------
def total(chunk):
    return sum(e[2] for e in chunk)


def test_long_prompt_is_cut_to_the_budget_and_finishes_over_steps():
    # section 3.1: a prompt longer than the budget is split so that every chunk stays within it
    remaining, ctx, steps = 1000, 0, []
    while remaining:
        chunk = S.schedule_chunk(256, 32, [(7, P, remaining, ctx)])
        assert len(chunk) == 1 and chunk[0][:2] == (7, P) and chunk[0][3] == ctx
        steps.append(chunk[0][2])
        remaining -= chunk[0][2]
        ctx += chunk[0][2]
    assert steps == [256, 256, 256, 232]          # no decode waiting: prefill-only chunks use the whole budget


def test_reserved_slots_keep_decodes_running_next_to_a_long_prefill():
    queue = [(0, P, 5000, 0)] + [(10 + i, D, 1, 100 + i) for i in range(40)]
    chunk = S.schedule_chunk(256, 32, queue)
    assert total(chunk) == 256
    assert chunk[0] == (0, P, 224, 0)             # prefill has T - R
    assert [e[0] for e in chunk[1:]] == list(range(10, 42))   # the first 32 decodes, queue order
    # nothing else waiting: the decodes left over in rule 1 fill the budget in rule 3
    chunk = S.schedule_chunk(256, 32, queue[1:])
    assert total(chunk) == 40 and all(e[1] == D for e in chunk)


def test_verify_segment_is_never_cut_and_smaller_entries_pass_it():
    queue = [(1, V, 31, 500), (2, D, 1, 50), (3, V, 15, 70), (4, P, 100, 0)]
    chunk = S.schedule_chunk(64, 16, queue)
    # rule 1 (R = 16): 31 does not fit, the decode does, 15 fits exactly; rule 2: prefill gets 64 - 16 = 48;
    # rule 3: 31 no longer fits
    assert chunk == [(4, P, 48, 0), (2, D, 1, 50), (3, V, 15, 70)]
    chunk = S.schedule_chunk(64, 16, queue[:3])
    assert chunk == [(1, V, 31, 500), (2, D, 1, 50), (3, V, 15, 70)]   # rule 3 picks it up when there is room


@pytest.mark.parametrize("seed", range(30))
def test_scheduler_invariants_random(seed):
    rng = np.random.default_rng(seed)
    t = int(rng.integers(1, 600))
    r = int(rng.integers(0, t + 1))
    queue = []
    for i in range(int(rng.integers(0, 40))):
        kind = int(rng.integers(0, 3))
        tokens = int(rng.integers(1, 2000)) if kind == P else 1 if kind == D else int(rng.integers(1, 64))
        queue.append((i, kind, tokens, int(rng.integers(0, 5000))))
    chunk = S.schedule_chunk(t, r, queue)
    by_id = {e[0]: e for e in queue}
    assert total(chunk) <= t
    assert len({e[0] for e in chunk}) == len(chunk)
    for req, kind, ql, ctx in chunk:
        assert kind == by_id[req][1] and ctx == by_id[req][3] and 1 <= ql <= by_id[req][2]
        if kind != P:
            assert ql == by_id[req][2]                      # decode / verify whole
    cut = [e for e in chunk if e[1] == P and e[2] < by_id[e[0]][2]]
    assert len(cut) <= 1 and (not cut or total(chunk) == t)  # only the last prefill is cut, and then the budget is full
    waiting_dv = [e for e in queue if e[1] != P]
    if waiting_dv and min(e[2] for e in waiting_dv) <= r:
        assert any(e[1] != P for e in chunk)                 # no prefill-only chunk while a decode that fits R waits
    # prefill is prioritised: it is never left with less than T - R while it still has tokens waiting
    pf_wait = sum(e[2] for e in queue if e[1] == P)
    pf_got = sum(e[2] for e in chunk if e[1] == P)
    assert pf_got >= min(pf_wait, t - r)
    # work conserving: budget left over means nothing that fits was left out
    left = t - total(chunk)
    chosen = {e[0] for e in chunk}
    for e in queue:
        if e[0] not in chosen:
            assert e[2] > left or e[1] == P and left == 0 or (e[1] == P and cut)


# ---- block manager ----------------------------------------------------------------------------
class Shadow:
    """Token ids per cache slot, maintained the way a caller maintains K/V rows."""

    def __init__(self, num_blocks, b):
        self.b = b
        self.data = -np.ones((num_blocks, b), dtype=np.int64)
        self.tokens = {}        # seq id -> all tokens of the sequence

    def opened(self, m, sid, tokens, cached, copies):
        for src, dst, rows in copies:
            self.data[dst, :rows] = self.data[src, :rows]
        self.tokens[sid] = list(tokens[:cached])

    def extended(self, m, sid, new):
        row = m.block_row(sid)
        start = len(self.tokens[sid])
        for k, tok in enumerate(new):
            pos = start + k
            self.data[row[pos // self.b], pos % self.b] = tok
        self.tokens[sid] += list(new)

    def check(self, m):
        for sid, toks in self.tokens.items():
            row = m.block_row(sid)
            assert m.length(sid) == len(toks)
            assert len(row) == -(-len(toks) // self.b)
            got = [int(self.data[row[p // self.b], p % self.b]) for p in range(len(toks))]
            assert got == toks, f"sequence {sid} does not read back its own tokens"
        owned = [blk for sid in self.tokens for blk in m.block_row(sid)]
        # a block may be shared between sequences only through the tree (identical prefixes)
        for sid in self.tokens:
            for other in self.tokens:
                if sid < other:
                    ra, rb = m.block_row(sid), m.block_row(other)
                    for i, (x, y) in enumerate(zip(ra, rb)):
                        if x == y:
                            a, b_ = self.tokens[sid], self.tokens[other]
                            assert a[i * self.b:(i + 1) * self.b] == b_[i * self.b:(i + 1) * self.b] and len(a) >= (i + 1) * self.b
        return owned


def open_full(m, sh, tokens):
    """open + extend with the rest of the prompt, the way a prefill does."""
    res = m.open(tokens)
    assert res is not None
    sid, cached, copies = res
    sh.opened(m, sid, tokens, cached, copies)
    assert m.extend(sid, tokens[cached:])
    sh.extended(m, sid, tokens[cached:])
    sh.check(m)
    return sid, cached, copies


def test_token_wise_prefix_reuse_and_copy_on_write():
    b = 4
    m, sh = S.BlockManagerOracle(32, b), Shadow(32, b)
    a = list(range(100, 114))                         # 14 tokens: 3 full blocks + 2
    sid_a, cached, copies = open_full(m, sh, a)
    assert cached == 0 and copies == []
    row_a = m.block_row(sid_a)
    assert row_a == [0, 1, 2, 3]                      # free list in ascending order
    # same first 10 tokens, then different: two whole blocks and half of the third are reused
    c = a[:10] + [900, 901, 902, 903, 904]
    sid_c, cached, copies = open_full(m, sh, c)
    assert cached == 10
    assert copies == [(row_a[2], m.block_row(sid_c)[2], 2)]           # copy-on-write of the partly matching block
    assert m.block_row(sid_c)[:2] == row_a[:2] and m.block_row(sid_c)[2] != row_a[2]
    # an identical prompt reuses the three full blocks; the two tokens of the first sequence's tail are
    # still private to it (not in the tree), so they are computed again
    sid_d, cached, copies = open_full(m, sh, list(a))
    assert cached == 12 and copies == []
    # a prompt that is a strict prefix ending on a block boundary keeps one token to compute
    sid_e, cached, _ = open_full(m, sh, a[:8])
    assert cached == 7


def test_partial_tail_of_an_open_sequence_is_not_shared_until_full():
    b = 4
    m, sh = S.BlockManagerOracle(16, b), Shadow(16, b)
    sid_a, _, _ = open_full(m, sh, [1, 2, 3, 4, 5, 6])            # one full block in the tree, tail of 2 private
    sid_b, cached, copies = open_full(m, sh, [1, 2, 3, 4, 5, 6, 7, 8, 9])
    assert cached == 4 and copies == []                           # the private tail (5, 6) is invisible
    assert m.extend(sid_a, [7, 8]); sh.extended(m, sid_a, [7, 8]); sh.check(m)
    # both sequences now hold a full block (5, 6, 7, 8): the first to fill it put it in the tree
    sid_c, cached, _ = open_full(m, sh, [1, 2, 3, 4, 5, 6, 7, 8, 42, 43])
    assert cached == 8


def test_lru_eviction_takes_unpinned_leaves_oldest_first_and_never_a_pinned_block():
    b = 2
    m, sh = S.BlockManagerOracle(6, b), Shadow(6, b)
    s1, _, _ = open_full(m, sh, [1, 2, 3, 4, 5])                 # blocks 0, 1 in tree, 2 private tail
    s2, _, _ = open_full(m, sh, [7, 8, 9])                       # block 3 in tree, 4 private tail
    m.close(s1); del sh.tokens[s1]
    m.close(s2); del sh.tokens[s2]
    assert m.stats()["free"] == 3 and m.stats()["cached"] == 3    # tails returned, full blocks stay cached
    s3, cached, _ = open_full(m, sh, [7, 8, 20, 21, 22, 23, 24])  # reuses (7, 8); needs 3 more blocks: all free ones
    assert cached == 2 and m.stats()["free"] == 0
    # next allocation must evict: leaves are (3, 4) [stamp of s1's close] and ... (7, 8) is pinned by s3
    s4, cached, _ = open_full(m, sh, [50, 51, 52])
    assert m.stats()["evictions"] == 2                            # (3,4) then its parent (1,2), now a leaf
    assert m.block_row(s4) == [1, 0]
    sh.check(m)
    # everything is pinned or private now: a request for more blocks than can be had fails and leaves the sequence alone
    before = (m.block_row(s4), m.length(s4))
    assert m.extend(s4, list(range(60, 80))) is False
    assert (m.block_row(s4), m.length(s4)) == before
    sh.check(m)


@pytest.mark.parametrize("seed", range(12))
def test_random_serving_traffic_keeps_every_sequence_readable(seed):
    rng = np.random.default_rng(100 + seed)
    b = int(rng.choice([2, 4, 8]))
    nblocks = int(rng.integers(24, 80))
    m, sh = S.BlockManagerOracle(nblocks, b), Shadow(nblocks, b)
    library = [list(rng.integers(0, 5, size=int(rng.integers(3, 40)))) for _ in range(6)]   # few symbols: many shared prefixes
    for _ in range(300):
        op = rng.random()
        if op < 0.35 or not sh.tokens:
            base = library[int(rng.integers(0, len(library)))]
            toks = base[:int(rng.integers(1, len(base) + 1))] + list(rng.integers(0, 5, size=int(rng.integers(0, 6))))
            res = m.open(toks)
            if res is None:
                continue
            sid, cached, copies = res
            assert 0 <= cached <= len(toks) - 1
            sh.opened(m, sid, toks, cached, copies)
            if m.extend(sid, toks[cached:]):
                sh.extended(m, sid, toks[cached:])
            else:
                m.close(sid); del sh.tokens[sid]
        elif op < 0.8:
            sid = list(sh.tokens)[int(rng.integers(0, len(sh.tokens)))]
            new = list(rng.integers(0, 5, size=int(rng.integers(1, 7))))
            if m.extend(sid, new):
                sh.extended(m, sid, new)
        else:
            sid = list(sh.tokens)[int(rng.integers(0, len(sh.tokens)))]
            m.close(sid); del sh.tokens[sid]
        owned = sh.check(m)
        st = m.stats()
        # conservation: every block is free, in the tree, or private to an open sequence -- exactly once
        private = sum(len(m.block_row(s)) for s in sh.tokens) - sum(len(m.seqs[s].path) for s in sh.tokens)
        assert st["free"] + st["cached"] + private == nblocks
