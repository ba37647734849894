"""Host-side producers of the attention inputs, written out rule by rule (TEST INFRASTRUCTURE ONLY).

Two pieces of the paper's serving loop sit in front of the attention kernel and
decide what it is asked to do:

* the token-wise scheduler (section 3.1): every step it picks at most a fixed
  budget of tokens from the queues -- prefill tokens, decode tokens, speculative
  (verify) tokens -- and long prompts are cut so that a chunk stays in budget;
* the K/V block manager (section 4.1.1): a radix tree whose nodes are K/V cache
  blocks; a new prompt reuses the longest cached prefix token by token, a block
  that matches only in part is continued through copy-on-write, new blocks hang
  below the block where the prompts part, and when room is needed the least
  recently used leaf blocks are evicted.

The paper gives the behaviour in prose; the rules below are the written contract
(readings of the open points are marked) that the C++ implementation reproduces
exactly, operation by operation.

Scheduler rules
---------------
Input: ``token_budget`` T, ``reserved_decode_slots`` R (0 <= R <= T) and the queue
in arrival order; an entry is ``(request, kind, tokens, context_len)`` with
``tokens`` = the rest of the prompt (PREFILL), 1 (DECODE) or the draft length
(VERIFY).
1. Decode and verify entries, in queue order, receive slots while the slots
   handed out in this pass stay <= R; an entry that does not fit in what is left
   of R is passed over (a verify segment is never cut: its tree mask is one unit).
2. Prefill entries, in queue order, receive what is left of T; the first one
   that does not fit whole is cut to the remaining budget (chunked prefill) and
   ends the pass.
3. If budget is left, the decode / verify entries passed over in 1 are visited
   again in queue order and receive slots while they fit.
The chunk lists the chosen entries in the order prefill, then decode / verify (each
in queue order), as ``(request, kind, query_len, context_len)``.
Consequences the tests pin: a chunk never exceeds T; with R > 0 a chunk made of
prefill tokens alone occurs only when no decode / verify entry is waiting that
fits R; prefill always has T - R tokens available ("prefill is prioritised").

Block manager rules
-------------------
State: ``num_blocks`` physical blocks of ``block_size`` B tokens; a free list handed
out in ascending block id; a radix tree of FULL blocks, each node keyed under its
parent by the B token ids it holds; per node a pin count and a last-use stamp
(a counter that increases with every open / extend / close call).
open(tokens):
  a. walk from the root while the next B tokens equal a child's key and at least
     one token would still be left to compute afterwards (a prompt is never
     reused whole: its last token must be run to produce an output); pin and
     stamp every node on the way;
  b. partial reuse: among the children of the last node reached, take the one with
     the longest common prefix m >= 1 with the tokens that follow (lowest block id
     among equals), again leaving at least one token to compute; if there is one,
     allocate a private block for the sequence and record the copy
     ``(src block, dst block, m rows)`` -- copy-on-write: the shared block is
     never written;
  c. the sequence now holds ``cached = full * B + m`` tokens; the caller extends it
     with the rest.
extend(seq, tokens): append token by token; when the private tail block is full
  it is inserted into the tree below the sequence's last tree node, keyed by its
  tokens, pinned by this sequence (if a node with that key already exists the
  sequence adopts nothing: it keeps its block private for good and stops
  inserting); when a new block is needed it is allocated.
allocate: lowest free block id; if none is free, evict the tree LEAF (no
  children, pin count 0) with the smallest stamp (lowest block id among equals),
  remove it from the tree and hand out its block; if there is none the operation
  fails: the sequence is left as it was, blocks already taken for this call go
  (back) to the free list, leaves evicted for it stay evicted.
close(seq): unpin the sequence's tree nodes (they stay cached), return its
  private blocks to the free list.
"""
from __future__ import annotations

PREFILL, DECODE, VERIFY = 0, 1, 2


def schedule_chunk(token_budget, reserved_decode_slots, queue):
    """queue: list of (request, kind, tokens, context_len) in arrival order.
    Returns the chunk as a list of (request, kind, query_len, context_len)."""
    t, r = int(token_budget), int(reserved_decode_slots)
    assert 0 <= r <= t
    used = 0
    dv, passed = [], []
    for e in queue:                       # rule 1
        if e[1] == PREFILL:
            continue
        if used + e[2] <= r:
            dv.append((e[0], e[1], e[2], e[3]))
            used += e[2]
        else:
            passed.append(e)
    pf = []
    for e in queue:                       # rule 2
        if e[1] != PREFILL or used >= t:
            continue
        take = min(e[2], t - used)
        pf.append((e[0], PREFILL, take, e[3]))
        used += take
        if take < e[2]:
            break
    for e in passed:                      # rule 3
        if used + e[2] <= t:
            dv.append((e[0], e[1], e[2], e[3]))
            used += e[2]
    # decode / verify entries keep queue order
    order = {e[0]: i for i, e in enumerate(queue)}
    dv.sort(key=lambda x: order[x[0]])
    return pf + dv


class _Node:
    __slots__ = ("block", "key", "parent", "children", "pins", "stamp")

    def __init__(self, block, key, parent):
        self.block, self.key, self.parent = block, key, parent
        self.children = {}
        self.pins = 0
        self.stamp = 0


class _Seq:
    __slots__ = ("path", "private", "tail_tokens", "length", "inserting")

    def __init__(self):
        self.path = []          # tree nodes, root excluded
        self.private = []       # private block ids after the path (the last one may be partly filled)
        self.tail_tokens = []   # token ids in the last private block
        self.length = 0
        self.inserting = True


class BlockManagerOracle:
    def __init__(self, num_blocks, block_size):
        self.b = int(block_size)
        self.free = list(range(int(num_blocks)))
        self.root = _Node(-1, None, None)
        self.clock = 0
        self.seqs = {}
        self.next_seq = 0
        self.evictions = 0

    # -- helpers ---------------------------------------------------------------------------
    def _leaves(self, node, out):
        for ch in node.children.values():
            if ch.children:
                self._leaves(ch, out)
            elif ch.pins == 0:
                out.append(ch)
        return out

    def _allocate(self):
        if self.free:
            self.free.sort()
            return self.free.pop(0)
        leaves = self._leaves(self.root, [])
        if not leaves:
            return None
        victim = min(leaves, key=lambda n: (n.stamp, n.block))
        del victim.parent.children[victim.key]
        self.evictions += 1
        return victim.block

    # -- operations ------------------------------------------------------------------------
    def open(self, tokens):
        """Returns (seq id, cached tokens, copies) with copies = [(src block, dst block, rows)];
        None if a block was needed and none could be had (state unchanged)."""
        tokens = [int(x) for x in tokens]
        n, b = len(tokens), self.b
        node, path, pos = self.root, [], 0
        while pos + b <= n - 1:                             # a. whole blocks, one token left to compute
            ch = node.children.get(tuple(tokens[pos:pos + b]))
            if ch is None:
                break
            path.append(ch)
            node, pos = ch, pos + b
        best, best_m = None, 0                              # b. partial block
        limit = min(b, n - 1 - pos)
        for ch in node.children.values():
            m = 0
            while m < limit and ch.key[m] == tokens[pos + m]:
                m += 1
            if m > best_m or (m == best_m and m > 0 and ch.block < best.block):
                best, best_m = ch, m
        # pin the path first so that an eviction for the copy cannot take it
        for p in path:
            p.pins += 1
        copies, private, tail = [], [], []
        if best_m > 0:
            best.pins += 1                                  # the source must survive the allocation
            blk = self._allocate()
            best.pins -= 1
            if blk is None:
                for p in path:
                    p.pins -= 1
                return None
            copies.append((best.block, blk, best_m))
            private, tail = [blk], tokens[pos:pos + best_m]
        self.clock += 1
        for p in path:
            p.stamp = self.clock
        if best_m > 0:
            best.stamp = self.clock
        s = _Seq()
        s.path, s.private, s.tail_tokens, s.length = path, private, tail, pos + best_m
        sid = self.next_seq
        self.next_seq += 1
        self.seqs[sid] = s
        return sid, s.length, copies

    def extend(self, sid, tokens):
        """Append tokens; returns True, or False (sequence unchanged) if a block could not be had."""
        s, b = self.seqs[sid], self.b
        tokens = [int(x) for x in tokens]
        # blocks needed beyond the current tail
        room = (b - len(s.tail_tokens)) if s.private else 0
        need = max(0, -(-(len(tokens) - room) // b))
        got = []
        for _ in range(need):
            blk = self._allocate()
            if blk is None:
                self.free.extend(got)          # evicted nodes stay evicted; blocks return to the free list
                return False
            got.append(blk)
        self.clock += 1
        for t in tokens:
            if not s.private or len(s.tail_tokens) == b:
                s.private.append(got.pop(0))
                s.tail_tokens = []
            s.tail_tokens.append(t)
            s.length += 1
            if len(s.tail_tokens) == b and s.inserting:     # a full private block joins the tree
                parent = s.path[-1] if s.path else self.root
                key = tuple(s.tail_tokens)
                if len(s.private) == 1 and key not in parent.children:
                    nd = _Node(s.private.pop(0), key, parent)
                    nd.pins, nd.stamp = 1, self.clock
                    parent.children[key] = nd
                    s.path.append(nd)
                    s.tail_tokens = []
                else:
                    s.inserting = False
        for p in s.path:
            p.stamp = self.clock
        return True

    def block_row(self, sid):
        s = self.seqs[sid]
        return [p.block for p in s.path] + list(s.private)

    def length(self, sid):
        return self.seqs[sid].length

    def close(self, sid):
        s = self.seqs.pop(sid)
        self.clock += 1
        for p in s.path:
            p.pins -= 1
            p.stamp = self.clock
        self.free.extend(s.private)

    def stats(self):
        def count(node):
            return sum(1 + count(ch) for ch in node.children.values())
        return {"free": len(self.free), "cached": count(self.root), "evictions": self.evictions,
                "open": len(self.seqs)}
