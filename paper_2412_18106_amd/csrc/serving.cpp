// Host-side producers of the attention inputs (paper sections 3.1 and 4.1.1): the token-budget chunk
// scheduler and the radix-tree K/V block manager.  Integers only, no GPU.  The rules are stated in
// xy_serve.h; an independent Python implementation of the same rules is what the tests compare with,
// operation by operation.
#include <algorithm>
#include <cstdint>
#include <map>
#include <new>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

#include "xy_serve.h"

// ---- scheduler ------------------------------------------------------------------------------

extern "C" int xy_serve_schedule_chunk(int32_t token_budget, int32_t reserved, const xy_queue_entry* queue,
                                       int32_t n, xy_chunk_entry* chunk, int32_t* num_chunk) {
  if (n < 0 || !num_chunk || (n > 0 && (!queue || !chunk))) return XY_ERR_ARG;
  if (token_budget < 1 || reserved < 0 || reserved > token_budget) return XY_ERR_ARG;
  for (int32_t i = 0; i < n; ++i) {
    const xy_queue_entry& e = queue[i];
    if (e.kind != XY_PREFILL && e.kind != XY_DECODE && e.kind != XY_VERIFY) return XY_ERR_ARG;
    if (e.tokens < 1 || e.context_len < 0 || (e.kind == XY_DECODE && e.tokens != 1)) return XY_ERR_ARG;
  }
  try {
    std::vector<int32_t> take(n, 0);           // tokens granted per queue position
    std::vector<int32_t> passed;
    int64_t used = 0;
    for (int32_t i = 0; i < n; ++i) {          // 1. reserved slots for decode / verify
      if (queue[i].kind == XY_PREFILL) continue;
      if (used + queue[i].tokens <= reserved) {
        take[i] = queue[i].tokens;
        used += queue[i].tokens;
      } else {
        passed.push_back(i);
      }
    }
    for (int32_t i = 0; i < n; ++i) {          // 2. prefill takes the rest, the last one cut
      if (queue[i].kind != XY_PREFILL || used >= token_budget) continue;
      const int32_t t = (int32_t)std::min<int64_t>(queue[i].tokens, token_budget - used);
      take[i] = t;
      used += t;
      if (t < queue[i].tokens) break;
    }
    for (int32_t i : passed)                    // 3. left-over budget for what was passed over
      if (used + queue[i].tokens <= token_budget) {
        take[i] = queue[i].tokens;
        used += queue[i].tokens;
      }
    int32_t m = 0;
    for (int pass = 0; pass < 2; ++pass)        // prefill first, then decode / verify, each in queue order
      for (int32_t i = 0; i < n; ++i)
        if (take[i] > 0 && ((queue[i].kind == XY_PREFILL) == (pass == 0)))
          chunk[m++] = xy_chunk_entry{queue[i].request, queue[i].kind, take[i], queue[i].context_len};
    *num_chunk = m;
  } catch (const std::bad_alloc&) {
    return XY_ERR_NOMEM;
  }
  return XY_OK;
}

// ---- block manager ----------------------------------------------------------------------------

namespace {

struct Node {
  int32_t block = -1;
  std::vector<int32_t> key;                     // the block_size token ids this block holds
  Node* parent = nullptr;
  std::map<std::vector<int32_t>, Node*> children;
  int32_t pins = 0;
  int64_t stamp = 0;
};

struct Seq {
  std::vector<Node*> path;                      // tree blocks, root excluded
  std::vector<int32_t> priv;                    // private blocks behind the path; the last may be partly filled
  std::vector<int32_t> tail;                    // token ids in the last private block
  int64_t length = 0;
  bool inserting = true;
};

}  // namespace

struct xy_kv_manager {
  int32_t b = 0;
  int32_t num_blocks = 0;
  std::set<int32_t> free_blocks;
  Node root;
  int64_t clock = 0;
  int64_t evictions = 0;
  int64_t cached = 0;
  int32_t next_seq = 0;
  std::unordered_map<int32_t, Seq> seqs;
  std::set<std::pair<int64_t, int32_t>> evictable;           // (stamp, block) of unpinned leaves
  std::unordered_map<int32_t, Node*> node_of_block;          // tree blocks only

  static bool is_evictable(const Node* nd) { return nd->pins == 0 && nd->children.empty(); }

  // every change of pins / stamp / children of a tree node goes through one of these two
  void before_change(Node* nd) {
    if (nd != &root && is_evictable(nd)) evictable.erase(std::make_pair(nd->stamp, nd->block));
  }
  void after_change(Node* nd) {
    if (nd != &root && is_evictable(nd)) evictable.insert(std::make_pair(nd->stamp, nd->block));
  }

  int32_t allocate() {
    if (!free_blocks.empty()) {
      const int32_t blk = *free_blocks.begin();
      free_blocks.erase(free_blocks.begin());
      return blk;
    }
    if (evictable.empty()) return -1;
    const int32_t blk = evictable.begin()->second;             // smallest stamp, then lowest block id
    Node* victim = node_of_block[blk];
    evictable.erase(evictable.begin());
    Node* parent = victim->parent;
    before_change(parent);
    parent->children.erase(victim->key);
    after_change(parent);
    node_of_block.erase(blk);
    delete victim;
    ++evictions;
    --cached;
    return blk;
  }

  void pin(Node* nd, int delta) {
    before_change(nd);
    nd->pins += delta;
    after_change(nd);
  }
  void touch(Node* nd) {
    before_change(nd);
    nd->stamp = clock;
    after_change(nd);
  }

  void free_tree(Node* nd) {
    for (auto& kv : nd->children) {
      free_tree(kv.second);
      delete kv.second;
    }
    nd->children.clear();
  }
};

extern "C" int xy_kv_create(int32_t num_blocks, int32_t block_size, xy_kv_manager** out) {
  if (!out || num_blocks < 1 || block_size < 1) return XY_ERR_ARG;
  *out = nullptr;
  xy_kv_manager* m = new (std::nothrow) xy_kv_manager();
  if (!m) return XY_ERR_NOMEM;
  try {
    m->b = block_size;
    m->num_blocks = num_blocks;
    for (int32_t i = 0; i < num_blocks; ++i) m->free_blocks.insert(m->free_blocks.end(), i);
  } catch (const std::bad_alloc&) {
    delete m;
    return XY_ERR_NOMEM;
  }
  *out = m;
  return XY_OK;
}

extern "C" void xy_kv_destroy(xy_kv_manager* m) {
  if (!m) return;
  m->free_tree(&m->root);
  delete m;
}

extern "C" int xy_kv_open(xy_kv_manager* m, const int32_t* tokens, int32_t n, int32_t* seq, int32_t* cached_tokens,
                          xy_kv_copy* copy, int32_t* num_copies) {
  if (!m || !tokens || n < 1 || !seq || !cached_tokens || !copy || !num_copies) return XY_ERR_ARG;
  try {
    const int32_t b = m->b;
    Node* node = &m->root;
    std::vector<Node*> path;
    int32_t pos = 0;
    std::vector<int32_t> key((size_t)b);
    while (pos + b <= n - 1) {                  // a. whole blocks; one token stays to be computed
      key.assign(tokens + pos, tokens + pos + b);
      auto it = node->children.find(key);
      if (it == node->children.end()) break;
      node = it->second;
      path.push_back(node);
      pos += b;
    }
    Node* best = nullptr;                       // b. longest common prefix with one more block
    int32_t best_m = 0;
    const int32_t limit = std::min(b, n - 1 - pos);
    for (auto& kv : node->children) {
      Node* ch = kv.second;
      int32_t c = 0;
      while (c < limit && ch->key[c] == tokens[pos + c]) ++c;
      if (c > best_m || (c == best_m && c > 0 && ch->block < best->block)) {
        best = ch;
        best_m = c;
      }
    }
    for (Node* p : path) m->pin(p, +1);         // pinned before allocating: an eviction cannot take them
    Seq s;
    *num_copies = 0;
    if (best_m > 0) {
      m->pin(best, +1);                         // the source must survive the allocation
      const int32_t blk = m->allocate();
      m->pin(best, -1);
      if (blk < 0) {
        for (Node* p : path) m->pin(p, -1);
        return XY_ERR_CAPACITY;
      }
      *copy = xy_kv_copy{best->block, blk, best_m};
      *num_copies = 1;
      s.priv.push_back(blk);
      s.tail.assign(tokens + pos, tokens + pos + best_m);
    }
    ++m->clock;
    for (Node* p : path) m->touch(p);
    if (best_m > 0) m->touch(best);
    s.path = std::move(path);
    s.length = pos + best_m;
    const int32_t sid = m->next_seq++;
    m->seqs.emplace(sid, std::move(s));
    *seq = sid;
    *cached_tokens = pos + best_m;
  } catch (const std::bad_alloc&) {
    return XY_ERR_NOMEM;
  }
  return XY_OK;
}

extern "C" int xy_kv_extend(xy_kv_manager* m, int32_t seq, const int32_t* tokens, int32_t n) {
  if (!m || n < 0 || (n > 0 && !tokens)) return XY_ERR_ARG;
  auto it = m->seqs.find(seq);
  if (it == m->seqs.end()) return XY_ERR_ARG;
  try {
    Seq& s = it->second;
    const int32_t b = m->b;
    const int64_t room = s.priv.empty() ? 0 : b - (int64_t)s.tail.size();
    const int64_t need = n > room ? (n - room + b - 1) / b : 0;
    std::vector<int32_t> got;
    for (int64_t i = 0; i < need; ++i) {
      const int32_t blk = m->allocate();
      if (blk < 0) {
        for (int32_t g : got) m->free_blocks.insert(g);
        return XY_ERR_CAPACITY;
      }
      got.push_back(blk);
    }
    ++m->clock;
    size_t next = 0;
    for (int32_t i = 0; i < n; ++i) {
      if (s.priv.empty() || (int32_t)s.tail.size() == b) {
        s.priv.push_back(got[next++]);
        s.tail.clear();
      }
      s.tail.push_back(tokens[i]);
      ++s.length;
      if ((int32_t)s.tail.size() == b && s.inserting) {        // a full private block joins the tree
        Node* parent = s.path.empty() ? &m->root : s.path.back();
        if (s.priv.size() == 1 && parent->children.find(s.tail) == parent->children.end()) {
          Node* nd = new Node();
          nd->block = s.priv[0];
          nd->key = s.tail;
          nd->parent = parent;
          nd->pins = 1;
          nd->stamp = m->clock;
          m->before_change(parent);
          parent->children.emplace(nd->key, nd);
          m->after_change(parent);
          m->node_of_block[nd->block] = nd;
          ++m->cached;
          s.path.push_back(nd);
          s.priv.clear();
          s.tail.clear();
        } else {
          s.inserting = false;
        }
      }
    }
    for (Node* p : s.path) m->touch(p);
  } catch (const std::bad_alloc&) {
    return XY_ERR_NOMEM;
  }
  return XY_OK;
}

extern "C" int xy_kv_block_row(const xy_kv_manager* m, int32_t seq, int32_t* row, int32_t capacity,
                               int32_t* num_blocks, int32_t* length) {
  if (!m) return XY_ERR_ARG;
  auto it = m->seqs.find(seq);
  if (it == m->seqs.end()) return XY_ERR_ARG;
  const Seq& s = it->second;
  const int32_t nb = (int32_t)(s.path.size() + s.priv.size());
  if (num_blocks) *num_blocks = nb;
  if (length) *length = (int32_t)s.length;
  if (row) {
    if (capacity < nb) return XY_ERR_ARG;
    int32_t k = 0;
    for (const Node* p : s.path) row[k++] = p->block;
    for (int32_t blk : s.priv) row[k++] = blk;
  }
  return XY_OK;
}

extern "C" int xy_kv_close(xy_kv_manager* m, int32_t seq) {
  if (!m) return XY_ERR_ARG;
  auto it = m->seqs.find(seq);
  if (it == m->seqs.end()) return XY_ERR_ARG;
  ++m->clock;
  for (Node* p : it->second.path) {
    m->before_change(p);
    p->pins -= 1;
    p->stamp = m->clock;
    m->after_change(p);
  }
  for (int32_t blk : it->second.priv) m->free_blocks.insert(blk);
  m->seqs.erase(it);
  return XY_OK;
}

extern "C" int xy_kv_stats(const xy_kv_manager* m, int64_t out[4]) {
  if (!m || !out) return XY_ERR_ARG;
  out[0] = (int64_t)m->free_blocks.size();
  out[1] = m->cached;
  out[2] = m->evictions;
  out[3] = (int64_t)m->seqs.size();
  return XY_OK;
}
