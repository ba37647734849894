// Fuzz driver for the host-side code (planner, chunk scheduler, K/V block manager), built by the test suite with
// the host compiler under -fsanitize=address,undefined (no HIP, no GPU).  It feeds seeded random batches, queues
// and token streams through the C ABI and checks the structural invariants of what comes back; the sanitizers
// catch what the invariants cannot (reads past a vector, use after free, signed overflow).  Exit status 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <vector>

#include "xy_serve.h"

// the planner frees a plan's GPU memory through this hook; there is none here
struct xy_attn_plan;
void xy_plan_free_device(xy_attn_plan*) {}

namespace {

uint64_t g_state = 0x2412181060000001ull;
uint64_t rnd() {                       // splitmix64
  uint64_t z = (g_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}
int64_t uni(int64_t lo, int64_t hi) { return lo + (int64_t)(rnd() % (uint64_t)(hi - lo + 1)); }

#define CHECK(cond)                                                            \
  do {                                                                         \
    if (!(cond)) {                                                             \
      std::fprintf(stderr, "host_fuzz: %s failed at line %d\n", #cond, __LINE__); \
      std::exit(1);                                                            \
    }                                                                          \
  } while (0)

void check_plan(const xy_attn_plan* plan, const xy_attn_config& cfg, const std::vector<xy_seq_desc>& descs) {
  const xy_work_unit* units = nullptr;
  const int32_t* offs = nullptr;
  const xy_merge_item* merges = nullptr;
  int64_t n = 0, nm = 0;
  CHECK(xy_attn_plan_get(plan, &units, &n, &offs, &merges, &nm) == XY_OK);
  size_t ws = 0;
  CHECK(xy_attn_plan_workspace_bytes(plan, &ws) == XY_OK);
  CHECK(offs[0] == 0);
  for (int32_t w = 0; w < cfg.num_workers; ++w) CHECK(offs[w] <= offs[w + 1]);
  CHECK(offs[cfg.num_workers] <= n);
  // every (sequence, head, query token) is covered by exactly one family, whose pieces partition its K/V tiles
  std::map<std::pair<int64_t, int64_t>, std::vector<std::pair<int32_t, int32_t>>> pieces;   // (seq, head*2^20+q) -> ranges
  int64_t rows_total = 0;
  for (int64_t i = 0; i < n; ++i) {
    const xy_work_unit& u = units[i];
    CHECK(u.seq >= 0 && u.seq < (int32_t)descs.size());
    const xy_seq_desc& s = descs[u.seq];
    CHECK(u.q_begin >= 0 && u.q_count >= 1 && u.q_begin + u.q_count <= s.query_len);
    CHECK(u.head_begin >= 0 && u.head_count >= 1 && u.head_begin + u.head_count <= cfg.num_q_heads);
    CHECK((int64_t)u.q_count * u.head_count <= 256);
    CHECK(u.kv_block_begin >= 0 && u.kv_block_begin < u.kv_block_end);
    const int64_t last = s.mask_kind == XY_MASK_TREE ? (int64_t)s.context_len + s.query_len
                                                     : (int64_t)s.context_len + u.q_begin + u.q_count;
    CHECK(u.kv_block_end <= (last + 127) / 128);
    CHECK(u.split_index >= 0 && u.split_index < u.num_splits);
    CHECK((u.num_splits == 1) == (u.ws_offset < 0));
    if (u.ws_offset >= 0) CHECK((size_t)(u.ws_offset + (int64_t)u.q_count * u.head_count * 130) * 4 <= ws);
    if (u.split_index == 0) rows_total += (int64_t)u.q_count * u.head_count;
    pieces[{u.seq, ((int64_t)u.head_begin << 20) + u.q_begin}].push_back({u.kv_block_begin, u.kv_block_end});
  }
  int64_t want_rows = 0;
  for (const xy_seq_desc& s : descs) want_rows += (int64_t)s.query_len * cfg.num_q_heads;
  CHECK(rows_total == want_rows);
  for (auto& kv : pieces) {
    std::set<std::pair<int32_t, int32_t>> sorted(kv.second.begin(), kv.second.end());
    int32_t at = 0;
    for (auto& r : sorted) {
      CHECK(r.first == at);
      at = r.second;
    }
  }
  for (int64_t i = 0; i < nm; ++i) CHECK(merges[i].num_splits >= 2 && merges[i].ws_offset >= 0);
}

void fuzz_planner(int rounds) {
  xy_attn_plan* reused = nullptr;
  for (int r = 0; r < rounds; ++r) {
    const int32_t hkv = (int32_t)(1 << uni(0, 3)), group = (int32_t)(1 << uni(0, 3));
    std::vector<xy_seq_desc> descs((size_t)uni(0, 40));
    int64_t longest = 1, mask_words = 0;
    for (xy_seq_desc& s : descs) {
      const int kind = (int)uni(0, 2);
      s.kind = kind;
      s.mask_kind = XY_MASK_CAUSAL;
      s.mask_word_offset = 0;
      s.context_len = (int32_t)uni(0, uni(0, 1) ? 300 : 40000);
      if (kind == XY_PREFILL) s.query_len = (int32_t)uni(1, 1500);
      else if (kind == XY_DECODE) s.query_len = 1;
      else {
        s.query_len = (int32_t)uni(1, 64);
        if (uni(0, 1)) {
          s.mask_kind = XY_MASK_TREE;
          s.mask_word_offset = mask_words;
          mask_words += (int64_t)s.query_len * ((s.query_len + 31) / 32);
        }
      }
      longest = std::max<int64_t>(longest, (int64_t)s.context_len + s.query_len);
    }
    const int32_t bs = (int32_t)(16 << uni(0, 3));
    xy_attn_config cfg;
    CHECK(xy_attn_default_config(hkv * group, hkv, (int32_t)((longest + bs - 1) / bs), &cfg) == XY_OK);
    cfg.block_size = bs;
    const int32_t workers[] = {1, 7, 64, 256, 304};
    cfg.num_workers = workers[uni(0, 4)];
    cfg.assign_policy = (int32_t)uni(0, 2);
    const int32_t splits[] = {XY_SPLIT_AUTO, 0, 1, 3, 16};
    cfg.split_kv_blocks = splits[uni(0, 4)];
    if (uni(0, 3) == 0) cfg.cost_row_floor = 1;
    if (uni(0, 3) == 0) {
      cfg.prefill_heads_per_unit = 1;
      cfg.prefill_tile_tokens = (int32_t)uni(1, 256);
    }
    if (uni(0, 3) == 0) cfg.verify_tile_tokens = (int32_t)uni(1, 256 / group);
    xy_attn_plan* plan = nullptr;
    CHECK(xy_attn_plan_create(&cfg, descs.data(), (int32_t)descs.size(), &plan) == XY_OK && plan);
    check_plan(plan, cfg, descs);
    // the same batch in a reused object
    if (!reused) CHECK(xy_attn_plan_create(&cfg, nullptr, 0, &reused) == XY_OK);
    CHECK(xy_attn_plan_rebuild(reused, &cfg, descs.data(), (int32_t)descs.size()) == XY_OK);
    check_plan(reused, cfg, descs);
    // refused inputs leave no damage
    if (!descs.empty()) {
      std::vector<xy_seq_desc> bad = descs;
      bad[uni(0, (int64_t)bad.size() - 1)].query_len = 0;
      xy_attn_plan* none = nullptr;
      CHECK(xy_attn_plan_create(&cfg, bad.data(), (int32_t)bad.size(), &none) == XY_ERR_DESC && !none);
      CHECK(xy_attn_plan_rebuild(reused, &cfg, bad.data(), (int32_t)bad.size()) == XY_ERR_DESC);
      check_plan(reused, cfg, descs);
    }
    xy_attn_plan_destroy(plan);
  }
  xy_attn_plan_destroy(reused);
  xy_attn_plan_destroy(nullptr);
}

void fuzz_scheduler(int rounds) {
  for (int r = 0; r < rounds; ++r) {
    const int32_t budget = (int32_t)uni(1, 600), reserved = (int32_t)uni(0, budget);
    std::vector<xy_queue_entry> q((size_t)uni(0, 50));
    for (size_t i = 0; i < q.size(); ++i) {
      const int kind = (int)uni(0, 2);
      q[i] = xy_queue_entry{(int32_t)i, kind, kind == XY_DECODE ? 1 : (int32_t)uni(1, kind == XY_PREFILL ? 900 : 31),
                            (int32_t)uni(0, 5000)};
    }
    std::vector<xy_chunk_entry> chunk(q.size() + 1);
    int32_t m = -1;
    CHECK(xy_serve_schedule_chunk(budget, reserved, q.data(), (int32_t)q.size(), chunk.data(), &m) == XY_OK);
    CHECK(m >= 0 && m <= (int32_t)q.size());
    int64_t used = 0;
    std::set<int32_t> seen;
    for (int32_t i = 0; i < m; ++i) {
      const xy_chunk_entry& c = chunk[i];
      CHECK(c.request >= 0 && c.request < (int32_t)q.size() && seen.insert(c.request).second);
      const xy_queue_entry& e = q[c.request];
      CHECK(c.kind == e.kind && c.context_len == e.context_len && c.query_len >= 1 && c.query_len <= e.tokens);
      if (e.kind != XY_PREFILL) CHECK(c.query_len == e.tokens);      // only a prefill is ever cut
      used += c.query_len;
    }
    CHECK(used <= budget);
  }
  int32_t m = 0;
  CHECK(xy_serve_schedule_chunk(0, 0, nullptr, 0, nullptr, &m) == XY_ERR_ARG);
}

void fuzz_block_manager(int rounds) {
  for (int r = 0; r < rounds; ++r) {
    const int32_t bs = (int32_t)(4 << uni(0, 3)), nb = (int32_t)uni(4, 60);
    xy_kv_manager* m = nullptr;
    CHECK(xy_kv_create(nb, bs, &m) == XY_OK && m);
    std::vector<int32_t> open;
    std::map<int32_t, int32_t> length;
    for (int op = 0; op < 300; ++op) {
      const int what = (int)uni(0, 9);
      if (what < 3) {                                              // admit a prompt from a tiny vocabulary (prefixes repeat)
        std::vector<int32_t> toks((size_t)uni(1, 5 * bs));
        for (int32_t& t : toks) t = (int32_t)uni(0, 2);
        int32_t seq = -1, cached = -1, nc = -1;
        xy_kv_copy cp{};
        const int rc = xy_kv_open(m, toks.data(), (int32_t)toks.size(), &seq, &cached, &cp, &nc);
        CHECK(rc == XY_OK || rc == XY_ERR_CAPACITY);
        if (rc == XY_OK) {
          CHECK(cached >= 0 && cached < (int32_t)toks.size() && (nc == 0 || nc == 1));
          if (nc) CHECK(cp.rows >= 1 && cp.rows < bs && cp.src_block != cp.dst_block && cp.dst_block >= 0 && cp.dst_block < nb);
          open.push_back(seq);
          length[seq] = cached;
        }
      } else if (what < 8 && !open.empty()) {                      // extend a sequence
        const int32_t seq = open[uni(0, (int64_t)open.size() - 1)];
        std::vector<int32_t> toks((size_t)uni(0, 2 * bs));
        for (int32_t& t : toks) t = (int32_t)uni(0, 2);
        const int rc = xy_kv_extend(m, seq, toks.data(), (int32_t)toks.size());
        CHECK(rc == XY_OK || rc == XY_ERR_CAPACITY);
        if (rc == XY_OK) length[seq] += (int32_t)toks.size();
      } else if (!open.empty()) {                                  // close one
        const size_t k = (size_t)uni(0, (int64_t)open.size() - 1);
        CHECK(xy_kv_close(m, open[k]) == XY_OK);
        length.erase(open[k]);
        open.erase(open.begin() + (long)k);
      }
      // block rows: right length, ids in range, no private block shared between two open sequences' tails
      std::map<int32_t, int> last_block_users;
      for (int32_t seq : open) {
        int32_t nblk = -1, len = -1;
        CHECK(xy_kv_block_row(m, seq, nullptr, 0, &nblk, &len) == XY_OK);
        CHECK(len == length[seq] && nblk == (len + bs - 1) / bs);
        std::vector<int32_t> row((size_t)nblk + 1);
        CHECK(xy_kv_block_row(m, seq, row.data(), nblk, &nblk, &len) == XY_OK);
        for (int32_t b = 0; b < nblk; ++b) CHECK(row[b] >= 0 && row[b] < nb);
        if (len % bs) CHECK(++last_block_users[row[nblk - 1]] == 1);   // a partly filled block is private
      }
      int64_t st[4];
      CHECK(xy_kv_stats(m, st) == XY_OK && st[0] >= 0 && st[0] <= nb && st[3] == (int64_t)open.size());
    }
    CHECK(xy_kv_close(m, 12345) == XY_ERR_ARG);
    xy_kv_destroy(m);
  }
}

}  // namespace

int main(int argc, char** argv) {
  const int scale = argc > 1 ? std::atoi(argv[1]) : 1;
  fuzz_planner(150 * scale);
  fuzz_scheduler(400 * scale);
  fuzz_block_manager(40 * scale);
  std::puts("host_fuzz: ok");
  return 0;
}
