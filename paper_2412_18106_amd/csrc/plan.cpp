// Host planner: Token-Table -> tiling units -> Task-Table.
//
// Decomposition follows the paper's section 3.2.1 (each stage is cut into
// tileSize-token tiling blocks, each block into head units, purely logically);
// reordering follows section 3.3.1 (load = tileSize x kvLen, largest first,
// symmetric round-robin over the workers).  The K/V extent of a unit is
// mask-aware (section 4.2.2): blocks past the tile's last visible key are not
// visited.  Splitting a long decode / verify unit along K/V across workers is
// this library's addition; its partial results are merged like the paper's
// Update stage (section 4.2.1).
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <utility>

#include "plan_internal.h"

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Units visit K/V in tiles of 128 keys (the kernel's tile); a tile is 128 / block_size consecutive
// entries of the sequence's block-table row.
constexpr int64_t kKvTile = 128;
// XY_SPLIT_AUTO: units of at most kNarrowRows rows are processed one per wavefront, kNarrowSlotsPerWorker
// wavefronts per worker (the unit kernel's workgroup size / 64)
constexpr int64_t kNarrowRows = 32;
constexpr int32_t kNarrowSlotsPerWorker = 4;
constexpr int64_t kAutoSplitMin = 2, kAutoSplitPieceOverhead = 1;
// unequal families: a wavefront's share of the tiles, but at most 16 tiles while that leaves a wavefront fewer than
// two and a half pieces, at most two fifths of the share beyond (a piece costs about a tile and a half on top of
// its own, and with some three pieces per wavefront the shared list still evens out), never more than 64
constexpr int64_t kAutoSplitMaxSmall = 16, kAutoSplitMaxLarge = 64;
constexpr int32_t kAutoSplitWide = 16;
constexpr int64_t kAutoSplitWideMin = 8;      // tiles: a wide unit costs about four tiles' time around its loop
// XY_ASSIGN_DYNAMIC without a unit of more than 32 rows: a shared list only if some unit visits more tiles than this
constexpr int32_t kSharedListMinTiles = 2;
// L2 domains (XCDs) of the GPU the unit kernel is written for
constexpr int64_t kChiplets = 8;

// Token tile of a DECODE / VERIFY sequence.  XY_TILE_AUTO: the narrow tile of 32 / G tokens (32 rows, one wavefront
// per unit), except for a segment of more tokens than that on at least kWholeSegmentTiles K/V tiles: its narrow
// tiles would each stream the same K/V, so it becomes one wide unit per KV head (and per 256 / G tokens).
constexpr int64_t kWholeSegmentTiles = 32;
inline int32_t verify_tile_of(const xy_attn_config& c, const xy_seq_desc& s, int32_t group) {
  if (c.verify_tile_tokens != XY_TILE_AUTO) return c.verify_tile_tokens;
  const int32_t narrow = std::max(1, 32 / group);
  if (s.query_len <= narrow || ceil_div((int64_t)s.context_len + s.query_len, kKvTile) < kWholeSegmentTiles) return narrow;
  return std::min(s.query_len, std::max(1, 256 / group));
}

int validate_config(const xy_attn_config& c) {
  if (c.num_q_heads < 1 || c.num_kv_heads < 1 || c.num_q_heads % c.num_kv_heads != 0) return XY_ERR_ARG;
  if (c.head_dim != 128) return XY_ERR_ARG;
  if (c.block_size != 16 && c.block_size != 32 && c.block_size != 64 && c.block_size != 128) return XY_ERR_ARG;
  if (c.max_blocks_per_seq < 1 || c.num_workers < 1) return XY_ERR_ARG;
  const int32_t group = c.num_q_heads / c.num_kv_heads;
  if (group > 256) return XY_ERR_ARG;     // a unit holds the group's heads of at least one token: rows <= 256
  if (c.prefill_tile_tokens < 1 || (c.verify_tile_tokens < 1 && c.verify_tile_tokens != XY_TILE_AUTO)) return XY_ERR_ARG;
  if (c.prefill_heads_per_unit < 1 || group % c.prefill_heads_per_unit != 0) return XY_ERR_ARG;
  if ((int64_t)c.prefill_tile_tokens * c.prefill_heads_per_unit > 256) return XY_ERR_ARG;
  if (c.verify_tile_tokens != XY_TILE_AUTO && (int64_t)c.verify_tile_tokens * group > 256) return XY_ERR_ARG;
  if ((c.split_kv_blocks < 0 && c.split_kv_blocks != XY_SPLIT_AUTO) || c.cost_row_floor < 1) return XY_ERR_ARG;
  if (c.assign_policy != XY_ASSIGN_SNAKE && c.assign_policy != XY_ASSIGN_LEAST_LOADED &&
      c.assign_policy != XY_ASSIGN_DYNAMIC)
    return XY_ERR_ARG;
  return XY_OK;
}

}  // namespace

extern "C" int xy_attn_default_config(int32_t hq, int32_t hkv, int32_t max_blocks, xy_attn_config* out) {
  if (!out || hq < 1 || hkv < 1 || hq % hkv != 0 || max_blocks < 1) return XY_ERR_ARG;
  const int32_t group = hq / hkv;
  if (group > 256) return XY_ERR_ARG;
  xy_attn_config c;
  c.num_q_heads = hq;
  c.num_kv_heads = hkv;
  c.head_dim = 128;
  c.block_size = 128;
  c.max_blocks_per_seq = max_blocks;
  c.num_workers = 256;
  c.prefill_heads_per_unit = group;
  c.prefill_tile_tokens = std::max(1, 256 / group);
  c.verify_tile_tokens = XY_TILE_AUTO;              // rows <= 32 (the bandwidth-bound unit shape) unless a long verify segment is cheaper whole
  c.split_kv_blocks = XY_SPLIT_AUTO;
  c.cost_row_floor = 128;
  c.assign_policy = XY_ASSIGN_DYNAMIC;
  *out = c;
  return XY_OK;
}

namespace {

// Everything of a plan that depends on the batch, written into an existing object (its vectors keep their
// capacity, its device arena stays).  Nothing of the object is touched before the arguments have been validated.
int build_plan(xy_attn_plan* plan, const xy_attn_config* cfg, const xy_seq_desc* descs, int32_t num_seqs) {
  if (!cfg || num_seqs < 0 || (num_seqs > 0 && !descs)) return XY_ERR_ARG;
  if (int rc = validate_config(*cfg)) return rc;
  const xy_attn_config& c = *cfg;
  const int32_t group = c.num_q_heads / c.num_kv_heads;
  const int64_t B = c.block_size, D = c.head_dim;

  // --- validate the Token-Table -------------------------------------------
  int64_t total = 0;
  for (int32_t i = 0; i < num_seqs; ++i) {
    const xy_seq_desc& s = descs[i];
    if (s.kind != XY_PREFILL && s.kind != XY_DECODE && s.kind != XY_VERIFY) return XY_ERR_DESC;
    if (s.mask_kind != XY_MASK_CAUSAL && s.mask_kind != XY_MASK_TREE) return XY_ERR_DESC;
    if (s.query_len < 1 || s.context_len < 0) return XY_ERR_DESC;
    if (s.kind == XY_DECODE && s.query_len != 1) return XY_ERR_DESC;
    if (s.mask_kind == XY_MASK_TREE && (s.kind != XY_VERIFY || s.mask_word_offset < 0 || s.query_len > 64))
      return XY_ERR_DESC;
    if (ceil_div((int64_t)s.context_len + s.query_len, B) > c.max_blocks_per_seq) return XY_ERR_CAPACITY;
    total += s.query_len;
    if (total > INT32_MAX) return XY_ERR_CAPACITY;
  }

  auto give_up = [&](int rc) {      // what is left is an empty plan
    plan->num_seqs = 0;
    plan->total_tokens = 0;
    plan->units.clear();
    plan->merges.clear();
    plan->workspace_floats = 0;
    return rc;
  };
  try {
    plan->device_stale = true;
    plan->cfg = c;
    plan->num_seqs = num_seqs;
    plan->total_tokens = total;
    if (descs != plan->descs.data()) plan->descs.assign(descs, descs + num_seqs);
    plan->token_start.resize(num_seqs);
    plan->units.clear();
    plan->merges.clear();
    plan->workspace_floats = 0;
    plan->max_merge_rows = 0;
    plan->has_tree = false;

    // --- size of the K/V split (see XY_SPLIT_AUTO) ---------------------------
    int32_t split_narrow = c.split_kv_blocks, split_wide = c.split_kv_blocks;
    int64_t wide_pieces = 1;      // XY_SPLIT_AUTO: pieces a family of more than kNarrowRows rows may be cut into
    if (c.split_kv_blocks == XY_SPLIT_AUTO) {
      // Fewer wide families than workers, and so little narrow work that the other workers would be done with
      // it before a wide family is (a prefill chunk with no or few decodes beside it): the wide families are
      // cut to fill the workers.  Loads as in the cost model, max(rows, floor) x tiles.
      int64_t wide_families = 0, wide_max = 0, narrow_total = 0;
      for (int32_t i = 0; i < num_seqs; ++i) {
        const xy_seq_desc& s = descs[i];
        const bool pre = s.kind == XY_PREFILL, tree = s.mask_kind == XY_MASK_TREE;
        const int32_t tile = pre ? c.prefill_tile_tokens : verify_tile_of(c, s, group);
        const int32_t hc = pre ? c.prefill_heads_per_unit : group;
        for (int32_t qb = 0; qb < s.query_len; qb += tile) {
          const int32_t qc = std::min(tile, s.query_len - qb);
          const int64_t rows = (int64_t)qc * hc;
          const int64_t last_excl = tree ? (int64_t)s.context_len + s.query_len : (int64_t)s.context_len + qb + qc;
          const int64_t load = std::max<int64_t>(rows, c.cost_row_floor) * ceil_div(last_excl, kKvTile);
          if (rows > kNarrowRows) {
            wide_families += c.num_q_heads / hc;
            wide_max = std::max(wide_max, load);
          } else {
            narrow_total += load * (c.num_q_heads / hc);
          }
        }
      }
      if (wide_families > 0 && wide_families < c.num_workers &&
          narrow_total * 2 < wide_max * (c.num_workers - wide_families))
        wide_pieces = c.num_workers / wide_families;
      int64_t tiles_total = 0;
      int64_t first_nb = -1;
      bool uniform = true;
      for (int32_t i = 0; i < num_seqs; ++i) {
        const xy_seq_desc& s = descs[i];
        if (s.kind == XY_PREFILL) continue;
        const bool tree = s.mask_kind == XY_MASK_TREE;
        const int32_t vtile = verify_tile_of(c, s, group);
        for (int32_t qb = 0; qb < s.query_len; qb += vtile) {
          const int32_t qc = std::min(vtile, s.query_len - qb);
          if ((int64_t)qc * group > kNarrowRows) continue;
          const int64_t last_excl = tree ? (int64_t)s.context_len + s.query_len : (int64_t)s.context_len + qb + qc;
          const int64_t nb = ceil_div(last_excl, kKvTile);
          tiles_total += nb * c.num_kv_heads;
          if (first_nb < 0) first_nb = nb;
          uniform = uniform && nb == first_nb;
        }
      }
      const int64_t slots = (int64_t)kNarrowSlotsPerWorker * c.num_workers;
      if (uniform && first_nb > 0) {
        // equal families: pieces per family that minimise (rounds of slots) x (tiles per piece + what a
        // piece costs on top of its tiles: set-up, partial result and its share of the merge, about one tile)
        const int64_t families = tiles_total / first_nb;
        int64_t best_k = 1, best = ceil_div(families, slots) * (first_nb + kAutoSplitPieceOverhead);
        for (int64_t k = 2; k <= first_nb; ++k) {
          const int64_t piece = ceil_div(first_nb, k);
          const int64_t cost = ceil_div(families * k, slots) * (piece + kAutoSplitPieceOverhead);
          if (cost < best) {
            best = cost;
            best_k = k;
          }
        }
        split_narrow = (int32_t)ceil_div(first_nb, best_k);
      } else {
        const int64_t share = ceil_div(tiles_total, slots);
        const int64_t most = std::max<int64_t>(kAutoSplitMaxSmall, std::min<int64_t>(kAutoSplitMaxLarge, 2 * share / 5));
        split_narrow = (int32_t)std::min<int64_t>(std::max<int64_t>(share, kAutoSplitMin), most);
      }
      split_wide = kAutoSplitWide;
    }

    // --- decomposition (section 3.2.1) + K/V split -------------------------
    // The units are made in the order (sequence, token tile, head group, piece); the sort below breaks ties in
    // the order (sequence, head group, token tile, piece).  A unit's place in that second order is known as soon
    // as its sequence is done (the pieces of a token tile number the same for every head group), so the units
    // can be laid out in that order by counting, and only their costs are left to sort by.
    std::vector<xy_work_unit>& fam = plan->scratch.fam;
    std::vector<int64_t>& place = plan->scratch.place;
    fam.clear();
    place.clear();
    int64_t ws = 0;
    int32_t start = 0;
    int64_t seq_base = 0;
    for (int32_t i = 0; i < num_seqs; ++i) {
      const xy_seq_desc& s = descs[i];
      plan->token_start[i] = start;
      start += s.query_len;
      const bool prefill = s.kind == XY_PREFILL;
      const bool tree = s.mask_kind == XY_MASK_TREE;
      plan->has_tree |= tree;
      const int32_t tile = prefill ? c.prefill_tile_tokens : verify_tile_of(c, s, group);
      const int32_t hc = prefill ? c.prefill_heads_per_unit : group;
      const int32_t head_groups = c.num_q_heads / hc;
      const int32_t kind_flags = s.kind | (s.mask_kind << 2);
      const size_t seq_first = fam.size();
      int64_t pieces_before = 0;            // pieces of the sequence's earlier token tiles, per head group
      for (int32_t qb = 0; qb < s.query_len; qb += tile) {
        const int32_t qc = std::min(tile, s.query_len - qb);
        const int64_t last_excl = tree ? (int64_t)s.context_len + s.query_len : (int64_t)s.context_len + qb + qc;
        const int32_t nb = (int32_t)ceil_div(last_excl, kKvTile);   // 128-key tiles, whatever the page size
        // pieces of a family and their size: the same for every head group of the token tile
        const int64_t rows = (int64_t)qc * hc;
        int32_t k = 1;
        int32_t split = rows <= kNarrowRows ? split_narrow : split_wide;
        bool may_split = !prefill;
        if (rows > kNarrowRows && wide_pieces > 1) {     // PREFILL too: nothing else would use the idle workers
          split = (int32_t)std::max<int64_t>(kAutoSplitWideMin, ceil_div(nb, wide_pieces));
          may_split = true;
        }
        if (may_split && split > 0 && nb > split) k = (nb + split - 1) / split;
        const int64_t slab = ((rows * (D + 2) + 3) / 4) * 4;   // keeps every partial 16-byte aligned
        // piece p covers tiles [floor(p nb / k), floor((p + 1) nb / k)): walked with a running remainder
        const int32_t whole = nb / k, rest = nb % k;
        const int64_t unit_rows = std::max<int64_t>(rows, c.cost_row_floor);
        const size_t at = fam.size();
        fam.resize(at + (size_t)k * head_groups);
        place.resize(fam.size());
        xy_work_unit* u = fam.data() + at;
        int64_t* where = place.data() + at;
        if (k > 1) plan->max_merge_rows = std::max<int32_t>(plan->max_merge_rows, (int32_t)rows);
        for (int32_t hb = 0, hg = 0; hb < c.num_q_heads; hb += hc, ++hg) {
          int64_t base = -1;
          if (k > 1) {
            base = ws;
            ws += (int64_t)k * slab;
            plan->merges.push_back(xy_merge_item{i, hb, hc, qb, qc, k, base});
          }
          int32_t piece_begin = 0, carry = 0;
          for (int32_t p = 0; p < k; ++p, ++u, ++where) {
            u->seq = i;
            u->head_begin = hb;
            u->head_count = hc;
            u->q_begin = qb;
            u->q_count = qc;
            u->kv_block_begin = piece_begin;
            carry += rest;
            piece_begin += whole;
            if (carry >= k) {
              carry -= k;
              ++piece_begin;
            }
            u->kv_block_end = piece_begin;
            u->split_index = p;
            u->num_splits = k;
            u->kind_flags = kind_flags;
            u->cost = unit_rows * (u->kv_block_end - u->kv_block_begin);
            u->ws_offset = k == 1 ? -1 : base + (int64_t)p * slab;
            *where = ((int64_t)hg << 32) | (pieces_before + p);      // head group, place inside it
          }
        }
        pieces_before += k;
      }
      // pieces_before is now the number of units per head group of this sequence
      if (fam.size() > (size_t)INT32_MAX) return give_up(XY_ERR_CAPACITY);      // unit numbers are 32-bit, here and in the kernels
      for (size_t x = seq_first; x < fam.size(); ++x)
        place[x] = seq_base + (place[x] >> 32) * pieces_before + (place[x] & 0xffffffff);
      seq_base += pieces_before * head_groups;
    }
    plan->workspace_floats = ws;

    // --- reordering (section 3.3.1): largest load first ---------------------
    // (cost descending, then sequence, head group, token tile, piece ascending): the units are laid out in the
    // tie order (their places) and then sorted by cost with a stable byte-wise radix sort, lowest byte first,
    // over the bytes of the cost in which any two units differ (two or three passes for real batches; a
    // comparison sort of the same list costs three to four times as much, most of it mispredicted branches).
    const size_t n = fam.size();
    std::vector<int32_t>&order = plan->scratch.order, &other = plan->scratch.order_tmp;
    std::vector<uint64_t>& key = plan->scratch.key;
    order.resize(n);
    other.resize(n);
    key.resize(n);
    uint64_t differ = 0;
    for (size_t x = 0; x < n; ++x) {
      order[place[x]] = (int32_t)x;
      key[x] = ~(uint64_t)fam[x].cost;              // ascending key = descending cost
      differ |= key[x] ^ key[0];
    }
    for (int shift = 0; shift < 64; shift += 8) {
      if (((differ >> shift) & 0xff) == 0) continue;
      size_t first[257] = {0};
      for (size_t i = 0; i < n; ++i) ++first[((key[order[i]] >> shift) & 0xff) + 1];
      for (int digit = 0; digit < 256; ++digit) first[digit + 1] += first[digit];
      for (size_t i = 0; i < n; ++i) other[first[(key[order[i]] >> shift) & 0xff]++] = order[i];
      order.swap(other);
    }

    // --- assignment onto W workers -> Task-Table -----------------------------
    // Snake: the paper's symmetric round-robin, 0..W-1 then W-1..0 and so on.  Least-loaded: the
    // same sorted list, each unit to the worker whose load so far is smallest (lowest index on
    // ties); with equal costs inside a round both give the same balance, with mixed wide and
    // narrow units only the second one compensates the heavy first round.
    // Dynamic: the wide units as in least-loaded, the narrow ones stay one sorted list for all workers,
    // unless there is nothing to even out (no wide unit and all narrow costs equal) or nothing worth it (no wide
    // unit and no narrow unit of more than kSharedListMinTiles K/V tiles: drawing such a unit from the shared
    // cursor takes about as long as the unit): then the plan is the least-loaded one.
    const int64_t W = c.num_workers;
    constexpr int32_t kShared = -1;            // worker_of value of a unit on the shared list
    std::vector<int32_t>&count = plan->scratch.count, &worker_of = plan->scratch.worker_of;
    count.assign(W, 0);
    worker_of.resize(fam.size());
    bool share = false;
    if (c.assign_policy == XY_ASSIGN_DYNAMIC) {
      int64_t narrow_cost = -1;
      int32_t longest_narrow = 0;
      bool any_wide = false, differ = false;
      for (const xy_work_unit& u : fam) {
        if ((int64_t)u.q_count * u.head_count > kNarrowRows) {
          any_wide = true;
          continue;
        }
        longest_narrow = std::max(longest_narrow, u.kv_block_end - u.kv_block_begin);
        if (narrow_cost < 0) narrow_cost = u.cost;
        else if (u.cost != narrow_cost) differ = true;
      }
      share = any_wide || (differ && longest_narrow > kSharedListMinTiles);
    }
    if (c.assign_policy == XY_ASSIGN_SNAKE) {
      for (int64_t pos = 0; pos < (int64_t)order.size(); ++pos) {
        const int64_t round = pos / W, lane = pos % W;
        worker_of[pos] = (int32_t)((round % 2 == 0) ? lane : W - 1 - lane);
      }
    } else {
      // Chiplet-aware placement of the wide units.  The unit kernel gives each of the kChiplets L2 domains a
      // contiguous range of W / kChiplets workers (when W is a multiple).  Wide units that read the same K/V -
      // the token tiles and head groups of one (sequence, KV head) - are kept on one chiplet, so that their
      // K/V stream is fetched from HBM once and found in that L2 by the others: the groups go, heaviest first,
      // to the chiplet with the least load, and a unit then to the least-loaded worker of its group's chiplet.
      // If the groups do not spread evenly (heaviest chiplet more than 3 % above the mean) they are not used.
      const int64_t per_chip = (W % kChiplets == 0) ? W / kChiplets : 0;
      std::vector<int32_t>& chip_of_group = plan->scratch.chip_of_group;
      chip_of_group.clear();
      const int64_t group_heads = c.num_q_heads / c.num_kv_heads;
      auto group_key = [&](const xy_work_unit& u) { return (int64_t)u.seq * c.num_kv_heads + u.head_begin / group_heads; };
      if (per_chip > 0) {
        const int64_t ngroups = (int64_t)num_seqs * c.num_kv_heads;
        std::vector<int64_t>& group_cost = plan->scratch.group_cost;
        group_cost.assign(ngroups, 0);
        int64_t total = 0;
        for (const xy_work_unit& u : fam)
          if ((int64_t)u.q_count * u.head_count > kNarrowRows) {
            group_cost[group_key(u)] += u.cost;
            total += u.cost;
          }
        std::vector<int64_t>& by_cost = plan->scratch.by_cost;
        by_cost.clear();
        for (int64_t g = 0; g < ngroups; ++g)
          if (group_cost[g] > 0) by_cost.push_back(g);
        std::stable_sort(by_cost.begin(), by_cost.end(),
                         [&](int64_t x, int64_t y) { return group_cost[x] > group_cost[y]; });
        chip_of_group.assign(ngroups, -1);
        std::vector<int64_t> chip_load(kChiplets, 0);
        for (int64_t g : by_cost) {
          const int64_t x = std::min_element(chip_load.begin(), chip_load.end()) - chip_load.begin();
          chip_of_group[g] = (int32_t)x;
          chip_load[x] += group_cost[g];
        }
        const int64_t heaviest = *std::max_element(chip_load.begin(), chip_load.end());
        if (heaviest * kChiplets * 100 > total * 103) chip_of_group.clear();
      }
      typedef std::pair<int64_t, int32_t> Entry;   // (load, worker): smallest load, then lowest index
      // one heap per chiplet (one in all without chiplets), side by side in one array; the least-loaded worker
      // overall is the best top.  Workers in index order with no load yet are a heap already.
      const int64_t nheaps = per_chip > 0 ? kChiplets : 1, per_heap = per_chip > 0 ? per_chip : W;
      std::vector<Entry>& heap = plan->scratch.heap;
      heap.resize(W);
      for (int32_t w = 0; w < W; ++w) heap[w] = Entry(0, w);
      auto top = [&](int64_t h) -> Entry& { return heap[h * per_heap]; };
      auto add_to_top = [&](int64_t h, int64_t cost) {        // the top worker takes a unit and sinks to its new place
        Entry* first = heap.data() + h * per_heap;
        Entry e = first[0];
        e.first += cost;
        int64_t hole = 0;
        for (;;) {
          int64_t child = 2 * hole + 1;
          if (child >= per_heap) break;
          if (child + 1 < per_heap && first[child + 1] < first[child]) ++child;
          if (!(first[child] < e)) break;
          first[hole] = first[child];
          hole = child;
        }
        first[hole] = e;
      };
      for (int64_t pos = 0; pos < (int64_t)order.size(); ++pos) {
        const xy_work_unit& u = fam[order[pos]];
        const bool narrow = (int64_t)u.q_count * u.head_count <= kNarrowRows;
        if (share && narrow) {
          worker_of[pos] = kShared;
          continue;
        }
        int64_t h = 0;
        if (!narrow && !chip_of_group.empty()) {
          h = chip_of_group[group_key(u)];
        } else {
          for (int64_t x = 1; x < nheaps; ++x)
            if (top(x) < top(h)) h = x;
        }
        worker_of[pos] = top(h).second;
        add_to_top(h, u.cost);
      }
    }
    for (int64_t pos = 0; pos < (int64_t)order.size(); ++pos)
      if (worker_of[pos] != kShared) ++count[worker_of[pos]];
    plan->worker_offsets.assign(W + 1, 0);
    for (int64_t w = 0; w < W; ++w) plan->worker_offsets[w + 1] = plan->worker_offsets[w] + count[w];
    plan->units.resize(fam.size());
    std::vector<int32_t>& cursor = plan->scratch.cursor;
    cursor.assign(plan->worker_offsets.begin(), plan->worker_offsets.end() - 1);
    int32_t shared_cursor = plan->worker_offsets[W];        // the shared list follows the workers' lists
    for (int64_t pos = 0; pos < (int64_t)order.size(); ++pos) {
      if (worker_of[pos] == kShared) plan->units[shared_cursor++] = fam[order[pos]];
      else plan->units[cursor[worker_of[pos]]++] = fam[order[pos]];
    }
  } catch (const std::bad_alloc&) {
    return give_up(XY_ERR_NOMEM);
  }
  return XY_OK;
}

}  // namespace

extern "C" int xy_attn_plan_create(const xy_attn_config* cfg, const xy_seq_desc* descs, int32_t num_seqs,
                                   xy_attn_plan** out) {
  if (!out) return XY_ERR_ARG;
  *out = nullptr;
  xy_attn_plan* plan = new (std::nothrow) xy_attn_plan();
  if (!plan) return XY_ERR_NOMEM;
  if (int rc = build_plan(plan, cfg, descs, num_seqs)) {
    delete plan;
    return rc;
  }
  *out = plan;
  return XY_OK;
}

extern "C" int xy_attn_plan_rebuild(xy_attn_plan* plan, const xy_attn_config* cfg, const xy_seq_desc* descs,
                                    int32_t num_seqs) {
  if (!plan) return XY_ERR_ARG;
  return build_plan(plan, cfg, descs, num_seqs);
}

extern "C" int xy_attn_plan_get(const xy_attn_plan* plan, const xy_work_unit** units, int64_t* num_units,
                                const int32_t** worker_offsets, const xy_merge_item** merges,
                                int64_t* num_merges) {
  if (!plan) return XY_ERR_ARG;
  if (units) *units = plan->units.data();
  if (num_units) *num_units = (int64_t)plan->units.size();
  if (worker_offsets) *worker_offsets = plan->worker_offsets.data();
  if (merges) *merges = plan->merges.data();
  if (num_merges) *num_merges = (int64_t)plan->merges.size();
  return XY_OK;
}

extern "C" int xy_attn_plan_workspace_bytes(const xy_attn_plan* plan, size_t* bytes) {
  if (!plan || !bytes) return XY_ERR_ARG;
  *bytes = (size_t)plan->workspace_floats * sizeof(float);
  return XY_OK;
}

extern "C" void xy_attn_plan_destroy(xy_attn_plan* plan) {
  if (!plan) return;
  xy_plan_free_device(plan);
  delete plan;
}

extern "C" const char* xy_attn_strerror(int status) {
  switch (status) {
    case XY_OK: return "ok";
    case XY_ERR_ARG: return "invalid argument";
    case XY_ERR_DESC: return "invalid sequence descriptor";
    case XY_ERR_CAPACITY: return "sequence exceeds block-table capacity";
    case XY_ERR_WORKSPACE: return "workspace too small or misaligned";
    case XY_ERR_HIP: return "HIP runtime error";
    case XY_ERR_NOMEM: return "out of host memory";
    default: return "unknown status";
  }
}
