// Private layout of a plan object, shared by the host planner and the launcher.
#pragma once
#include <cstdint>
#include <utility>
#include <vector>

#include "xy_attn.h"

// Compact per-unit record read by the persistent kernel.
struct XyDevUnit {
  int32_t seq, head_begin, head_count, q_begin, q_count, kv_begin, kv_end, flags;
  int64_t ws_offset;
};

// Per-sequence record read by the kernels.
struct XyDevSeq {
  int32_t q_len, ctx_len, token_start, mask_kind;
  int64_t mask_off;
};

// Working arrays of the planner, kept between rebuilds so that planning a step allocates nothing once the
// object has seen a batch of that size.
struct XyPlanScratch {
  std::vector<xy_work_unit> fam;            // the units in the order they are made
  std::vector<int64_t> place;               // a unit's place in the order that breaks ties of the sort
  std::vector<uint64_t> key;                // a unit's cost, complemented
  std::vector<int32_t> order_tmp;
  std::vector<int32_t> order, worker_of, count, cursor, chip_of_group;
  std::vector<int64_t> group_cost, by_cost;
  std::vector<std::pair<int64_t, int32_t>> heap;
};

struct xy_attn_plan {
  xy_attn_config cfg;
  int32_t num_seqs = 0;
  int64_t total_tokens = 0;
  std::vector<xy_seq_desc> descs;
  std::vector<int32_t> token_start;
  std::vector<xy_work_unit> units;          // grouped by worker
  std::vector<int32_t> worker_offsets;      // W + 1
  std::vector<xy_merge_item> merges;
  int64_t workspace_floats = 0;
  int32_t max_merge_rows = 0;
  bool has_tree = false;
  XyPlanScratch scratch;
  // Device copy of the tables (owned): one arena on one device and a pinned staging buffer of the same size,
  // both kept and reused when the plan is rebuilt; the table pointers point into the arena.
  int device = -1;                          // device of the arena, -1 while there is none
  bool device_stale = true;                 // the host tables changed since they were last copied
  void* d_arena = nullptr;
  void* h_stage = nullptr;                  // pinned host memory the copy kernel reads from
  void* h_stage_dev = nullptr;              // the same memory as the device sees it
  size_t arena_capacity = 0;
  void* copied = nullptr;                   // hipEvent_t recorded behind the last copy: the staging buffer is free again after it
  void* d_units = nullptr;
  void* d_offsets = nullptr;
  void* d_seqs = nullptr;
  void* d_merges = nullptr;
  void* d_counters = nullptr;               // XY_ASSIGN_DYNAMIC: shared-list cursor and finished-workgroup counts (null without a shared list)
};

// Implemented in the HIP translation unit; frees the arena, the staging buffer and the event.
void xy_plan_free_device(xy_attn_plan* plan);
