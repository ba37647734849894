// Private layout of a plan object, shared by the host planner and the launcher.
#pragma once
#include <cstdint>
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
  // device copies (owned; created by upload)
  int device = -1;
  void* d_units = nullptr;
  void* d_offsets = nullptr;
  void* d_seqs = nullptr;
  void* d_merges = nullptr;
  void* d_counters = nullptr;               // XY_ASSIGN_DYNAMIC: shared-list cursor and finished-workgroup counts
};

// Implemented in the HIP translation unit; frees the device copies.
void xy_plan_free_device(xy_attn_plan* plan);
