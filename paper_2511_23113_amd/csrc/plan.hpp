// Internal layout of a plan: host arrays built by the planner, device mirrors used by the kernels.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "dbsp.h"

struct dbsp_host_plan {
  int32_t H = 0, nQ = 0, nK = 0, block = 0;
  int32_t P = 0, mode = 0, max_item_len = 0, item_overhead = 0;
  int64_t nnz = 0;
  std::vector<int32_t> row_cnt;          // [R]
  std::vector<int64_t> blocks_per_head;  // [H]
  std::vector<int32_t> row_ptr;          // [R+1]
  std::vector<int32_t> kv_idx;           // [nnz]
  std::vector<int32_t> items;            // [n_items*4]
  std::vector<int32_t> item_slot;        // [n_items]
  std::vector<int32_t> split_rows;       // [n_split*4]
  std::vector<int32_t> empty_rows;       // [n_empty]
  std::vector<int32_t> part_ptr;         // [P+1]
  std::vector<int32_t> part_items;       // [n_items]
  std::vector<int64_t> part_load;        // [P]
  int32_t n_slots = 0;
  double rho_naive = 1.0, rho_balanced = 1.0, rho_mode = 1.0;  // rho_mode: of the placement actually used
  bool reused = false;       // the placement was carried over from a previous plan
  double rho_reuse = 0.0;    // rho_s of this mask under the previous plan's placement (0 if none was tried)
  int64_t n_items() const { return (int64_t)item_slot.size(); }
};

// Device mirror.  One pooled allocation (`blob`) holds the int32 arrays, the busy-time capture
// buffers and the split-row scratch for one batch entry at d = 128; a larger batch gets a
// separate scratch allocation on first use.
struct dbsp_device_plan {
  bool resident = false;
  int device = -1;
  unsigned char* blob = nullptr;
  size_t blob_bytes = 0;          // capacity as handed out by the pool
  void* staging = nullptr;        // pinned host copy of the uploaded part; lives as long as the plan
  size_t staging_bytes = 0;
  void* uploaded = nullptr;       // hipEvent_t: the upload has finished
  void* last_use = nullptr;       // hipEvent_t: recorded after every forward launch
  bool used = false;
  const int32_t* row_ptr = nullptr;
  const int32_t* kv_idx = nullptr;
  const int32_t* items = nullptr;
  const int32_t* item_slot = nullptr;
  const int32_t* split_rows = nullptr;
  const int32_t* empty_rows = nullptr;
  const int32_t* part_ptr = nullptr;
  const int32_t* part_items = nullptr;
  uint64_t* busy = nullptr;       // [P]
  uint32_t* hw_id = nullptr;      // [P]
  float* part_o = nullptr;        // split-row partial outputs, f32 [batches][n_slots][block][d]
  float* part_lse = nullptr;      // f32 [batches][n_slots][block]
  float* big_scratch = nullptr;   // separate allocation when the in-blob scratch is too small
  int64_t scratch_floats = 0;     // capacity of part_o in floats
  int64_t scratch_rows = 0;       // capacity of part_lse in floats
};

struct dbsp_plan {
  dbsp_host_plan host;
  mutable dbsp_device_plan dev;
  double plan_usec = 0.0;
};

// Host planner (pure integer work, no HIP).  Returns DBSP_OK or a negative status; fills `err`.
// `prev` (may be null) is a plan of the same geometry whose placement is kept if the new mask's
// rho_s under it does not exceed `reuse_threshold`.
int dbsp_build_host_plan(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                         int32_t P, int32_t mode, int32_t max_item_len, int32_t item_overhead,
                         int32_t locality_groups, const int32_t* partition_cost, const dbsp_host_plan* prev,
                         double reuse_threshold, dbsp_host_plan& out, std::string& err);

double dbsp_rho(const int64_t* work, int32_t periods, int32_t partitions);

// Records the calling thread's error text (returned by dbsp_last_error) and hands `code` back.
int dbsp_set_error(int code, const std::string& msg);
