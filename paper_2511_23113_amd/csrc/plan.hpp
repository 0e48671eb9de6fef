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
  int64_t n_items() const { return (int64_t)item_slot.size(); }
};

// Device mirror: one allocation holding every int32 array, plus scratch.
struct dbsp_device_plan {
  bool resident = false;
  int device = -1;
  int32_t* blob = nullptr;  // all int32 arrays back to back
  const int32_t* row_ptr = nullptr;
  const int32_t* kv_idx = nullptr;
  const int32_t* items = nullptr;
  const int32_t* item_slot = nullptr;
  const int32_t* split_rows = nullptr;
  const int32_t* empty_rows = nullptr;
  const int32_t* part_ptr = nullptr;
  const int32_t* part_items = nullptr;
  uint64_t* busy = nullptr;     // [P]
  uint32_t* hw_id = nullptr;    // [P]
  float* part_o = nullptr;      // split-row partial outputs, f32 [ws_batches][n_slots][block][ws_d]
  float* part_lse = nullptr;    // f32 [ws_batches][n_slots][block]
  int32_t ws_batches = 0, ws_d = 0;
};

struct dbsp_plan {
  dbsp_host_plan host;
  mutable dbsp_device_plan dev;
  double plan_usec = 0.0;
};

// Host planner (pure integer work, no HIP).  Returns DBSP_OK or a negative status; fills `err`.
int dbsp_build_host_plan(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                         int32_t P, int32_t mode, int32_t max_item_len, int32_t item_overhead,
                         dbsp_host_plan& out, std::string& err);

double dbsp_rho(const int64_t* work, int32_t periods, int32_t partitions);
