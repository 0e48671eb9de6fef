// Internal layout of a plan: host arrays built by the planner, device mirrors used by the kernels.
#pragma once

#include <cstdint>
#include <functional>
#include <mutex>
#include <string>
#include <vector>

#include "dbsp.h"

struct dbsp_host_plan {
  int32_t H = 0, nQ = 0, nK = 0, block = 0;   // nQ: rows per head of the PLAN (pair mode: pairs of query blocks)
  bool pair = false;                          // pair mode: a row is two query blocks, a unit of work a pair of KV blocks
  int32_t nQ_blocks = 0;                      // query blocks per head of the MASK
  int32_t P = 0, mode = 0, max_item_len = 0, item_overhead = 0;
  int64_t nnz = 0;
  std::vector<int32_t> row_cnt;          // [R]
  std::vector<int64_t> blocks_per_head;  // [H]
  std::vector<int32_t> row_ptr;          // [R+1]
  const int32_t* kv_idx = nullptr;       // [nnz] (pair mode: [2 nnz], j0 and j1 | flags << 24 per super block): in kv_store (host-only plans) or in the plan's pinned staging buffer
  std::vector<int32_t> kv_store;
  std::vector<int32_t> items;            // [n_items*4]
  std::vector<int32_t> item_slot;        // [n_items]
  std::vector<int32_t> split_rows;       // [n_split*4]
  std::vector<int32_t> empty_rows;       // [n_empty]
  std::vector<int32_t> part_ptr;         // [P+1]
  std::vector<int32_t> part_items;       // [n_items - n_tail]
  std::vector<int32_t> tail_items;       // [n_tail]: items no partition owns; taken from a shared queue at run time
  std::vector<int64_t> part_load;        // [P]
  std::vector<int32_t> partition_cost;   // [P] or empty (unit cost): copy of the caller's array
  int32_t n_slots = 0;
  double rho_mode = 1.0;                 // rho_s of the placement actually used
  // rho_s of the naive and of the greedy placement of the same items: known at once when that is
  // the placement used, else worked out on the first dbsp_plan_stats call that asks (see dbsp_plan)
  mutable double rho_naive = 1.0, rho_balanced = 1.0;
  mutable bool have_rho_naive = false, have_rho_balanced = false;
  bool reused = false;       // the placement was carried over from a previous plan
  double rho_reuse = 0.0;    // rho_s of this mask under the previous plan's placement (0 if none was tried)
  int64_t n_items() const { return (int64_t)item_slot.size(); }
  int64_t kv_ints() const { return pair ? 2 * nnz : nnz; }   // length of kv_idx
  int32_t tile_rows() const { return pair ? 2 * block : block; }   // query rows one work item covers
};

// Device mirror.  One pooled allocation (`blob`) holds the int32 arrays, the busy-time capture
// buffers and the split-row scratch for max_batch batch entries at d = 128.
struct dbsp_device_plan {
  bool resident = false;
  int device = -1;
  unsigned char* blob = nullptr;
  size_t blob_bytes = 0;          // capacity as handed out by the pool
  void* staging = nullptr;        // pinned host copy of the uploaded small arrays; lives as long as the plan
  size_t staging_bytes = 0;
  void* staging_kv = nullptr;     // pinned host memory the index lists are compacted into (the plan's kv_idx)
  size_t staging_kv_bytes = 0;
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
  const int32_t* tail_items = nullptr;
  uint32_t* queue = nullptr;      // [2 + n_tail]: next queue position, workgroups that have left, take count per tail item
  uint64_t* busy = nullptr;       // [P]
  uint32_t* hw_id = nullptr;      // [P]
  float* part_o = nullptr;        // split-row partial outputs, f32 [batches][n_slots][block][d]
  float* part_lse = nullptr;      // f32 [batches][n_slots][block]
  int32_t max_batch = 1;          // batch entries the split-row scratch was sized for
};

struct dbsp_plan {
  dbsp_host_plan host;
  mutable dbsp_device_plan dev;
  double plan_usec = 0.0;
  mutable std::mutex lazy_mu;   // guards host.rho_naive / rho_balanced and their flags
};

// Host planner (pure integer work, no HIP), in three phases so that the caller can provide the
// destination of the index lists (pinned memory) and overlap their compaction with the placement:
//   dbsp_plan_count      per-row counts, row offsets, per-head sums, nnz
//   dbsp_compact_begin   starts writing the ascending KV block ids of every row to dst (kv_ints() + 8
//                        elements) on helper threads; dbsp_compact_end waits (true = all went well).
//                        The mask and the plan's counts must stay untouched in between.
//   dbsp_plan_place      work items, placement, per-partition lists, rho_s (needs the counts only)
// dbsp_build_host_plan runs all of them with the lists in the plan's own memory.
// All return DBSP_OK or a negative status and fill `err`.  `prev` (may be null) is a plan of the
// same geometry whose placement is kept if the new mask's rho_s under it does not exceed
// `reuse_threshold`.
struct dbsp_place_opts {
  int32_t P = 0, mode = 0, max_item_len = 0, item_overhead = 0, locality_groups = 0;
  const int32_t* partition_cost = nullptr;
  bool pair = false;          // pair mode (see dbsp_host_plan)
  int32_t dynamic_tail = 0;   // permille of the total weight left to the shared queue (round-based placement)
  double reward = 0.0;        // R_b of DBSP_MODE_REWARD
};
struct dbsp_compaction {
  std::function<void(int)> body;
  void* pool = nullptr;    // set between begin and end
  void* state = nullptr;
};
int dbsp_plan_count(const uint8_t* mask, int32_t H, int32_t nQ_blocks, int32_t nK, int32_t block, bool pair, dbsp_host_plan& out, std::string& err);
void dbsp_compact_begin(const uint8_t* mask, const dbsp_host_plan& hp, int32_t* dst, dbsp_compaction& job);
bool dbsp_compact_end(dbsp_compaction& job);
int dbsp_plan_place(const dbsp_place_opts& opts, const dbsp_host_plan* prev, double reuse_threshold,
                    dbsp_host_plan& hp, std::string& err);
int dbsp_build_host_plan(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                         const dbsp_place_opts& opts, const dbsp_host_plan* prev,
                         double reuse_threshold, dbsp_host_plan& out, std::string& err);

// rho_s of the naive and / or the greedy longest-first placement of the plan's items (each costs a placement pass).
void dbsp_host_plan_lazy_rhos(const dbsp_host_plan& hp, bool want_naive, bool want_balanced, double* rho_naive, double* rho_balanced);

double dbsp_rho(const int64_t* work, int32_t periods, int32_t partitions);

// Records the calling thread's error text (returned by dbsp_last_error) and hands `code` back.
int dbsp_set_error(int code, const std::string& msg);
