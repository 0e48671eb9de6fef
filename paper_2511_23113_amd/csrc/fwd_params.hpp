// Kernel argument block of the forward pass (device pointers and sizes only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

struct dbsp_fwd_params {
  const uint16_t* q;   // bf16 [B,H,nQ*BLK,D]
  const uint16_t* k;   // bf16 [B,H,nK*BLK,D]
  const uint16_t* v;   // bf16 [B,H,nK*BLK,D]
  uint16_t* o;         // bf16 [B,H,nQ*BLK,D]
  float* lse;          // f32  [B,H,nQ*BLK] or null
  const int32_t* row_ptr;
  const int32_t* kv_idx;
  const int32_t* items;       // 4 x int32 per item
  const int32_t* item_slot;
  const int32_t* split_rows;  // 4 x int32 per split row
  const int32_t* empty_rows;
  const int32_t* part_ptr;
  const int32_t* part_items;
  const int32_t* tail_items;  // items no partition owns, in queue order
  uint32_t* queue;            // [0] next queue position, [1] workgroups that have left, [2 + t] times tail item t was taken
  float* part_o;       // f32 [B][n_slots][BLK][D]
  float* part_lse;     // f32 [B][n_slots][BLK]
  uint64_t* busy;      // [P]
  uint32_t* hw_id;     // [P]
  int32_t B, H, nQ, nK;     // nQ: rows per head of the plan (pair mode: pairs of query blocks); nK: KV blocks
  int32_t Nq, Nk;           // tokens per head
  int32_t n_slots, n_split, n_empty, n_tail;
  float scale;         // softmax scale
  float scale_log2;    // softmax scale * log2(e)
};

// Enqueues the persistent kernel (grid = P workgroups) and, if needed, the fix-up kernel.
// pair: the plan's rows are pairs of 64-token query blocks and its units pairs of 64-token KV blocks (d = 128 only).
hipError_t dbsp_launch_fwd(const dbsp_fwd_params& p, int block, int d, bool pair, int P, hipStream_t stream);
