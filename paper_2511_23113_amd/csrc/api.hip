// C ABI of libdbsp: argument checks, plan life cycle, device upload, kernel launches.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "dbsp.h"
#include "fwd_params.hpp"
#include "plan.hpp"

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();  // clear the sticky error so that later calls report their own
  return DBSP_EHIP;
}

#define DBSP_HIP(call)                                  \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return fail_hip(e_, #call);   \
  } while (0)

void free_device(dbsp_device_plan& d) {
  if (d.blob) (void)hipFree(d.blob);
  if (d.busy) (void)hipFree(d.busy);
  if (d.hw_id) (void)hipFree(d.hw_id);
  if (d.part_o) (void)hipFree(d.part_o);
  if (d.part_lse) (void)hipFree(d.part_lse);
  d = dbsp_device_plan();
}

// Grows the split-row scratch so that it holds `batches` batch entries at head dim `d`.
int ensure_scratch(const dbsp_plan* plan, int32_t batches, int32_t d) {
  dbsp_device_plan& dv = plan->dev;
  const dbsp_host_plan& hp = plan->host;
  if (hp.n_slots == 0) return DBSP_OK;
  if (dv.part_o && (int64_t)dv.ws_batches * dv.ws_d >= (int64_t)batches * d) return DBSP_OK;
  if (dv.part_o) { (void)hipFree(dv.part_o); dv.part_o = nullptr; }
  if (dv.part_lse) { (void)hipFree(dv.part_lse); dv.part_lse = nullptr; }
  const size_t rows = (size_t)batches * hp.n_slots * hp.block;
  hipError_t e = hipMalloc(&dv.part_o, rows * d * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&dv.part_lse, rows * sizeof(float));
  if (e != hipSuccess) {
    if (dv.part_o) { (void)hipFree(dv.part_o); dv.part_o = nullptr; }
    dv.ws_batches = dv.ws_d = 0;
    (void)hipGetLastError();
    return fail(DBSP_ENOMEM, std::string("split-row scratch: ") + hipGetErrorString(e));
  }
  dv.ws_batches = batches;
  dv.ws_d = d;
  return DBSP_OK;
}

int upload(dbsp_plan* plan) {
  dbsp_host_plan& hp = plan->host;
  dbsp_device_plan& dv = plan->dev;
  DBSP_HIP(hipGetDevice(&dv.device));
  const std::vector<int32_t>* arrays[] = {&hp.row_ptr,    &hp.kv_idx,     &hp.items,    &hp.item_slot,
                                          &hp.split_rows, &hp.empty_rows, &hp.part_ptr, &hp.part_items};
  size_t off[9];
  off[0] = 0;
  for (int i = 0; i < 8; ++i) off[i + 1] = off[i] + ((arrays[i]->size() + 3) & ~size_t(3));  // keep 16-byte alignment
  std::vector<int32_t> staging(off[8] ? off[8] : 4, 0);
  for (int i = 0; i < 8; ++i)
    if (!arrays[i]->empty()) std::memcpy(staging.data() + off[i], arrays[i]->data(), arrays[i]->size() * sizeof(int32_t));
  DBSP_HIP(hipMalloc(&dv.blob, staging.size() * sizeof(int32_t)));
  DBSP_HIP(hipMemcpy(dv.blob, staging.data(), staging.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  dv.row_ptr = dv.blob + off[0];
  dv.kv_idx = dv.blob + off[1];
  dv.items = dv.blob + off[2];
  dv.item_slot = dv.blob + off[3];
  dv.split_rows = dv.blob + off[4];
  dv.empty_rows = dv.blob + off[5];
  dv.part_ptr = dv.blob + off[6];
  dv.part_items = dv.blob + off[7];
  DBSP_HIP(hipMalloc(&dv.busy, hp.P * sizeof(uint64_t)));
  DBSP_HIP(hipMalloc(&dv.hw_id, hp.P * sizeof(uint32_t)));
  DBSP_HIP(hipMemset(dv.busy, 0, hp.P * sizeof(uint64_t)));
  DBSP_HIP(hipMemset(dv.hw_id, 0, hp.P * sizeof(uint32_t)));
  dv.resident = true;
  return ensure_scratch(plan, 1, 128);
}

}  // namespace

extern "C" {

const char* dbsp_last_error(void) { return g_err.c_str(); }

int plan_sparse_attn(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                     const dbsp_plan_opts* opts, dbsp_plan** out_plan) {
  const auto t_start = std::chrono::steady_clock::now();
  if (out_plan) *out_plan = nullptr;
  if (!mask_host || !out_plan) return fail(DBSP_EINVAL, "plan_sparse_attn: null pointer");
  if (H <= 0 || nQ <= 0 || nK <= 0 || block <= 0) return fail(DBSP_EINVAL, "plan_sparse_attn: H, nQ, nK and block must be positive");
  if ((int64_t)H * nQ >= INT32_MAX) return fail(DBSP_EINVAL, "plan_sparse_attn: too many rows");
  dbsp_plan_opts o;
  std::memset(&o, 0, sizeof(o));
  if (opts) o = *opts;
  if (o.num_partitions < 0 || o.item_overhead < 0 || (o.mode != DBSP_MODE_BALANCED && o.mode != DBSP_MODE_NAIVE && o.mode != DBSP_MODE_ROUNDS) ||
      (o.flags & ~DBSP_PLAN_HOST_ONLY))
    return fail(DBSP_EINVAL, "plan_sparse_attn: bad option (partitions < 0, overhead < 0, unknown mode or flag)");
  const bool host_only = (o.flags & DBSP_PLAN_HOST_ONLY) != 0;
  int32_t P = o.num_partitions;
  if (P == 0) {
    P = 256;
    if (!host_only) {
      int dev = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        P = prop.multiProcessorCount;
      else
        (void)hipGetLastError();
    }
    // a 64-token block is served by a one-wave workgroup: four of them fill a compute unit
    if (block <= 64) P *= 4;
  }
  dbsp_plan* plan = new (std::nothrow) dbsp_plan();
  if (!plan) return fail(DBSP_ENOMEM, "plan_sparse_attn: out of host memory");
  std::string err;
  int rc = dbsp_build_host_plan(mask_host, H, nQ, nK, block, P, o.mode, o.max_item_len, o.item_overhead, plan->host, err);
  if (rc != DBSP_OK) {
    delete plan;
    return fail(rc, "plan_sparse_attn: " + err);
  }
  if (!host_only) {
    rc = upload(plan);
    if (rc != DBSP_OK) {
      free_device(plan->dev);
      delete plan;
      return rc;
    }
  }
  plan->plan_usec = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t_start).count();
  *out_plan = plan;
  return DBSP_OK;
}

void dbsp_plan_destroy(dbsp_plan* plan) {
  if (!plan) return;
  if (plan->dev.resident || plan->dev.blob) free_device(plan->dev);
  delete plan;
}

int sparse_attn_fwd(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                    float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                    void* stream) {
  if (!plan || !q || !k || !v || !o) return fail(DBSP_EINVAL, "sparse_attn_fwd: null pointer");
  const dbsp_host_plan& hp = plan->host;
  if (B <= 0) return fail(DBSP_EINVAL, "sparse_attn_fwd: B must be positive");
  if (d != 64 && d != 128) return fail(DBSP_EINVAL, "sparse_attn_fwd: head dim must be 64 or 128");
  if (hp.block != 64 && hp.block != 128) return fail(DBSP_EINVAL, "sparse_attn_fwd: the plan's block size must be 64 or 128");
  if (Nq <= 0 || Nk <= 0 || Nq % hp.block != 0 || Nk % hp.block != 0)
    return fail(DBSP_ESHAPE, "sparse_attn_fwd: sequence lengths must be positive multiples of the block size");
  if (Nq / hp.block != hp.nQ || Nk / hp.block != hp.nK)
    return fail(DBSP_ESHAPE, "sparse_attn_fwd: Nq/Nk do not match the plan's block grid");
  if (!plan->dev.resident) return fail(DBSP_EINVAL, "sparse_attn_fwd: the plan was built host-only");
  if (!(softmax_scale == softmax_scale)) return fail(DBSP_EINVAL, "sparse_attn_fwd: softmax_scale is NaN");
  int rc = ensure_scratch(plan, B, d);
  if (rc != DBSP_OK) return rc;

  const dbsp_device_plan& dv = plan->dev;
  dbsp_fwd_params p;
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.v = static_cast<const uint16_t*>(v);
  p.o = static_cast<uint16_t*>(o);
  p.lse = lse;
  p.row_ptr = dv.row_ptr;
  p.kv_idx = dv.kv_idx;
  p.items = dv.items;
  p.item_slot = dv.item_slot;
  p.split_rows = dv.split_rows;
  p.empty_rows = dv.empty_rows;
  p.part_ptr = dv.part_ptr;
  p.part_items = dv.part_items;
  p.part_o = dv.part_o;
  p.part_lse = dv.part_lse;
  p.busy = dv.busy;
  p.hw_id = dv.hw_id;
  p.B = B; p.H = hp.H; p.nQ = hp.nQ; p.nK = hp.nK;
  p.n_slots = hp.n_slots;
  p.n_split = (int32_t)(hp.split_rows.size() / 4);
  p.n_empty = (int32_t)hp.empty_rows.size();
  p.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)d);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  hipError_t e = dbsp_launch_fwd(p, hp.block, d, hp.P, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "sparse_attn_fwd launch");
  return DBSP_OK;
}

int imbalance_ratio(const int64_t* work, int32_t periods, int32_t partitions, double* rho_out) {
  if (!work || !rho_out) return fail(DBSP_EINVAL, "imbalance_ratio: null pointer");
  if (periods <= 0 || partitions <= 0) return fail(DBSP_EINVAL, "imbalance_ratio: periods and partitions must be positive");
  for (int64_t i = 0; i < (int64_t)periods * partitions; ++i)
    if (work[i] < 0) return fail(DBSP_EINVAL, "imbalance_ratio: negative work entry");
  *rho_out = dbsp_rho(work, periods, partitions);
  return DBSP_OK;
}

int dbsp_plan_get(const dbsp_plan* plan, int32_t what, const void** data, int64_t* count) {
  if (!plan || !data || !count) return fail(DBSP_EINVAL, "dbsp_plan_get: null pointer");
  const dbsp_host_plan& hp = plan->host;
#define DBSP_ARR(vec) do { *data = (vec).data(); *count = (int64_t)(vec).size(); return DBSP_OK; } while (0)
  switch (what) {
    case DBSP_ROW_PTR: DBSP_ARR(hp.row_ptr);
    case DBSP_KV_IDX: DBSP_ARR(hp.kv_idx);
    case DBSP_ITEMS: DBSP_ARR(hp.items);
    case DBSP_ITEM_SLOT: DBSP_ARR(hp.item_slot);
    case DBSP_SPLIT_ROWS: DBSP_ARR(hp.split_rows);
    case DBSP_PART_PTR: DBSP_ARR(hp.part_ptr);
    case DBSP_PART_ITEMS: DBSP_ARR(hp.part_items);
    case DBSP_PART_LOAD: DBSP_ARR(hp.part_load);
    case DBSP_BLOCKS_PER_HEAD: DBSP_ARR(hp.blocks_per_head);
    case DBSP_ROW_CNT: DBSP_ARR(hp.row_cnt);
    case DBSP_EMPTY_ROWS: DBSP_ARR(hp.empty_rows);
    default: return fail(DBSP_EINVAL, "dbsp_plan_get: unknown array id");
  }
#undef DBSP_ARR
}

int dbsp_plan_stats(const dbsp_plan* plan, double* rho_naive, double* rho_balanced, double* rho_plan,
                    int64_t* nnz, int64_t* n_items, int32_t* num_partitions, int32_t* max_item_len,
                    double* plan_usec) {
  if (!plan) return fail(DBSP_EINVAL, "dbsp_plan_stats: null plan");
  const dbsp_host_plan& hp = plan->host;
  if (rho_naive) *rho_naive = hp.rho_naive;
  if (rho_balanced) *rho_balanced = hp.rho_balanced;
  if (rho_plan) *rho_plan = hp.rho_mode;
  if (nnz) *nnz = hp.nnz;
  if (n_items) *n_items = hp.n_items();
  if (num_partitions) *num_partitions = hp.P;
  if (max_item_len) *max_item_len = hp.max_item_len;
  if (plan_usec) *plan_usec = plan->plan_usec;
  return DBSP_OK;
}

int dbsp_plan_busy(const dbsp_plan* plan, uint64_t* busy_ticks, uint32_t* hw_id, void* stream) {
  if (!plan) return fail(DBSP_EINVAL, "dbsp_plan_busy: null plan");
  if (!plan->dev.resident) return fail(DBSP_EINVAL, "dbsp_plan_busy: the plan was built host-only");
  DBSP_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  if (busy_ticks) DBSP_HIP(hipMemcpy(busy_ticks, plan->dev.busy, plan->host.P * sizeof(uint64_t), hipMemcpyDeviceToHost));
  if (hw_id) DBSP_HIP(hipMemcpy(hw_id, plan->dev.hw_id, plan->host.P * sizeof(uint32_t), hipMemcpyDeviceToHost));
  return DBSP_OK;
}

}  // extern "C"
