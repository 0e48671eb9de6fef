// C ABI of libdbsp: argument checks, plan life cycle, device upload, kernel launches.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "dbsp.h"
#include "fwd_params.hpp"
#include "plan.hpp"

namespace {
thread_local std::string g_err;
}

int dbsp_set_error(int code, const std::string& msg) {
  g_err = msg;
  return code;
}

namespace {

int fail(int code, const std::string& msg) { return dbsp_set_error(code, msg); }

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

// ---- process-wide resources: upload stream, device and pinned-host buffer pools -------------
// Plans are created and destroyed per attention call when masks are dynamic, so their buffers are
// recycled instead of going through hipMalloc / hipFree (which synchronises the device) each time.
// Entries remember the device that was current when they were allocated and only go back to it.
struct BufferPool {
  struct Entry { void* ptr; size_t bytes; int device; };
  std::vector<Entry> free_list;
  static constexpr size_t kMaxCached = 8;
};

constexpr int kMaxDevices = 64;
std::mutex g_mu;
hipStream_t g_upload_stream[kMaxDevices] = {};
BufferPool g_dev_pool, g_pin_pool;

hipError_t pool_get(BufferPool& pool, bool pinned, int device, size_t bytes, void** out, size_t* cap) {
  {
    std::lock_guard<std::mutex> lk(g_mu);
    int best = -1;
    for (size_t i = 0; i < pool.free_list.size(); ++i)
      if (pool.free_list[i].device == device && pool.free_list[i].bytes >= bytes &&
          (best < 0 || pool.free_list[i].bytes < pool.free_list[best].bytes))
        best = (int)i;
    if (best >= 0) {
      *out = pool.free_list[best].ptr;
      *cap = pool.free_list[best].bytes;
      pool.free_list.erase(pool.free_list.begin() + best);
      return hipSuccess;
    }
  }
  const size_t rounded = (bytes + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);   // 1 MiB granules
  hipError_t e = pinned ? hipHostMalloc(out, rounded, hipHostMallocDefault) : hipMalloc(out, rounded);
  *cap = rounded;
  return e;
}

void pool_put(BufferPool& pool, bool pinned, int device, void* ptr, size_t bytes) {
  if (!ptr) return;
  void* victim = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    pool.free_list.push_back({ptr, bytes, device});
    if (pool.free_list.size() > BufferPool::kMaxCached) {
      size_t smallest = 0;
      for (size_t i = 1; i < pool.free_list.size(); ++i)
        if (pool.free_list[i].bytes < pool.free_list[smallest].bytes) smallest = i;
      victim = pool.free_list[smallest].ptr;
      pool.free_list.erase(pool.free_list.begin() + smallest);
    }
  }
  if (victim) (void)(pinned ? hipHostFree(victim) : hipFree(victim));
}

// One upload stream per device (created on first use, with that device current).
hipError_t upload_stream(int device, hipStream_t* out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_upload_stream[device]) {
    hipError_t e = hipStreamCreateWithFlags(&g_upload_stream[device], hipStreamNonBlocking);
    if (e != hipSuccess) return e;
  }
  *out = g_upload_stream[device];
  return hipSuccess;
}

// Waits until nothing on the device still uses the plan's buffers, then recycles them.
void free_device(dbsp_device_plan& d) {
  if (d.last_use && d.used) (void)hipEventSynchronize(static_cast<hipEvent_t>(d.last_use));
  if (d.uploaded) (void)hipEventSynchronize(static_cast<hipEvent_t>(d.uploaded));
  if (d.last_use) (void)hipEventDestroy(static_cast<hipEvent_t>(d.last_use));
  if (d.uploaded) (void)hipEventDestroy(static_cast<hipEvent_t>(d.uploaded));
  pool_put(g_dev_pool, false, d.device, d.blob, d.blob_bytes);
  pool_put(g_pin_pool, true, d.device, d.staging, d.staging_bytes);
  pool_put(g_pin_pool, true, d.device, d.staging_kv, d.staging_kv_bytes);
  (void)hipGetLastError();
  d = dbsp_device_plan();
}

// Pinned memory for the index lists (the plan's kv_ints() + 8 int32): the compaction writes straight into it, it is
// the source of the upload and the plan's host copy of the lists.
int get_kv_staging(dbsp_plan* plan) {
  dbsp_device_plan& dv = plan->dev;
  DBSP_HIP(hipGetDevice(&dv.device));
  const size_t bytes = ((size_t)plan->host.kv_ints() + 8) * sizeof(int32_t);
  hipError_t e = pool_get(g_pin_pool, true, dv.device, bytes, &dv.staging_kv, &dv.staging_kv_bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return fail(DBSP_ENOMEM, std::string("plan staging buffer: ") + hipGetErrorString(e)); }
  return DBSP_OK;
}

// Copies the plan to the device: the index lists from their pinned buffer, the small arrays through
// a second pinned staging buffer, both asynchronously on the library's upload stream, and one event
// that forward launches wait for.  The host does not wait.
int upload(dbsp_plan* plan) {
  dbsp_host_plan& hp = plan->host;
  dbsp_device_plan& dv = plan->dev;
  const std::vector<int32_t>* arrays[] = {&hp.row_ptr,    &hp.items,      &hp.item_slot, &hp.split_rows,
                                          &hp.empty_rows, &hp.part_ptr,   &hp.part_items, &hp.tail_items};
  constexpr int NA = 8;
  size_t off[NA + 1];   // in int32 units, each array 16-byte aligned
  off[0] = 0;
  for (int i = 0; i < NA; ++i) off[i + 1] = off[i] + ((arrays[i]->size() + 3) & ~size_t(3));
  const size_t ints_bytes = off[NA] * sizeof(int32_t);
  const size_t busy_off = (ints_bytes + 255) & ~size_t(255);
  const size_t hw_off = busy_off + (((size_t)hp.P * sizeof(uint64_t) + 255) & ~size_t(255));
  // shared queue of the dynamic tail: [0] next position, [1] workgroups that have left, then one take count per tail item
  const size_t queue_off = hw_off + (((size_t)hp.P * sizeof(uint32_t) + 255) & ~size_t(255));
  const size_t up_bytes = queue_off + (((2 + hp.tail_items.size()) * sizeof(uint32_t) + 255) & ~size_t(255));   // staged part ends here
  const size_t kv_off = up_bytes;
  const size_t kv_bytes = (size_t)hp.kv_ints() * sizeof(int32_t);
  // split-row scratch for max_batch batch entries at d = 128
  const int64_t rows = (int64_t)dv.max_batch * hp.n_slots * hp.tile_rows();
  const size_t lse_off = (kv_off + kv_bytes + 255) & ~size_t(255);
  const size_t po_off = lse_off + (((size_t)rows * sizeof(float) + 255) & ~size_t(255));
  const size_t total = po_off + (size_t)rows * 128 * sizeof(float);

  void* blob = nullptr;
  hipError_t e = pool_get(g_dev_pool, false, dv.device, total, &blob, &dv.blob_bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return fail(DBSP_ENOMEM, std::string("plan device buffer: ") + hipGetErrorString(e)); }
  dv.blob = static_cast<unsigned char*>(blob);
  e = pool_get(g_pin_pool, true, dv.device, up_bytes, &dv.staging, &dv.staging_bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return fail(DBSP_ENOMEM, std::string("plan staging buffer: ") + hipGetErrorString(e)); }

  unsigned char* st = static_cast<unsigned char*>(dv.staging);
  for (int i = 0; i < NA; ++i)
    if (!arrays[i]->empty()) std::memcpy(st + off[i] * sizeof(int32_t), arrays[i]->data(), arrays[i]->size() * sizeof(int32_t));
  std::memset(st + busy_off, 0, up_bytes - busy_off);   // busy ticks, hardware ids, the queue's counters start at zero

  hipEvent_t ev_up, ev_use;
  DBSP_HIP(hipEventCreateWithFlags(&ev_up, hipEventDisableTiming));
  dv.uploaded = ev_up;
  DBSP_HIP(hipEventCreateWithFlags(&ev_use, hipEventDisableTiming));
  dv.last_use = ev_use;
  hipStream_t us;
  DBSP_HIP(upload_stream(dv.device, &us));
  DBSP_HIP(hipMemcpyAsync(dv.blob, st, up_bytes, hipMemcpyHostToDevice, us));
  if (kv_bytes) DBSP_HIP(hipMemcpyAsync(dv.blob + kv_off, dv.staging_kv, kv_bytes, hipMemcpyHostToDevice, us));
  DBSP_HIP(hipEventRecord(ev_up, us));

  const int32_t* ints = reinterpret_cast<const int32_t*>(dv.blob);
  dv.row_ptr = ints + off[0];
  dv.items = ints + off[1];
  dv.item_slot = ints + off[2];
  dv.split_rows = ints + off[3];
  dv.empty_rows = ints + off[4];
  dv.part_ptr = ints + off[5];
  dv.part_items = ints + off[6];
  dv.tail_items = ints + off[7];
  dv.queue = reinterpret_cast<uint32_t*>(dv.blob + queue_off);
  dv.kv_idx = reinterpret_cast<const int32_t*>(dv.blob + kv_off);
  dv.busy = reinterpret_cast<uint64_t*>(dv.blob + busy_off);
  dv.hw_id = reinterpret_cast<uint32_t*>(dv.blob + hw_off);
  dv.part_lse = reinterpret_cast<float*>(dv.blob + lse_off);
  dv.part_o = reinterpret_cast<float*>(dv.blob + po_off);
  dv.resident = true;
  return DBSP_OK;
}

// ---- scratch for callers that cannot allocate ------------------------------------------------
// The split-row partials of sparse_attn_fwd_static go here instead of into the plan's buffer.
// One copy of the array exists per GPU the library runs on, for the life of the process; every
// call on a GPU shares it.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device and used from then on.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;   // 32 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (the device must be current).
int static_scratch(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return fail(DBSP_EINVAL, "sparse_attn_fwd_static: device index out of range");
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    if (!ptr) return fail(DBSP_EHIP, "sparse_attn_fwd_static: the static scratch has no device address");
    g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return DBSP_OK;
}

}  // namespace

extern "C" {

const char* dbsp_last_error(void) { return g_err.c_str(); }

static int make_plan(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                     const dbsp_plan_opts* opts, const dbsp_plan* previous, double reuse_threshold,
                     dbsp_plan** out_plan, const char* who) {
  const auto t_start = std::chrono::steady_clock::now();
  if (out_plan) *out_plan = nullptr;
  if (!mask_host || !out_plan) return fail(DBSP_EINVAL, std::string(who) + ": null pointer");
  if (H <= 0 || nQ <= 0 || nK <= 0 || block <= 0) return fail(DBSP_EINVAL, std::string(who) + ": H, nQ, nK and block must be positive");
  if ((int64_t)H * nQ >= INT32_MAX) return fail(DBSP_EINVAL, std::string(who) + ": too many rows");
  dbsp_plan_opts o;
  std::memset(&o, 0, sizeof(o));
  if (opts) o = *opts;
  if (o.num_partitions < 0 || o.item_overhead < 0 ||
      (o.mode != DBSP_MODE_BALANCED && o.mode != DBSP_MODE_NAIVE && o.mode != DBSP_MODE_ROUNDS && o.mode != DBSP_MODE_REWARD) ||
      (o.flags & ~(DBSP_PLAN_HOST_ONLY | DBSP_PLAN_PAIR_ROWS | DBSP_PLAN_PAIR_AUTO)) || o.locality_groups < 0 || o.max_batch < 0)
    return fail(DBSP_EINVAL, std::string(who) + ": bad option (partitions < 0, overhead < 0, groups < 0, max_batch < 0, unknown mode or flag)");
  if (o.dynamic_tail < 0 || o.dynamic_tail >= 1000 || (o.dynamic_tail > 0 && o.mode != DBSP_MODE_ROUNDS))
    return fail(DBSP_EINVAL, std::string(who) + ": dynamic_tail is a permille in [0, 1000) and goes with DBSP_MODE_ROUNDS only");
  if (!(o.reward >= 0.0) || (o.reward != 0.0 && o.mode != DBSP_MODE_REWARD) || (o.mode == DBSP_MODE_REWARD && o.partition_cost))
    return fail(DBSP_EINVAL, std::string(who) + ": reward must be >= 0, goes with DBSP_MODE_REWARD only, and that mode takes no partition_cost");
  if (o.head_dim != 0 && o.head_dim != 64 && o.head_dim != 128)
    return fail(DBSP_EINVAL, std::string(who) + ": head_dim is 0 (unknown), 64 or 128");
  const bool host_only = (o.flags & DBSP_PLAN_HOST_ONLY) != 0;
  bool pair = (o.flags & DBSP_PLAN_PAIR_ROWS) != 0;
  const bool pair_auto = (o.flags & DBSP_PLAN_PAIR_AUTO) != 0;
  if (pair && pair_auto) return fail(DBSP_EINVAL, std::string(who) + ": DBSP_PLAN_PAIR_ROWS and DBSP_PLAN_PAIR_AUTO exclude each other");
  if ((pair || pair_auto) && block != 64) return fail(DBSP_EINVAL, std::string(who) + ": pair rows go with 64-token blocks");
  if (pair_auto && o.head_dim != 128) return fail(DBSP_EINVAL, std::string(who) + ": DBSP_PLAN_PAIR_AUTO needs head_dim = 128 (pair rows run at that head dim only)");
  // DBSP_PLAN_PAIR_AUTO: a chain of plans keeps the first one's choice (items of the two kinds do not
  // match each other); else both counts are taken and pair rows chosen from a flag fill of 5 / 8
  // (2 x the mask's active blocks >= 5 x the super blocks), the measured break-even
  dbsp_host_plan counted;
  bool have_counts = false;
  if (pair_auto) {
    if (previous) {
      pair = previous->host.pair;
    } else {
      std::string cerr;
      dbsp_host_plan plain;
      int rc = dbsp_plan_count(mask_host, H, nQ, nK, block, true, counted, cerr);
      if (rc == DBSP_OK) rc = dbsp_plan_count(mask_host, H, nQ, nK, block, false, plain, cerr);
      if (rc != DBSP_OK) return fail(rc, std::string(who) + ": " + cerr);
      pair = 2 * plain.nnz >= 5 * counted.nnz;
      if (!pair) counted = std::move(plain);
      have_counts = true;
    }
  }
  if (previous && previous->host.pair != pair) return fail(DBSP_ESHAPE, std::string(who) + ": the previous plan differs in DBSP_PLAN_PAIR_ROWS");
  int32_t P = o.num_partitions;
  if (P == 0 && previous) P = previous->host.P;
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
    // a 64-token block is served by a two-wave workgroup: four of them fill a compute unit at d = 64
    // (at d = 128 two are resident at a time; the plan does not know d, and an even split runs in two rounds);
    // pair rows are served by eight-wave workgroups, one per compute unit
    if (block <= 64 && !pair) P *= (o.head_dim == 128 ? 2 : 4);
  }
  if (previous && (previous->host.H != H || previous->host.nQ_blocks != nQ || previous->host.nK != nK || previous->host.P != P))
    return fail(DBSP_ESHAPE, std::string(who) + ": the previous plan has a different geometry or partition count");
  if (o.locality_groups > 1 && P % o.locality_groups != 0)
    return fail(DBSP_EINVAL, std::string(who) + ": locality_groups must divide the number of partitions");
  if (o.partition_cost)
    for (int32_t g = 0; g < P; ++g)
      if (o.partition_cost[g] <= 0) return fail(DBSP_EINVAL, std::string(who) + ": partition_cost must be positive");
  dbsp_plan* plan = new (std::nothrow) dbsp_plan();
  if (!plan) return fail(DBSP_ENOMEM, std::string(who) + ": out of host memory");
  std::string err;
  dbsp_place_opts po;
  po.P = P; po.mode = o.mode; po.max_item_len = o.max_item_len; po.item_overhead = o.item_overhead;
  po.locality_groups = o.locality_groups; po.partition_cost = o.partition_cost;
  po.dynamic_tail = o.dynamic_tail; po.reward = o.reward; po.pair = pair;
  if (host_only) {
    int rc = dbsp_build_host_plan(mask_host, H, nQ, nK, block, po, previous ? &previous->host : nullptr, reuse_threshold, plan->host, err);
    if (rc != DBSP_OK) {
      delete plan;
      return fail(rc, std::string(who) + ": " + err);
    }
  } else {
    // counts first; then the index lists are compacted into pinned memory on helper threads while
    // this thread builds the items and the placement; then everything is sent to the device
    dbsp_host_plan& hp = plan->host;
    plan->dev.max_batch = o.max_batch > 0 ? o.max_batch : 1;
    int rc = DBSP_OK;
    if (have_counts) hp = std::move(counted);
    else rc = dbsp_plan_count(mask_host, H, nQ, nK, block, pair, hp, err);
    if (rc != DBSP_OK) {
      delete plan;
      return fail(rc, std::string(who) + ": " + err);
    }
    rc = get_kv_staging(plan);
    if (rc != DBSP_OK) {
      free_device(plan->dev);
      delete plan;
      return rc;
    }
    hp.kv_idx = static_cast<const int32_t*>(plan->dev.staging_kv);
    dbsp_compaction job;
    dbsp_compact_begin(mask_host, hp, static_cast<int32_t*>(plan->dev.staging_kv), job);
    rc = dbsp_plan_place(po, previous ? &previous->host : nullptr, reuse_threshold, hp, err);
    const bool compacted = dbsp_compact_end(job);
    if (rc == DBSP_OK && !compacted) { rc = DBSP_ENOMEM; err = "out of host memory while planning"; }
    if (rc != DBSP_OK) {
      free_device(plan->dev);
      delete plan;
      return fail(rc, std::string(who) + ": " + err);
    }
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

int dbsp_plan_pair_rows(const dbsp_plan* plan, int32_t* pair_rows) {
  if (!plan || !pair_rows) return fail(DBSP_EINVAL, "dbsp_plan_pair_rows: null pointer");
  *pair_rows = plan->host.pair ? 1 : 0;
  return DBSP_OK;
}

int plan_sparse_attn(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                     const dbsp_plan_opts* opts, dbsp_plan** out_plan) {
  return make_plan(mask_host, H, nQ, nK, block, opts, nullptr, 0.0, out_plan, "plan_sparse_attn");
}

int plan_sparse_attn_reuse(const dbsp_plan* previous, const uint8_t* mask_host, const dbsp_plan_opts* opts,
                           double reuse_threshold, dbsp_plan** out_plan, int32_t* reused, double* rho_under_previous) {
  if (reused) *reused = 0;
  if (rho_under_previous) *rho_under_previous = 0.0;
  if (!previous) {
    if (out_plan) *out_plan = nullptr;
    return fail(DBSP_EINVAL, "plan_sparse_attn_reuse: null previous plan");
  }
  if (!(reuse_threshold >= 1.0)) {
    if (out_plan) *out_plan = nullptr;
    return fail(DBSP_EINVAL, "plan_sparse_attn_reuse: the threshold must be at least 1");
  }
  const dbsp_host_plan& ph = previous->host;
  int rc = make_plan(mask_host, ph.H, ph.nQ_blocks, ph.nK, ph.block, opts, previous, reuse_threshold, out_plan, "plan_sparse_attn_reuse");
  if (rc != DBSP_OK) return rc;
  if (reused) *reused = (*out_plan)->host.reused ? 1 : 0;
  if (rho_under_previous) *rho_under_previous = (*out_plan)->host.rho_reuse;
  return DBSP_OK;
}

void dbsp_plan_destroy(dbsp_plan* plan) {
  if (!plan) return;
  if (plan->dev.resident || plan->dev.blob) free_device(plan->dev);
  delete plan;
}

static int forward(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                   float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                   void* stream, bool static_scratch_wanted, const char* who) {
  const std::string w(who);
  if (!plan || !q || !k || !v || !o) return fail(DBSP_EINVAL, w + ": null pointer");
  const dbsp_host_plan& hp = plan->host;
  if (B <= 0) return fail(DBSP_EINVAL, w + ": B must be positive");
  if (d != 64 && d != 128) return fail(DBSP_EINVAL, w + ": head dim must be 64 or 128");
  if (hp.block != 64 && hp.block != 128) return fail(DBSP_EINVAL, w + ": the plan's block size must be 64 or 128");
  if (Nq <= 0 || Nk <= 0 || Nq % hp.block != 0 || Nk % hp.block != 0)
    return fail(DBSP_ESHAPE, w + ": sequence lengths must be positive multiples of the block size");
  if (Nq / hp.block != hp.nQ_blocks || Nk / hp.block != hp.nK)
    return fail(DBSP_ESHAPE, w + ": Nq/Nk do not match the plan's block grid");
  if (hp.pair && d != 128) return fail(DBSP_EINVAL, w + ": a plan made with DBSP_PLAN_PAIR_ROWS needs head dim 128");
  if (!plan->dev.resident) return fail(DBSP_EINVAL, w + ": the plan was built host-only");
  if (!(softmax_scale == softmax_scale)) return fail(DBSP_EINVAL, w + ": softmax_scale is NaN");
  int cur = -1;
  DBSP_HIP(hipGetDevice(&cur));
  if (cur != plan->dev.device) return fail(DBSP_EINVAL, w + ": the plan lives on another device than the current one");

  const dbsp_device_plan& dv = plan->dev;
  float* part_o = dv.part_o;
  float* part_lse = dv.part_lse;
  if (static_scratch_wanted) {
    // partial outputs f32 [B][n_slots][block][d], then their LSE f32 [B][n_slots][block]
    const size_t rows = (size_t)B * hp.n_slots * hp.tile_rows();
    const size_t lse_off = (rows * d * sizeof(float) + 255) & ~size_t(255);
    const size_t need = lse_off + rows * sizeof(float);
    if (need > kStaticScratchBytes)
      return fail(DBSP_EINVAL, w + ": the split rows of this plan need " + std::to_string(need) + " bytes of scratch for B = " +
                                   std::to_string(B) + ", the static buffer holds " + std::to_string(kStaticScratchBytes));
    unsigned char* base = nullptr;
    const int rc = static_scratch(cur, &base);
    if (rc != DBSP_OK) return rc;
    part_o = reinterpret_cast<float*>(base);
    part_lse = reinterpret_cast<float*>(base + lse_off);
  } else if (B > dv.max_batch && hp.n_slots > 0) {
    return fail(DBSP_EINVAL, w + ": B exceeds the max_batch the plan's split-row scratch was sized for");
  }

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
  p.tail_items = dv.tail_items;
  p.queue = dv.queue;
  p.n_tail = (int32_t)hp.tail_items.size();
  p.part_o = part_o;
  p.part_lse = part_lse;
  p.busy = dv.busy;
  p.hw_id = dv.hw_id;
  p.B = B; p.H = hp.H; p.nQ = hp.nQ; p.nK = hp.nK;
  p.Nq = Nq; p.Nk = Nk;
  p.n_slots = hp.n_slots;
  p.n_split = (int32_t)(hp.split_rows.size() / 4);
  p.n_empty = (int32_t)hp.empty_rows.size();
  p.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)d);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  DBSP_HIP(hipStreamWaitEvent(st, static_cast<hipEvent_t>(dv.uploaded), 0));   // the plan's upload is asynchronous
  hipError_t e = dbsp_launch_fwd(p, hp.block, d, hp.pair, hp.P, st);
  if (e != hipSuccess) return fail_hip(e, (w + " launch").c_str());
  DBSP_HIP(hipEventRecord(static_cast<hipEvent_t>(dv.last_use), st));
  plan->dev.used = true;
  return DBSP_OK;
}

int sparse_attn_fwd(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                    float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                    void* stream) {
  return forward(plan, q, k, v, o, lse, B, Nq, Nk, d, softmax_scale, stream, false, "sparse_attn_fwd");
}

int sparse_attn_fwd_static(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                           float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                           void* stream) {
  return forward(plan, q, k, v, o, lse, B, Nq, Nk, d, softmax_scale, stream, true, "sparse_attn_fwd_static");
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
    case DBSP_KV_IDX: *data = hp.kv_idx; *count = hp.kv_ints(); return DBSP_OK;
    case DBSP_ITEMS: DBSP_ARR(hp.items);
    case DBSP_ITEM_SLOT: DBSP_ARR(hp.item_slot);
    case DBSP_SPLIT_ROWS: DBSP_ARR(hp.split_rows);
    case DBSP_PART_PTR: DBSP_ARR(hp.part_ptr);
    case DBSP_PART_ITEMS: DBSP_ARR(hp.part_items);
    case DBSP_PART_LOAD: DBSP_ARR(hp.part_load);
    case DBSP_BLOCKS_PER_HEAD: DBSP_ARR(hp.blocks_per_head);
    case DBSP_ROW_CNT: DBSP_ARR(hp.row_cnt);
    case DBSP_EMPTY_ROWS: DBSP_ARR(hp.empty_rows);
    case DBSP_TAIL_ITEMS: DBSP_ARR(hp.tail_items);
    default: return fail(DBSP_EINVAL, "dbsp_plan_get: unknown array id");
  }
#undef DBSP_ARR
}

int dbsp_plan_stats(const dbsp_plan* plan, double* rho_naive, double* rho_balanced, double* rho_plan,
                    int64_t* nnz, int64_t* n_items, int32_t* num_partitions, int32_t* max_item_len,
                    double* plan_usec) {
  if (!plan) return fail(DBSP_EINVAL, "dbsp_plan_stats: null plan");
  const dbsp_host_plan& hp = plan->host;
  if (rho_naive || rho_balanced) {
    std::lock_guard<std::mutex> lk(plan->lazy_mu);
    const bool need_n = rho_naive && !hp.have_rho_naive, need_b = rho_balanced && !hp.have_rho_balanced;
    if (need_n || need_b) {
      try {
        dbsp_host_plan_lazy_rhos(hp, need_n, need_b, &hp.rho_naive, &hp.rho_balanced);
      } catch (const std::bad_alloc&) {
        return fail(DBSP_ENOMEM, "dbsp_plan_stats: out of host memory");
      }
      hp.have_rho_naive = hp.have_rho_naive || need_n;
      hp.have_rho_balanced = hp.have_rho_balanced || need_b;
    }
    if (rho_naive) *rho_naive = hp.rho_naive;
    if (rho_balanced) *rho_balanced = hp.rho_balanced;
  }
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

int dbsp_plan_tail_takes(const dbsp_plan* plan, uint32_t* takes, void* stream) {
  if (!plan || !takes) return fail(DBSP_EINVAL, "dbsp_plan_tail_takes: null pointer");
  if (!plan->dev.resident) return fail(DBSP_EINVAL, "dbsp_plan_tail_takes: the plan was built host-only");
  DBSP_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  const size_t n = plan->host.tail_items.size();
  if (n) DBSP_HIP(hipMemcpy(takes, plan->dev.queue + 2, n * sizeof(uint32_t), hipMemcpyDeviceToHost));
  return DBSP_OK;
}

int dbsp_plan_calibrate(const dbsp_plan* plan, int32_t* cost, void* stream) {
  if (!plan || !cost) return fail(DBSP_EINVAL, "dbsp_plan_calibrate: null pointer");
  if (!plan->dev.resident) return fail(DBSP_EINVAL, "dbsp_plan_calibrate: the plan was built host-only");
  const int32_t P = plan->host.P;
  std::vector<uint64_t> busy(P);
  DBSP_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  DBSP_HIP(hipMemcpy(busy.data(), plan->dev.busy, P * sizeof(uint64_t), hipMemcpyDeviceToHost));
  // cost[g] = round(1024 * (busy[g] / load[g]) / (sum busy / sum load)), exact, round half up
  unsigned __int128 sb = 0, sl = 0;
  for (int32_t g = 0; g < P; ++g)
    if (busy[g] > 0 && plan->host.part_load[g] > 0) {
      sb += busy[g];
      sl += (uint64_t)plan->host.part_load[g];
    }
  for (int32_t g = 0; g < P; ++g) {
    const int64_t l = plan->host.part_load[g];
    if (busy[g] == 0 || l <= 0 || sb == 0) { cost[g] = 1024; continue; }
    const unsigned __int128 num = (unsigned __int128)busy[g] * 1024 * sl, den = (unsigned __int128)(uint64_t)l * sb;
    const unsigned __int128 q = (2 * num + den) / (2 * den);
    cost[g] = q < 512 ? 512 : q > 2048 ? 2048 : (int32_t)q;
  }
  return DBSP_OK;
}

}  // extern "C"
