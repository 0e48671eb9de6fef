// Host planner: block-mask compaction, work items, greedy longest-first placement, rho_s.
//
// Cost model and rules come from db-SP (arXiv 2511.23113): the work of a unit is its number of
// dense mask blocks (Background, "Block-wise Sparse Attention"); rho_s is Eq. 1 (Motivation);
// placement is the greedy of "Head-level Partitioning" / Alg. 1's first loop, applied to
// (head, query block, KV range) items and P partitions instead of heads and GPUs.
// Everything here is integer arithmetic; the only floating point is the final rho_s division.

#include <emmintrin.h>   // SSE2: baseline of every x86-64 host

#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <system_error>
#include <thread>

#include "plan.hpp"

namespace {

// Bit 7 of every byte of the result is set exactly where the byte of w is nonzero.
inline uint64_t nonzero_bytes(uint64_t w) {
  const uint64_t low7 = 0x7f7f7f7f7f7f7f7fULL;
  return (((w & low7) + low7) | w) & ~low7;
}

// Number of nonzero bytes of row[0..n).
inline int32_t count_row(const uint8_t* row, int32_t n) {
  int32_t c = 0, j = 0;
  for (; j + 8 <= n; j += 8) {
    uint64_t w;
    std::memcpy(&w, row + j, 8);
    c += __builtin_popcountll(nonzero_bytes(w));
  }
  for (; j < n; ++j) c += row[j] != 0;
  return c;
}

// Table for the compaction below: byte t of entry m is the position of the t-th set bit of m.
struct CompactTable {
  uint64_t e[256];
  CompactTable() {
    for (int m = 0; m < 256; ++m) {
      uint64_t v = 0;
      int t = 0;
      for (int k = 0; k < 8; ++k)
        if (m & (1 << k)) v |= (uint64_t)k << (8 * t++);
      e[m] = v;
    }
  }
};
const CompactTable g_compact;

// Writes the ascending indices of the nonzero bytes of row[0..n) to out; returns one past the last.
// Branch-free per 8-byte word (a test per byte mispredicts all the time at 30 % density): the
// word's nonzero-byte mask selects a table entry holding the positions of its set bits, which are
// widened to 32 bits, offset and stored as 8 values; the cursor advances by the mask's popcount.
// The destination therefore needs 8 elements of slack past the last valid one.
inline int32_t* compact_row(const uint8_t* row, int32_t n, int32_t* out) {
  const __m128i zero = _mm_setzero_si128();
  int32_t j = 0;
  for (; j + 8 <= n; j += 8) {
    uint64_t w;
    std::memcpy(&w, row + j, 8);
    if (w == 0) continue;
    // bit 7 of byte k -> bit k of the top byte (the multiplier's terms never collide, so no carries)
    const uint32_t m = (uint32_t)(((nonzero_bytes(w) >> 7) * 0x0102040810204080ULL) >> 56);
    const __m128i b = _mm_cvtsi64_si128((long long)g_compact.e[m]);
    const __m128i h = _mm_unpacklo_epi8(b, zero);
    const __m128i base = _mm_set1_epi32(j);
    _mm_storeu_si128(reinterpret_cast<__m128i*>(out), _mm_add_epi32(_mm_unpacklo_epi16(h, zero), base));
    _mm_storeu_si128(reinterpret_cast<__m128i*>(out + 4), _mm_add_epi32(_mm_unpackhi_epi16(h, zero), base));
    out += __builtin_popcount(m);
  }
  for (; j < n; ++j) {
    *out = j;
    out += (row[j] != 0);
  }
  return out;
}

// Pair mode (two query blocks per row): number of KV blocks either of the two mask rows needs.
inline int32_t count_union(const uint8_t* row0, const uint8_t* row1, int32_t n) {
  if (!row1) return count_row(row0, n);
  int32_t c = 0, j = 0;
  for (; j + 8 <= n; j += 8) {
    uint64_t a, b;
    std::memcpy(&a, row0 + j, 8);
    std::memcpy(&b, row1 + j, 8);
    c += __builtin_popcountll(nonzero_bytes(a) | nonzero_bytes(b));
  }
  for (; j < n; ++j) c += (row0[j] | row1[j]) != 0;
  return c;
}

// Pair mode: the super blocks of one super-row: consecutive pairs (j0, j1) of the ascending union of
// the two rows' KV blocks, stored as j0 and j1 | flags << 24, flags bit (q + 2k) = "query block q
// needs KV block j_k".  A union of odd length ends with j1 = j0 and no flag for the second slot.
inline void compact_pair(const uint8_t* row0, const uint8_t* row1, int32_t n, int32_t* out) {
  int32_t have = -1, have_f = 0;
  for (int32_t j = 0; j < n; ++j) {
    const int32_t f = (row0[j] != 0 ? 1 : 0) | ((row1 && row1[j] != 0) ? 2 : 0);
    if (!f) continue;
    if (have < 0) { have = j; have_f = f; continue; }
    *out++ = have;
    *out++ = j | ((have_f | (f << 2)) << 24);
    have = -1;
  }
  if (have >= 0) {
    *out++ = have;
    *out++ = have | (have_f << 24);
  }
}

// Binary min-heap over partitions keyed by (load, index): the root is the least-loaded
// partition, lowest index among equals.  Only the root's key ever grows, so one sift-down
// per placement is enough.
// With per-partition costs the key is accumulated time, weight * cost, instead of weight.
struct LoadHeap {
  std::vector<int64_t> load;
  std::vector<int32_t> heap;  // partition ids
  const int32_t* cost;        // may be null (unit cost)
  LoadHeap(int32_t P, const int32_t* cost_) : load(P, 0), heap(P), cost(cost_) {
    for (int32_t g = 0; g < P; ++g) heap[g] = g;  // all loads equal: ascending ids form a valid heap
  }
  bool less(int32_t a, int32_t b) const { return load[a] < load[b] || (load[a] == load[b] && a < b); }
  int32_t place(int64_t w) {
    const int32_t g = heap[0];
    load[g] += cost ? w * cost[g] : w;
    const size_t n = heap.size();
    size_t i = 0;
    for (;;) {
      size_t l = 2 * i + 1, r = l + 1, m = i;
      if (l < n && less(heap[l], heap[m])) m = l;
      if (r < n && less(heap[r], heap[m])) m = r;
      if (m == i) break;
      std::swap(heap[i], heap[m]);
      i = m;
    }
    return g;
  }
};


// Persistent helper threads for the two row passes (starting and joining threads per plan costs
// more than the passes themselves on a 2-3 MB mask).  The pool is created on first use, lives
// until the process ends (its threads sleep on a condition variable in between) and is used by
// one planner at a time: a planner that finds it busy simply runs its passes on its own thread.
// A forked child starts a pool of its own.
class RowPool {
 public:
  static constexpr int kMaxThreads = 8;
  // Runs body(k) for k in [0, n): k = 0 on the calling thread, the rest on helpers (or on the
  // calling thread too, for helpers that could not be started).  Returns false if a body threw.
  bool run(int n, const std::function<void(int)>& body) {
    std::unique_lock<std::mutex> user(user_mu_, std::try_to_lock);
    if (!user.owns_lock() || n <= 1) return run_inline(n, body);
    ensure_workers(n - 1);
    const int helpers = std::min<int>(n - 1, (int)workers_);
    {
      std::lock_guard<std::mutex> lk(mu_);
      body_ = &body;
      job_base_ = 1;
      n_jobs_ = helpers;
      pending_ = helpers;
      failed_ = false;
      ++generation_;
    }
    cv_work_.notify_all();
    bool ok = true;
    try {
      body(0);
      for (int k = helpers + 1; k < n; ++k) body(k);
    } catch (...) { ok = false; }
    std::unique_lock<std::mutex> lk(mu_);
    cv_done_.wait(lk, [&] { return pending_ == 0; });
    body_ = nullptr;
    return ok && !failed_;
  }
  // Asynchronous form: begin() hands jobs [0, n) to helper threads and returns at once; finish()
  // runs whatever no helper took on the calling thread, waits for the helpers and reports
  // whether every job ran without throwing.  Every begin() needs its finish(), from the same
  // thread, with the same Async record (the caller's: several planners may be at it at once, and
  // only the one that found the pool free gets helpers).
  struct Async {
    const std::function<void(int)>* body = nullptr;
    int n = 0, started = 0;
    bool locked = false;
  };
  void begin(int n, const std::function<void(int)>& body, Async& a) {
    a.n = n;
    a.body = &body;
    a.started = 0;
    a.locked = n > 0 && user_mu_.try_lock();
    if (!a.locked) return;
    ensure_workers(n);
    const int helpers = std::min<int>(n, (int)workers_);
    {
      std::lock_guard<std::mutex> lk(mu_);
      body_ = &body;
      job_base_ = 0;
      n_jobs_ = helpers;
      pending_ = helpers;
      failed_ = false;
      ++generation_;
    }
    a.started = helpers;
    if (helpers) cv_work_.notify_all();
  }
  bool finish(Async& a) {
    bool ok = true;
    try {
      for (int k = a.started; k < a.n; ++k) (*a.body)(k);
    } catch (...) { ok = false; }
    if (a.locked) {
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_done_.wait(lk, [&] { return pending_ == 0; });
        body_ = nullptr;
        ok = ok && !failed_;
      }
      user_mu_.unlock();
      a.locked = false;
    }
    a.n = a.started = 0;
    return ok;
  }
  static RowPool& instance() {
    static std::mutex make_mu;
    static RowPool* pool = nullptr;
    static pid_t owner = 0;
    std::lock_guard<std::mutex> lk(make_mu);
    if (!pool || owner != getpid()) {   // first use, or first use in a forked child (the parent's threads are not there)
      pool = new RowPool();
      owner = getpid();
    }
    return *pool;
  }

 private:
  static bool run_inline(int n, const std::function<void(int)>& body) {
    try {
      for (int k = 0; k < n; ++k) body(k);
    } catch (...) { return false; }
    return true;
  }
  void ensure_workers(int want) {
    want = std::min(want, kMaxThreads);
    while ((int)workers_ < want) {
      try {
        std::thread(&RowPool::worker, this, (int)workers_).detach();
      } catch (const std::system_error&) {
        return;   // no more threads to be had: the caller takes the remaining ranges
      }
      ++workers_;
    }
  }
  void worker(int id) {
    uint64_t seen = 0;
    std::unique_lock<std::mutex> lk(mu_);
    for (;;) {
      cv_work_.wait(lk, [&] { return generation_ != seen; });
      seen = generation_;
      if (id >= n_jobs_) continue;
      const std::function<void(int)>* body = body_;
      const int job = id + job_base_;
      lk.unlock();
      bool ok = true;
      try { (*body)(job); } catch (...) { ok = false; }
      lk.lock();
      if (!ok) failed_ = true;
      if (--pending_ == 0) cv_done_.notify_all();
    }
  }
  std::mutex user_mu_, mu_;
  std::condition_variable cv_work_, cv_done_;
  const std::function<void(int)>* body_ = nullptr;
  uint64_t generation_ = 0;
  int n_jobs_ = 0, pending_ = 0, job_base_ = 0;
  size_t workers_ = 0;
  bool failed_ = false;
};

// Stable descending order of items by weight through a counting sort: weights are bounded, and
// filling each bucket in ascending id keeps ties stable.
template <class Weight>
void order_by_weight_desc(int64_t n_items, int64_t wmax, Weight weight, std::vector<int32_t>& order) {
  std::vector<int64_t> bucket_start(wmax + 2, 0);
  for (int64_t i = 0; i < n_items; ++i) bucket_start[wmax - weight(i) + 1]++;
  for (int64_t w = 0; w <= wmax; ++w) bucket_start[w + 1] += bucket_start[w];
  order.resize(n_items);
  for (int64_t i = 0; i < n_items; ++i) order[bucket_start[wmax - weight(i)]++] = (int32_t)i;
}

std::vector<int64_t> loads_of(const dbsp_host_plan& hp, const std::vector<int32_t>& assign) {
  std::vector<int64_t> ld(hp.P, 0);
  const int64_t n_items = hp.n_items();
  for (int64_t i = 0; i < n_items; ++i)
    if (assign[i] >= 0) ld[assign[i]] += hp.items[4 * i + 3] - hp.items[4 * i + 2];   // -1: left to the shared queue
  return ld;
}

// naive placement: items in generation order, contiguous runs of ceil(n_items / P)
std::vector<int32_t> place_naive(const dbsp_host_plan& hp) {
  const int64_t n_items = hp.n_items();
  std::vector<int32_t> assign(n_items);
  const int64_t run = n_items ? (n_items + hp.P - 1) / hp.P : 1;
  for (int64_t i = 0; i < n_items; ++i) assign[i] = (int32_t)(i / run);
  return assign;
}

// greedy longest-first placement (Alg. 1, first loop)
std::vector<int32_t> place_greedy(const dbsp_host_plan& hp) {
  const int64_t n_items = hp.n_items();
  std::vector<int32_t> assign(n_items), order;
  const int64_t ov = hp.item_overhead;
  auto weight = [&](int64_t i) { return (int64_t)(hp.items[4 * i + 3] - hp.items[4 * i + 2]) + ov; };
  order_by_weight_desc(n_items, (int64_t)hp.nK + ov, weight, order);
  LoadHeap heap(hp.P, hp.partition_cost.empty() ? nullptr : hp.partition_cost.data());
  for (int64_t t = 0; t < n_items; ++t) assign[order[t]] = heap.place(weight(order[t]));
  return assign;
}

// Greedy longest-first placement with the paper's reward factor R_b (Methodology, "Block-level
// Partitioning", overhead mitigation; Alg. 1, second loop) carried onto cache groups: partition p
// belongs to group p mod G, an item's home group is q_block * G / nQ (contiguous layout), and
// before the argmin the load of every partition of the home group is lowered by reward * weight
// (compared in double; ties: lowest partition index).  Inside a group the offset is the same for
// all, so the group's candidate is its least-loaded partition: one (load, index) heap per group,
// and the argmin runs over the G heap roots.
std::vector<int32_t> place_reward(const dbsp_host_plan& hp, int32_t G, double reward) {
  const int64_t n_items = hp.n_items();
  const int32_t P = hp.P, per = P / G;
  std::vector<int32_t> assign(n_items), order;
  const int64_t ov = hp.item_overhead;
  auto weight = [&](int64_t i) { return (int64_t)(hp.items[4 * i + 3] - hp.items[4 * i + 2]) + ov; };
  order_by_weight_desc(n_items, (int64_t)hp.nK + ov, weight, order);
  std::vector<int64_t> load(P, 0);
  std::vector<int32_t> heap((size_t)G * per);       // group g: heap[g*per ..], partition ids g, g+G, g+2G, ...
  for (int32_t g = 0; g < G; ++g)
    for (int32_t k = 0; k < per; ++k) heap[(size_t)g * per + k] = g + k * G;   // equal loads, ascending ids: a valid heap
  auto less = [&](int32_t a, int32_t b) { return load[a] < load[b] || (load[a] == load[b] && a < b); };
  for (int64_t t = 0; t < n_items; ++t) {
    const int32_t i = order[t];
    const int64_t w = weight(i);
    const int32_t home = (int32_t)((int64_t)hp.items[4 * (int64_t)i + 1] * G / hp.nQ);
    int32_t best_g = -1, best_p = -1;
    double best_val = 0.0;
    for (int32_t g = 0; g < G; ++g) {
      const int32_t pt = heap[(size_t)g * per];
      const double val = (double)load[pt] - (g == home ? reward * (double)w : 0.0);
      if (best_g < 0 || val < best_val || (val == best_val && pt < best_p)) { best_g = g; best_p = pt; best_val = val; }
    }
    assign[i] = best_p;
    load[best_p] += w;
    int32_t* hg = heap.data() + (size_t)best_g * per;     // only the root's key grew: one sift-down
    size_t at = 0;
    for (;;) {
      size_t l = 2 * at + 1, r = l + 1, m = at;
      if (l < (size_t)per && less(hg[l], hg[m])) m = l;
      if (r < (size_t)per && less(hg[r], hg[m])) m = r;
      if (m == at) break;
      std::swap(hg[at], hg[m]);
      at = m;
    }
  }
  return assign;
}

}  // namespace

void dbsp_host_plan_lazy_rhos(const dbsp_host_plan& hp, bool want_naive, bool want_balanced, double* rho_naive, double* rho_balanced) {
  if (want_naive) {
    const std::vector<int64_t> ld = loads_of(hp, place_naive(hp));
    *rho_naive = dbsp_rho(ld.data(), 1, hp.P);
  }
  if (want_balanced) {
    const std::vector<int64_t> ld = loads_of(hp, place_greedy(hp));
    *rho_balanced = dbsp_rho(ld.data(), 1, hp.P);
  }
}

double dbsp_rho(const int64_t* work, int32_t periods, int32_t partitions) {
  int64_t total = 0, num = 0;
  for (int32_t i = 0; i < periods; ++i) {
    int64_t mx = 0;
    for (int32_t g = 0; g < partitions; ++g) {
      const int64_t w = work[(int64_t)i * partitions + g];
      total += w;
      mx = std::max(mx, w);
    }
    num += mx;
  }
  if (total == 0) return 1.0;
  return (double)num / ((double)total / (double)partitions);
}

namespace {
int row_threads(int64_t mask_bytes) {
  if (mask_bytes < (int64_t)1 << 20) return 1;
  const unsigned hw = std::thread::hardware_concurrency();
  return (int)std::min<int64_t>(std::min<unsigned>(hw ? hw : 1, RowPool::kMaxThreads), mask_bytes >> 19);
}
}  // namespace

int dbsp_plan_count(const uint8_t* mask, int32_t H, int32_t nQ_blocks, int32_t nK, int32_t block, bool pair, dbsp_host_plan& hp, std::string& err) {
  try {
    // pair mode: a row of the plan is two query blocks of the mask, and what is counted are super
    // blocks (pairs of KV blocks of the union list)
    const int32_t nQ = pair ? (nQ_blocks + 1) / 2 : nQ_blocks;
    const int64_t R = (int64_t)H * nQ;
    if (pair && nK >= (1 << 24)) { err = "pair mode packs flags above 24 bits of a KV block id"; return DBSP_EINVAL; }
    hp.H = H; hp.nQ = nQ; hp.nK = nK; hp.block = block;
    hp.pair = pair; hp.nQ_blocks = nQ_blocks;
    // per-row counts (Alg. 1's get_blocks_per_head, kept per row), row offsets.  Rows are
    // independent: large masks are cut into contiguous row ranges, one per thread.
    hp.row_cnt.resize(R);
    hp.row_ptr.resize(R + 1);
    hp.blocks_per_head.assign(H, 0);
    const int n_thr = row_threads((int64_t)H * nQ_blocks * nK);
    const std::function<void(int)> job = [&](int k) {
      for (int64_t r = R * k / n_thr; r < R * (k + 1) / n_thr; ++r) {
        if (!pair) { hp.row_cnt[r] = count_row(mask + r * nK, nK); continue; }
        const int64_t h = r / nQ, q0 = 2 * (r % nQ);
        const uint8_t* row0 = mask + (h * nQ_blocks + q0) * nK;
        hp.row_cnt[r] = (count_union(row0, q0 + 1 < nQ_blocks ? row0 + nK : nullptr, nK) + 1) / 2;
      }
    };
    if (n_thr <= 1) job(0);
    else if (!RowPool::instance().run(n_thr, job)) { err = "out of host memory while planning"; return DBSP_ENOMEM; }
    hp.row_ptr[0] = 0;
    int64_t total = 0;
    for (int64_t r = 0; r < R; ++r) {
      total += hp.row_cnt[r];
      // offsets into the index lists are int32 (pair mode: two words per super block)
      if (total > (int64_t)INT32_MAX / (pair ? 2 : 1)) { err = "more than 2^31-1 index-list entries"; return DBSP_EINVAL; }
      hp.row_ptr[r + 1] = (int32_t)total;
      hp.blocks_per_head[r / nQ] += hp.row_cnt[r];
    }
    hp.nnz = total;
    return DBSP_OK;
  } catch (const std::bad_alloc&) {
    err = "out of host memory while planning";
    return DBSP_ENOMEM;
  }
}

// Ascending KV block ids of every row, written to dst[row_ptr[r] ...) (dst holds kv_ints() + 8 elements;
// pair mode: two words per super block at dst[2 * row_ptr[r] ...), see compact_pair).
// compact_row stores up to 8 elements past a row's end: harmless while that stays inside the
// thread's own range (later rows overwrite them) or in the slack at the very end; a row whose
// spill would reach the next thread's range goes through a bounce buffer.
void dbsp_compact_begin(const uint8_t* mask, const dbsp_host_plan& hp, int32_t* dst, dbsp_compaction& job) {
  const int64_t R = (int64_t)hp.H * hp.nQ;
  const int32_t nK = hp.nK;
  const int n_thr = row_threads((int64_t)hp.H * hp.nQ_blocks * nK);
  const dbsp_host_plan* php = &hp;
  job.body = [=](int k) {
    const dbsp_host_plan& h = *php;
    const int64_t r0 = R * k / n_thr, r1 = R * (k + 1) / n_thr;
    if (h.pair) {     // two ints per super block, written exactly: no slack between rows needed
      for (int64_t r = r0; r < r1; ++r) {
        if (!h.row_cnt[r]) continue;
        const int64_t hd = r / h.nQ, q0 = 2 * (r % h.nQ);
        const uint8_t* row0 = mask + (hd * h.nQ_blocks + q0) * nK;
        compact_pair(row0, q0 + 1 < h.nQ_blocks ? row0 + nK : nullptr, nK, dst + 2 * (int64_t)h.row_ptr[r]);
      }
      return;
    }
    std::vector<int32_t> bounce;
    for (int64_t r = r0; r < r1; ++r) {
      if (!h.row_cnt[r]) continue;
      if (r1 == R || (int64_t)h.row_ptr[r + 1] + 8 <= (int64_t)h.row_ptr[r1]) {
        compact_row(mask + r * nK, nK, dst + h.row_ptr[r]);
      } else {
        bounce.resize((size_t)nK + 8);
        compact_row(mask + r * nK, nK, bounce.data());
        std::memcpy(dst + h.row_ptr[r], bounce.data(), sizeof(int32_t) * (size_t)h.row_cnt[r]);
      }
    }
  };
  if (n_thr <= 1 && (int64_t)hp.H * hp.nQ_blocks * nK < ((int64_t)1 << 18)) {   // a small mask: done before a helper thread would have woken up
    job.pool = nullptr;
    job.body(0);
    return;
  }
  job.pool = &RowPool::instance();
  auto* async = new RowPool::Async();
  job.state = async;
  static_cast<RowPool*>(job.pool)->begin(n_thr, job.body, *async);
}

bool dbsp_compact_end(dbsp_compaction& job) {
  if (!job.pool) return true;
  auto* async = static_cast<RowPool::Async*>(job.state);
  const bool ok = static_cast<RowPool*>(job.pool)->finish(*async);
  delete async;
  job.pool = job.state = nullptr;
  return ok;
}

int dbsp_plan_place(const dbsp_place_opts& opts, const dbsp_host_plan* prev, double reuse_threshold,
                    dbsp_host_plan& hp, std::string& err) {
  try {
    const int32_t P = opts.P, mode = opts.mode, max_item_len = opts.max_item_len, item_overhead = opts.item_overhead;
    const int32_t locality_groups = opts.locality_groups;
    const int32_t* partition_cost = opts.partition_cost;
    const int32_t H = hp.H, nQ = hp.nQ, nK = hp.nK;
    const int64_t R = (int64_t)H * nQ;
    hp.P = P; hp.mode = mode; hp.item_overhead = item_overhead;
    hp.tail_items.clear();

    // split threshold
    int32_t L = max_item_len;
    if (L == 0) L = (int32_t)std::max<int64_t>(4, hp.nnz / (2 * (int64_t)P));   // half the mean partition load
    hp.max_item_len = L;

    // items in row-major order: sizes first, then indexed writes
    int64_t ni = 0, n_split = 0, n_empty = 0;
    for (int64_t r = 0; r < R; ++r) {
      const int32_t c = hp.row_cnt[r];
      if (c == 0) ++n_empty;
      else if (L < 0 || c <= L) ++ni;
      else { ni += (c + L - 1) / L; ++n_split; }
    }
    if (ni > (int64_t)INT32_MAX / 4) { err = "too many work items"; return DBSP_EINVAL; }
    hp.items.resize(4 * ni); hp.item_slot.resize(ni); hp.split_rows.resize(4 * n_split); hp.empty_rows.resize(n_empty);
    hp.n_slots = 0;
    {
      int32_t* it = hp.items.data();
      int32_t* sl = hp.item_slot.data();
      int32_t* sr = hp.split_rows.data();
      int32_t* er = hp.empty_rows.data();
      int64_t r = 0;
      for (int32_t h = 0; h < H; ++h)
        for (int32_t I = 0; I < nQ; ++I, ++r) {
          const int32_t c = hp.row_cnt[r];
          if (c == 0) { *er++ = (int32_t)r; continue; }
          if (L < 0 || c <= L) {
            it[0] = h; it[1] = I; it[2] = 0; it[3] = c;
            it += 4;
            *sl++ = -1;
            continue;
          }
          const int32_t k = (c + L - 1) / L, base = c / k, extra = c % k;
          sr[0] = (int32_t)r; sr[1] = hp.n_slots; sr[2] = k; sr[3] = 0;
          sr += 4;
          int32_t pos = 0;
          for (int32_t t = 0; t < k; ++t) {
            const int32_t len = base + (t < extra ? 1 : 0);
            it[0] = h; it[1] = I; it[2] = pos; it[3] = pos + len;
            it += 4;
            *sl++ = hp.n_slots++;
            pos += len;
          }
        }
    }
    const int64_t n_items = hp.n_items();

    // Plan reuse (paper: Methodology, "Head-level Partitioning", overhead mitigation; Alg. 1's
    // first test): keep the previous step's placement while the current mask's rho_s under it
    // stays at or below the threshold P_s.  The placement is carried over per (row, chunk index);
    // items the previous plan did not have go, in item order, to the least-loaded partition.
    std::vector<int32_t> assign_reuse;
    if (prev && prev->H == H && prev->nQ == nQ && prev->nK == nK && prev->P == P) {
      const int64_t pn = prev->n_items();
      std::vector<int32_t> prev_part(pn, -1), prev_first(R + 1, 0);   // -1: the item was in the previous plan's shared queue
      for (int32_t g = 0; g < P; ++g)
        for (int32_t k = prev->part_ptr[g]; k < prev->part_ptr[g + 1]; ++k) prev_part[prev->part_items[k]] = g;
      for (int64_t i = 0; i < pn; ++i) prev_first[(int64_t)prev->items[4 * i] * nQ + prev->items[4 * i + 1] + 1]++;
      for (int64_t r = 0; r < R; ++r) prev_first[r + 1] += prev_first[r];   // prev items of row r: [prev_first[r], prev_first[r+1])
      assign_reuse.assign(n_items, -1);
      std::vector<int64_t> load(P, 0);
      int64_t row_prev = -1, chunk = 0;
      for (int64_t i = 0; i < n_items; ++i) {
        const int64_t r = (int64_t)hp.items[4 * i] * nQ + hp.items[4 * i + 1];
        chunk = (r == row_prev) ? chunk + 1 : 0;
        row_prev = r;
        if (prev_first[r] + chunk < prev_first[r + 1] && prev_part[prev_first[r] + chunk] >= 0) {
          assign_reuse[i] = prev_part[prev_first[r] + chunk];
          load[assign_reuse[i]] += hp.items[4 * i + 3] - hp.items[4 * i + 2];
        }
      }
      for (int64_t i = 0; i < n_items; ++i) {
        if (assign_reuse[i] >= 0) continue;
        int32_t best = 0;
        for (int32_t g = 1; g < P; ++g)
          if (load[g] < load[best]) best = g;
        assign_reuse[i] = best;
        load[best] += hp.items[4 * i + 3] - hp.items[4 * i + 2];
      }
      hp.rho_reuse = dbsp_rho(load.data(), 1, P);
      hp.reused = hp.rho_reuse <= reuse_threshold;
    }

    // The placement asked for; rho_s of the other ones is worked out only when dbsp_plan_stats asks.
    hp.partition_cost.assign(partition_cost ? partition_cost : nullptr, partition_cost ? partition_cost + P : nullptr);
    std::vector<int32_t> assign_naive, assign_lpt;
    if (!hp.reused && mode == DBSP_MODE_NAIVE) assign_naive = place_naive(hp);
    if (!hp.reused && mode == DBSP_MODE_BALANCED) assign_lpt = place_greedy(hp);
    if (!hp.reused && mode == DBSP_MODE_REWARD) assign_lpt = place_reward(hp, locality_groups > 1 ? locality_groups : 1, opts.reward);

    // round-based greedy (DBSP_MODE_ROUNDS): heads in descending order of their block count
    // (the sort of Alg. 1), their items cut into consecutive rounds of P; inside a round the
    // k-th heaviest item goes to the k-th least-loaded partition.  Every partition works on the
    // same head at about the same time, which is what lets the KV blocks be reused from L2.
    std::vector<int32_t> assign_rounds, seq;
    if (mode == DBSP_MODE_ROUNDS && !hp.reused) {
      auto weight = [&](int64_t i) { return (int64_t)(hp.items[4 * i + 3] - hp.items[4 * i + 2]) + item_overhead; };
      std::vector<int32_t> head_order(H);
      for (int32_t h = 0; h < H; ++h) head_order[h] = h;
      std::stable_sort(head_order.begin(), head_order.end(),
                       [&](int32_t a, int32_t b) { return hp.blocks_per_head[a] > hp.blocks_per_head[b]; });
      std::vector<int64_t> head_begin(H + 1, 0);   // items are generated head-major
      for (int64_t i = 0; i < n_items; ++i) head_begin[hp.items[4 * i] + 1]++;
      for (int32_t h = 0; h < H; ++h) head_begin[h + 1] += head_begin[h];
      seq.reserve(n_items);
      for (int32_t h : head_order)
        for (int64_t i = head_begin[h]; i < head_begin[h + 1]; ++i) seq.push_back((int32_t)i);
      assign_rounds.assign(n_items, -1);
      // With G > 1 locality groups (partition p belongs to group p mod G: the partitions behind
      // one cache) a round is cut into G contiguous chunks of P/G items -- runs of neighbouring
      // query blocks -- and the same greedy runs one level up: heaviest chunk first, each to the
      // least-loaded group that has no chunk yet in this round.
      const int32_t G = locality_groups > 1 ? locality_groups : 1, per = P / G;
      const int64_t wmax = (int64_t)nK + item_overhead;
      std::vector<int64_t> load(P, 0), chunk_w(G), group_load(G);
      std::vector<int32_t> chunk_order(G);
      std::vector<char> taken(G);
      std::vector<int32_t> wseq(n_items);            // weights in sequence order
      for (int64_t t = 0; t < n_items; ++t) wseq[t] = (int32_t)weight(seq[t]);
      // Both orders inside a chunk -- items by weight, descending and stable; a group's partitions
      // by accumulated load, ascending and stable -- are orders of distinct integers
      // (key << 20 | position) and come from plain integer sorts.  The keys hold a position in 20
      // bits and a weight or a load above it; inputs too large for that take the comparison sorts.
      int64_t cost_max = 1;
      if (partition_cost) cost_max = *std::max_element(partition_cost, partition_cost + P);
      const bool packed_keys = per < (1 << 20) && wmax < ((int64_t)1 << 40) &&
                               (hp.nnz + (int64_t)item_overhead * n_items) < (((int64_t)1 << 43) / cost_max);
      std::vector<uint64_t> item_key(per), part_key(per);
      std::vector<int32_t> item_pos(per), part_rank(per);   // part_rank: positions k of a group's partitions (partition = g + k G), by load
      auto insertion_sort = [](auto* first, int64_t n, auto less) {
        for (int64_t a = 1; a < n; ++a) {
          auto v = first[a];
          int64_t b = a;
          for (; b > 0 && less(v, first[b - 1]); --b) first[b] = first[b - 1];
          first[b] = v;
        }
      };
      // Dynamic tail: the longest suffix of the sequence whose weight is at most dynamic_tail / 1000
      // of the total is left to a queue all partitions share (the greedy rule decided at run time,
      // with measured finishing times as the loads); the placed part is cut back to whole rounds.
      int64_t n_static = n_items;
      if (opts.dynamic_tail > 0) {
        int64_t total_w = 0;
        for (int64_t t = 0; t < n_items; ++t) total_w += wseq[t];
        const int64_t budget = total_w * opts.dynamic_tail / 1000;
        int64_t tail = 0, acc = 0;
        while (tail < n_items && acc + wseq[n_items - 1 - tail] <= budget) acc += wseq[n_items - 1 - tail++];
        if (tail > 0) {
          n_static = n_items - tail;
          n_static -= n_static % P;
        }
      }
      hp.tail_items.assign(seq.begin() + n_static, seq.end());
      for (int64_t r0 = 0; r0 < n_static; r0 += P) {
        const int64_t r1 = std::min<int64_t>(n_static, r0 + P);
        for (int32_t j = 0; j < G; ++j) {
          chunk_w[j] = 0;
          for (int64_t t = r0 + (int64_t)j * per; t < std::min<int64_t>(r1, r0 + (int64_t)(j + 1) * per); ++t) chunk_w[j] += wseq[t];
          chunk_order[j] = j;
          taken[j] = 0;
          group_load[j] = 0;
        }
        for (int32_t k = 0, p = 0; k < per; ++k)
          for (int32_t g = 0; g < G; ++g, ++p) group_load[g] += load[p];
        // heaviest chunk first, stable (insertion sort is stable)
        insertion_sort(chunk_order.data(), G, [&](int32_t a, int32_t b) { return chunk_w[a] > chunk_w[b]; });
        for (int32_t j : chunk_order) {
          int32_t gamma = -1;
          for (int32_t g = 0; g < G; ++g)
            if (!taken[g] && (gamma < 0 || group_load[g] < group_load[gamma])) gamma = g;
          taken[gamma] = 1;
          const int64_t c0 = r0 + (int64_t)j * per, c1 = std::min<int64_t>(r1, c0 + per);
          if (c0 >= c1) continue;
          // k-th heaviest item (stable) to the group's k-th least-loaded partition (stable)
          const int64_t n_c = c1 - c0;
          int32_t* rank = part_rank.data();
          if (packed_keys) {
            for (int64_t t = 0; t < n_c; ++t) item_key[t] = ((uint64_t)(wmax - wseq[c0 + t]) << 20) | (uint64_t)t;
            std::sort(item_key.begin(), item_key.begin() + n_c);
            for (int64_t t = 0; t < n_c; ++t) item_pos[t] = (int32_t)(item_key[t] & 0xFFFFF);
            for (int32_t k = 0; k < per; ++k) part_key[k] = ((uint64_t)load[gamma + k * G] << 20) | (uint64_t)k;
            std::sort(part_key.begin(), part_key.end());
            for (int32_t k = 0; k < per; ++k) rank[k] = (int32_t)(part_key[k] & 0xFFFFF);
          } else {
            for (int64_t t = 0; t < n_c; ++t) item_pos[t] = (int32_t)t;
            std::stable_sort(item_pos.begin(), item_pos.begin() + n_c, [&](int32_t a, int32_t b) { return wseq[c0 + a] > wseq[c0 + b]; });
            for (int32_t k = 0; k < per; ++k) rank[k] = k;
            std::stable_sort(rank, rank + per, [&](int32_t a, int32_t b) { return load[gamma + a * G] < load[gamma + b * G]; });
          }
          for (int64_t k = 0; k < n_c; ++k) {
            const int32_t it = seq[c0 + item_pos[k]];
            const int32_t pt = gamma + rank[k] * G;
            assign_rounds[it] = pt;
            load[pt] += partition_cost ? (int64_t)wseq[c0 + item_pos[k]] * partition_cost[pt] : (int64_t)wseq[c0 + item_pos[k]];
          }
        }
      }
    }

    const std::vector<int32_t>& assign = hp.reused ? assign_reuse
        : (mode == DBSP_MODE_NAIVE) ? assign_naive : (mode == DBSP_MODE_ROUNDS) ? assign_rounds : assign_lpt;
    hp.part_load = loads_of(hp, assign);
    hp.rho_mode = dbsp_rho(hp.part_load.data(), 1, P);
    hp.have_rho_naive = hp.have_rho_balanced = false;
    if (!hp.reused && mode == DBSP_MODE_NAIVE) { hp.rho_naive = hp.rho_mode; hp.have_rho_naive = true; }
    if (!hp.reused && mode == DBSP_MODE_BALANCED) { hp.rho_balanced = hp.rho_mode; hp.have_rho_balanced = true; }

    // per-partition lists: ascending item id (= ascending head, q_block, kv_begin), or, for the
    // round-based placement, the order of the rounds
    hp.part_ptr.assign(P + 1, 0);
    for (int64_t i = 0; i < n_items; ++i)
      if (assign[i] >= 0) hp.part_ptr[assign[i] + 1]++;
    for (int32_t g = 0; g < P; ++g) hp.part_ptr[g + 1] += hp.part_ptr[g];
    hp.part_items.resize(hp.part_ptr[P]);
    std::vector<int32_t> cursor(hp.part_ptr.begin(), hp.part_ptr.end() - 1);
    if (mode == DBSP_MODE_ROUNDS && !hp.reused) {
      for (int32_t i : seq)
        if (assign[i] >= 0) hp.part_items[cursor[assign[i]]++] = i;
    } else {
      for (int64_t i = 0; i < n_items; ++i) hp.part_items[cursor[assign[i]]++] = (int32_t)i;
    }
    return DBSP_OK;
  } catch (const std::bad_alloc&) {
    err = "out of host memory while planning";
    return DBSP_ENOMEM;
  }
}

int dbsp_build_host_plan(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                         const dbsp_place_opts& opts, const dbsp_host_plan* prev,
                         double reuse_threshold, dbsp_host_plan& hp, std::string& err) {
  int rc = dbsp_plan_count(mask, H, nQ, nK, block, opts.pair, hp, err);
  if (rc != DBSP_OK) return rc;
  try {
    hp.kv_store.resize(hp.kv_ints() + 8);
  } catch (const std::bad_alloc&) {
    err = "out of host memory while planning";
    return DBSP_ENOMEM;
  }
  hp.kv_idx = hp.kv_store.data();
  dbsp_compaction job;
  dbsp_compact_begin(mask, hp, hp.kv_store.data(), job);     // runs beside the placement
  rc = dbsp_plan_place(opts, prev, reuse_threshold, hp, err);
  const bool ok = dbsp_compact_end(job);
  if (rc == DBSP_OK && !ok) { err = "out of host memory while planning"; rc = DBSP_ENOMEM; }
  return rc;
}
