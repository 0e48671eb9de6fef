// Host planner: block-mask compaction, work items, greedy longest-first placement, rho_s.
//
// Cost model and rules come from db-SP (arXiv 2511.23113): the work of a unit is its number of
// dense mask blocks (Background, "Block-wise Sparse Attention"); rho_s is Eq. 1 (Motivation);
// placement is the greedy of "Head-level Partitioning" / Alg. 1's first loop, applied to
// (head, query block, KV range) items and P partitions instead of heads and GPUs.
// Everything here is integer arithmetic; the only floating point is the final rho_s division.

#include <emmintrin.h>   // SSE2: baseline of every x86-64 host

#include <algorithm>
#include <cstring>
#include <atomic>
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

}  // namespace

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

int dbsp_build_host_plan(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                         int32_t P, int32_t mode, int32_t max_item_len, int32_t item_overhead,
                         int32_t locality_groups, const int32_t* partition_cost, const dbsp_host_plan* prev,
                         double reuse_threshold, dbsp_host_plan& hp, std::string& err) {
  try {
    const int64_t R = (int64_t)H * nQ;
    hp.H = H; hp.nQ = nQ; hp.nK = nK; hp.block = block;
    hp.P = P; hp.mode = mode; hp.item_overhead = item_overhead;

    // pass 1: per-row counts (Alg. 1's get_blocks_per_head, kept per row), row offsets.
    // Rows are independent: large masks are cut into contiguous row ranges, one per thread.
    hp.row_cnt.resize(R);
    hp.row_ptr.resize(R + 1);
    hp.blocks_per_head.assign(H, 0);
    const int64_t mask_bytes = R * nK;
    int n_thr = 1;
    if (mask_bytes >= (int64_t)1 << 20) {
      const unsigned hw = std::thread::hardware_concurrency();
      n_thr = (int)std::min<int64_t>(std::min<unsigned>(hw ? hw : 1, 8), mask_bytes >> 19);
    }
    std::atomic<bool> worker_failed{false};
    auto for_row_ranges = [&](auto&& body) {   // body(first_row, last_row_exclusive)
      if (n_thr <= 1) { body((int64_t)0, R); return; }
      auto guarded = [&](int64_t r0, int64_t r1) {
        try { body(r0, r1); } catch (...) { worker_failed = true; }
      };
      std::vector<std::thread> pool;
      pool.reserve(n_thr - 1);
      int started = 1;
      try {
        for (; started < n_thr; ++started) pool.emplace_back(guarded, R * started / n_thr, R * (started + 1) / n_thr);
      } catch (const std::system_error&) {
        // no more threads to be had: this thread takes the ranges that were not started
      }
      guarded((int64_t)0, R / n_thr);
      if (started < n_thr) guarded(R * started / n_thr, R);
      for (auto& th : pool) th.join();
    };
    for_row_ranges([&](int64_t r0, int64_t r1) {
      for (int64_t r = r0; r < r1; ++r) hp.row_cnt[r] = count_row(mask + r * nK, nK);
    });
    hp.row_ptr[0] = 0;
    int64_t total = 0;
    for (int64_t r = 0; r < R; ++r) {
      total += hp.row_cnt[r];
      if (total > (int64_t)INT32_MAX) { err = "more than 2^31-1 active blocks"; return DBSP_EINVAL; }
      hp.row_ptr[r + 1] = (int32_t)total;
      hp.blocks_per_head[r / nQ] += hp.row_cnt[r];
    }
    hp.nnz = total;
    // pass 2: ascending KV block ids of every row.  compact_row stores up to 8 elements past a
    // row's end: harmless while that stays inside the thread's own range (later rows overwrite
    // them) or in the slack at the very end; a row whose spill would reach the next thread's
    // range goes through a bounce buffer.
    hp.kv_idx.resize(total + 8);
    for_row_ranges([&](int64_t r0, int64_t r1) {
      int32_t* base = hp.kv_idx.data();
      std::vector<int32_t> bounce;
      for (int64_t r = r0; r < r1; ++r) {
        if (!hp.row_cnt[r]) continue;
        if (r1 == R || (int64_t)hp.row_ptr[r + 1] + 8 <= (int64_t)hp.row_ptr[r1]) {
          compact_row(mask + r * nK, nK, base + hp.row_ptr[r]);
        } else {
          bounce.resize((size_t)nK + 8);
          compact_row(mask + r * nK, nK, bounce.data());
          std::memcpy(base + hp.row_ptr[r], bounce.data(), sizeof(int32_t) * (size_t)hp.row_cnt[r]);
        }
      }
    });
    hp.kv_idx.resize(total);
    if (worker_failed) { err = "out of host memory while planning"; return DBSP_ENOMEM; }

    // split threshold
    int32_t L = max_item_len;
    if (L == 0) L = (int32_t)std::max<int64_t>(4, hp.nnz / (2 * (int64_t)P));   // half the mean partition load
    hp.max_item_len = L;

    // items in row-major order
    hp.items.clear(); hp.item_slot.clear(); hp.split_rows.clear(); hp.empty_rows.clear();
    hp.items.reserve(4 * (R + 64)); hp.item_slot.reserve(R + 64);
    hp.n_slots = 0;
    for (int64_t r = 0; r < R; ++r) {
      const int32_t c = hp.row_cnt[r];
      const int32_t h = (int32_t)(r / nQ), I = (int32_t)(r % nQ);
      if (c == 0) { hp.empty_rows.push_back((int32_t)r); continue; }
      if (L < 0 || c <= L) {
        hp.items.insert(hp.items.end(), {h, I, 0, c});
        hp.item_slot.push_back(-1);
        continue;
      }
      const int32_t k = (c + L - 1) / L, base = c / k, extra = c % k;
      hp.split_rows.insert(hp.split_rows.end(), {(int32_t)r, hp.n_slots, k, 0});
      int32_t pos = 0;
      for (int32_t t = 0; t < k; ++t) {
        const int32_t len = base + (t < extra ? 1 : 0);
        hp.items.insert(hp.items.end(), {h, I, pos, pos + len});
        hp.item_slot.push_back(hp.n_slots++);
        pos += len;
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
      std::vector<int32_t> prev_part(pn), prev_first(R + 1, 0);
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
        if (prev_first[r] + chunk < prev_first[r + 1]) {
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

    // naive placement: contiguous runs of ceil(n_items / P)
    std::vector<int32_t> assign_naive(n_items), assign_lpt(n_items);
    const int64_t run = n_items ? (n_items + P - 1) / P : 1;
    for (int64_t i = 0; i < n_items; ++i) assign_naive[i] = (int32_t)(i / run);

    // greedy placement.  Stable descending order by weight through a counting sort: weights
    // are bounded by nK + item_overhead, and filling each bucket in ascending id keeps ties stable.
    {
      const int64_t wmax = (int64_t)nK + item_overhead;
      std::vector<int64_t> bucket_start(wmax + 2, 0);
      auto weight = [&](int64_t i) { return (int64_t)(hp.items[4 * i + 3] - hp.items[4 * i + 2]) + item_overhead; };
      for (int64_t i = 0; i < n_items; ++i) bucket_start[wmax - weight(i) + 1]++;
      for (int64_t w = 0; w <= wmax; ++w) bucket_start[w + 1] += bucket_start[w];
      std::vector<int32_t> order(n_items);
      for (int64_t i = 0; i < n_items; ++i) order[bucket_start[wmax - weight(i)]++] = (int32_t)i;
      LoadHeap heap(P, partition_cost);
      for (int64_t t = 0; t < n_items; ++t) {
        const int32_t i = order[t];
        assign_lpt[i] = heap.place(weight(i));
      }
    }

    // round-based greedy (DBSP_MODE_ROUNDS): heads in descending order of their block count
    // (the sort of Alg. 1), their items cut into consecutive rounds of P; inside a round the
    // k-th heaviest item goes to the k-th least-loaded partition.  Every partition works on the
    // same head at about the same time, which is what lets the KV blocks be reused from L2.
    std::vector<int32_t> assign_rounds, seq;
    if (mode == DBSP_MODE_ROUNDS) {
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
      assign_rounds.assign(n_items, 0);
      // With G > 1 locality groups (partition p belongs to group p mod G: the partitions behind
      // one cache) a round is cut into G contiguous chunks of P/G items -- runs of neighbouring
      // query blocks -- and the same greedy runs one level up: heaviest chunk first, each to the
      // least-loaded group that has no chunk yet in this round.
      const int32_t G = locality_groups > 1 ? locality_groups : 1, per = P / G;
      std::vector<int64_t> load(P, 0), chunk_w(G), group_load(G);
      std::vector<int32_t> parts(per), idx, chunk_order(G);
      std::vector<char> taken(G);
      for (int64_t r0 = 0; r0 < n_items; r0 += P) {
        const int64_t r1 = std::min<int64_t>(n_items, r0 + P);
        for (int32_t j = 0; j < G; ++j) {
          chunk_w[j] = 0;
          for (int64_t t = r0 + (int64_t)j * per; t < std::min<int64_t>(r1, r0 + (int64_t)(j + 1) * per); ++t) chunk_w[j] += weight(seq[t]);
          chunk_order[j] = j;
          taken[j] = 0;
          group_load[j] = 0;
        }
        for (int32_t p = 0; p < P; ++p) group_load[p % G] += load[p];
        std::stable_sort(chunk_order.begin(), chunk_order.end(), [&](int32_t a, int32_t b) { return chunk_w[a] > chunk_w[b]; });
        for (int32_t j : chunk_order) {
          int32_t gamma = -1;
          for (int32_t g = 0; g < G; ++g)
            if (!taken[g] && (gamma < 0 || group_load[g] < group_load[gamma])) gamma = g;
          taken[gamma] = 1;
          const int64_t c0 = r0 + (int64_t)j * per, c1 = std::min<int64_t>(r1, c0 + per);
          if (c0 >= c1) continue;
          idx.assign(seq.begin() + c0, seq.begin() + c1);
          std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) { return weight(a) > weight(b); });
          for (int32_t k = 0; k < per; ++k) parts[k] = gamma + k * G;
          std::stable_sort(parts.begin(), parts.end(), [&](int32_t a, int32_t b) { return load[a] < load[b]; });
          for (size_t k = 0; k < idx.size(); ++k) {
            assign_rounds[idx[k]] = parts[k];
            load[parts[k]] += partition_cost ? weight(idx[k]) * partition_cost[parts[k]] : weight(idx[k]);
          }
        }
      }
    }

    auto loads_of = [&](const std::vector<int32_t>& a) {
      std::vector<int64_t> ld(P, 0);
      for (int64_t i = 0; i < n_items; ++i) ld[a[i]] += hp.items[4 * i + 3] - hp.items[4 * i + 2];
      return ld;
    };
    const std::vector<int64_t> ld_naive = loads_of(assign_naive), ld_lpt = loads_of(assign_lpt);
    hp.rho_naive = dbsp_rho(ld_naive.data(), 1, P);
    hp.rho_balanced = dbsp_rho(ld_lpt.data(), 1, P);

    const std::vector<int32_t>& assign = hp.reused ? assign_reuse
        : (mode == DBSP_MODE_NAIVE) ? assign_naive : (mode == DBSP_MODE_ROUNDS) ? assign_rounds : assign_lpt;
    hp.part_load = loads_of(assign);
    hp.rho_mode = dbsp_rho(hp.part_load.data(), 1, P);

    // per-partition lists: ascending item id (= ascending head, q_block, kv_begin), or, for the
    // round-based placement, the order of the rounds
    hp.part_ptr.assign(P + 1, 0);
    for (int64_t i = 0; i < n_items; ++i) hp.part_ptr[assign[i] + 1]++;
    for (int32_t g = 0; g < P; ++g) hp.part_ptr[g + 1] += hp.part_ptr[g];
    hp.part_items.resize(n_items);
    std::vector<int32_t> cursor(hp.part_ptr.begin(), hp.part_ptr.end() - 1);
    if (mode == DBSP_MODE_ROUNDS && !hp.reused) {
      for (int32_t i : seq) hp.part_items[cursor[assign[i]]++] = i;
    } else {
      for (int64_t i = 0; i < n_items; ++i) hp.part_items[cursor[assign[i]]++] = (int32_t)i;
    }
    return DBSP_OK;
  } catch (const std::bad_alloc&) {
    err = "out of host memory while planning";
    return DBSP_ENOMEM;
  }
}
