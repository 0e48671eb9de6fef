// Host-side planners for several GPUs: heads over a Ulysses group, Q blocks over a ring's GPUs,
// KV blocks over the ring's iterations, and the ring form of the sparse imbalance ratio.
// Pure host code: nothing here touches a GPU.
//
// Paper: Methodology, "Head-level Partitioning" and "Block-level Partitioning" (greedy, reward
// factor R_b), Alg. 1 (both branches), Eq. 2 and Eq. 3.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "dbsp.h"
#include "plan.hpp"

namespace {

// unit j of n starts in group j / ceil(n / groups): the contiguous layout sequence parallelism begins with
inline int32_t contiguous_owner(int64_t j, int64_t n, int32_t groups) {
  const int64_t run = (n + groups - 1) / groups;
  return (int32_t)(j / run);
}

// Greedy of Alg. 1: units by descending count (stable), each to the bin whose accumulated count,
// minus reward * count for the unit's initial bin, is smallest among bins that are not full.
// `initial` may be null (no reward).  where[n]; list[n] grouped by bin in placement order; ptr[groups+1].
void biased_greedy(const int64_t* counts, int64_t n, int32_t groups, double reward, const int32_t* initial,
                   int32_t capacity, int32_t* where, int32_t* list, int32_t* ptr, int64_t* load_out) {
  std::vector<int32_t> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return counts[a] > counts[b]; });
  std::vector<int64_t> load(groups, 0);
  std::vector<int32_t> held(groups, 0);
  std::vector<int32_t> seq(n);           // placement sequence number of each unit
  for (int64_t t = 0; t < n; ++t) {
    const int32_t j = order[t];
    const int64_t w = counts[j];
    int32_t best = -1;
    double best_val = 0.0;
    for (int32_t g = 0; g < groups; ++g) {
      if (capacity > 0 && held[g] >= capacity) continue;
      double val = (double)load[g];
      if (initial && reward != 0.0 && g == initial[j]) {
        const double bonus = reward * (double)w;
        val = val - bonus;
      }
      if (best < 0 || val < best_val) {
        best = g;
        best_val = val;
      }
    }
    where[j] = best;
    load[best] += w;
    held[best] += 1;
    seq[t] = j;
  }
  std::vector<int32_t> cursor(groups + 1, 0);
  for (int64_t j = 0; j < n; ++j) cursor[where[j] + 1]++;
  for (int32_t g = 0; g < groups; ++g) cursor[g + 1] += cursor[g];
  if (ptr) std::copy(cursor.begin(), cursor.end(), ptr);
  if (list)
    for (int64_t t = 0; t < n; ++t) list[cursor[where[seq[t]]]++] = seq[t];
  if (load_out) std::copy(load.begin(), load.end(), load_out);
}

// acc[i][j] = number of heads whose block (i, j) is dense
void accumulate_heads(const uint8_t* mask, int32_t H, int32_t nQ, int32_t nK, std::vector<int32_t>& acc) {
  acc.assign((size_t)nQ * nK, 0);
  for (int32_t h = 0; h < H; ++h) {
    const uint8_t* m = mask + (size_t)h * nQ * nK;
    for (size_t e = 0; e < (size_t)nQ * nK; ++e) acc[e] += m[e] != 0;
  }
}

// Eq. 3: work[i][g] = C[g][(i + g) mod y], C[g][c] = dense blocks between GPU g's Q blocks and chunk c's KV blocks
void ring_work_from(const std::vector<int32_t>& acc, int32_t nQ, int32_t nK, int32_t y, const int32_t* gpu_of_q,
                    const int32_t* chunk_of_kv, int64_t* work) {
  std::vector<int64_t> C((size_t)y * y, 0);
  for (int32_t i = 0; i < nQ; ++i) {
    int64_t* row = &C[(size_t)gpu_of_q[i] * y];
    const int32_t* a = &acc[(size_t)i * nK];
    for (int32_t j = 0; j < nK; ++j) row[chunk_of_kv[j]] += a[j];
  }
  for (int32_t i = 0; i < y; ++i)
    for (int32_t g = 0; g < y; ++g) work[(size_t)i * y + g] = C[(size_t)g * y + (i + g) % y];
}

bool valid_map(const int32_t* map, int64_t n, int32_t groups) {
  for (int64_t j = 0; j < n; ++j)
    if (map[j] < 0 || map[j] >= groups) return false;
  return true;
}

}  // namespace

extern "C" {

int dbsp_partition_heads(const int64_t* blocks_per_head, int32_t H, int32_t x, int32_t capacity,
                         const int32_t* previous_gpu_of_head, double reuse_threshold, int32_t* gpu_of_head,
                         int32_t* head_list, int32_t* list_ptr, int64_t* load, double* rho_contiguous,
                         double* rho_previous, double* rho, int32_t* reused) {
  if (!blocks_per_head || !gpu_of_head) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: null pointer");
  if (H <= 0 || x <= 0 || capacity < 0) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: H and x must be positive, capacity >= 0");
  if (capacity > 0 && (int64_t)capacity * x < H) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: capacity * x < H");
  for (int32_t h = 0; h < H; ++h)
    if (blocks_per_head[h] < 0) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: negative block count");
  if (previous_gpu_of_head) {
    if (!(reuse_threshold >= 1.0)) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: the threshold must be at least 1");
    if (!valid_map(previous_gpu_of_head, H, x)) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_heads: previous plan names a GPU outside [0, x)");
  }
  std::vector<int64_t> ld(x, 0);
  for (int32_t h = 0; h < H; ++h) ld[contiguous_owner(h, H, x)] += blocks_per_head[h];
  if (rho_contiguous) *rho_contiguous = dbsp_rho(ld.data(), 1, x);
  bool keep = false;
  double rp = 0.0;
  if (previous_gpu_of_head) {
    std::fill(ld.begin(), ld.end(), 0);
    for (int32_t h = 0; h < H; ++h) ld[previous_gpu_of_head[h]] += blocks_per_head[h];
    rp = dbsp_rho(ld.data(), 1, x);
    keep = x == 1 || rp <= reuse_threshold;
  }
  if (rho_previous) *rho_previous = rp;
  if (reused) *reused = keep ? 1 : 0;
  if (keep) {
    // lists in ascending head id
    std::vector<int32_t> cursor(x + 1, 0);
    for (int32_t h = 0; h < H; ++h) {
      gpu_of_head[h] = previous_gpu_of_head[h];
      cursor[gpu_of_head[h] + 1]++;
    }
    for (int32_t g = 0; g < x; ++g) cursor[g + 1] += cursor[g];
    if (list_ptr) std::copy(cursor.begin(), cursor.end(), list_ptr);
    if (head_list)
      for (int32_t h = 0; h < H; ++h) head_list[cursor[gpu_of_head[h]]++] = h;
  } else if (x == 1) {
    // nothing to partition (Alg. 1's guard x > 1): heads stay in their order
    ld[0] = 0;
    for (int32_t h = 0; h < H; ++h) {
      gpu_of_head[h] = 0;
      if (head_list) head_list[h] = h;
      ld[0] += blocks_per_head[h];
    }
    if (list_ptr) { list_ptr[0] = 0; list_ptr[1] = H; }
  } else {
    biased_greedy(blocks_per_head, H, x, 0.0, nullptr, capacity, gpu_of_head, head_list, list_ptr, ld.data());
  }
  if (load) std::copy(ld.begin(), ld.end(), load);
  if (rho) *rho = dbsp_rho(ld.data(), 1, x);
  return DBSP_OK;
}

int dbsp_partition_blocks(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t y, double reward,
                          int32_t capacity_q, int32_t capacity_kv, int32_t* gpu_of_q, int32_t* q_list, int32_t* q_ptr,
                          int32_t* chunk_of_kv, int32_t* kv_list, int32_t* kv_ptr, int64_t* work,
                          double* rho_contiguous, double* rho, int64_t* moved_q, int64_t* moved_kv) {
  if (!mask_host || !gpu_of_q || !chunk_of_kv) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_blocks: null pointer");
  if (H <= 0 || nQ <= 0 || nK <= 0 || y <= 0) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_blocks: H, nQ, nK and y must be positive");
  if (!(reward >= 0.0) || !std::isfinite(reward)) return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_blocks: the reward must be finite and >= 0");
  if (capacity_q < 0 || capacity_kv < 0 || (capacity_q > 0 && (int64_t)capacity_q * y < nQ) ||
      (capacity_kv > 0 && (int64_t)capacity_kv * y < nK))
    return dbsp_set_error(DBSP_EINVAL, "dbsp_partition_blocks: a capacity is negative or too small to hold every block");
  try {
    std::vector<int32_t> acc;
    accumulate_heads(mask_host, H, nQ, nK, acc);
    std::vector<int64_t> per_q(nQ, 0), per_kv(nK, 0);
    for (int32_t i = 0; i < nQ; ++i)
      for (int32_t j = 0; j < nK; ++j) {
        per_q[i] += acc[(size_t)i * nK + j];
        per_kv[j] += acc[(size_t)i * nK + j];
      }
    std::vector<int32_t> q0(nQ), kv0(nK);
    for (int32_t i = 0; i < nQ; ++i) q0[i] = contiguous_owner(i, nQ, y);
    for (int32_t j = 0; j < nK; ++j) kv0[j] = contiguous_owner(j, nK, y);
    // y == 1: nothing to partition (Alg. 1's guard); the greedy gives the same single list but
    // in sorted order, so the identity plan is written out directly
    if (y == 1) {
      for (int32_t i = 0; i < nQ; ++i) { gpu_of_q[i] = 0; if (q_list) q_list[i] = i; }
      for (int32_t j = 0; j < nK; ++j) { chunk_of_kv[j] = 0; if (kv_list) kv_list[j] = j; }
      if (q_ptr) { q_ptr[0] = 0; q_ptr[1] = nQ; }
      if (kv_ptr) { kv_ptr[0] = 0; kv_ptr[1] = nK; }
    } else {
      biased_greedy(per_q.data(), nQ, y, reward, q0.data(), capacity_q, gpu_of_q, q_list, q_ptr, nullptr);
      biased_greedy(per_kv.data(), nK, y, reward, kv0.data(), capacity_kv, chunk_of_kv, kv_list, kv_ptr, nullptr);
    }
    std::vector<int64_t> w((size_t)y * y);
    if (rho_contiguous) {
      ring_work_from(acc, nQ, nK, y, q0.data(), kv0.data(), w.data());
      *rho_contiguous = dbsp_rho(w.data(), y, y);
    }
    ring_work_from(acc, nQ, nK, y, gpu_of_q, chunk_of_kv, w.data());
    if (work) std::copy(w.begin(), w.end(), work);
    if (rho) *rho = dbsp_rho(w.data(), y, y);
    if (moved_q) {
      *moved_q = 0;
      for (int32_t i = 0; i < nQ; ++i) *moved_q += gpu_of_q[i] != q0[i];
    }
    if (moved_kv) {
      *moved_kv = 0;
      for (int32_t j = 0; j < nK; ++j) *moved_kv += chunk_of_kv[j] != kv0[j];
    }
  } catch (const std::bad_alloc&) {
    return dbsp_set_error(DBSP_ENOMEM, "dbsp_partition_blocks: out of host memory");
  }
  return DBSP_OK;
}

int dbsp_ring_work(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t y, const int32_t* gpu_of_q,
                   const int32_t* chunk_of_kv, int64_t* work, double* rho) {
  if (!mask_host || (!work && !rho)) return dbsp_set_error(DBSP_EINVAL, "dbsp_ring_work: null pointer");
  if (H <= 0 || nQ <= 0 || nK <= 0 || y <= 0) return dbsp_set_error(DBSP_EINVAL, "dbsp_ring_work: H, nQ, nK and y must be positive");
  if ((gpu_of_q && !valid_map(gpu_of_q, nQ, y)) || (chunk_of_kv && !valid_map(chunk_of_kv, nK, y)))
    return dbsp_set_error(DBSP_EINVAL, "dbsp_ring_work: a map names a GPU or chunk outside [0, y)");
  try {
    std::vector<int32_t> acc, q0, kv0;
    accumulate_heads(mask_host, H, nQ, nK, acc);
    if (!gpu_of_q) {
      q0.resize(nQ);
      for (int32_t i = 0; i < nQ; ++i) q0[i] = contiguous_owner(i, nQ, y);
      gpu_of_q = q0.data();
    }
    if (!chunk_of_kv) {
      kv0.resize(nK);
      for (int32_t j = 0; j < nK; ++j) kv0[j] = contiguous_owner(j, nK, y);
      chunk_of_kv = kv0.data();
    }
    std::vector<int64_t> w((size_t)y * y);
    ring_work_from(acc, nQ, nK, y, gpu_of_q, chunk_of_kv, w.data());
    if (work) std::copy(w.begin(), w.end(), work);
    if (rho) *rho = dbsp_rho(w.data(), y, y);
  } catch (const std::bad_alloc&) {
    return dbsp_set_error(DBSP_ENOMEM, "dbsp_ring_work: out of host memory");
  }
  return DBSP_OK;
}

}  // extern "C"
