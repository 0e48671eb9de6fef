/*
 * dbsp.h -- C ABI of libdbsp: balanced block-sparse attention forward on one AMD MI355X.
 *
 * The library carries the workload-balancing idea of db-SP (arXiv 2511.23113) from "GPUs of
 * a sequence-parallel group" onto "compute units of one GPU":
 *   - the cost of a piece of attention work is its number of dense mask blocks
 *     (paper: Background, "Block-wise Sparse Attention");
 *   - the sparse imbalance ratio rho_s = (sum over sync periods of the max per-partition
 *     block count) / (total block count / number of partitions) (paper: Motivation, Eq. 1;
 *     one-period form Eq. 2);
 *   - work is balanced with the greedy rule of Alg. 1 / "Head-level Partitioning": sort
 *     units by block count, descending, and give each to the least-loaded partition.
 * Attention itself is O = softmax(Q K^T / sqrt(d)) V per head (paper: Background, "Visual
 * Generative Models"), evaluated only on the dense blocks of a per-head block mask.
 *
 * Conventions for every function:
 *   - returns DBSP_OK (0) on success, a negative dbsp_status on error; never throws;
 *     dbsp_last_error() gives a thread-local message for the last error on this thread;
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on
 *     the current device; the library never takes ownership of caller memory;
 *   - calls on distinct plans are thread-safe; calls that use the same plan must not
 *     overlap (a plan owns scratch buffers that a forward call writes).
 */
#ifndef DBSP_H
#define DBSP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dbsp_status {
  DBSP_OK = 0,
  DBSP_EINVAL = -1, /* null pointer, non-positive size, unsupported head dim / block size, bad option */
  DBSP_ESHAPE = -2, /* sequence length not a multiple of the block size, or shapes disagree with the plan */
  DBSP_ENOMEM = -3, /* host or device allocation failed */
  DBSP_EHIP = -4    /* a HIP runtime call failed; dbsp_last_error() holds its message */
} dbsp_status;

/* Opaque, library-owned plan.  Immutable after creation except for its scratch buffers. */
typedef struct dbsp_plan dbsp_plan;

enum { DBSP_MODE_BALANCED = 0, DBSP_MODE_NAIVE = 1, DBSP_MODE_ROUNDS = 2, DBSP_MODE_REWARD = 3 };
enum {
  DBSP_PLAN_HOST_ONLY = 1, /* flags bit: build the plan on the host only (no device, no upload);
                              such a plan cannot be passed to sparse_attn_fwd */
  DBSP_PLAN_PAIR_ROWS = 2, /* flags bit, block == 64 only, forward pass at d == 128 only: 64-token blocks (the block
                              size of the paper's PAROAttention masks: Methodology, "Block-level Partitioning") served
                              by 128-query workgroups.  A row of the plan is then a pair of neighbouring query blocks
                              (2p, 2p+1) of a head and its KV list the ascending union of the two rows' lists, cut into
                              consecutive pairs ("super blocks", the unit of work and of every count, length and rho_s
                              of such a plan); the (query block, KV block) combinations of a super block that the
                              mask does not have are computed with the rest and given probability zero, so K and V
                              must be finite in every block that either row of a pair uses.  It pays when neighbouring
                              rows are alike: from about 5 / 8 of the flags set (the mask's active blocks / (4 x the
                              plan's nnz)) it is faster than the plain plan, up to 1.57 times.  DBSP_ROW_CNT /
                              ROW_PTR / ITEMS then refer to pair rows (ceil(nQ / 2) per head) and super blocks,
                              and DBSP_KV_IDX holds two int32 per super block: j0, and j1 | flags << 24
                              with flags bit (q + 2k) = "query block 2p+q needs KV block j_k" (a union of odd length
                              ends with j1 = j0 and no flag for the second slot) */
  DBSP_PLAN_PAIR_AUTO = 4  /* flags bit, block == 64 and head_dim == 128 only, not together with DBSP_PLAN_PAIR_ROWS:
                              the library counts the mask both ways and plans with pair rows if at least 5 / 8 of the
                              flags would be set (2 x active blocks >= 5 x super blocks), else plainly;
                              dbsp_plan_pair_rows tells which.  plan_sparse_attn_reuse keeps the previous plan's kind */
};

typedef struct dbsp_plan_opts {
  int32_t num_partitions; /* P >= 1; 0 -> number of compute units of the current device (256 when no device),
                             times 4 when block <= 64 without DBSP_PLAN_PAIR_ROWS (those workgroups are two
                             waves each: four fill a compute unit at d = 64; at d = 128 their tiles leave room
                             for two at a time: times 2 if head_dim says so, else the other half of the
                             workgroups follow as the first finish, which costs about a tenth) */
  int32_t mode;           /* DBSP_MODE_BALANCED: greedy longest-first placement (Alg. 1, first loop);
                             DBSP_MODE_NAIVE: items in row-major order dealt in contiguous runs of
                             ceil(n_items / P) -- the unbalanced baseline rho_s is quoted against;
                             DBSP_MODE_ROUNDS: the greedy applied round by round: heads in descending
                             order of their block count (Alg. 1's sort), their items cut into consecutive
                             rounds of P, and inside a round the k-th heaviest item goes to the k-th
                             least-loaded partition.  All partitions then work on the same head at about
                             the same time, so KV blocks are reused from L2: balance traded for locality,
                             the trade-off the paper steers with its reward factor R_b;
                             DBSP_MODE_REWARD: the greedy longest-first placement with the paper's reward factor
                             itself (Methodology, "Block-level Partitioning", overhead mitigation; Alg. 1, second
                             loop): partition p belongs to group p mod locality_groups (the compute units behind
                             one L2), an item's home group is q_block * G / nQ (neighbouring query blocks, which
                             share KV blocks, have one home), and before each argmin the accumulated load of
                             every partition of the home group is lowered by reward * (the item's weight),
                             compared in double; ties go to the lowest partition index */
  int32_t max_item_len;   /* split threshold in blocks: a row with more active blocks is cut into
                             ceil(cnt / max_item_len) near-equal chunks. 0 -> max(4, nnz / (2 P)); < 0 -> never split */
  int32_t item_overhead;  /* >= 0; constant added to every item's weight for the greedy placement only
                             (rho_s is always computed from pure block counts). 0 = the paper's cost model */
  int32_t flags;          /* DBSP_PLAN_HOST_ONLY, DBSP_PLAN_PAIR_ROWS or DBSP_PLAN_PAIR_AUTO, or'ed; or 0 */
  int32_t locality_groups; /* DBSP_MODE_ROUNDS only: G > 1 keeps runs of neighbouring query blocks inside one
                             group of partitions that share a cache (partition p belongs to group p mod G;
                             on MI355X workgroup p runs on XCD p mod 8, each XCD has its own L2).  A round is
                             cut into G contiguous chunks of P/G items; chunks go, heaviest first, to the
                             group with the least accumulated load that has none yet in this round; inside
                             the group the k-th heaviest item goes to its k-th least-loaded partition.
                             G must divide P.  0 or 1 = one group (plain rounds) */
  const int32_t* partition_cost; /* host, int32 [P] or NULL: relative time partition g needs per block (> 0), e.g.
                             from dbsp_plan_calibrate.  The greedy placements (balanced, rounds) then compare
                             accumulated time, sum of weight * cost[g], instead of accumulated weight (list
                             scheduling on compute units of different speed); equal costs or NULL give the
                             paper's rule.  Read during the call only.  rho_s stays on pure block counts */
  int32_t max_batch;      /* >= 0; the largest B sparse_attn_fwd will be called with on this plan (0 -> 1).  Rows
                             that are split need device scratch per batch entry; it is allocated here, at plan
                             time, so that the forward call never allocates or waits */
  int32_t dynamic_tail;   /* DBSP_MODE_ROUNDS only, permille in [0, 1000): the end of the item sequence -- the longest
                             suffix whose weight is at most dynamic_tail / 1000 of the total, plus whatever a partial
                             last round would hold -- is placed on no partition: the workgroups take those items from
                             a shared queue, one by one, as they run out of placed work.  This is the greedy rule
                             ("each unit to the least-loaded partition", Alg. 1's first loop) decided at run time,
                             with real finishing times as loads; it absorbs speed differences between compute
                             units.  Heads come in descending order of block count, so the queue holds the lightest
                             rows.  Results do not depend on who computes an item.  0 = everything placed */
  double reward;          /* DBSP_MODE_REWARD only: R_b >= 0 (0 = plain greedy) */
  int32_t head_dim;       /* 0, 64 or 128: the head dim the plan will run at, if known.  Only the default of
                             num_partitions looks at it: 64-token blocks without pair rows at head dim 128 keep two
                             workgroups per compute unit resident, so the default is twice the compute units there */
} dbsp_plan_opts;

/*
 * plan_sparse_attn -- compact a block mask and build the (balanced) work list.
 *
 * mask_host: host, uint8 [H, nQ, nK] row-major; nonzero = the (query block, key block) pair is
 *            computed (a "dense block").  Read during the call only.
 * block:     block size b in tokens; the forward pass supports 64 and 128.
 * opts:      host, may be NULL (all zero = defaults).
 * out_plan:  receives the plan; free it with dbsp_plan_destroy.
 *
 * Steps (all integer): per-row counts and per-head sums (Alg. 1, get_blocks_per_head); ascending
 * KV-block index list per row; work items (head, q_block, kv_begin, kv_end) in row-major order
 * with long rows split; greedy placement: stable sort by weight descending, each item to the
 * partition with the smallest accumulated weight (ties: lowest index); each partition's list
 * in ascending item order (round order for DBSP_MODE_ROUNDS); rho_s of the chosen placement (Eq. 1
 * with one period; that of the naive and of the greedy placement on request, see dbsp_plan_stats).
 * Unless DBSP_PLAN_HOST_ONLY is set, the arrays are then copied to the current device, next to
 * scratch for split rows (max_batch batch entries) and busy-time capture.  The copy is
 * asynchronous (a stream of the library's own, pinned staging, buffers recycled from a
 * process-wide pool): the call returns without waiting for it, and sparse_attn_fwd makes its
 * stream wait for the copy, so planning the next call overlaps with the device's work on the
 * current one.  Masks over 1 MB are counted on up to 8 host threads; the index lists are written
 * straight into pinned memory by helper threads while the calling thread builds items and
 * placement (the helpers belong to a process-wide pool and sleep between plans; all of them are
 * done before the call returns).
 * Errors: DBSP_EINVAL, DBSP_ENOMEM, DBSP_EHIP.  Rows with no active block are legal.
 */
int plan_sparse_attn(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t block,
                     const dbsp_plan_opts* opts, dbsp_plan** out_plan);

/* Whether the plan was made with pair rows (DBSP_PLAN_PAIR_ROWS, or DBSP_PLAN_PAIR_AUTO's choice): 1 or 0.
 * Errors: DBSP_EINVAL (null pointer). */
int dbsp_plan_pair_rows(const dbsp_plan* plan, int32_t* pair_rows);

/*
 * plan_sparse_attn_reuse -- plan for the next mask of a sequence (denoising steps), keeping the
 * previous plan's placement when it is still balanced enough (paper: Methodology, "Head-level
 * Partitioning", overhead mitigation: the plan of the last step is reused if the current rho_s
 * falls below a threshold P_s; Alg. 1 re-plans only if rho_s > P_s).
 *
 * previous: a plan of the same geometry (H, nQ, nK, block are taken from it) and partition count.
 * mask_host: host, uint8 [H, nQ, nK], the new mask.  opts as for plan_sparse_attn
 * (num_partitions 0 = the previous plan's).  reuse_threshold: P_s >= 1.
 * Counts, index lists and items are always rebuilt for the new mask.  Its rho_s under the previous
 * placement is evaluated by carrying the placement over per (row, chunk index); items the
 * previous plan did not have go, in item order, to the least-loaded partition.  If that rho_s
 * <= P_s the carried-over placement is used (*reused = 1), else the mask is planned afresh in
 * opts->mode (*reused = 0).  *rho_under_previous receives the evaluated rho_s.  The new plan is
 * independent of `previous`, which may be destroyed afterwards.  reused / rho_under_previous may
 * be NULL.  Errors: DBSP_EINVAL, DBSP_ESHAPE (geometry or partition count differ), DBSP_ENOMEM, DBSP_EHIP.
 */
int plan_sparse_attn_reuse(const dbsp_plan* previous, const uint8_t* mask_host, const dbsp_plan_opts* opts,
                           double reuse_threshold, dbsp_plan** out_plan, int32_t* reused,
                           double* rho_under_previous);

/*
 * sparse_attn_fwd -- block-sparse attention forward over a plan's work list: per head,
 * O = softmax(Q K^T / sqrt(d)) V (paper: Background, "Visual Generative Models") with the
 * scores of every (query block, key block) pair outside the mask left out, i.e. computed on the
 * dense blocks only (paper: Background, "Block-wise Sparse Attention": the dense-block count is
 * the workload), in the order and on the compute units the plan's work list fixes.
 *
 * q:   device, bf16 [B, H, Nq, d] contiguous (d fastest);  k, v: device, bf16 [B, H, Nk, d].
 * o:   device, bf16 [B, H, Nq, d], written.  lse: device, f32 [B, H, Nq], written; may be NULL.
 *      LSE = natural log of the sum of exp(softmax_scale * q.k) over the row's active keys.
 * Nq == nQ * block and Nk == nK * block of the plan (else DBSP_ESHAPE); d in {64, 128} (128 only
 * for a plan made with DBSP_PLAN_PAIR_ROWS, else DBSP_EINVAL);
 * the mask has no batch axis: every batch entry uses the same per-head mask.
 * softmax_scale <= 0 selects 1 / sqrt(d).  A query row with no active block gets O = 0, LSE = -inf.
 * stream: a hipStream_t (NULL = default stream).  The call only enqueues work: one persistent
 * kernel with one workgroup per partition, plus a small fix-up kernel when rows were split or
 * are empty.  It neither allocates nor synchronises with the host.  bf16 inputs, f32 accumulation.
 * Errors: DBSP_EINVAL (also: B above the plan's max_batch when rows are split), DBSP_ESHAPE, DBSP_EHIP.
 */
int sparse_attn_fwd(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                    float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                    void* stream);

/*
 * sparse_attn_fwd_static -- sparse_attn_fwd for callers that cannot allocate device memory or
 * have it allocated for them: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same results as sparse_attn_fwd; the one
 * difference is where the partial results of split rows go: into a static device array of the
 * library (32 MiB per GPU, there from the moment the library is loaded until the process ends)
 * instead of the scratch the plan allocated.  It therefore works for any B whatever the plan's
 * max_batch, as long as  B * n_split_chunks * block * (d + 1) * 4 bytes (plus alignment; with pair
 * rows 2 * block in place of block) fit in the 32 MiB; beyond that it returns DBSP_EINVAL and the message names both sizes.  The call makes
 * no allocation of any kind (its first use on a device looks up the array's device address).
 * Nothing in the array needs clearing: every slot a launch reads was written by that launch.
 * All calls on one GPU share the array: two such calls must not overlap on the device (different
 * streams without ordering, or concurrent host threads), or they race on it.
 * Errors: as sparse_attn_fwd.
 */
int sparse_attn_fwd_static(const dbsp_plan* plan, const void* q, const void* k, const void* v, void* o,
                           float* lse, int32_t B, int32_t Nq, int32_t Nk, int32_t d, float softmax_scale,
                           void* stream);

/*
 * imbalance_ratio -- Eq. 1 on a host matrix work[periods][partitions] (row-major, int64, >= 0):
 * rho = sum_i max_g work[i][g] / (sum_{i,g} work[i][g] / partitions), in double.  Zero total
 * work gives 1.0.  Errors: DBSP_EINVAL (null pointer, non-positive size, negative entry).
 */
int imbalance_ratio(const int64_t* work, int32_t periods, int32_t partitions, double* rho_out);

/*
 * dbsp_fit_cost_model -- least-squares fit of  time = a * blocks + c * items + t0  over n
 * per-partition samples (paper: Methodology, "Sparsity-aware Strategy Selection": compute time
 * proportional to the dense-block count plus a constant, constants fitted from profiles; the
 * per-item term accounts for the fixed cost of starting a work item).
 * blocks, items: host int64 [n] (PART_LOAD and the list lengths of a plan); time: host double [n]
 * in any unit (e.g. the ticks of dbsp_plan_busy).  Out: a, c, t0 in that unit (required);
 * rms_residual may be NULL.  Errors: DBSP_EINVAL (null pointer, n < 3, non-finite sample, or
 * samples that do not determine the constants: blocks or items constant, or proportional).
 */
int dbsp_fit_cost_model(const int64_t* blocks, const int64_t* items, const double* time, int32_t n,
                        double* a, double* c, double* t0, double* rms_residual);

/*
 * Planners for several GPUs (host only: every pointer below is host memory, nothing touches a
 * GPU).  They produce the plans a U_x R_y deployment would exchange data by; one GPU cannot run
 * that exchange, so only the plans and their rho_s are computed.  "Initial" owner of unit j of n
 * over g groups is j / ceil(n / g), the contiguous layout sequence parallelism starts from.
 * Sorts are stable; ties of the argmin go to the lowest index.  Optional outputs may be NULL.
 */

/*
 * dbsp_partition_heads -- head-level partitioning over a Ulysses group of x GPUs (paper:
 * Methodology, "Head-level Partitioning"; Alg. 1, first branch).
 *
 * blocks_per_head: int64 [H], dense blocks of each head (>= 0).  capacity: 0 = no limit, else
 * the most heads one GPU may hold (capacity * x >= H).  previous_gpu_of_head: int32 [H] or
 * NULL, the last step's plan; it is kept (*reused = 1) if rho_s of the current counts under it
 * (*rho_previous) is <= reuse_threshold (>= 1), or if x == 1.  Otherwise heads are taken in
 * descending count order, each going to the GPU with the least accumulated count that is not full.
 * Out: gpu_of_head int32 [H] (required); head_list int32 [H] = head ids grouped by GPU, in
 * placement order (ascending id when reused), list_ptr int32 [x+1]; load int64 [x];
 * rho_contiguous = rho_s (Eq. 2) of the initial layout, rho = of the returned plan.
 * Errors: DBSP_EINVAL.
 */
int dbsp_partition_heads(const int64_t* blocks_per_head, int32_t H, int32_t x, int32_t capacity,
                         const int32_t* previous_gpu_of_head, double reuse_threshold, int32_t* gpu_of_head,
                         int32_t* head_list, int32_t* list_ptr, int64_t* load, double* rho_contiguous,
                         double* rho_previous, double* rho, int32_t* reused);

/*
 * dbsp_partition_blocks -- block-level partitioning for a ring of y GPUs (paper: Methodology,
 * "Block-level Partitioning", reward factor R_b; Alg. 1, second branch).
 *
 * mask_host: uint8 [H, nQ, nK]; it is summed over heads.  Q blocks, in descending order of their
 * row sums, go greedily to GPUs; KV blocks, in descending order of their column sums, go
 * greedily to KV chunks (chunk c is processed by GPU g in iteration (c - g) mod y).  Before each
 * argmin the load of the block's initial GPU / chunk is lowered by reward * (the block's own
 * sum), compared in double; reward >= 0, 0 = plain greedy.  capacity_q / capacity_kv: 0 = no
 * limit, else the most blocks per GPU / chunk.  y == 1 returns the identity plan.
 * Out: gpu_of_q int32 [nQ], chunk_of_kv int32 [nK] (required); q_list [nQ] with q_ptr [y+1] and
 * kv_list [nK] with kv_ptr [y+1]: ids grouped by GPU / chunk in placement order; work int64
 * [y, y] = Eq. 3's b[i][g] under the plan (row = iteration); rho = its rho_s, rho_contiguous =
 * rho_s of the initial layout; moved_q / moved_kv = blocks that leave their initial owner.
 * Errors: DBSP_EINVAL, DBSP_ENOMEM.
 */
int dbsp_partition_blocks(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t y, double reward,
                          int32_t capacity_q, int32_t capacity_kv, int32_t* gpu_of_q, int32_t* q_list, int32_t* q_ptr,
                          int32_t* chunk_of_kv, int32_t* kv_list, int32_t* kv_ptr, int64_t* work,
                          double* rho_contiguous, double* rho, int64_t* moved_q, int64_t* moved_kv);

/*
 * dbsp_ring_work -- Eq. 3's work matrix and rho_s for given maps: work[i][g] = dense blocks,
 * over all heads, between the Q blocks of GPU g and the KV blocks of chunk (i + g) mod y.
 * gpu_of_q int32 [nQ] / chunk_of_kv int32 [nK]: values in [0, y); NULL = the initial layout.
 * work int64 [y, y] and rho: at least one must be given.  Errors: DBSP_EINVAL, DBSP_ENOMEM.
 */
int dbsp_ring_work(const uint8_t* mask_host, int32_t H, int32_t nQ, int32_t nK, int32_t y, const int32_t* gpu_of_q,
                   const int32_t* chunk_of_kv, int64_t* work, double* rho);

/* Plan arrays (host copies, owned by the plan, valid until dbsp_plan_destroy). */
enum dbsp_plan_array {
  DBSP_ROW_PTR = 0,         /* int32 [H*nQ + 1]  CSR offsets over rows r = h*nQ + I                  */
  DBSP_KV_IDX = 1,          /* int32 [nnz]       ascending active KV block ids of each row (pair rows: [2 nnz]) */
  DBSP_ITEMS = 2,           /* int32 [n_items*4] (head, q_block, kv_begin, kv_end); begin/end are
                               positions inside the row's list                                        */
  DBSP_ITEM_SLOT = 3,       /* int32 [n_items]   -1 = whole row; else index of this chunk among all
                               chunks of split rows, in item order                                    */
  DBSP_SPLIT_ROWS = 4,      /* int32 [n_split*4] (row, first_slot, n_chunks, 0)                       */
  DBSP_PART_PTR = 5,        /* int32 [P + 1]     offsets into PART_ITEMS                              */
  DBSP_PART_ITEMS = 6,      /* int32 [n_items]   item ids of each partition, in processing order      */
  DBSP_PART_LOAD = 7,       /* int64 [P]         active blocks per partition (pure block counts)      */
  DBSP_BLOCKS_PER_HEAD = 8, /* int64 [H]         active blocks per head                               */
  DBSP_ROW_CNT = 9,         /* int32 [H*nQ]      active blocks per row                                */
  DBSP_EMPTY_ROWS = 10,     /* int32 [n_empty]   rows with no active block                            */
  DBSP_TAIL_ITEMS = 11      /* int32 [n_tail]    items left to the shared queue (dynamic_tail), in queue order;
                               they appear in no partition's list, and PART_LOAD / rho_plan leave them out */
};

/* dbsp_plan_get: *data points to the array, *count is its number of ELEMENTS of the type above. */
int dbsp_plan_get(const dbsp_plan* plan, int32_t what, const void** data, int64_t* count);

/* dbsp_plan_stats: any output pointer may be NULL.  rho_* are Eq. 1 (one period) on pure block
 * counts of the SAME item list under three placements: naive, greedy longest-first (balanced),
 * and the one this plan uses (rho_plan; equals one of the other two unless the mode is
 * DBSP_MODE_ROUNDS or the placement was carried over).  rho_naive / rho_balanced of a placement
 * the plan does not use are worked out on the first call that asks for them (one placement pass
 * each, on the calling thread; ask with NULL to skip it).  plan_usec is the host time spent inside
 * plan_sparse_attn (including handing the upload to the device).  Errors: DBSP_EINVAL, DBSP_ENOMEM. */
int dbsp_plan_stats(const dbsp_plan* plan, double* rho_naive, double* rho_balanced, double* rho_plan,
                    int64_t* nnz, int64_t* n_items, int32_t* num_partitions, int32_t* max_item_len,
                    double* plan_usec);

/* dbsp_plan_calibrate: relative time per block of every partition in the LAST sparse_attn_fwd on this plan,
 * for dbsp_plan_opts.partition_cost of later plans with the same partition count (compute units of one
 * chip differ by a few percent in speed, systematically).  cost: host, int32 [P], written:
 * cost[g] = round(1024 * (busy[g] / load[g]) / (sum busy / sum load)) in exact integer arithmetic (round
 * half up), clamped to [512, 2048]; 1024 for a partition without work or measurement.  Synchronises
 * `stream` before reading.  Errors: DBSP_EINVAL (null pointer, host-only plan), DBSP_EHIP. */
int dbsp_plan_calibrate(const dbsp_plan* plan, int32_t* cost, void* stream);

/* dbsp_plan_tail_takes: how often each item of the shared queue (DBSP_TAIL_ITEMS) has been taken since the plan was
 * made: after n forward calls with batch size B every entry must read n * B (each item taken exactly once per batch
 * entry and launch).  takes: host, uint32 [n_tail], written.  Synchronises `stream` before reading.
 * Errors: DBSP_EINVAL (null pointer, host-only plan), DBSP_EHIP. */
int dbsp_plan_tail_takes(const dbsp_plan* plan, uint32_t* takes, void* stream);

/* dbsp_plan_busy: per-partition busy time of the LAST sparse_attn_fwd on this plan.
 * busy_ticks: host, uint64 [P], ticks of the 100 MHz constant clock summed over the partition's
 * items; hw_id: host, uint32 [P], (XCC id << 16) | (SE id << 8) | CU id the workgroup ran on;
 * either may be NULL.  Synchronises `stream` before reading. */
int dbsp_plan_busy(const dbsp_plan* plan, uint64_t* busy_ticks, uint32_t* hw_id, void* stream);

/* dbsp_plan_destroy: waits (on the host) until the last sparse_attn_fwd enqueued with this plan
 * and the plan's upload have finished, then recycles its buffers.  NULL is ignored. */
void dbsp_plan_destroy(dbsp_plan* plan);

const char* dbsp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DBSP_H */
