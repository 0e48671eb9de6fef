"""Oracle: block-mask compaction, work items, greedy (longest-first) partitioning, rho_s.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is followed:
  * cost of a unit of work = its number of dense mask blocks (Background, "Block-wise
    Sparse Attention": the dense-block count is the workload);
  * sparse imbalance ratio rho_s (Motivation, Eq. 1; one-period form: Eq. 2; ring form:
    Eq. 3);
  * greedy head-level partitioning (Methodology, "Head-level Partitioning" and the first
    loop of Alg. 1): sort units by dense-block count, descending; hand each to the
    partition whose accumulated count is currently smallest.

The paper balances heads over GPUs.  Here the same greedy rule balances finer units --
(head, query block, range of that row's active KV blocks) -- over P partitions (the
persistent workgroups of one GPU).  Steps are taken in the paper's order; plain Python
integers throughout, so results are exact.

Readings where the paper is silent or garbled (all integer rules):
  * the descending sort is stable: equal weights keep ascending item id;
  * argmin ties go to the lowest partition index;
  * Alg. 1's loop header "in enumerate(sorted ids)" is read as "over the sorted ids";
  * "sum_per_gpu.update()" is read as load[g] += weight of the unit just placed;
  * partitions have no capacity limit (the published text states none);
  * rho_s of zero total work is 1.0;
  * rho_s is always computed from pure block counts, even when a per-item overhead
    steers the greedy placement.
"""

from __future__ import annotations

import numpy as np

MODE_BALANCED = 0
MODE_NAIVE = 1
MODE_ROUNDS = 2
MODE_REWARD = 3


def row_counts(mask):
    """cnt[h*nQ+I] = number of active KV blocks of row (h, I); per-head sums; total.

    `blocks_per_head` is Alg. 1's get_blocks_per_head.
    """
    active = np.asarray(mask) != 0
    cnt = active.sum(axis=2, dtype=np.int64)          # [H, nQ]
    per_head = [int(x) for x in cnt.sum(axis=1)]
    flat = [int(x) for x in cnt.reshape(-1)]
    return flat, per_head, sum(per_head)


def compact(mask):
    """CSR over rows r = h*nQ + I: ascending active KV block ids per row."""
    mask = np.asarray(mask)
    H, nQ, nK = mask.shape
    row_ptr = [0]
    kv_idx = []
    for h in range(H):
        for I in range(nQ):
            kv_idx.extend(int(J) for J in np.flatnonzero(mask[h, I] != 0))   # ascending J
            row_ptr.append(len(kv_idx))
    return row_ptr, kv_idx


def pair_rows(mask):
    """Query blocks taken two at a time (for 64-token blocks served by 128-query workgroups: the
    block size of the paper's PAROAttention masks, Methodology, "Block-level Partitioning").

    Super-row (h, p) covers query blocks 2p and 2p+1 (the second may not exist when nQ is odd).
    Its KV list is the ascending union of the two rows' active KV blocks, cut into consecutive
    pairs ("super blocks", what one workgroup step streams): (j0, j1, flags) with flags bit
    (q + 2k) set when query block 2p+q needs KV block j_k.  A union of odd length ends with a
    super block whose second slot repeats j0 with no flag set.
    Returns (cnt [H*ceil(nQ/2)] super blocks per super-row, row_ptr, list of (j0, j1, flags))."""
    mask = np.asarray(mask)
    H, nQ, nK = mask.shape
    nQ2 = (nQ + 1) // 2
    cnt, row_ptr, sbs = [], [0], []
    for h in range(H):
        for p in range(nQ2):
            r0 = mask[h, 2 * p] != 0
            r1 = mask[h, 2 * p + 1] != 0 if 2 * p + 1 < nQ else np.zeros(nK, dtype=bool)
            union = [int(j) for j in np.flatnonzero(r0 | r1)]
            need = lambda j: int(r0[j]) | (int(r1[j]) << 1)
            for t in range(0, len(union), 2):
                j0 = union[t]
                if t + 1 < len(union):
                    j1 = union[t + 1]
                    sbs.append((j0, j1, need(j0) | (need(j1) << 2)))
                else:
                    sbs.append((j0, j0, need(j0)))
            cnt.append((len(union) + 1) // 2)
            row_ptr.append(len(sbs))
    return cnt, row_ptr, sbs


def pair_rows_pay(mask) -> bool:
    """The library's rule for choosing pair rows by itself: at least 5 / 8 of the (query block, KV block)
    combinations of the super blocks are the mask's own, i.e. active blocks / (4 * super blocks) >= 5 / 8
    (the measured break-even against the plain plan), taken in integers."""
    cnt, _, _ = pair_rows(mask)
    return 2 * int((np.asarray(mask) != 0).sum()) >= 5 * sum(cnt)


def auto_max_item_len(total_blocks: int, P: int) -> int:
    """Split threshold when the caller gives none: max(4, total // (2 P)).

    With every item at most half of the mean partition load, list scheduling's bound
    (max load <= mean + largest item) keeps rho_s <= 1.5 in the worst case; the greedy lands
    far closer, and every split costs a chunk's fixed work plus a merge.
    """
    return max(4, total_blocks // (2 * P))


def make_items(cnt, nQ: int, max_len: int):
    """Work items in row-major order.

    An item is (head, q_block, kv_begin, kv_end): positions [kv_begin, kv_end) inside the
    row's compacted list.  Empty rows give no item.  max_len < 0: never split.  A row with
    cnt > max_len is cut into k = ceil(cnt / max_len) consecutive chunks, chunk t having
    cnt // k + (1 if t < cnt % k else 0) blocks.

    Also returns, per item, `slot` (-1 for a whole row, else the index of the chunk among
    all chunks of split rows, in generation order) and the list of split rows as
    (row, first_slot, n_chunks).
    """
    items, slot, split_rows = [], [], []
    n_slots = 0
    for r, c in enumerate(cnt):
        if c == 0:
            continue
        h, I = divmod(r, nQ)
        if max_len < 0 or c <= max_len:
            items.append((h, I, 0, c))
            slot.append(-1)
            continue
        k = -(-c // max_len)
        base, extra = divmod(c, k)
        split_rows.append((r, n_slots, k))
        pos = 0
        for t in range(k):
            ln = base + (1 if t < extra else 0)
            items.append((h, I, pos, pos + ln))
            slot.append(n_slots)
            n_slots += 1
            pos += ln
        assert pos == c
    return items, slot, split_rows


def lpt_partition(weights, P: int, cost=None):
    """Greedy of Alg. 1 (first loop): returns (assignment per item, load per partition).

    cost[g] (positive integers, optional) is the relative time partition g needs per unit of
    weight; the greedy then compares accumulated time, sum of weight * cost[g], instead of
    accumulated weight (list scheduling on machines of different speed).  Equal costs give the
    paper's rule."""
    cost = [1] * P if cost is None else [int(x) for x in cost]
    order = sorted(range(len(weights)), key=lambda i: -weights[i])   # Python's sort is stable
    time = np.zeros(P, dtype=np.int64)                               # accumulated time per partition
    assign = [0] * len(weights)
    for i in order:
        g = int(np.argmin(time))                                     # first minimum: lowest index wins ties
        assign[i] = g
        time[g] += int(weights[i]) * cost[g]
    loads = [0] * P
    for i, g in enumerate(assign):
        loads[g] += weights[i]
    return assign, loads


def naive_partition(n_items: int, P: int):
    """Items in generation order, dealt in contiguous runs of ceil(n_items / P)."""
    if n_items == 0:
        return []
    run = -(-n_items // P)
    return [i // run for i in range(n_items)]


def dynamic_tail_length(seq, weights, permille: int) -> int:
    """Number of items at the end of the sequence `seq` that are left to a shared queue instead
    of being placed: the longest suffix whose weight is at most permille/1000 of the total
    weight (integer arithmetic: total * permille // 1000).  The compute units take those items
    one by one as they run out of placed work, which is the greedy rule of Alg. 1's first loop
    ("each unit to the least-loaded partition") decided at run time, with the measured
    finishing times as the loads.  Heads come in descending order of their block count, so the
    suffix holds the lightest rows: the last item taken is a short one."""
    budget = sum(weights) * int(permille) // 1000
    n, acc = 0, 0
    for i in reversed(seq):
        if acc + weights[i] > budget:
            break
        acc += weights[i]
        n += 1
    return n


def static_length(n_items: int, tail: int, P: int) -> int:
    """Items that are placed when `tail` items would go to the shared queue: the rest, cut back
    to whole rounds of P (a partial last round would leave the placed loads uneven by an item;
    its items join the queue instead)."""
    n_static = n_items - tail
    return n_static - n_static % P if tail > 0 else n_static


def rounds_partition(item_heads, weights, blocks_per_head, P: int, groups: int = 1, cost=None, tail_permille: int = 0):
    """Round-based greedy placement (locality-preserving variant of the greedy of Alg. 1).

    Heads are taken in descending order of their dense-block count (Alg. 1's sort of
    blocks_per_head; stable).  Their items, in generation order, form one sequence that is
    cut into consecutive rounds of P items.  Inside a round the k-th heaviest item (stable)
    goes to the k-th least-loaded partition (ties: lowest index), so every partition gets at
    most one item per round and all partitions work on the same head at about the same
    time.  This trades a little balance for data reuse, the trade-off the paper steers with
    its reward factor R_b (Methodology, "Block-level Partitioning", overhead mitigation).

    With groups = G > 1 (G divides P; partition p belongs to group p mod G -- the partitions
    that share a cache) the round is first cut into G contiguous chunks of P/G items, i.e.
    runs of neighbouring query blocks.  Chunks are handed to groups by the same greedy one
    level up: heaviest chunk first (stable), each to the group with the least accumulated
    load that has not received a chunk in this round (ties: lowest index).  Inside its group
    a chunk is spread as before: k-th heaviest item to the group's k-th least-loaded partition.
    With cost[g] given (see lpt_partition) "load" is accumulated time, weight * cost[g], everywhere.
    With tail_permille > 0 the items of the sequence past static_length(...) are not placed
    (assignment -1): they form the shared queue.
    Returns (assignment per item, the item sequence).
    """
    cost = [1] * P if cost is None else [int(x) for x in cost]
    if groups < 1 or P % groups != 0:
        raise ValueError("groups must divide the number of partitions")
    H = len(blocks_per_head)
    head_order = sorted(range(H), key=lambda h: -blocks_per_head[h])
    by_head = [[] for _ in range(H)]
    for i, h in enumerate(item_heads):
        by_head[h].append(i)
    seq = [i for h in head_order for i in by_head[h]]
    n_static = static_length(len(seq), dynamic_tail_length(seq, weights, tail_permille) if tail_permille > 0 else 0, P)
    assign = [-1] * len(weights)
    load = [0] * P
    per = P // groups
    for r0 in range(0, n_static, P):
        rnd = seq[r0:min(r0 + P, n_static)]
        chunks = [rnd[j * per:(j + 1) * per] for j in range(groups)]
        chunk_order = sorted(range(groups), key=lambda j: -sum(weights[i] for i in chunks[j]))
        free = list(range(groups))
        for j in chunk_order:
            gamma = min(free, key=lambda g: (sum(load[p] for p in range(g, P, groups)), g))
            free.remove(gamma)
            idx = sorted(chunks[j], key=lambda i: -weights[i])
            parts = sorted(range(gamma, P, groups), key=lambda p: load[p])
            for k, i in enumerate(idx):
                assign[i] = parts[k]
                load[parts[k]] += weights[i] * cost[parts[k]]
    return assign, seq


def reward_partition(q_blocks, weights, nQ: int, P: int, groups: int, reward: float):
    """Greedy longest-first placement with the paper's reward factor R_b (Methodology,
    "Block-level Partitioning", overhead mitigation; Alg. 1, second loop): before the argmin the
    accumulated load of the unit's initial GPU is lowered by R_b times the unit's own count, so a
    unit stays where its data already is unless another GPU is clearly less loaded.

    Carried onto one GPU: partition p belongs to group p mod G (the compute units behind one
    L2); the "initial" group of an item is that of its query block under the contiguous layout,
    q_block * G // nQ, so neighbouring query blocks, which share most of their KV blocks, prefer
    one L2.  Every partition of the home group gets the reward.  Items are taken in descending
    weight order (stable); the biased loads  load[p] - reward * weight  (home group) or
    load[p]  (elsewhere) are compared in float64; first minimum wins (lowest partition index).
    Returns the assignment per item."""
    if groups < 1 or P % groups != 0:
        raise ValueError("groups must divide the number of partitions")
    group_of = np.arange(P) % groups
    load = np.zeros(P, dtype=np.int64)
    assign = [0] * len(weights)
    for i in sorted(range(len(weights)), key=lambda j: -weights[j]):
        home = int(q_blocks[i]) * groups // nQ
        biased = load.astype(np.float64)
        biased[group_of == home] -= float(reward) * float(weights[i])
        p = int(np.argmin(biased))
        assign[i] = p
        load[p] += int(weights[i])
    return assign


def imbalance_ratio(work):
    """Eq. 1: sum_i max_g b[i][g] / (sum_{i,g} b[i][g] / |G|); work is [periods][partitions]."""
    work = [[int(x) for x in row] for row in work]
    G = len(work[0])
    total = sum(sum(row) for row in work)
    if total == 0:
        return 1.0
    num = sum(max(row) for row in work)
    return float(num) / (float(total) / float(G))


def ring_work_matrix(chunk_blocks):
    """Eq. 3's b[i][g]: dense blocks between Q chunk g and KV chunk (i+g) mod |G|.

    chunk_blocks[q][kv] = dense blocks (summed over heads) between Q chunk q and KV chunk kv.
    """
    G = len(chunk_blocks)
    return [[int(chunk_blocks[g][(i + g) % G]) for g in range(G)] for i in range(G)]


def carry_over_partition(previous, items, nQ: int, P: int):
    """Placement of `items` taken from a previous plan (paper: Methodology, "Head-level
    Partitioning", overhead mitigation -- the last step's plan is kept while rho_s stays under
    a threshold P_s; Alg. 1, first test).

    The paper carries a head -> GPU map over; here the unit is a work item, named by its row
    and its ordinal among that row's items.  An item the previous plan also had keeps that
    item's partition.  The others (a row that was empty before, or that is now cut into more
    pieces, or whose item the previous plan had left to its shared queue) are taken in item order, each going to the partition with the least load in blocks
    (lowest index on ties), after all carried-over items are in place.
    Returns (assign, loads)."""
    prev_part = {}
    for g in range(P):
        for i in previous["part_items"][previous["part_ptr"][g]:previous["part_ptr"][g + 1]]:
            prev_part[i] = g
    by_key = {}
    ordinal = {}
    for i, (h, qb, _, _) in enumerate(previous["items"]):
        t = ordinal.get((h, qb), 0)
        ordinal[(h, qb)] = t + 1
        by_key[(h, qb, t)] = prev_part.get(i)      # None: the item sat in the previous plan's shared queue
    assign = [None] * len(items)
    loads = [0] * P
    ordinal = {}
    for i, (h, qb, b, e) in enumerate(items):
        t = ordinal.get((h, qb), 0)
        ordinal[(h, qb)] = t + 1
        g = by_key.get((h, qb, t))
        if g is not None:
            assign[i] = g
            loads[g] += e - b
    for i, (h, qb, b, e) in enumerate(items):
        if assign[i] is None:
            g = min(range(P), key=lambda j: (loads[j], j))
            assign[i] = g
            loads[g] += e - b
    return assign, loads


def plan(mask, P: int, mode: int = MODE_BALANCED, max_item_len: int = 0, item_overhead: int = 0,
         previous=None, reuse_threshold: float = 1.0, locality_groups: int = 1, partition_cost=None,
         dynamic_tail: int = 0, reward: float = 0.0, pair: bool = False):
    """Full plan as plain Python lists/ints (the arrays the library must reproduce bit-exactly).

    With `previous` (a plan of the same geometry and P), the previous placement is kept when the
    new mask's rho_s under it is <= reuse_threshold; `reused` and `rho_reuse` report the outcome.
    dynamic_tail (permille of the total weight, round-based placement only, not with a carried-over
    placement): the end of the item sequence goes to `tail_items`, a queue shared by all partitions,
    and is in no partition's list; part_load and rho_plan then cover the placed items only.
    reward (MODE_REWARD only): the paper's R_b, see reward_partition.
    pair: rows are the super-rows of pair_rows (two query blocks each) and the unit of work is the
    super block; nQ, cnt, row_ptr, items, nnz are then in those units and kv_idx holds, per super
    block, j0 and j1 | flags << 24.  pair = "auto": decided by pair_rows_pay (a chain of plans keeps the
    first one's choice); the result's "pair" says which."""
    mask = np.asarray(mask)
    H, nQ, nK = mask.shape
    if pair == "auto":
        pair = previous["pair"] if previous is not None else pair_rows_pay(mask)
    if pair:
        cnt, row_ptr, sbs = pair_rows(mask)
        nQ = (nQ + 1) // 2
        per_head = [sum(cnt[h * nQ:(h + 1) * nQ]) for h in range(H)]
        total = sum(cnt)
        kv_idx = [v for (j0, j1, f) in sbs for v in (j0, j1 | (f << 24))]
    else:
        cnt, per_head, total = row_counts(mask)
        row_ptr, kv_idx = compact(mask)
    L = auto_max_item_len(total, P) if max_item_len == 0 else max_item_len
    items, slot, split_rows = make_items(cnt, nQ, L)
    lens = [e - b for (_, _, b, e) in items]
    weights = [ln + item_overhead for ln in lens]

    lpt_assign, _ = lpt_partition(weights, P, partition_cost)
    nv_assign = naive_partition(len(items), P)

    def loads_of(assign):
        ld = [0] * P
        for i, g in enumerate(assign):
            if g >= 0:
                ld[g] += lens[i]
        return ld

    rho_bal = imbalance_ratio([loads_of(lpt_assign)])
    rho_naive = imbalance_ratio([loads_of(nv_assign)])
    order = range(len(items))
    reused, rho_reuse = False, 0.0
    if previous is not None:
        ru_assign, ru_loads = carry_over_partition(previous, items, nQ, P)
        rho_reuse = imbalance_ratio([ru_loads])
        reused = rho_reuse <= reuse_threshold
    if reused:
        assign = ru_assign
    elif mode == MODE_BALANCED:
        assign = lpt_assign
    elif mode == MODE_NAIVE:
        assign = nv_assign
    elif mode == MODE_REWARD:
        assign = reward_partition([it[1] for it in items], weights, nQ, P, max(1, locality_groups), reward)
    else:
        assign, order = rounds_partition([it[0] for it in items], weights, per_head, P, max(1, locality_groups), partition_cost,
                                         tail_permille=dynamic_tail)
    tail_items = [i for i in order if assign[i] < 0]

    # per-partition lists: ascending item id = ascending (head, q_block, kv_begin); for the
    # round-based placement, the order of the rounds
    lists = [[] for _ in range(P)]
    for i in order:
        if assign[i] >= 0:
            lists[assign[i]].append(i)
    part_ptr = [0]
    part_items = []
    for g in range(P):
        part_items.extend(lists[g])
        part_ptr.append(len(part_items))

    return dict(
        H=H, nQ=nQ, nK=nK, P=P, max_item_len=L,
        cnt=cnt, blocks_per_head=per_head, nnz=total,
        row_ptr=row_ptr, kv_idx=kv_idx,
        items=items, item_slot=slot, split_rows=split_rows,
        part_ptr=part_ptr, part_items=part_items, tail_items=tail_items,
        part_load=loads_of(assign),
        rho_naive=rho_naive, rho_balanced=rho_bal, rho_plan=imbalance_ratio([loads_of(assign)]),
        reused=reused, rho_reuse=rho_reuse, pair=bool(pair),
    )


def calibrate_cost(busy, load):
    """Relative time per block of every partition from one launch's busy times, as integers with
    mean about 1024: cost[g] = round(1024 * (busy[g] / load[g]) / (sum busy / sum load)), in
    exact integer arithmetic (round half up), clamped to [512, 2048]; 1024 for a partition
    without work or without a measurement.  Feeding it back to the placement evens out compute
    units that run at different speeds (the paper fits its latency constants from profiles:
    Methodology, "Sparsity-aware Strategy Selection")."""
    pairs = [(int(b), int(l)) for b, l in zip(busy, load)]
    sb = sum(b for b, l in pairs if b > 0 and l > 0)
    sl = sum(l for b, l in pairs if b > 0 and l > 0)
    out = []
    for b, l in pairs:
        if b <= 0 or l <= 0 or sb == 0:
            out.append(1024)
            continue
        num, den = b * 1024 * sl, l * sb
        out.append(min(2048, max(512, (2 * num + den) // (2 * den))))
    return out
