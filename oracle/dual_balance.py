"""Oracle: the dual-balancing partitioning across GPUs (heads over a Ulysses group of x GPUs,
Q blocks over a ring of y GPUs and KV blocks over its y iterations), and the ring form of rho_s.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is followed:
  * head-level greedy (Methodology, "Head-level Partitioning"; Alg. 1, first branch): heads in
    descending order of their dense-block count, each to the GPU with the least accumulated
    count; the last step's plan is kept while rho_s of the current mask under it is <= P_s;
  * block-level greedy (Methodology, "Block-level Partitioning"; Alg. 1, second branch): the
    mask is summed over heads; Q blocks sorted by their row sums go greedily to GPUs, KV blocks
    sorted by their column sums go greedily to ring iterations (= KV chunks);
  * reward factor R_b (same section, overhead mitigation): before the argmin, the load of the
    block's initial GPU is lowered by R_b times the block's own count;
  * ring rho_s (Eq. 3): b[i][g] = dense blocks between Q chunk g and KV chunk (i+g) mod y,
    accumulated over all heads; rho_s = sum_i max_g b[i][g] / (sum b / y).

Readings where the paper is silent, garbled or at odds with itself:
  * sorts are stable (equal counts keep ascending id); argmin ties go to the lowest GPU index;
  * reward: the prose (R_b times the block's count, scale-free) is taken, not the listing's
    absolute "s - R_b"; the comparison is done in float64 on  load - R_b*w;
  * the initial GPU of block j of n is j // ceil(n / y) (contiguous chunks, the layout sequence
    parallelism starts from); the same rule gives a KV block's initial chunk and a head's GPU
    under the unbalanced contiguous Ulysses split;
  * capacity: the published text states no limit, an earlier draft fills only groups that are
    "not yet full"; capacity = 0 means no limit, capacity = c > 0 skips GPUs already holding c
    units (needed when the exchange must move equal-sized chunks);
  * per-GPU lists hold ids in the order they were placed (the order of the listing's append);
  * the reuse test evaluates the *current* counts under the *previous* head -> GPU map; equality
    with P_s keeps the plan; with x == 1 nothing is partitioned (Alg. 1's guard).
"""

from __future__ import annotations

import numpy as np


def rho_one_period(loads):
    """Eq. 2 (one synchronisation period): max_g / mean_g; 1.0 when there is no work."""
    total = sum(int(v) for v in loads)
    if total == 0:
        return 1.0
    return float(max(int(v) for v in loads)) / (float(total) / float(len(loads)))


def contiguous_owner(n: int, groups: int):
    """Initial layout: unit j of n sits in group j // ceil(n / groups)."""
    run = -(-n // groups) if n else 1
    return [j // run for j in range(n)]


def biased_greedy(counts, groups: int, reward: float = 0.0, initial=None, capacity: int = 0):
    """Greedy placement of units with the given counts onto `groups` bins.

    Units are taken in descending count order (stable).  For each, the candidate loads are the
    bins' accumulated counts, except that the unit's initial bin is credited reward * count;
    the unit goes to the smallest candidate among bins that are not full (lowest index on
    ties).  Returns (bin of each unit, per-bin lists in placement order, per-bin loads)."""
    n = len(counts)
    if capacity and capacity * groups < n:
        raise ValueError("capacity too small to hold every unit")
    load = np.zeros(groups, dtype=np.int64)
    units = np.zeros(groups, dtype=np.int64)
    where = [0] * n
    lists = [[] for _ in range(groups)]
    for j in sorted(range(n), key=lambda u: -int(counts[u])):          # descending, stable
        w = int(counts[j])
        biased = load.astype(np.float64)                               # what the argmin looks at
        if initial is not None and reward != 0.0:
            biased[initial[j]] -= float(reward) * float(w)             # the unit's own GPU looks emptier
        if capacity:
            biased[units >= capacity] = np.inf                         # full GPUs are out
        g = int(np.argmin(biased))                                     # first minimum: lowest index on ties
        where[j] = g
        lists[g].append(j)
        load[g] += w
        units[g] += 1
    return where, lists, [int(v) for v in load]


def partition_heads(blocks_per_head, x: int, capacity: int = 0, previous=None, reuse_threshold: float = 1.0):
    """Head-level partitioning with plan reuse.  Returns a dict:
    gpu_of_head, lists, loads, rho_contiguous (heads dealt in contiguous runs), rho (of the
    returned plan), rho_previous (current counts under `previous`, 0.0 if none), reused."""
    H = len(blocks_per_head)
    cont = contiguous_owner(H, x)
    cont_loads = [0] * x
    for h, g in enumerate(cont):
        cont_loads[g] += int(blocks_per_head[h])
    rho_prev, reused = 0.0, False
    if previous is not None:
        prev_loads = [0] * x
        for h, g in enumerate(previous):
            prev_loads[g] += int(blocks_per_head[h])
        rho_prev = rho_one_period(prev_loads)
        reused = x == 1 or rho_prev <= reuse_threshold
    if reused:
        where = [int(g) for g in previous]
        lists = [[h for h in range(H) if where[h] == g] for g in range(x)]
        loads = prev_loads
    elif x == 1:
        where, lists, loads = [0] * H, [list(range(H))], [sum(int(v) for v in blocks_per_head)]
    else:
        where, lists, loads = biased_greedy(blocks_per_head, x, capacity=capacity)
    return dict(gpu_of_head=where, lists=lists, loads=loads, rho_contiguous=rho_one_period(cont_loads),
                rho=rho_one_period(loads), rho_previous=rho_prev, reused=reused)


def chunk_blocks(mask, gpu_of_q, chunk_of_kv, y: int):
    """C[g][c] = dense blocks, over all heads, between the Q blocks of GPU g and the KV blocks of chunk c."""
    acc = (np.asarray(mask) != 0).sum(axis=0)
    C = [[0] * y for _ in range(y)]
    for i in range(acc.shape[0]):
        for j in range(acc.shape[1]):
            C[gpu_of_q[i]][chunk_of_kv[j]] += int(acc[i, j])
    return C


def ring_work(mask, gpu_of_q, chunk_of_kv, y: int):
    """Eq. 3's matrix: work[i][g] = C[g][(i + g) mod y] for iteration i and GPU g."""
    C = chunk_blocks(mask, gpu_of_q, chunk_of_kv, y)
    return [[C[g][(i + g) % y] for g in range(y)] for i in range(y)]


def ring_rho(work):
    """Eq. 3: sum over iterations of the slowest GPU's count, over the per-GPU mean of all work."""
    y = len(work)
    total = sum(sum(row) for row in work)
    if total == 0:
        return 1.0
    return float(sum(max(row) for row in work)) / (float(total) / float(y))


def partition_blocks(mask, y: int, reward: float = 0.0, capacity_q: int = 0, capacity_kv: int = 0):
    """Block-level partitioning of one mask [H, nQ, nK] for a ring of y GPUs.  Returns a dict:
    gpu_of_q, q_lists, chunk_of_kv, kv_lists, work (Eq. 3's matrix under the plan), rho (its
    rho_s), rho_contiguous (rho_s of the contiguous layout), moved_q / moved_kv (blocks that
    leave their initial GPU / chunk)."""
    acc = (np.asarray(mask) != 0).sum(axis=0)            # blocks_accum_by_head
    nQ, nK = acc.shape
    per_q = [int(v) for v in acc.sum(axis=1)]            # for each Q block, its KV blocks
    per_kv = [int(v) for v in acc.sum(axis=0)]           # for each KV block, its Q blocks
    q0, kv0 = contiguous_owner(nQ, y), contiguous_owner(nK, y)
    if y == 1:
        gq, ql, gkv, kvl = [0] * nQ, [list(range(nQ))], [0] * nK, [list(range(nK))]
    else:
        gq, ql, _ = biased_greedy(per_q, y, reward, q0, capacity_q)
        gkv, kvl, _ = biased_greedy(per_kv, y, reward, kv0, capacity_kv)
    work = ring_work(mask, gq, gkv, y)
    return dict(gpu_of_q=gq, q_lists=ql, chunk_of_kv=gkv, kv_lists=kvl, work=work, rho=ring_rho(work),
                rho_contiguous=ring_rho(ring_work(mask, q0, kv0, y)),
                moved_q=sum(1 for a, b in zip(gq, q0) if a != b), moved_kv=sum(1 for a, b in zip(gkv, kv0) if a != b))
