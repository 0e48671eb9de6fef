"""Pins for the multi-GPU planner oracle (oracle/dual_balance.py): hand-traced runs of the greedy
with and without reward and capacity, a second independent greedy (a priority-queue one written in the test), a step-by-step replay of
the placement rule, the classical 4/3 - 1/(3m) bound against a brute-force optimum, brute-force
ring work on tiny masks, and the special cases whose rho_s is known in closed form."""

import itertools

import numpy as np
import pytest

import synth
from oracle import dual_balance as db
from oracle import planner as op


def test_heads_by_hand():
    # 9,7,6,5,4,3 on 2 GPUs: 9->g0, 7->g1, 6->g1 (13), 5->g0 (14), 4->g1 (17), 3->g0 (17)
    r = db.partition_heads([9, 7, 6, 5, 4, 3], 2)
    assert r["gpu_of_head"] == [0, 1, 1, 0, 1, 0] and r["loads"] == [17, 17] and r["rho"] == 1.0
    assert r["lists"] == [[0, 3, 5], [1, 2, 4]]
    # contiguous split {9,7,6} / {5,4,3} = 22 / 12 -> rho = 22 / 17
    assert r["rho_contiguous"] == 22 / 17 and not r["reused"] and r["rho_previous"] == 0.0
    # unsorted input, ties: equal counts keep ascending head id, equal loads go to the lowest GPU
    r = db.partition_heads([2, 5, 2, 5], 3)
    assert r["gpu_of_head"] == [2, 0, 2, 1] and r["loads"] == [5, 5, 4] and r["lists"] == [[1], [3], [0, 2]]


def test_heads_reuse_by_hand():
    prev = [0, 1, 1, 0, 1, 0]                        # the plan of test_heads_by_hand
    # new counts 10,7,6,5,4,3: under prev {10+5+3, 7+6+4} = {18, 17}: rho = 18 / 17.5
    r = db.partition_heads([10, 7, 6, 5, 4, 3], 2, previous=prev, reuse_threshold=1.05)
    assert r["reused"] and r["rho_previous"] == 18 / 17.5 == r["rho"] and r["gpu_of_head"] == prev and r["loads"] == [18, 17]
    assert r["lists"] == [[0, 3, 5], [1, 2, 4]]
    r = db.partition_heads([10, 7, 6, 5, 4, 3], 2, previous=prev, reuse_threshold=1.02)
    assert not r["reused"] and r["rho_previous"] == 18 / 17.5
    # fresh: 10->g0, 7->g1, 6->g1 (13), 5->g0 (15), 4->g1 (17), 3->g0 (18): same loads, re-planned anyway
    assert r["loads"] == [18, 17]
    # equality keeps the plan; one GPU never partitions
    assert db.partition_heads([10, 7, 6, 5, 4, 3], 2, previous=prev, reuse_threshold=18 / 17.5)["reused"]
    one = db.partition_heads([3, 1], 1, previous=[0, 0], reuse_threshold=1.0)
    assert one["reused"] and one["rho"] == 1.0 and db.partition_heads([3, 1], 1)["lists"] == [[0, 1]]


def test_capacity_by_hand():
    # 10,1,1,1 on 2 GPUs: free -> {10} {1,1,1}; with at most 2 heads per GPU the last 1 must join the 10
    assert db.biased_greedy([10, 1, 1, 1], 2)[2] == [10, 3]
    where, lists, loads = db.biased_greedy([10, 1, 1, 1], 2, capacity=2)
    assert where == [0, 1, 1, 0] and lists == [[0, 3], [1, 2]] and loads == [11, 2]
    with pytest.raises(ValueError):
        db.biased_greedy([1, 1, 1], 2, capacity=1)
    rng = np.random.default_rng(0)
    for _ in range(50):
        g = int(rng.integers(1, 6))
        cap = int(rng.integers(1, 5))
        n = int(rng.integers(0, g * cap + 1))
        where, lists, loads = db.biased_greedy(rng.integers(0, 50, n).tolist(), g, capacity=cap)
        assert all(len(l) <= cap for l in lists) and sorted(sum(lists, [])) == list(range(n))


def test_reward_by_hand():
    # per-block counts 4,4,2,2 over 2 GPUs, initial owners 0,0,1,1
    init = [0, 0, 1, 1]
    # no reward: 4->g0, 4->g1, 2->g0 (tie, lowest), 2->g1
    assert db.biased_greedy([4, 4, 2, 2], 2, 0.0, init)[0] == [0, 1, 0, 1]
    # R_b = 0.6: b0: [0-2.4, 0] -> g0.  b1: [4-2.4, 0] -> g1.  b2 (home g1): [4, 4-1.2] -> g1.  b3 (home g1): [4, 6-1.2] -> g0
    where, lists, loads = db.biased_greedy([4, 4, 2, 2], 2, 0.6, init)
    assert where == [0, 1, 1, 0] and loads == [6, 6] and lists == [[0, 3], [1, 2]]
    # R_b = 1.5: b1: [4-6, 0] -> stays on g0.  b2: [8, 0-3] -> g1.  b3: [8, 2-3] -> g1: nothing moves
    where, lists, loads = db.biased_greedy([4, 4, 2, 2], 2, 1.5, init)
    assert where == init and loads == [8, 4]


def _heap_greedy(w, g):
    # the same rule written a second way: a priority queue of (load, bin) instead of a scan
    import heapq
    heap = [(0, b) for b in range(g)]
    where = [0] * len(w)
    for j in sorted(range(len(w)), key=lambda u: (-w[u], u)):
        load, b = heapq.heappop(heap)
        where[j] = b
        heapq.heappush(heap, (load + w[j], b))
    return where


def test_unbiased_greedy_equals_a_priority_queue_greedy():
    rng = np.random.default_rng(1)
    for _ in range(200):
        n, g = int(rng.integers(0, 40)), int(rng.integers(1, 9))
        w = rng.integers(0, 30, n).tolist()
        where, _, loads = db.biased_greedy(w, g)
        assign, loads2 = op.lpt_partition(w, g)
        assert where == assign == _heap_greedy(w, g) and loads == loads2


def test_every_unit_lands_on_the_smallest_biased_load_among_open_bins():
    # replay the returned placement in the order it was made (descending count, stable) and check
    # the rule itself at every step: among bins that are not full, none had a smaller load after
    # crediting the unit's home bin with reward * count, and no lower-indexed bin had an equal one
    rng = np.random.default_rng(7)
    for _ in range(300):
        g = int(rng.integers(1, 6))
        n = int(rng.integers(0, 14))
        cap = int(rng.integers(0, 5))
        if cap and cap * g < n:
            cap = 0
        w = rng.integers(0, 12, n).tolist()
        home = rng.integers(0, g, n).tolist()
        reward = float(rng.choice([0.0, 0.25, 0.6, 1.0, 3.0]))
        where, lists, loads = db.biased_greedy(w, g, reward, home, cap)
        load, held = [0] * g, [0] * g
        for j in sorted(range(n), key=lambda u: (-w[u], u)):
            seen = {b: load[b] - (reward * w[j] if b == home[j] else 0.0) for b in range(g) if not cap or held[b] < cap}
            lowest = min(seen.values())
            assert where[j] == min(b for b, val in seen.items() if val == lowest), (w, home, reward, cap, j)
            load[where[j]] += w[j]
            held[where[j]] += 1
        assert load == loads and [sorted(l) for l in lists] == [sorted(j for j in range(n) if where[j] == b) for b in range(g)]


def _optimal_makespan(w, g):
    best = sum(w)
    for assign in itertools.product(range(g), repeat=len(w)):
        loads = [0] * g
        for wi, a in zip(w, assign):
            loads[a] += wi
        best = min(best, max(loads))
    return best


def test_greedy_is_within_the_longest_first_bound_of_the_optimum():
    # Graham's bound for longest-processing-time-first: makespan <= (4/3 - 1/(3m)) * optimum
    rng = np.random.default_rng(2)
    for _ in range(60):
        g = int(rng.integers(2, 4))
        w = rng.integers(1, 20, int(rng.integers(1, 8))).tolist()
        loads = db.biased_greedy(w, g)[2]
        assert max(loads) <= (4 / 3 - 1 / (3 * g)) * _optimal_makespan(w, g) + 1e-9


def test_large_reward_keeps_every_block_at_home():
    mask = synth.random_mask(3, 12, 20, 0.4, seed=4)
    r = db.partition_blocks(mask, 4, reward=1e9)
    assert r["gpu_of_q"] == db.contiguous_owner(12, 4) and r["chunk_of_kv"] == db.contiguous_owner(20, 4)
    assert r["moved_q"] == 0 and r["moved_kv"] == 0 and r["rho"] == r["rho_contiguous"]


def test_ring_by_hand():
    # one head, 2x2 blocks, mask [[1,1],[0,1]], 2 GPUs, contiguous: C = [[1,1],[0,1]]
    # iteration 0: GPU0 x chunk0 = 1, GPU1 x chunk1 = 1;  iteration 1: GPU0 x chunk1 = 1, GPU1 x chunk0 = 0
    mask = np.array([[[1, 1], [0, 1]]], dtype=np.uint8)
    work = db.ring_work(mask, [0, 1], [0, 1], 2)
    assert work == [[1, 1], [1, 0]] and db.ring_rho(work) == 2 / 1.5
    # swapping the KV chunks: iteration 0: GPU0 x chunk0 (= kv block 1) = 1, GPU1 x chunk1 (= kv block 0) = 0
    assert db.ring_work(mask, [0, 1], [1, 0], 2) == [[1, 0], [1, 1]]
    # 3 GPUs, one Q block each, KV block c in chunk c, one head: work[i][g] = mask[g][(i+g) % 3]
    m = np.array([[[1, 0, 1], [1, 1, 0], [0, 0, 1]]], dtype=np.uint8)
    assert db.ring_work(m, [0, 1, 2], [0, 1, 2], 3) == [[1, 1, 1], [0, 0, 0], [1, 1, 0]]
    assert db.ring_rho([[1, 1, 1], [0, 0, 0], [1, 1, 0]]) == 2 / (5 / 3)


def test_ring_work_brute_force():
    rng = np.random.default_rng(5)
    for _ in range(20):
        H, nQ, nK, y = int(rng.integers(1, 4)), int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 5))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=int(rng.integers(1 << 30)))
        gq, gk = rng.integers(0, y, nQ).tolist(), rng.integers(0, y, nK).tolist()
        expect = [[0] * y for _ in range(y)]
        for h in range(H):
            for i in range(nQ):
                for j in range(nK):
                    if mask[h, i, j]:
                        g, c = gq[i], gk[j]
                        expect[(c - g) % y][g] += 1          # GPU g meets chunk c in iteration (c - g) mod y
        work = db.ring_work(mask, gq, gk, y)
        assert work == expect and sum(map(sum, work)) == int((mask != 0).sum())
        assert db.ring_rho(work) == op.imbalance_ratio(work)     # Eq. 3 is Eq. 1 with y periods and y GPUs


def test_closed_form_cases():
    ones = np.ones((2, 8, 8), dtype=np.uint8)
    for y in (1, 2, 4, 8):
        r = db.partition_blocks(ones, y)
        assert r["rho"] == 1.0 and r["rho_contiguous"] == 1.0
    # all the work in the first Q chunk: every iteration waits for GPU 0 -> rho_s = y
    top = np.zeros((1, 8, 8), dtype=np.uint8)
    top[:, :2, :] = 1
    r = db.partition_blocks(top, 4)
    assert r["rho_contiguous"] == 4.0
    # the two busy Q blocks go to two GPUs, two KV blocks per chunk: each of the 4 iterations costs 2 on
    # the slowest GPU = 8, against 16 blocks / 4 GPUs = 4 -> rho_s = 2 (two of four GPUs can be kept busy)
    assert r["rho"] == 2.0 and sorted(r["gpu_of_q"][:2]) == [0, 1]
    # block-diagonal mask in the contiguous layout: all work happens in iteration 0, evenly -> rho_s = 1
    diag = np.zeros((1, 8, 8), dtype=np.uint8)
    for g in range(4):
        diag[0, 2 * g:2 * g + 2, 2 * g:2 * g + 2] = 1
    assert db.partition_blocks(diag, 4, reward=1e9)["rho"] == 1.0
    # empty mask
    z = db.partition_blocks(np.zeros((1, 4, 4), dtype=np.uint8), 2)
    assert z["rho"] == 1.0 and z["work"] == [[0, 0], [0, 0]]
    # one GPU: identity plan
    one = db.partition_blocks(synth.random_mask(2, 5, 7, 0.5, seed=1), 1)
    assert one["q_lists"] == [list(range(5))] and one["kv_lists"] == [list(range(7))] and one["rho"] == 1.0


def test_partition_invariants_and_effect_on_the_paper_shaped_masks():
    # the paper reports rho_s <= 1.1 after head-level and <= 1.05 after block-level partitioning on
    # its video masks (Methodology); the synthetic masks of the same shape statistics get there too
    for cfg, x in ((2, 8), (3, 8), (4, 8)):
        mask = synth.mask_for_config(cfg)
        per_head = (mask != 0).sum(axis=(1, 2)).tolist()
        r = db.partition_heads(per_head, x)
        assert sorted(sum(r["lists"], [])) == list(range(len(per_head))) and sum(r["loads"]) == sum(per_head)
        assert r["rho"] <= r["rho_contiguous"] and r["rho"] <= 1.1
    mask = synth.mask_for_config(5)
    for y in (2, 4, 8):
        r = db.partition_blocks(mask, y)
        assert sorted(sum(r["q_lists"], [])) == list(range(mask.shape[1]))
        assert sorted(sum(r["kv_lists"], [])) == list(range(mask.shape[2]))
        assert sum(map(sum, r["work"])) == int((mask != 0).sum())
        assert r["rho"] <= r["rho_contiguous"] and r["rho"] <= 1.05
    # reward trades balance for data that stays put: moved blocks never increase with R_b here
    moved = [db.partition_blocks(mask, 4, reward=rb)["moved_q"] for rb in (0.0, 0.5, 2.0, 1e9)]
    assert moved[-1] == 0 and moved[0] >= moved[-1]
