"""Host-side checks of libdbsp through its C ABI (no GPU needed): the library loads and
exports every symbol dbsp.h declares, argument errors map to the documented codes, and the
planner's integer arrays and rho_s equal the oracle's bit for bit."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
from oracle import planner as op
import paper_2511_23113_amd as dbsp
from paper_2511_23113_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):       # the boundary and the diagnostics header
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(?:int|void|const char\s*\*)\s+([a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def _plan_raw(mask_ptr, H, nQ, nK, block, opts=None):
    lib = B.load_library()
    out = C.c_void_p()
    rc = lib.plan_sparse_attn(mask_ptr, H, nQ, nK, block, C.byref(opts) if opts is not None else None, C.byref(out))
    return rc, out


def test_argument_errors():
    lib = B.load_library()
    m = np.ones((1, 2, 2), dtype=np.uint8)
    mp = m.ctypes.data_as(C.c_void_p)
    host = B.PlanOpts(4, 0, 0, 0, B.PLAN_HOST_ONLY)
    assert _plan_raw(None, 1, 2, 2, 64, host)[0] == B.DBSP_EINVAL
    assert lib.plan_sparse_attn(mp, 1, 2, 2, 64, C.byref(host), None) == B.DBSP_EINVAL
    for bad in ((0, 2, 2, 64), (1, 0, 2, 64), (1, 2, -1, 64), (1, 2, 2, 0)):
        assert _plan_raw(mp, *bad, host)[0] == B.DBSP_EINVAL
    assert b"positive" in lib.dbsp_last_error()
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(-1, 0, 0, 0, B.PLAN_HOST_ONLY))[0] == B.DBSP_EINVAL
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(4, 7, 0, 0, B.PLAN_HOST_ONLY))[0] == B.DBSP_EINVAL
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(4, 0, 0, -2, B.PLAN_HOST_ONLY))[0] == B.DBSP_EINVAL
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(4, 0, 0, 0, 8))[0] == B.DBSP_EINVAL
    rc, plan = _plan_raw(mp, 1, 2, 2, 64, host)
    assert rc == B.DBSP_OK and plan.value
    one = C.c_void_p(16)  # never dereferenced: every call below must fail on its checks first
    fwd = lambda *a: lib.sparse_attn_fwd(*a)
    assert fwd(None, one, one, one, one, None, 1, 128, 128, 64, 0.0, None) == B.DBSP_EINVAL
    assert fwd(plan, None, one, one, one, None, 1, 128, 128, 64, 0.0, None) == B.DBSP_EINVAL
    assert fwd(plan, one, one, one, one, None, 0, 128, 128, 64, 0.0, None) == B.DBSP_EINVAL
    assert fwd(plan, one, one, one, one, None, 1, 128, 128, 96, 0.0, None) == B.DBSP_EINVAL
    assert fwd(plan, one, one, one, one, None, 1, 130, 128, 64, 0.0, None) == B.DBSP_ESHAPE
    assert fwd(plan, one, one, one, one, None, 1, 128, 256, 64, 0.0, None) == B.DBSP_ESHAPE
    assert fwd(plan, one, one, one, one, None, 1, 128, 128, 64, 0.0, None) == B.DBSP_EINVAL  # host-only plan
    assert b"host-only" in lib.dbsp_last_error()
    assert lib.dbsp_plan_busy(plan, None, None, None) == B.DBSP_EINVAL
    data, cnt = C.c_void_p(), C.c_int64()
    assert lib.dbsp_plan_get(plan, 99, C.byref(data), C.byref(cnt)) == B.DBSP_EINVAL
    assert lib.dbsp_plan_get(plan, B.ROW_PTR, None, C.byref(cnt)) == B.DBSP_EINVAL
    lib.dbsp_plan_destroy(plan)
    lib.dbsp_plan_destroy(None)
    # unsupported block size is a forward-pass error, not a planning error
    rc, plan = _plan_raw(mp, 1, 2, 2, 32, host)
    assert rc == B.DBSP_OK
    assert fwd(plan, one, one, one, one, None, 1, 64, 64, 64, 0.0, None) == B.DBSP_EINVAL
    lib.dbsp_plan_destroy(plan)
    rho = C.c_double()
    w = np.array([[1, 2]], dtype=np.int64)
    assert lib.imbalance_ratio(None, 1, 2, C.byref(rho)) == B.DBSP_EINVAL
    assert lib.imbalance_ratio(w.ctypes.data_as(C.c_void_p), 0, 2, C.byref(rho)) == B.DBSP_EINVAL
    wn = np.array([[1, -2]], dtype=np.int64)
    assert lib.imbalance_ratio(wn.ctypes.data_as(C.c_void_p), 1, 2, C.byref(rho)) == B.DBSP_EINVAL


def test_imbalance_ratio_matches_oracle_and_hand_values():
    assert B.imbalance_ratio([[12, 4]]) == 1.5
    assert B.imbalance_ratio([[4, 3], [0, 1]]) == 1.25
    assert B.imbalance_ratio([[0, 0, 0]]) == 1.0
    rng = np.random.default_rng(5)
    for _ in range(100):
        w = rng.integers(0, 1000, size=(int(rng.integers(1, 6)), int(rng.integers(1, 20))))
        assert B.imbalance_ratio(w) == op.imbalance_ratio(w.tolist())


def _assert_plan_equal(mask, block, P, mode, L, c0, G=0, cost=None, tail=0, reward=0.0, pair=False):
    pl = B.plan_sparse_attn(mask, block, num_partitions=P, mode=mode, max_item_len=L, item_overhead=c0, host_only=True,
                            locality_groups=G, partition_cost=cost, dynamic_tail=tail, reward=reward, pair_rows=pair)
    ref = op.plan(mask, P, mode=mode, max_item_len=L, item_overhead=c0, locality_groups=G, partition_cost=cost,
                  dynamic_tail=tail, reward=reward, pair=pair)
    st = pl.stats()
    assert st["nnz"] == ref["nnz"] and st["n_items"] == len(ref["items"])
    assert st["num_partitions"] == P and st["max_item_len"] == ref["max_item_len"]
    assert st["rho_naive"] == ref["rho_naive"] and st["rho_balanced"] == ref["rho_balanced"]   # bit-exact doubles
    assert st["rho_plan"] == ref["rho_plan"]
    eq = np.testing.assert_array_equal
    eq(pl.array(B.ROW_CNT), np.array(ref["cnt"], dtype=np.int32))
    eq(pl.array(B.BLOCKS_PER_HEAD), np.array(ref["blocks_per_head"], dtype=np.int64))
    eq(pl.array(B.ROW_PTR), np.array(ref["row_ptr"], dtype=np.int32))
    eq(pl.array(B.KV_IDX), np.array(ref["kv_idx"], dtype=np.int32))
    eq(pl.array(B.ITEMS), np.array(ref["items"], dtype=np.int32).reshape(-1))
    eq(pl.array(B.ITEM_SLOT), np.array(ref["item_slot"], dtype=np.int32))
    eq(pl.array(B.SPLIT_ROWS), np.array([(r, s, k, 0) for r, s, k in ref["split_rows"]], dtype=np.int32).reshape(-1))
    eq(pl.array(B.PART_PTR), np.array(ref["part_ptr"], dtype=np.int32))
    eq(pl.array(B.PART_ITEMS), np.array(ref["part_items"], dtype=np.int32))
    eq(pl.array(B.PART_LOAD), np.array(ref["part_load"], dtype=np.int64))
    eq(pl.array(B.TAIL_ITEMS), np.array(ref["tail_items"], dtype=np.int32))
    empty = [r for r, c in enumerate(ref["cnt"]) if c == 0]
    eq(pl.array(B.EMPTY_ROWS), np.array(empty, dtype=np.int32))
    pl.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_planner_bit_exact_on_configs(cfg):
    mask = synth.mask_for_config(cfg)
    block = synth.CONFIGS[cfg]["block"]
    for mode in (B.MODE_BALANCED, B.MODE_NAIVE, B.MODE_ROUNDS):
        _assert_plan_equal(mask, block, 256, mode, 0, 0)
    if cfg in (1, 5):
        _assert_plan_equal(mask, block, 8, B.MODE_BALANCED, 0, 0)
        _assert_plan_equal(mask, block, 304, B.MODE_BALANCED, 16, 3)
        _assert_plan_equal(mask, block, 256, B.MODE_BALANCED, -1, 0)


@pytest.mark.parametrize("seed", range(12))
def test_planner_bit_exact_random_small(seed):
    rng = np.random.default_rng(100 + seed)
    H, nQ, nK = int(rng.integers(1, 5)), int(rng.integers(1, 20)), int(rng.integers(1, 40))
    mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0.0, 1.0)), seed=seed)
    if seed % 4 == 0:
        mask[0, 0, :] = 0                      # an empty row
    for P in (1, 2, 5, 300):
        for mode in (B.MODE_BALANCED, B.MODE_NAIVE, B.MODE_ROUNDS):
            for L, c0 in ((0, 0), (-1, 0), (3, 0), (0, 2)):
                _assert_plan_equal(mask, 64, P, mode, L, c0)


def test_planner_degenerate_masks():
    _assert_plan_equal(np.zeros((2, 3, 5), dtype=np.uint8), 64, 4, B.MODE_BALANCED, 0, 0)
    _assert_plan_equal(np.ones((2, 3, 5), dtype=np.uint8), 64, 4, B.MODE_BALANCED, 0, 0)
    _assert_plan_equal(np.ones((1, 1, 9), dtype=np.uint8), 64, 4, B.MODE_NAIVE, 2, 0)
    _assert_plan_equal(np.zeros((2, 3, 5), dtype=np.uint8), 64, 4, B.MODE_ROUNDS, 0, 0)
    _assert_plan_equal(np.ones((3, 2, 9), dtype=np.uint8), 64, 4, B.MODE_ROUNDS, 2, 1)
    _assert_plan_equal(np.full((1, 2, 17), 255, dtype=np.uint8), 128, 1, B.MODE_BALANCED, 0, 0)   # any nonzero byte counts


def test_five_config5_steps_replan_bit_exact():
    # per-call replanning over the denoising-step sequence (first steps only, to stay quick)
    for step, mask in enumerate(synth.mask_sequence_cfg5(4)):
        _assert_plan_equal(mask, 128, 256, B.MODE_BALANCED, 0, 0)
        _assert_plan_equal(mask, 128, 256, B.MODE_ROUNDS, 0, 0)


def _arrays_equal(pl, ref):
    eq = np.testing.assert_array_equal
    eq(pl.array(B.ROW_PTR), np.array(ref["row_ptr"], dtype=np.int32))
    eq(pl.array(B.KV_IDX), np.array(ref["kv_idx"], dtype=np.int32))
    eq(pl.array(B.ITEMS), np.array(ref["items"], dtype=np.int32).reshape(-1))
    eq(pl.array(B.ITEM_SLOT), np.array(ref["item_slot"], dtype=np.int32))
    eq(pl.array(B.PART_PTR), np.array(ref["part_ptr"], dtype=np.int32))
    eq(pl.array(B.PART_ITEMS), np.array(ref["part_items"], dtype=np.int32))
    eq(pl.array(B.PART_LOAD), np.array(ref["part_load"], dtype=np.int64))
    st = pl.stats()
    assert st["rho_plan"] == ref["rho_plan"] and st["rho_balanced"] == ref["rho_balanced"] and st["rho_naive"] == ref["rho_naive"]


@pytest.mark.parametrize("threshold,mode", [(1.02, B.MODE_BALANCED), (1.05, B.MODE_ROUNDS), (1.20, B.MODE_BALANCED), (100.0, B.MODE_NAIVE)])
def test_plan_reuse_over_the_config5_sequence_bit_exact(threshold, mode):
    # chain of plans over the denoising-step masks: each step either keeps the previous placement
    # or re-plans; decisions, rho_s values and every array must equal the oracle's chain
    masks = list(synth.mask_sequence_cfg5(8))
    P = 256
    pl = B.plan_sparse_attn(masks[0], 128, num_partitions=P, mode=mode, host_only=True)
    ref = op.plan(masks[0], P, mode=mode)
    decisions = []
    for mask in masks[1:]:
        nxt, reused, rho = B.plan_sparse_attn_reuse(pl, mask, threshold, mode=mode, host_only=True)
        ref = op.plan(mask, P, mode=mode, previous=ref, reuse_threshold=threshold)
        assert reused == ref["reused"] and rho == ref["rho_reuse"]
        _arrays_equal(nxt, ref)
        pl.close()                      # the new plan does not depend on the old one
        pl = nxt
        decisions.append(reused)
    pl.close()
    if threshold >= 1.3:
        assert all(decisions)


@pytest.mark.parametrize("seed", range(6))
def test_plan_reuse_random_masks_bit_exact(seed):
    # unrelated masks (many unmatched items: rows appear, vanish, split differently), small P
    rng = np.random.default_rng(900 + seed)
    H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(2, 12)), int(rng.integers(4, 40))
    for P, L in ((3, 0), (7, 2), (1, 0)):
        m0 = synth.random_mask(H, nQ, nK, float(rng.uniform(0.1, 0.9)), seed=seed)
        pl = B.plan_sparse_attn(m0, 64, num_partitions=P, max_item_len=L, host_only=True)
        ref = op.plan(m0, P, max_item_len=L)
        for t in range(4):
            m = synth.random_mask(H, nQ, nK, float(rng.uniform(0.0, 1.0)), seed=50 * seed + t)
            thr = (1.0, 1.2, 5.0, 1.05)[t]
            nxt, reused, rho = B.plan_sparse_attn_reuse(pl, m, thr, max_item_len=L, host_only=True)
            ref = op.plan(m, P, max_item_len=L, previous=ref, reuse_threshold=thr)
            assert reused == ref["reused"] and rho == ref["rho_reuse"]
            _arrays_equal(nxt, ref)
            pl.close()
            pl = nxt
        pl.close()


def test_plan_reuse_argument_errors():
    lib = B.load_library()
    m = np.ones((1, 2, 2), dtype=np.uint8)
    pl = B.plan_sparse_attn(m, 64, num_partitions=4, host_only=True)
    out, reused, rho = C.c_void_p(), C.c_int32(), C.c_double()
    host = B.PlanOpts(0, 0, 0, 0, B.PLAN_HOST_ONLY)
    mp = m.ctypes.data_as(C.c_void_p)
    call = lambda prev, mask, opts, thr: lib.plan_sparse_attn_reuse(prev, mask, C.byref(opts), thr, C.byref(out), C.byref(reused), C.byref(rho))
    assert call(None, mp, host, 1.1) == B.DBSP_EINVAL
    assert call(pl.handle, None, host, 1.1) == B.DBSP_EINVAL
    assert call(pl.handle, mp, host, 0.5) == B.DBSP_EINVAL
    assert call(pl.handle, mp, host, float("nan")) == B.DBSP_EINVAL
    assert call(pl.handle, mp, B.PlanOpts(5, 0, 0, 0, B.PLAN_HOST_ONLY), 1.1) == B.DBSP_ESHAPE
    assert out.value is None
    # P = 0: the previous plan's 4; two rows of 2 blocks on 4 partitions: rho_s = 2 / (4 / 4)
    assert call(pl.handle, mp, host, 2.0) == B.DBSP_OK and reused.value == 1 and rho.value == 2.0
    lib.dbsp_plan_destroy(out)
    assert lib.plan_sparse_attn_reuse(pl.handle, mp, C.byref(host), 1.1, C.byref(out), None, None) == B.DBSP_OK
    lib.dbsp_plan_destroy(out)
    pl.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_rounds_with_locality_groups_bit_exact(cfg):
    mask = synth.mask_for_config(cfg)
    block = synth.CONFIGS[cfg]["block"]
    for P, G in ((256, 8), (256, 2), (64, 8), (8, 8), (24, 4)):
        _assert_plan_equal(mask, block, P, B.MODE_ROUNDS, 0, 0, G)
    _assert_plan_equal(mask, block, 256, B.MODE_ROUNDS, 16, 2, 8)


def test_locality_groups_random_and_errors():
    rng = np.random.default_rng(77)
    for seed in range(8):
        H, nQ, nK = int(rng.integers(1, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0.0, 1.0)), seed=seed)
        for P, G in ((4, 2), (12, 4), (6, 6), (5, 1), (9, 3)):
            _assert_plan_equal(mask, 64, P, B.MODE_ROUNDS, 0, 0, G)
            _assert_plan_equal(mask, 64, P, B.MODE_ROUNDS, 2, 1, G)
    m = np.ones((1, 2, 2), dtype=np.uint8)
    mp = m.ctypes.data_as(C.c_void_p)
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(6, B.MODE_ROUNDS, 0, 0, B.PLAN_HOST_ONLY, 4))[0] == B.DBSP_EINVAL
    assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(6, B.MODE_ROUNDS, 0, 0, B.PLAN_HOST_ONLY, -1))[0] == B.DBSP_EINVAL
    rc, pl = _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(6, B.MODE_ROUNDS, 0, 0, B.PLAN_HOST_ONLY, 3))
    assert rc == B.DBSP_OK
    B.load_library().dbsp_plan_destroy(pl)


def test_threaded_compaction_with_empty_and_tiny_rows_bit_exact():
    # a mask large enough for the multi-threaded row passes, with runs of empty rows and rows of one
    # or two blocks around the places where the row ranges of the threads meet
    rng = np.random.default_rng(2024)
    H, nQ, nK = 8, 512, 520                       # 2.1 MB; nK not a multiple of 8 (scalar tail)
    mask = (rng.random((H, nQ, nK)) < 0.2).astype(np.uint8)
    flat = mask.reshape(H * nQ, nK)
    flat[rng.random(H * nQ) < 0.3] = 0
    for n in range(2, 9):                         # ranges meet at R * t / n for n = 2..8 threads
        for t in range(1, n):
            r = H * nQ * t // n
            flat[max(0, r - 3):r] = 0
            if r - 4 >= 0:
                flat[r - 4] = 0
                flat[r - 4, rng.integers(0, nK, 2)] = 1
    _assert_plan_equal(mask, 128, 256, B.MODE_BALANCED, 0, 0)
    _assert_plan_equal(mask, 128, 256, B.MODE_ROUNDS, 0, 0, 8)


def test_partition_cost_bit_exact_and_errors():
    rng = np.random.default_rng(31)
    for cfg, P in ((5, 256), (1, 8), (3, 256)):
        mask = synth.mask_for_config(cfg)
        block = synth.CONFIGS[cfg]["block"]
        cost = rng.integers(960, 1090, P).tolist()
        _assert_plan_equal(mask, block, P, B.MODE_BALANCED, 0, 0, 0, cost)
        _assert_plan_equal(mask, block, P, B.MODE_ROUNDS, 0, 0, 8, cost)
        _assert_plan_equal(mask, block, P, B.MODE_ROUNDS, 0, 1, 0, cost)
        _assert_plan_equal(mask, block, P, B.MODE_NAIVE, 0, 0, 0, cost)          # ignored by the naive placement
        _assert_plan_equal(mask, block, P, B.MODE_BALANCED, 0, 0, 0, [3] * P)    # equal costs: the paper's rule
    for seed in range(6):
        H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=seed)
        for P, G in ((4, 2), (6, 3), (5, 1)):
            cost = rng.integers(1, 50, P).tolist()
            _assert_plan_equal(mask, 64, P, B.MODE_BALANCED, 2, 1, 0, cost)
            _assert_plan_equal(mask, 64, P, B.MODE_ROUNDS, 0, 0, G, cost)
    m = np.ones((1, 2, 2), dtype=np.uint8)
    with pytest.raises(B.DbspError):
        B.plan_sparse_attn(m, 64, num_partitions=3, host_only=True, partition_cost=[1, 0, 2])
    with pytest.raises(ValueError):
        B.plan_sparse_attn(m, 64, num_partitions=3, host_only=True, partition_cost=[1, 2])
    pl = B.plan_sparse_attn(m, 64, host_only=True, partition_cost=[5, 5, 5, 5])      # the array fixes P
    assert pl.stats()["num_partitions"] == 4
    lib = B.load_library()
    out = np.zeros(4, np.int32)
    assert lib.dbsp_plan_calibrate(pl.handle, out.ctypes.data_as(C.c_void_p), None) == B.DBSP_EINVAL   # host-only plan
    assert lib.dbsp_plan_calibrate(None, out.ctypes.data_as(C.c_void_p), None) == B.DBSP_EINVAL
    pl.close()


def test_concurrent_planners_share_the_helper_threads_and_agree():
    # several host threads plan a mask large enough for the threaded passes at the same time: one of
    # them gets the library's helper threads, the others run their passes themselves; every plan
    # must be the same as one made alone.  Also: negative max_batch is refused.
    import threading
    rng = np.random.default_rng(77)
    mask = (rng.random((6, 600, 512)) < 0.25).astype(np.uint8)            # 1.8 MB
    alone = dbsp.plan_sparse_attn(mask, 128, num_partitions=256, mode=B.MODE_ROUNDS, locality_groups=8, host_only=True)
    want = {k: alone.array(k).tolist() for k in (B.ROW_PTR, B.KV_IDX, B.ITEMS, B.PART_PTR, B.PART_ITEMS)}
    alone.close()
    got, errors = [], []

    def work():
        try:
            for _ in range(3):
                p = dbsp.plan_sparse_attn(mask, 128, num_partitions=256, mode=B.MODE_ROUNDS, locality_groups=8, host_only=True)
                got.append({k: p.array(k).tolist() for k in want})
                p.close()
        except Exception as exc:        # noqa: BLE001
            errors.append(exc)

    threads = [threading.Thread(target=work) for _ in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors and len(got) == 12 and all(g == want for g in got)
    m = np.ones((1, 2, 2), dtype=np.uint8)
    opts = B.PlanOpts(4, 0, 0, 0, B.PLAN_HOST_ONLY, 0, None, -1)
    assert _plan_raw(m.ctypes.data_as(C.c_void_p), 1, 2, 2, 64, opts)[0] == B.DBSP_EINVAL


def test_rho_of_the_unused_placements_is_worked_out_on_request():
    # the plan computes rho_s of its own placement; that of the naive and of the greedy placement
    # comes on the first dbsp_plan_stats call that asks, and equals the oracle's
    mask = synth.mask_for_config(5)
    ref = op.plan(mask, 256, mode=op.MODE_ROUNDS, locality_groups=8)
    p = dbsp.plan_sparse_attn(mask, 128, num_partitions=256, mode=B.MODE_ROUNDS, locality_groups=8, host_only=True)
    light = p.stats(with_rho=False)
    assert "rho_naive" not in light and light["rho_plan"] == ref["rho_plan"]
    full = p.stats()
    assert full["rho_naive"] == ref["rho_naive"] and full["rho_balanced"] == ref["rho_balanced"] and full["rho_plan"] == ref["rho_plan"]
    assert p.stats() == full                      # the second call reads the stored values
    p.close()


def test_dynamic_tail_bit_exact_and_errors():
    for cfg, P in ((3, 256), (5, 256), (2, 1024), (1, 8)):
        mask = synth.mask_for_config(cfg)
        block = synth.CONFIGS[cfg]["block"]
        for tail, G in ((30, 8), (100, 1), (999, 4)):
            _assert_plan_equal(mask, block, P, B.MODE_ROUNDS, 0, 0, G, None, tail)
    rng = np.random.default_rng(5)
    for seed in range(12):
        H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=seed)
        P = int(rng.choice([1, 2, 4, 6]))
        cost = rng.integers(1, 50, P).tolist() if seed % 3 == 0 else None
        _assert_plan_equal(mask, 64, P, B.MODE_ROUNDS, int(rng.choice([0, 2, -1])), int(rng.integers(0, 3)), 1, cost, int(rng.integers(1, 600)))
    # a plan with a queue as the previous plan of a reuse chain: queued items count as new ones
    seq = list(synth.mask_sequence_cfg5(3))
    prev = B.plan_sparse_attn(seq[0], 128, num_partitions=256, mode=B.MODE_ROUNDS, host_only=True, dynamic_tail=100)
    ref_prev = op.plan(seq[0], 256, mode=op.MODE_ROUNDS, dynamic_tail=100)
    assert len(ref_prev["tail_items"]) > 0
    nxt, reused, rho = B.plan_sparse_attn_reuse(prev, seq[1], 1.5, mode=B.MODE_ROUNDS, host_only=True)
    ref = op.plan(seq[1], 256, mode=op.MODE_ROUNDS, previous=ref_prev, reuse_threshold=1.5)
    assert reused == ref["reused"] and rho == ref["rho_reuse"] and nxt.array(B.PART_ITEMS).tolist() == ref["part_items"]
    assert nxt.array(B.TAIL_ITEMS).shape == (0,) or not reused
    prev.close()
    nxt.close()
    m = np.ones((1, 2, 2), dtype=np.uint8)
    mp = m.ctypes.data_as(C.c_void_p)
    for mode, tail in ((B.MODE_ROUNDS, 1000), (B.MODE_ROUNDS, -1), (B.MODE_BALANCED, 10)):
        assert _plan_raw(mp, 1, 2, 2, 64, B.PlanOpts(4, mode, 0, 0, B.PLAN_HOST_ONLY, 0, None, 0, tail, 0.0))[0] == B.DBSP_EINVAL


def test_reward_mode_bit_exact_and_errors():
    for cfg, P in ((3, 256), (5, 256), (1, 8)):
        mask = synth.mask_for_config(cfg)
        block = synth.CONFIGS[cfg]["block"]
        for G, rb in ((8, 0.0), (8, 0.5), (8, 2.0), (1, 1.0), (4, 1e6)):
            if P % G == 0:
                _assert_plan_equal(mask, block, P, B.MODE_REWARD, 0, 0, G, None, 0, rb)
    rng = np.random.default_rng(6)
    for seed in range(12):
        H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=seed)
        P, G = [(4, 2), (6, 3), (5, 1), (8, 4)][seed % 4]
        _assert_plan_equal(mask, 64, P, B.MODE_REWARD, int(rng.choice([0, 2, -1])), int(rng.integers(0, 3)), G, None, 0, float(rng.choice([0.0, 0.3, 1.0, 2.5])))
    m = np.ones((1, 2, 2), dtype=np.uint8)
    mp = m.ctypes.data_as(C.c_void_p)
    cost = (C.c_int32 * 4)(1, 1, 1, 1)
    bad = (B.PlanOpts(4, B.MODE_REWARD, 0, 0, B.PLAN_HOST_ONLY, 2, None, 0, 0, -1.0),
           B.PlanOpts(4, B.MODE_REWARD, 0, 0, B.PLAN_HOST_ONLY, 2, None, 0, 0, float("nan")),
           B.PlanOpts(4, B.MODE_BALANCED, 0, 0, B.PLAN_HOST_ONLY, 2, None, 0, 0, 1.0),
           B.PlanOpts(4, B.MODE_REWARD, 0, 0, B.PLAN_HOST_ONLY, 2, C.cast(cost, C.c_void_p), 0, 0, 1.0),
           B.PlanOpts(4, B.MODE_REWARD, 0, 0, B.PLAN_HOST_ONLY, 3, None, 0, 0, 1.0))
    for o in bad:
        assert _plan_raw(mp, 1, 2, 2, 64, o)[0] == B.DBSP_EINVAL


def test_pair_rows_bit_exact_reuse_and_errors():
    # 64-token blocks served two query blocks at a time: rows, counts and lists are those of pairs and super blocks
    rng = np.random.default_rng(8)
    for seed in range(24):
        H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(1, 14)), int(rng.integers(1, 30))
        mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=seed)
        if seed % 4 == 0 and nQ > 2:
            mask[:, 2:4] = 0
        P = int(rng.choice([1, 3, 4, 8]))
        mode = (B.MODE_BALANCED, B.MODE_NAIVE, B.MODE_ROUNDS)[seed % 3]
        tail = int(rng.integers(1, 500)) if mode == B.MODE_ROUNDS and seed % 2 else 0
        _assert_plan_equal(mask, 64, P, mode, int(rng.choice([0, 1, 2, -1])), int(rng.integers(0, 3)), 1 if tail else 0, None, tail, 0.0, True)
    cog = synth.mask_for_config(2)                      # 275 query blocks per head: an odd number
    _assert_plan_equal(cog, 64, 256, B.MODE_ROUNDS, 0, 0, 8, None, 40, 0.0, True)
    _assert_plan_equal(cog, 64, 256, B.MODE_BALANCED, 0, 0, 0, None, 0, 0.0, True)
    # the placement is carried over between pair-row plans like between plain ones
    m0, m1 = synth.random_mask(2, 7, 20, 0.5, seed=1), synth.random_mask(2, 7, 20, 0.5, seed=2)
    prev = B.plan_sparse_attn(m0, 64, num_partitions=4, host_only=True, pair_rows=True)
    ref_prev = op.plan(m0, 4, pair=True)
    nxt, reused, rho = B.plan_sparse_attn_reuse(prev, m1, 3.0, host_only=True)
    ref = op.plan(m1, 4, pair=True, previous=ref_prev, reuse_threshold=3.0)
    assert reused == ref["reused"] and rho == ref["rho_reuse"] and nxt.pair_rows
    assert nxt.array(B.PART_ITEMS).tolist() == list(ref["part_items"]) and nxt.array(B.KV_IDX).tolist() == list(ref["kv_idx"])
    # a plain plan cannot follow a pair-row plan, 128-token blocks have no pair rows
    lib = B.load_library()
    out = C.c_void_p()
    plain = B.PlanOpts(0, 0, 0, 0, B.PLAN_HOST_ONLY)
    assert lib.plan_sparse_attn_reuse(prev.handle, m1.ctypes.data_as(C.c_void_p), C.byref(plain), 3.0, C.byref(out), None, None) == B.DBSP_ESHAPE
    assert out.value is None
    prev.close()
    nxt.close()
    m = np.ones((1, 2, 2), dtype=np.uint8)
    assert _plan_raw(m.ctypes.data_as(C.c_void_p), 1, 2, 2, 128, B.PlanOpts(4, 0, 0, 0, B.PLAN_HOST_ONLY | B.PLAN_PAIR_ROWS))[0] == B.DBSP_EINVAL
    assert _plan_raw(m.ctypes.data_as(C.c_void_p), 1, 2, 2, 64, B.PlanOpts(4, 0, 0, 0, B.PLAN_HOST_ONLY | 4))[0] == B.DBSP_EINVAL
    # default partition counts without a device: 256 compute units assumed
    for kw, want in ((dict(), 1024), (dict(head_dim=64), 1024), (dict(head_dim=128), 512), (dict(pair_rows=True, head_dim=128), 256)):
        pl = B.plan_sparse_attn(m, 64, host_only=True, **kw)
        assert pl.stats(with_rho=False)["num_partitions"] == want
        pl.close()
    assert _plan_raw(m.ctypes.data_as(C.c_void_p), 1, 2, 2, 64, B.PlanOpts(4, 0, 0, 0, B.PLAN_HOST_ONLY, 0, None, 0, 0, 0.0, 96))[0] == B.DBSP_EINVAL


def test_pair_auto_chooses_like_the_oracle_and_errors():
    rng = np.random.default_rng(9)
    seen = set()
    for seed in range(16):
        H, nQ, nK = int(rng.integers(1, 4)), int(rng.integers(1, 10)), int(rng.integers(2, 24))
        base = synth.random_mask(H, (nQ + 1) // 2, nK, float(rng.uniform(0.2, 0.9)), seed=seed)
        # neighbouring rows alike to a varying degree: copies of one row with a share of the blocks dropped
        mask = np.repeat(base, 2, axis=1)[:, :nQ].copy()
        mask &= (rng.random(mask.shape) < float(rng.choice([1.0, 0.9, 0.6, 0.3]))).astype(np.uint8)
        pl = B.plan_sparse_attn(mask, 64, num_partitions=4, host_only=True, pair_rows="auto", head_dim=128)
        ref = op.plan(mask, 4, pair="auto")
        assert pl.pair_rows is ref["pair"]
        seen.add(pl.pair_rows)
        assert pl.array(B.KV_IDX).tolist() == list(ref["kv_idx"]) and pl.array(B.PART_ITEMS).tolist() == list(ref["part_items"])
        # a chain keeps the first plan's kind whatever the next mask looks like
        nxt, reused, rho = B.plan_sparse_attn_reuse(pl, 1 - mask, 1.0, host_only=True)
        assert nxt.pair_rows is pl.pair_rows
        pl.close()
        nxt.close()
    assert seen == {False, True}
    m = np.ones((1, 2, 2), dtype=np.uint8)
    mp = m.ctypes.data_as(C.c_void_p)
    host = B.PLAN_HOST_ONLY
    bad = (B.PlanOpts(4, 0, 0, 0, host | B.PLAN_PAIR_AUTO, 0, None, 0, 0, 0.0, 0),                      # head dim unknown
           B.PlanOpts(4, 0, 0, 0, host | B.PLAN_PAIR_AUTO, 0, None, 0, 0, 0.0, 64),
           B.PlanOpts(4, 0, 0, 0, host | B.PLAN_PAIR_AUTO | B.PLAN_PAIR_ROWS, 0, None, 0, 0, 0.0, 128))
    for o in bad:
        assert _plan_raw(mp, 1, 2, 2, 64, o)[0] == B.DBSP_EINVAL
    assert _plan_raw(mp, 1, 2, 2, 128, B.PlanOpts(4, 0, 0, 0, host | B.PLAN_PAIR_AUTO, 0, None, 0, 0, 0.0, 128))[0] == B.DBSP_EINVAL
    assert B.load_library().dbsp_plan_pair_rows(None, None) == B.DBSP_EINVAL
