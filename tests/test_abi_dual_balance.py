"""The library's host-only planners for several GPUs against the oracle, bit for bit (no GPU)."""

import ctypes as C

import numpy as np
import pytest

import synth
from oracle import dual_balance as db
from paper_2511_23113_amd import binding as B


def _same(got, ref, keys):
    for k in keys:
        assert got[k] == ref[k], k


HEAD_KEYS = ("gpu_of_head", "lists", "loads", "rho_contiguous", "rho", "rho_previous", "reused")
BLOCK_KEYS = ("gpu_of_q", "q_lists", "chunk_of_kv", "kv_lists", "work", "rho", "rho_contiguous", "moved_q", "moved_kv")


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_heads_on_configs(cfg):
    mask = synth.mask_for_config(cfg)
    per_head = (mask != 0).sum(axis=(1, 2)).tolist()
    H = len(per_head)
    for x in (1, 2, 4, 8):
        _same(B.partition_heads(per_head, x), db.partition_heads(per_head, x), HEAD_KEYS)
        cap = -(-H // x)
        _same(B.partition_heads(per_head, x, capacity=cap), db.partition_heads(per_head, x, capacity=cap), HEAD_KEYS)


def test_heads_reuse_chain_on_per_step_counts():
    # per-head counts drift from step to step; the chain of decisions must equal the oracle's
    rng = np.random.default_rng(3)
    cnt = rng.integers(2000, 30000, 40)
    for thr in (1.02, 1.05, 1.10):
        prev_l = prev_o = None
        kept = 0
        c = cnt.copy()
        for step in range(50):
            c = np.maximum(0, c + rng.integers(-600, 601, c.shape))
            got = B.partition_heads(c, 8, previous=prev_l, reuse_threshold=thr)
            ref = db.partition_heads(c.tolist(), 8, previous=prev_o, reuse_threshold=thr)
            _same(got, ref, HEAD_KEYS)
            prev_l, prev_o = got["gpu_of_head"], ref["gpu_of_head"]
            kept += got["reused"]
        assert 0 < kept < 50


@pytest.mark.parametrize("seed", range(10))
def test_blocks_random(seed):
    rng = np.random.default_rng(700 + seed)
    H, nQ, nK = int(rng.integers(1, 5)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
    mask = synth.random_mask(H, nQ, nK, float(rng.uniform(0, 1)), seed=seed)
    for y in (1, 2, 3, 8):
        for reward in (0.0, 0.3, 1.0, 7.5):
            _same(B.partition_blocks(mask, y, reward), db.partition_blocks(mask, y, reward), BLOCK_KEYS)
        cq, ck = -(-nQ // y), -(-nK // y)
        _same(B.partition_blocks(mask, y, 0.5, cq, ck), db.partition_blocks(mask, y, 0.5, cq, ck), BLOCK_KEYS)
        gq, gk = rng.integers(0, y, nQ).tolist(), rng.integers(0, y, nK).tolist()
        work, rho = B.ring_work(mask, y, gq, gk)
        ref = db.ring_work(mask, gq, gk, y)
        assert work == ref and rho == db.ring_rho(ref)
        work, rho = B.ring_work(mask, y)
        ref = db.ring_work(mask, db.contiguous_owner(nQ, y), db.contiguous_owner(nK, y), y)
        assert work == ref and rho == db.ring_rho(ref)


@pytest.mark.parametrize("cfg,y", [(5, 8), (3, 8), (2, 4)])
def test_blocks_on_configs(cfg, y):
    mask = synth.mask_for_config(cfg)
    for reward in (0.0, 0.25):
        _same(B.partition_blocks(mask, y, reward), db.partition_blocks(mask, y, reward), BLOCK_KEYS)


def test_argument_errors():
    lib = B.load_library()
    cnt = np.array([3, 2, 1], dtype=np.int64)
    out = np.empty(3, np.int32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    heads = lambda *a: lib.dbsp_partition_heads(*a, None, None, None, None, None, None, None)
    assert heads(None, 3, 2, 0, None, 1.0, p(out)) == B.DBSP_EINVAL
    assert heads(p(cnt), 3, 2, 0, None, 1.0, None) == B.DBSP_EINVAL
    assert heads(p(cnt), 0, 2, 0, None, 1.0, p(out)) == B.DBSP_EINVAL
    assert heads(p(cnt), 3, 0, 0, None, 1.0, p(out)) == B.DBSP_EINVAL
    assert heads(p(cnt), 3, 2, 1, None, 1.0, p(out)) == B.DBSP_EINVAL                 # capacity too small
    assert heads(p(np.array([3, -2, 1], dtype=np.int64)), 3, 2, 0, None, 1.0, p(out)) == B.DBSP_EINVAL
    bad_prev = np.array([0, 2, 0], dtype=np.int32)
    assert heads(p(cnt), 3, 2, 0, p(bad_prev), 1.1, p(out)) == B.DBSP_EINVAL
    assert heads(p(cnt), 3, 2, 0, p(np.zeros(3, np.int32)), 0.9, p(out)) == B.DBSP_EINVAL
    assert heads(p(cnt), 3, 2, 0, None, 1.0, p(out)) == B.DBSP_OK and out.tolist() == [0, 1, 1]
    m = np.ones((1, 2, 3), dtype=np.uint8)
    gq, gk = np.empty(2, np.int32), np.empty(3, np.int32)
    blocks = lambda mask, H, nQ, nK, y, rw, cq, ck, a, b: lib.dbsp_partition_blocks(mask, H, nQ, nK, y, rw, cq, ck, a, None, None, b, None, None,
                                                                                 None, None, None, None, None)
    assert blocks(None, 1, 2, 3, 2, 0.0, 0, 0, p(gq), p(gk)) == B.DBSP_EINVAL
    assert blocks(p(m), 1, 2, 3, 2, 0.0, 0, 0, None, p(gk)) == B.DBSP_EINVAL
    assert blocks(p(m), 1, 2, 3, 0, 0.0, 0, 0, p(gq), p(gk)) == B.DBSP_EINVAL
    assert blocks(p(m), 1, 2, 3, 2, -1.0, 0, 0, p(gq), p(gk)) == B.DBSP_EINVAL
    assert blocks(p(m), 1, 2, 3, 2, float("nan"), 0, 0, p(gq), p(gk)) == B.DBSP_EINVAL
    assert blocks(p(m), 1, 2, 3, 2, 0.0, 0, 1, p(gq), p(gk)) == B.DBSP_EINVAL         # 1 * 2 < 3 KV blocks
    assert blocks(p(m), 1, 2, 3, 2, 0.0, 0, 0, p(gq), p(gk)) == B.DBSP_OK
    rho = C.c_double()
    assert lib.dbsp_ring_work(p(m), 1, 2, 3, 2, None, None, None, None) == B.DBSP_EINVAL
    assert lib.dbsp_ring_work(p(m), 1, 2, 3, 2, p(np.array([0, 2], dtype=np.int32)), None, None, C.byref(rho)) == B.DBSP_EINVAL
    # 3 KV blocks in chunks of 2 and 1: iterations cost 2 and 2 on the slowest GPU against 6 / 2
    assert lib.dbsp_ring_work(p(m), 1, 2, 3, 2, None, None, None, C.byref(rho)) == B.DBSP_OK and rho.value == 4 / 3


def test_cost_model_fit_matches_the_oracle():
    from oracle import cost_model as cm
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(3, 400))
        b = rng.integers(100, 5000, n)
        i = rng.integers(1, 80, n)
        t = rng.uniform(1, 5) * b + rng.uniform(0, 100) * i + rng.uniform(0, 2000) + rng.normal(0, 30.0, n)
        try:
            ref = cm.fit(b, i, t)
        except ValueError:
            continue
        got = B.fit_cost_model(b, i, t)
        # same least-squares problem solved two ways (SVD there, centred normal equations here):
        # agreement to rounding amplified by the conditioning of the design (cond < 1e5 for these ranges)
        for g, r, scale in zip(got, ref, (1.0, 100.0, 5000.0, 30.0)):
            assert abs(g - r) <= 1e-8 * scale, (trial, got, ref)
    assert B.fit_cost_model([1, 3, 1], [1, 1, 2], [14.0, 18.0, 19.0])[:3] == (2.0, 5.0, 7.0)
    lib = B.load_library()
    for bad in (([1, 2], [1, 2], [1.0, 2.0]), ([2, 4, 6, 8], [1, 2, 3, 4], [1.0, 2.0, 3.0, 4.0]), ([5, 5, 5], [1, 2, 3], [1.0, 2.0, 3.0]),
                ([1, 3, 1], [1, 1, 2], [1.0, float("inf"), 2.0])):
        with pytest.raises(B.DbspError):
            B.fit_cost_model(*bad)
    assert b"determine" in lib.dbsp_last_error() or b"finite" in lib.dbsp_last_error()
