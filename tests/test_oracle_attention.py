"""Pins for oracle.attention: closed forms, invariants, a separately written dense
brute force, and a hand-worked fixture.  CPU only."""

import math
import os

import numpy as np
import pytest

import synth
from oracle import attention as oa
from oracle.dense_bruteforce import dense_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return synth.bf16_bits_to_f32(synth.normal_bf16(shape, seed)).astype(np.float64)


def _small(seed=0, B=1, H=2, nQ=3, nK=4, b=8, d=16):
    q = _rand((B, H, nQ * b, d), seed)
    k = _rand((B, H, nK * b, d), seed + 1)
    v = _rand((B, H, nK * b, d), seed + 2)
    return q, k, v


def test_hand_worked_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "attention_hand.txt")) if l.strip() and not l.startswith("#")]
    qv = np.array([float(r[0]) for r in rows])
    mask = np.array([[int(x) for x in r[1:4]] for r in rows], dtype=np.uint8)[None]   # [1,3,3]
    o_exp = np.array([float(r[4]) for r in rows])
    z_exp = np.array([float(r[5]) for r in rows])
    q = qv.reshape(1, 1, 3, 1)
    k = np.array([0.0, math.log(3.0), math.log(2.0)]).reshape(1, 1, 3, 1)
    v = np.array([4.0, 8.0, 100.0]).reshape(1, 1, 3, 1)
    O, L = oa.masked_attention(q, k, v, mask, block=1)
    np.testing.assert_allclose(O[0, 0, :, 0], o_exp, rtol=1e-13)
    np.testing.assert_allclose(np.exp(L[0, 0]), z_exp, rtol=1e-13)


def test_all_ones_mask_equals_dense_bruteforce():
    q, k, v = _small(seed=10)
    B, H, Nq, d = q.shape
    mask = np.ones((H, 3, 4), dtype=np.uint8)
    O, L = oa.masked_attention(q, k, v, mask, block=8)
    for h in range(H):
        Od, Ld = dense_attention(q[0, h], k[0, h], v[0, h])
        np.testing.assert_allclose(O[0, h], Od, atol=1e-12)
        np.testing.assert_allclose(L[0, h], Ld, atol=1e-12)


def test_float32_mode_close_to_float64():
    q, k, v = _small(seed=11)
    mask = synth.random_mask(2, 3, 4, 0.6, seed=5, keep_diag=True)
    O64, L64 = oa.masked_attention(q, k, v, mask, block=8)
    O32, L32 = oa.masked_attention(q, k, v, mask, block=8, dtype=np.float32)
    assert O32.dtype == np.float32
    assert np.abs(O32 - O64).max() < 1e-5
    assert np.abs(L32 - L64).max() < 1e-5


def test_explicit_scale_is_used():
    q, k, v = _small(seed=12, H=1)
    mask = np.ones((1, 3, 4), dtype=np.uint8)
    O, L = oa.masked_attention(q, k, v, mask, block=8, scale=0.37)
    Od, Ld = dense_attention(q[0, 0], k[0, 0], v[0, 0], scale=0.37)
    np.testing.assert_allclose(O[0, 0], Od, atol=1e-12)
    np.testing.assert_allclose(L[0, 0], Ld, atol=1e-12)


def test_q_zero_closed_form_pins_mask_counts_and_lse():
    # every score is 0 -> LSE = ln(b * active blocks of the row), O = mean of V over active keys
    B, H, nQ, nK, b, d = 2, 3, 4, 5, 4, 8
    mask = synth.random_mask(H, nQ, nK, 0.5, seed=3)
    mask[0, 0, :] = 0
    mask[0, 0, 2] = 1                       # a one-block row
    k = _rand((B, H, nK * b, d), 21)
    v = _rand((B, H, nK * b, d), 22)
    q = np.zeros((B, H, nQ * b, d))
    O, L = oa.masked_attention(q, k, v, mask, block=b)
    for bb in range(B):
        for h in range(H):
            for I in range(nQ):
                act = np.repeat(mask[h, I] != 0, b)
                rows = slice(I * b, (I + 1) * b)
                if act.sum() == 0:
                    assert np.all(O[bb, h, rows] == 0) and np.all(np.isneginf(L[bb, h, rows]))
                    continue
                np.testing.assert_allclose(L[bb, h, rows], math.log(act.sum()), atol=1e-13)
                np.testing.assert_allclose(O[bb, h, rows], np.broadcast_to(v[bb, h][act].mean(0), (b, d)), atol=1e-13)


def test_asymmetric_mask_is_not_transposed():
    # mask[h, I, J]: I indexes query blocks.  Row 0 sees only KV block 1; row 1 sees only KV block 0.
    b, d = 4, 8
    mask = np.array([[[0, 1], [1, 0]]], dtype=np.uint8)
    v = np.zeros((1, 1, 2 * b, d))
    v[0, 0, :b] = 1.0      # KV block 0 carries 1, block 1 carries 2
    v[0, 0, b:] = 2.0
    q = _rand((1, 1, 2 * b, d), 31)
    k = _rand((1, 1, 2 * b, d), 32)
    O, _ = oa.masked_attention(q, k, v, mask, block=b)
    np.testing.assert_allclose(O[0, 0, :b], 2.0, atol=1e-13)
    np.testing.assert_allclose(O[0, 0, b:], 1.0, atol=1e-13)


def test_rows_sum_to_one_and_block_mass():
    # V = ones -> O = 1.  V = indicator of KV block J -> O = probability mass on J; 0 when J inactive.
    q, k, _ = _small(seed=40)
    H, nQ, nK, b, d = 2, 3, 4, 8, 16
    mask = synth.random_mask(H, nQ, nK, 0.5, seed=9, keep_diag=True)
    ones = np.ones((1, H, nK * b, d))
    O, _ = oa.masked_attention(q, k, ones, mask, block=b)
    np.testing.assert_allclose(O, 1.0, atol=1e-13)
    mass = np.zeros((H, nQ * b, nK))
    for J in range(nK):
        ind = np.zeros((1, H, nK * b, d))
        ind[:, :, J * b:(J + 1) * b, :] = 1.0
        OJ, _ = oa.masked_attention(q, k, ind, mask, block=b)
        mass[:, :, J] = OJ[0, :, :, 0]
    np.testing.assert_allclose(mass.sum(-1), 1.0, atol=1e-13)
    for h in range(H):
        for I in range(nQ):
            for J in range(nK):
                blk = mass[h, I * b:(I + 1) * b, J]
                if mask[h, I, J]:
                    assert np.all(blk > 0)
                else:
                    assert np.all(blk == 0)


def test_diagonal_mask_equals_per_block_dense():
    b, d, n = 8, 16, 3
    q = _rand((1, 1, n * b, d), 50)
    k = _rand((1, 1, n * b, d), 51)
    v = _rand((1, 1, n * b, d), 52)
    mask = np.eye(n, dtype=np.uint8)[None]
    O, L = oa.masked_attention(q, k, v, mask, block=b)
    for I in range(n):
        s = slice(I * b, (I + 1) * b)
        Od, Ld = dense_attention(q[0, 0, s], k[0, 0, s], v[0, 0, s])
        np.testing.assert_allclose(O[0, 0, s], Od, atol=1e-12)
        np.testing.assert_allclose(L[0, 0, s], Ld, atol=1e-12)


def test_lse_bounds_and_shift():
    q, k, v = _small(seed=60)
    H, nQ, nK, b, d = 2, 3, 4, 8, 16
    mask = synth.random_mask(H, nQ, nK, 0.6, seed=2, keep_diag=True)
    scale = 1.0 / math.sqrt(d)
    O, L = oa.masked_attention(q, k, v, mask, block=b, scale=scale)
    for h in range(H):
        s = scale * q[0, h] @ k[0, h].T
        for I in range(nQ):
            act = np.repeat(mask[h, I] != 0, b)
            smax = s[I * b:(I + 1) * b][:, act].max(1)
            Lr = L[0, h, I * b:(I + 1) * b]
            assert np.all(Lr >= smax - 1e-12)
            assert np.all(Lr <= smax + math.log(act.sum()) + 1e-12)
    # adding a constant c to every score (one extra shared feature) shifts LSE by c, leaves O unchanged
    c = 1.7
    q2 = np.concatenate([q, np.ones(q.shape[:-1] + (1,))], axis=-1)
    k2 = np.concatenate([k, np.full(k.shape[:-1] + (1,), c / scale)], axis=-1)
    O2, L2 = oa.masked_attention(q2, k2, v, mask, block=b, scale=scale)
    np.testing.assert_allclose(O2, O, atol=1e-12)
    np.testing.assert_allclose(L2, L + c, atol=1e-12)


def test_split_and_merge_identity():
    q, k, v = _small(seed=70, H=1)
    b = 8
    mask = np.array([[[1, 1, 0, 1], [1, 1, 1, 1], [0, 1, 1, 0]]], dtype=np.uint8)
    m1 = mask.copy(); m1[:, :, 2:] = 0
    m2 = mask.copy(); m2[:, :, :2] = 0
    O, L = oa.masked_attention(q, k, v, mask, block=b)
    O1, L1 = oa.masked_attention(q, k, v, m1, block=b)
    O2, L2 = oa.masked_attention(q, k, v, m2, block=b)
    Om, Lm = oa.merge_partials(np.stack([O1[0, 0], O2[0, 0]]), np.stack([L1[0, 0], L2[0, 0]]))
    np.testing.assert_allclose(Om, O[0, 0], atol=1e-12)
    np.testing.assert_allclose(Lm, L[0, 0], atol=1e-12)
    # an empty part (LSE = -inf) contributes nothing
    Oe, Le = oa.merge_partials(np.stack([O[0, 0], np.zeros_like(O[0, 0])]),
                               np.stack([L[0, 0], np.full_like(L[0, 0], -np.inf)]))
    np.testing.assert_allclose(Oe, O[0, 0], atol=1e-13)
    np.testing.assert_allclose(Le, L[0, 0], atol=1e-13)


def test_permutation_invariance():
    # the property the paper's block reordering relies on (Methodology, "Block-level Partitioning")
    q, k, v = _small(seed=80)
    H, nQ, nK, b, d = 2, 3, 4, 8, 16
    mask = synth.random_mask(H, nQ, nK, 0.6, seed=4, keep_diag=True)
    O, L = oa.masked_attention(q, k, v, mask, block=b)
    rng = np.random.default_rng(0)
    pk = rng.permutation(nK)
    tok = (pk[:, None] * b + np.arange(b)[None]).reshape(-1)
    O2, L2 = oa.masked_attention(q, k[:, :, tok], v[:, :, tok], mask[:, :, pk], block=b)
    np.testing.assert_allclose(O2, O, atol=1e-12)
    np.testing.assert_allclose(L2, L, atol=1e-12)
    pq = rng.permutation(nQ)
    tq = (pq[:, None] * b + np.arange(b)[None]).reshape(-1)
    O3, L3 = oa.masked_attention(q[:, :, tq], k, v, mask[:, pq], block=b)
    np.testing.assert_allclose(O3, O[:, :, tq], atol=1e-12)
    np.testing.assert_allclose(L3, L[:, :, tq], atol=1e-12)
    ph = np.array([1, 0])
    O4, L4 = oa.masked_attention(q[:, ph], k[:, ph], v[:, ph], mask[ph], block=b)
    np.testing.assert_allclose(O4, O[:, ph], atol=1e-12)
    np.testing.assert_allclose(L4, L[:, ph], atol=1e-12)


def test_batch_entries_share_the_mask():
    q, k, v = _small(seed=90, B=2)
    mask = synth.random_mask(2, 3, 4, 0.5, seed=6, keep_diag=True)
    O, L = oa.masked_attention(q, k, v, mask, block=8)
    for bb in range(2):
        Ob, Lb = oa.masked_attention(q[bb:bb + 1], k[bb:bb + 1], v[bb:bb + 1], mask, block=8)
        np.testing.assert_array_equal(Ob[0], O[bb])
        np.testing.assert_array_equal(Lb[0], L[bb])


def test_rows_subset_matches_full():
    q, k, v = _small(seed=100)
    mask = synth.random_mask(2, 3, 4, 0.5, seed=8, keep_diag=True)
    O, L = oa.masked_attention(q, k, v, mask, block=8)
    Or, Lr = oa.masked_attention_rows(q, k, v, mask, 8, [(0, 1, 2), (0, 0, 0)])
    np.testing.assert_array_equal(Or[0], O[0, 1, 16:24])
    np.testing.assert_array_equal(Lr[1], L[0, 0, 0:8])


def test_bf16_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.0e-39, np.inf], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0078125)
    assert back[3] == -2.5 and np.isinf(back[5])
    import torch
    t = torch.from_numpy(np.random.default_rng(1).standard_normal(4096).astype(np.float32))
    ref = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(t.numpy()), ref)
