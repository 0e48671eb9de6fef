"""Pair mode (64-token mask blocks served by 128-query workgroups at d = 128) against the CPU oracle."""

import numpy as np
import pytest

import synth
from test_gpu_attention import _check_all_rows, _run

pytestmark = pytest.mark.gpu


def _qkv(B, H, nQ, nK, seed):
    return (synth.normal_bf16((B, H, nQ * 64, 128), seed), synth.normal_bf16((B, H, nK * 64, 128), seed + 1),
            synth.normal_bf16((B, H, nK * 64, 128), seed + 2))


@pytest.mark.parametrize("nQ,nK,density", [(5, 7, 0.5), (4, 9, 1.0), (6, 24, 0.15), (1, 3, 0.7), (8, 16, 0.85)])
def test_pair_rows_all_rows(nQ, nK, density):
    B, H = 2, 3
    mask = synth.random_mask(H, nQ, nK, density, seed=nQ * 100 + nK, keep_diag=False)
    if nQ >= 4:
        mask[1, 1, :] = 0            # one query block of a pair empty, its sibling not
        mask[1, 0, 0] = 1
        mask[2, 2, :] = 0            # a whole pair empty
        mask[2, 3, :] = 0
        mask[0, 0, :] = 1            # a full row
    qb, kb, vb = _qkv(B, H, nQ, nK, 41)
    for kw in (dict(num_partitions=4), dict(num_partitions=7, max_item_len=2), dict(num_partitions=64, max_item_len=1),
               dict(num_partitions=3, mode=1, max_item_len=-1), dict(num_partitions=5, mode=2, dynamic_tail=300)):
        print("pair case", nQ, nK, density, kw, flush=True)
        plan, O, L = _run(mask, 64, qb, kb, vb, pair_rows=True, **kw)
        _check_all_rows(mask, 64, qb, kb, vb, O, L)
        plan.close()


def test_pair_rows_zero_mask_and_plain_plan_agree():
    B, H, nQ, nK = 1, 2, 3, 4
    qb, kb, vb = _qkv(B, H, nQ, nK, 51)
    zero = np.zeros((H, nQ, nK), dtype=np.uint8)
    plan, O, L = _run(zero, 64, qb, kb, vb, pair_rows=True, num_partitions=8)
    assert np.all(O == 0) and np.all(np.isneginf(L))
    plan.close()
    mask = synth.random_mask(H, nQ, nK, 0.6, seed=5, keep_diag=True)
    plan, O1, L1 = _run(mask, 64, qb, kb, vb, pair_rows=True, num_partitions=8)
    plan.close()
    plan, O2, L2 = _run(mask, 64, qb, kb, vb, num_partitions=8)
    plan.close()
    assert np.abs(O1 - O2).max() <= 1e-2 and np.abs(L1 - L2).max() <= 1e-3


def test_pair_rows_full_size_sampled_rows():
    # the CogVideoX-like mask (48 heads, 275 x 275 blocks of 64 tokens: an odd number of query blocks) at d = 128,
    # in the launch configuration the benchmark's pair-row measurement uses
    from oracle import attention as oa
    from oracle import planner as op
    from test_gpu_attention import LSE_TOL, O_TOL, _sample_rows
    mask = synth.mask_for_config(2)
    H, nQ, nK = mask.shape
    qb, kb, vb = (synth.normal_bf16((1, H, n * 64, 128), 61 + t) for t, n in enumerate((nQ, nK, nK)))
    print("pair full size", mask.shape, flush=True)
    plan, O, L = _run(mask, 64, qb, kb, vb, pair_rows=True, mode=op.MODE_ROUNDS, locality_groups=8, dynamic_tail=40)
    ref = op.plan(mask, plan.stats()["num_partitions"], mode=op.MODE_ROUNDS, locality_groups=8, dynamic_tail=40, pair=True)
    rows = _sample_rows(mask, 2, seed=7) + [(0, h, nQ - 1) for h in range(0, H, 7)]     # the unpaired last block too
    for i in ref["tail_items"][:2] + ref["tail_items"][-2:]:
        rows += [(0, ref["items"][i][0], 2 * ref["items"][i][1])]
    for r, _, _ in ref["split_rows"][:6]:
        h, p = divmod(r, (nQ + 1) // 2)
        rows += [(0, h, 2 * p), (0, h, min(2 * p + 1, nQ - 1))]
    rows = sorted(set(rows))
    q32, k32, v32 = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
    Or, Lr = oa.masked_attention_rows(q32, k32, v32, mask, 64, rows)
    O = O.reshape(1, H, nQ, 64, 128)
    L = L.reshape(1, H, nQ, 64)
    for t, (b, h, I) in enumerate(rows):
        assert np.abs(O[b, h, I] - Or[t]).max() <= O_TOL, (h, I)
        assert np.abs(L[b, h, I] - Lr[t]).max() <= LSE_TOL, (h, I)
    assert np.isfinite(O).all() and np.isfinite(L).all()
    vmax = v32.max(axis=2)[:, :, None, None, :] + O_TOL
    vmin = v32.min(axis=2)[:, :, None, None, :] - O_TOL
    assert (O <= vmax).all() and (O >= vmin).all()
    st = plan.stats()
    assert st["rho_plan"] == ref["rho_plan"] and st["nnz"] == ref["nnz"] and st["num_partitions"] == 256
    assert plan.tail_takes().tolist() == [1] * len(ref["tail_items"])
    plan.close()


def test_pair_rows_scores_that_keep_growing_take_the_rescale_path():
    # growing keys and outliers (the speculative softmax redoes units again and again) while the two
    # query blocks of a pair use different KV blocks, so redone units and zero-probability units mix
    H, nQ, nK = 2, 4, 10
    mask = synth.random_mask(H, nQ, nK, 0.5, seed=77, keep_diag=True)
    mask[0, 0, :] = 1
    mask[0, 1, ::2] = 0
    rng = np.random.default_rng(98)
    q = rng.standard_normal((1, H, nQ * 64, 128)).astype(np.float32)
    k = rng.standard_normal((1, H, nK * 64, 128)).astype(np.float32)
    v = rng.uniform(-1.0, 1.0, (1, H, nK * 64, 128)).astype(np.float32)
    k *= np.linspace(0.2, 5.0, nK * 64, dtype=np.float32)[None, None, :, None]
    k[:, :, rng.integers(0, nK * 64, 12)] *= 4.0
    q[:, :, 5] = 1e-3 * q[:, :, 5]
    qb, kb, vb = (synth.f32_to_bf16_bits(x) for x in (q, k, v))
    for kw in (dict(num_partitions=4), dict(num_partitions=5, max_item_len=2)):
        plan, O, L = _run(mask, 64, qb, kb, vb, pair_rows=True, **kw)
        _check_all_rows(mask, 64, qb, kb, vb, O, L)
        plan.close()


def test_pair_rows_through_the_entry_point_that_allocates_nothing():
    # split pair rows put 128-row partials into the static scratch array: same results as with the plan's buffer
    import torch
    import paper_2511_23113_amd as dbsp
    from test_gpu_attention import _dev
    H, nQ, nK = 2, 5, 12
    mask = synth.random_mask(H, nQ, nK, 0.7, seed=12, keep_diag=True)
    qb, kb, vb = _qkv(2, H, nQ, nK, 71)
    plan = dbsp.plan_sparse_attn(mask, 64, num_partitions=16, max_item_len=2, pair_rows=True, max_batch=2)
    assert plan.stats(with_rho=False)["n_items"] > H * 3
    q, k, v = _dev(qb), _dev(kb), _dev(vb)
    o1, l1 = dbsp.sparse_attn_fwd(plan, q, k, v)
    o2, l2 = dbsp.sparse_attn_fwd(plan, q, k, v, static_scratch=True)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    _check_all_rows(mask, 64, qb, kb, vb, o2.float().cpu().numpy(), l2.cpu().numpy())
    plan.close()


def test_pair_auto_picks_a_kind_and_both_kinds_agree_with_the_oracle():
    # neighbouring rows alike -> pair rows; unrelated rows -> the plain plan; the results do not depend on the choice
    import paper_2511_23113_amd as dbsp
    H, nQ, nK = 2, 6, 16
    alike = np.repeat(synth.random_mask(H, nQ // 2, nK, 0.5, seed=3, keep_diag=False), 2, axis=1)
    unrelated = synth.random_mask(H, nQ, nK, 0.2, seed=4, keep_diag=False)
    qb, kb, vb = _qkv(1, H, nQ, nK, 81)
    for mask, want in ((alike, True), (unrelated, False)):
        plan, O, L = _run(mask, 64, qb, kb, vb, pair_rows="auto", head_dim=128, num_partitions=8)
        assert plan.pair_rows is want
        _check_all_rows(mask, 64, qb, kb, vb, O, L)
        plan.close()
    with pytest.raises(dbsp.DbspError):
        dbsp.plan_sparse_attn(alike, 64, pair_rows="auto")           # the head dim must be stated
