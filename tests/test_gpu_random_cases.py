"""Randomised parity of the HIP path with the CPU oracle: shapes, masks, placement options, split lengths,
batch sizes, scales and entry points drawn from one seeded stream; every row of every case is compared."""

import numpy as np
import pytest

import synth
from oracle import attention as oa

pytestmark = pytest.mark.gpu

O_TOL = 1e-2
LSE_TOL = 1e-3


def _case(rng, case):
    block, d = [(64, 64), (128, 128), (64, 128), (128, 64), (64, 128)][int(rng.integers(0, 5))]
    pair = bool(block == 64 and d == 128 and rng.random() < 0.6)
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    nQ, nK = int(rng.integers(1, 7)), int(rng.integers(1, 13))
    mask = (rng.random((H, nQ, nK)) < float(rng.choice([0.1, 0.3, 0.6, 0.9, 1.0]))).astype(np.uint8)
    if rng.random() < 0.3:
        mask[int(rng.integers(0, H)), int(rng.integers(0, nQ))] = 0          # an empty row
    mode = int(rng.choice([0, 1, 2]))
    P = int(rng.choice([1, 2, 3, 5, 8, 16, 64]))
    kw = dict(num_partitions=P, mode=mode, max_item_len=int(rng.choice([0, -1, 1, 2, 3])), max_batch=B, pair_rows=pair)
    if mode == 2:
        kw["dynamic_tail"] = int(rng.choice([0, 50, 300, 900]))
        G = int(rng.choice([1, 2, 4]))
        if P % G == 0:
            kw["locality_groups"] = G
    scale = float(rng.choice([0.0, 0.05, 0.2]))
    static = bool(rng.random() < 0.3)
    qb = synth.normal_bf16((B, H, nQ * block, d), 10000 + case)
    kb = synth.normal_bf16((B, H, nK * block, d), 20000 + case)
    # V in [-1, 1]: O is a convex combination of V rows, so the absolute bound applies as it stands
    v = np.random.Generator(np.random.PCG64(30000 + case)).uniform(-1.0, 1.0, (B, H, nK * block, d)).astype(np.float32)
    return block, d, mask, kw, scale, static, qb, kb, synth.f32_to_bf16_bits(v)


def test_random_cases_all_rows():
    import torch
    import paper_2511_23113_amd as dbsp
    from test_gpu_attention import _dev
    rng = np.random.default_rng(20251123)
    worst_o = worst_l = 0.0
    for case in range(200):
        block, d, mask, kw, scale, static, qb, kb, vb = _case(rng, case)
        what = (case, block, d, mask.shape, qb.shape[0], scale, static, kw)
        plan = dbsp.plan_sparse_attn(mask, block, **kw)
        o, lse = dbsp.sparse_attn_fwd(plan, _dev(qb), _dev(kb), _dev(vb), softmax_scale=scale, static_scratch=static)
        torch.cuda.synchronize()
        O, L = o.float().cpu().numpy(), lse.cpu().numpy()
        plan.close()
        q32, k32, v32 = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
        Or, Lr = oa.masked_attention(q32, k32, v32, mask, block, scale=(scale if scale > 0 else None))
        empty = np.isneginf(Lr)
        assert np.array_equal(np.isneginf(L), empty), what
        assert np.isfinite(O).all() and np.all(O[empty] == 0), what
        eo = float(np.abs(O - Or).max())
        el = float(np.abs(L[~empty] - Lr[~empty]).max()) if (~empty).any() else 0.0
        assert eo <= O_TOL and el <= LSE_TOL, (what, eo, el)
        worst_o, worst_l = max(worst_o, eo), max(worst_l, el)
    print(f"200 random cases: worst |dO| {worst_o:.2e}, worst |dLSE| {worst_l:.2e}")
