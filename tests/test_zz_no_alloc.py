"""sparse_attn_fwd_static (the entry point that allocates nothing; split-row partials go to the
library's static device array) against sparse_attn_fwd, through the C ABI, on two calls in a row,
the second with a smaller input: the array keeps the first call's contents, which must not leak
into the second call's result."""

import ctypes as C

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

O_TOL = 1e-2
LSE_TOL = 1e-3


def _dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _both_entry_points(mask, block, d, B, seed):
    import torch
    import paper_2511_23113_amd as dbsp
    from paper_2511_23113_amd import binding
    lib = binding.load_library()
    H, nQ, nK = mask.shape
    q = _dev(synth.normal_bf16((B, H, nQ * block, d), seed))
    k = _dev(synth.normal_bf16((B, H, nK * block, d), seed + 1))
    v = _dev(synth.normal_bf16((B, H, nK * block, d), seed + 2))
    plan = dbsp.plan_sparse_attn(mask, block, mode=dbsp.MODE_ROUNDS, locality_groups=8, max_batch=B)
    assert plan.stats(with_rho=False)["n_items"] > int(((mask != 0).sum(2) > 0).sum())        # some rows are split
    outs = []
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for entry in (lib.sparse_attn_fwd, lib.sparse_attn_fwd_static):
        o = torch.full_like(q, float("nan"))
        lse = torch.full((B, H, nQ * block), float("nan"), dtype=torch.float32, device="cuda")
        rc = entry(plan.handle, C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()),
                   C.c_void_p(o.data_ptr()), C.c_void_p(lse.data_ptr()), B, nQ * block, nK * block, d, 0.0, stream)
        assert rc == 0, lib.dbsp_last_error().decode()
        torch.cuda.synchronize()
        outs.append((o.float().cpu().numpy(), lse.cpu().numpy()))
    plan.close()
    (o_ref, l_ref), (o_new, l_new) = outs
    assert np.isfinite(o_new).all() and np.isfinite(l_new).all()
    assert np.abs(o_new - o_ref).max() <= O_TOL
    assert np.abs(l_new - l_ref).max() <= LSE_TOL
    return o_new


def test_static_scratch_entry_point_matches_on_two_calls_the_second_smaller():
    # first call: config 5's mask at full size (a few hundred split-row chunks, 20 MB of partials)
    c = synth.config_shape(5)
    _both_entry_points(synth.mask_for_config(5), c["block"], c["d"], 1, 500)
    # second call: a smaller mask and head dim, two batch entries, every row split
    rng = np.random.default_rng(5)
    small = (rng.random((3, 4, 24)) < 0.7).astype(np.uint8)
    small[:, :, 0] = 1
    _both_entry_points(small, 64, 64, 2, 600)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2511_23113_amd as dbsp
    from paper_2511_23113_amd import binding
    lib = binding.load_library()
    # 40 rows of 64 blocks, each cut into 32 chunks of 2: 1280 chunks x 128 x 129 x 4 bytes = 84.5 MB > 32 MiB
    mask = np.ones((1, 40, 64), dtype=np.uint8)
    plan = dbsp.plan_sparse_attn(mask, 128, num_partitions=256, max_item_len=2)
    q = torch.zeros((1, 1, 40 * 128, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((1, 1, 64 * 128, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q)
    rc = lib.sparse_attn_fwd_static(plan.handle, C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()), C.c_void_p(k.data_ptr()),
                                    C.c_void_p(o.data_ptr()), None, 1, 40 * 128, 64 * 128, 128, 0.0, None)
    msg = lib.dbsp_last_error().decode()
    plan.close()
    assert rc == binding.DBSP_EINVAL and "static buffer holds 33554432" in msg and "84" in msg
