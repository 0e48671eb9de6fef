#!/usr/bin/env python3
"""Benchmark of the block-sparse attention hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: plan_sparse_attn
(mask compaction, work items, greedy placement, rho_s, plan upload) followed by
sparse_attn_fwd (persistent kernel + fix-up).  Q/K/V live in HBM before the timed region; the
block mask is a host array, as the C ABI takes it.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (2.5 PFLOP/s)

# HBM-side bytes per launch of dbsp_fwd_kernel come from rocprofv3 --pmc runs of this command
# (FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for a plain 1 GiB copy).  They are not
# measured in this run: the line reports what the tracked counter summary states, together with the
# file and the commit it was taken at, or null when there is no summary for the workload.
TRAFFIC_SUMMARY = {3: "profiles/dbsp_fwd_kernel_config3_pmc.md", 2: "profiles/dbsp_fwd_kernel_config2_pmc.md",
                   5: "profiles/dbsp_fwd_kernel_config5_pmc.md"}


def recorded_traffic(cfg):
    """(bytes per launch, {"file", "commit"}) from the summary's line
    `roofline.traffic: <bytes> bytes per launch, measured at commit <hash>`; (None, None) if absent."""
    import re
    path = TRAFFIC_SUMMARY.get(cfg)
    if not path or not os.path.exists(os.path.join(ROOT, path)):
        return None, None
    m = re.search(r"roofline\.traffic:\s*([0-9.eE+]+)\s*bytes per launch, measured at commit\s+([0-9a-f]{7,40})",
                  open(os.path.join(ROOT, path)).read())
    if not m:
        return None, None
    return float(m.group(1)), {"file": path, "commit": m.group(2)}


def algorithmic_bytes(mask, block, d, B=1):
    """What the method must move if nothing is reused: K and V of every active pair, Q and O of every non-empty row, LSE."""
    pairs = int((mask != 0).sum())
    rows = int(((mask != 0).sum(2) > 0).sum())
    return B * (pairs * 4.0 * block * d + rows * (4.0 * block * d + 4.0 * block))


def cpu_baseline(cfg, c, mask, qb, kb, vb, budget_s=15.0):
    """The oracle as it stands, timed on this host on a bounded, seeded sample of rows."""
    import numpy as np
    import synth
    from oracle import attention as oa
    block, d = c["block"], c["d"]
    rng = np.random.default_rng(12345)
    H, nQ, _ = mask.shape
    cnt = (mask != 0).sum(2)
    t_used, blocks, rows = 0.0, 0, 0
    for h in range(H):                       # an equal share of the budget for every head
        q32, k32, v32 = (synth.bf16_bits_to_f32(x[:, h:h + 1]) for x in (qb, kb, vb))
        t_head = 0.0
        for I in rng.choice(nQ, size=min(nQ, 32), replace=False):
            t0 = time.perf_counter()
            oa.masked_attention_rows(q32, k32, v32, mask[h:h + 1], block, [(0, 0, int(I))])
            t_head += time.perf_counter() - t0
            blocks += int(cnt[h, I])
            rows += 1
            if t_head >= budget_s / H:
                break
        t_used += t_head
    tflops = blocks * 4.0 * block * block * d / t_used / 1e12
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": tflops, "unit": "TFLOP/s (active blocks)", "cores": min(threads, os.cpu_count() or threads),
            "kind": "oracle", "host_cpus": os.cpu_count(),
            "sample": f"{rows} seeded (head, q-block) rows of the same workload, {blocks} active blocks, "
                      f"{t_used:.1f} s of float64 numpy; throughput extrapolated by active-block count"}


def timed_launches(dbsp, torch, plan, qq, kk, vv, oo, ll, reps=3, warm=2):
    """Mean time of `reps` launches (HIP events on the launch stream), after `warm` untimed ones."""
    for _ in range(warm):
        dbsp.sparse_attn_fwd(plan, qq, kk, vv, o=oo, lse=ll)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dbsp.sparse_attn_fwd(plan, qq, kk, vv, o=oo, lse=ll)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def busy_rho_per_cu(np, plan):
    ticks, hw = plan.busy()
    percu = {}
    for tk, idv in zip(ticks.tolist(), hw.tolist()):
        percu[idv] = percu.get(idv, 0) + tk
    vals = np.array(list(percu.values()), dtype=np.float64)
    return (float(vals.max() / vals.mean()) if vals.sum() > 0 else 1.0), len(percu)


def low_density_heads(dbsp, torch, np, c, mask, q, k, v, o, lse, plan_kw):
    """The low-density heads of the workload on their own (extra launches): few rows share a KV block
    there, so the memory rate is what counts; reported as algorithmic bytes per second."""
    block, d = c["block"], c["d"]
    dens = (mask != 0).mean(axis=(1, 2))
    low = np.where(dens < 0.12)[0]
    if not len(low):
        return None
    m2 = mask.copy()
    m2[[h for h in range(mask.shape[0]) if h not in set(low.tolist())]] = 0
    plan = dbsp.plan_sparse_attn(m2, block, **plan_kw)
    ms = timed_launches(dbsp, torch, plan, q, k, v, o, lse, reps=10, warm=5)
    plan.close()
    pairs = int((m2 != 0).sum())
    return {"heads": low.tolist(), "density": [round(float(x), 4) for x in dens[low]], "active_blocks": pairs,
            "kernel_ms": ms, "algorithmic_GB_per_s": algorithmic_bytes(m2, block, d) / (ms * 1e-3) / 1e9,
            "tflops": pairs * 4.0 * block * block * d / (ms * 1e-3) / 1e12}


def pair_rows(dbsp, synth, torch, np, c, mask, q, k, v, o, lse, plan_kw, keeps=(1.0, 0.75, 0.5)):
    """64-token mask blocks at d = 128 (the paper's PAROAttention block size: Methodology, "Block-level
    Partitioning") on the workload's tensors: its mask refined to half blocks, served by the plain
    two-wave kernel and by 128-query workgroups over pair rows (extra launches).  flag_fill = share of
    the (query block, KV block) combinations of the super blocks that the mask has."""
    rows = []
    for keep in keeps:
        fine = synth.refine_to_half_blocks(mask, keep)
        nnz = int(fine.sum())
        flops = float(c["B"]) * nnz * 4.0 * 64 * 64 * c["d"]
        row = {"keep": keep, "active_blocks": nnz}
        for name, pair in (("plain", False), ("pair_rows", True)):
            plan = dbsp.plan_sparse_attn(fine, 64, **dict(plan_kw, num_partitions=0, partition_cost=None, pair_rows=pair, head_dim=c["d"]))
            ms = timed_launches(dbsp, torch, plan, q, k, v, o, lse, reps=5, warm=3)
            rho_busy, _ = busy_rho_per_cu(np, plan)
            st = plan.stats(with_rho=False)
            row[name] = {"kernel_ms": ms, "frac_of_bf16_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                         "partitions": st["num_partitions"], "plan_ms": st["plan_usec"] / 1e3, "rho_busy_per_cu": rho_busy}
            if pair:
                row[name]["flag_fill"] = nnz / (4.0 * st["nnz"])
            plan.close()
        auto = dbsp.plan_sparse_attn(fine, 64, **dict(plan_kw, num_partitions=0, partition_cost=None, pair_rows="auto", head_dim=c["d"],
                                                         host_only=True))
        row["auto_choice"] = "pair_rows" if auto.pair_rows else "plain"      # what DBSP_PLAN_PAIR_AUTO plans with
        auto.close()
        rows.append(row)
    return rows


def other_config(dbsp, synth, torch, np, cfg, plan_kw):
    """One of the other workload configs under the same placement options: kernel time, fraction of the
    bf16 MFMA peak, algorithmic bytes per second, planning time, busy-time imbalance (extra launches)."""
    c = synth.config_shape(cfg)
    block, d, B = c["block"], c["d"], c["B"]
    mask = synth.mask_for_config(cfg)
    qb, kb, vb = synth.qkv_for_config(cfg, B, c["H"], c["Nq"], c["Nk"], d)
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    q, k, v = dev(qb), dev(kb), dev(vb)
    o = torch.empty_like(q)
    lse = torch.empty((B, c["H"], c["Nq"]), dtype=torch.float32, device="cuda")
    plan_ms = []
    for _ in range(4):
        plan = dbsp.plan_sparse_attn(mask, block, **plan_kw)
        plan_ms.append(plan.stats(with_rho=False)["plan_usec"] / 1e3)
        if _ < 3:
            plan.close()
    # short kernels: enough warm-up launches for the clocks to come back up after the host-side set-up
    ms = timed_launches(dbsp, torch, plan, q, k, v, o, lse, reps=10 if cfg != 4 else 3, warm=10 if cfg != 4 else 2)
    rho_busy, _ = busy_rho_per_cu(np, plan)
    st = plan.stats()
    plan.close()
    nnz = int((mask != 0).sum())
    flops = float(B) * nnz * 4.0 * block * block * d
    del q, k, v, o, lse
    torch.cuda.empty_cache()
    return {"workload": f"config {cfg}: {c['name']} H={c['H']} Nq={c['Nq']} Nk={c['Nk']} d={d} block={block}", "active_blocks": nnz,
            "kernel_ms": ms, "frac_of_bf16_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "algorithmic_GB_per_s": algorithmic_bytes(mask, block, d, B) / (ms * 1e-3) / 1e9,
            "plan_ms": float(np.median(plan_ms)), "rho_busy_per_cu": rho_busy,
            "rho_s_planned": {"naive": st["rho_naive"], "balanced": st["rho_balanced"], "timed": st["rho_plan"]}}


def speedup_sweep(dbsp, synth, torch, np, q, k, v, o, lse, plan_kw, targets=(1.0, 1.25, 1.5, 2.0, 2.5, 3.0)):
    """Kernel time under the naive placement against the balanced one, over masks of the workload's
    shape whose imbalance under the naive placement is dialled from about 1 to about 3 (the one-GPU
    form of the paper's attention speed-up against imbalance ratio experiment)."""
    rows = []
    for tgt in targets:
        m = synth.imbalance_sweep_mask(tgt)
        res = {"target": tgt, "active_blocks": int((m != 0).sum())}
        for name, kw in (("naive", dict(mode=dbsp.MODE_NAIVE)), ("balanced", plan_kw)):
            plan = dbsp.plan_sparse_attn(m, 128, **kw)
            res[name + "_ms"] = timed_launches(dbsp, torch, plan, q, k, v, o, lse, reps=3)
            res["rho_busy_" + name], _ = busy_rho_per_cu(np, plan)
            st = plan.stats()
            res["rho_s_naive"] = st["rho_naive"]
            res["rho_s_" + name] = st["rho_plan"]
            plan.close()
        res["speedup"] = res["naive_ms"] / res["balanced_ms"]
        rows.append(res)
    return rows


def placement_sweep(dbsp, torch, np, mask, block, q, k, v, o, lse):
    """The locality / balance trade-off on the workload: the round-based placement over the number of
    locality groups G, and the greedy placement with the paper's reward factor R_b over R_b and G.
    Three launches each (the first untimed), in the order listed: a rocprofv3 --pmc run of this command
    sees the dbsp_fwd_kernel dispatches in that order."""
    variants = [("greedy", dict(mode=dbsp.MODE_BALANCED))]
    variants += [(f"rounds G={g}", dict(mode=dbsp.MODE_ROUNDS, locality_groups=g)) for g in (1, 2, 4, 8, 16, 32)]
    variants += [(f"reward G=8 R_b={r}", dict(mode=dbsp.MODE_REWARD, locality_groups=8, reward=r)) for r in (0.0, 0.25, 0.5, 1.0, 2.0, 8.0)]
    variants += [(f"reward G={g} R_b=1.0", dict(mode=dbsp.MODE_REWARD, locality_groups=g, reward=1.0)) for g in (1, 2, 4, 16, 32)]
    rows = []
    for name, kw in variants:
        plan = dbsp.plan_sparse_attn(mask, block, **kw)
        ms = timed_launches(dbsp, torch, plan, q, k, v, o, lse, reps=2, warm=1)
        rho_busy, _ = busy_rho_per_cu(np, plan)
        rows.append({"placement": name, "rho_s": plan.stats(with_rho=False)["rho_plan"], "kernel_ms": ms, "rho_busy_per_cu": rho_busy,
                     "launches": 3})
        plan.close()
    return rows


def extras(dbsp, synth, torch, np, cfg, c, mask, q, k, v, o, lse):
    """Side measurements (not part of the timed region)."""
    res = {}

    def timed(plan, qq, kk, vv, oo, ll, reps=3):
        return timed_launches(dbsp, torch, plan, qq, kk, vv, oo, ll, reps=reps)

    # kernel time against the number of active blocks: the cost of a mask is its dense-block count
    # (paper: Background, "Block-wise Sparse Attention"), so this should be a straight line.  The masks are
    # config 5's first mask restricted to its first 1..H heads, then the first masks of its sequence.
    c5 = synth.config_shape(5)
    qb, kb, vb = synth.qkv_for_config(5, c5["B"], c5["H"], c5["Nq"], c5["Nk"], c5["d"])
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    q5, k5, v5 = dev(qb), dev(kb), dev(vb)
    o5 = torch.empty_like(q5)
    l5 = torch.empty((c5["B"], c5["H"], c5["Nq"]), dtype=torch.float32, device="cuda")
    seq = list(synth.mask_sequence_cfg5(8))
    masks = []
    for nh in range(1, c5["H"] + 1):
        m = seq[0].copy()
        m[nh:] = 0
        masks.append(m)
    masks += seq[1:]
    xs, ys = [], []
    for m in masks:
        plan = dbsp.plan_sparse_attn(m, c5["block"], mode=dbsp.MODE_ROUNDS, locality_groups=8)
        ys.append(timed(plan, q5, k5, v5, o5, l5))
        xs.append(int((m != 0).sum()))
        plan.close()
    xs, ys = np.array(xs, dtype=np.float64), np.array(ys)
    slope, icpt = np.polyfit(xs, ys, 1)
    r2 = 1.0 - ((ys - (slope * xs + icpt)) ** 2).sum() / ((ys - ys.mean()) ** 2).sum()
    res["config5_time_vs_blocks"] = {"masks": len(xs), "blocks": [int(x) for x in xs], "kernel_ms": [round(float(y), 4) for y in ys],
                                     "us_per_1000_blocks": float(slope * 1e6), "intercept_ms": float(icpt), "r_squared": float(r2)}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload config (3 = Wan-14B-like 480p, the headline shape)")
    ap.add_argument("--partitions", type=int, default=0, help="0 = one per compute unit")
    ap.add_argument("--reuse-plan", action="store_true", help="static-mask mode: plan once outside the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=12.0, help="seconds of oracle time to spend on the CPU baseline sample")
    ap.add_argument("--compare-placements", action="store_true",
                    help="also time the kernel under the naive and the greedy longest-first placement (extra launches)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (3x), so that a rocprofv3 --pmc run of this "
                         "command can scale FETCH_SIZE / WRITE_SIZE by what they read for a copy of known size")
    ap.add_argument("--locality-groups", type=int, default=8,
                    help="round-based placement: keep runs of neighbouring query blocks inside one of G groups of partitions "
                         "(partition p is in group p mod G; 8 = the XCDs of an MI355X, each with its own L2); 0 or 1 = one group")
    ap.add_argument("--dynamic-tail", type=int, default=40,
                    help="permille of the work left to the queue all workgroups share (taken at run time by whoever runs out of "
                         "placed work); 0 = everything placed")
    ap.add_argument("--no-side-measurements", action="store_true",
                    help="leave out the low-density heads and the other workload configs (extra launches after the timed region): "
                         "for profiler runs that should see the timed launches only")
    ap.add_argument("--half-blocks", action="store_true",
                    help="run the 64-token-block side measurement (plain kernel against pair rows) even with --no-side-measurements")
    ap.add_argument("--speedup-sweep", action="store_true",
                    help="also time the naive against the balanced placement over masks whose imbalance is dialled from 1 to 3")
    ap.add_argument("--placement-sweep", action="store_true",
                    help="also time the round-based placement over the number of locality groups and the reward-biased greedy over R_b")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the few-millisecond measurement of the chip's sustained MFMA rate")
    ap.add_argument("--extras", action="store_true",
                    help="also measure (extra launches, outside the timed region) kernel time against active-block count over "
                         "masks of config 5")
    ap.add_argument("--zero-data", action="store_true",
                    help="power experiment, not the benchmark: all-zero Q, K, V (same instruction stream and cycle count, far fewer "
                         "bit flips, so the chip holds a higher clock)")
    ap.add_argument("--calibrate", action="store_true",
                    help="feed the per-compute-unit speeds measured in the last warm-up launch back into the placement "
                         "(worth about 1 %% once clocks have settled: use a long warm-up)")
    ap.add_argument("--item-overhead", type=int, default=0, help="per-item cost, in blocks, the placement adds to an item's weight")
    ap.add_argument("--fit-cost-model", action="store_true",
                    help="also fit time = a*blocks + c*items + t0 on per-partition busy times of extra launches under several "
                         "placements and split lengths, and compare its prediction for the timed plan with the measured kernel time")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (one GPU's share of the workload "
              "at its real shape is what is measured).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2511_23113_amd as dbsp
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = args.config
    c = synth.config_shape(cfg)
    block, d, B = c["block"], c["d"], c["B"]
    mask = synth.mask_for_config(cfg)
    qb, kb, vb = synth.qkv_for_config(cfg, B, c["H"], c["Nq"], c["Nk"], d)
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    q, k, v = dev(qb), dev(kb), dev(vb)
    if args.zero_data:
        q.zero_(), k.zero_(), v.zero_()
    o = torch.empty_like(q)
    lse = torch.empty((B, c["H"], c["Nq"]), dtype=torch.float32, device="cuda")
    nnz = int((mask != 0).sum())
    flops = float(B) * nnz * 4.0 * block * block * d

    part_cost = {"v": None}  # relative time per block of every partition, measured in the last warm-up launch

    sustained = None
    if not args.no_mfma_probe:
        try:
            tf, ghz = dbsp.mfma_probe()            # back-to-back MFMAs on random operands on every compute unit, ~40 ms
            sustained = {"mfma_tflops": tf, "clock_ghz": ghz}
        except dbsp.DbspError as exc:              # a diagnostic only: never fail the benchmark over it
            print(f"bench.py: MFMA probe failed: {exc}", file=sys.stderr)

    def plan_kw(mode):
        rounds = mode == dbsp.MODE_ROUNDS
        return dict(num_partitions=args.partitions, mode=mode, item_overhead=args.item_overhead,
                    locality_groups=args.locality_groups if rounds else 0, dynamic_tail=args.dynamic_tail if rounds else 0,
                    partition_cost=part_cost["v"] if mode != dbsp.MODE_NAIVE else None)

    def one_plan(mode):
        return dbsp.plan_sparse_attn(mask, block, **plan_kw(mode))

    def measured_rho(plan):
        return busy_rho_per_cu(np, plan)

    # placements: planned rho_s (Eq. 1 on block counts) of the naive, the greedy longest-first and the
    # round-based placement come from the planner alone; kernel times and busy-time imbalance of all
    # three need extra launches of the same kernel and are only taken with --compare-placements, so
    # that a profile of the default command sees one kind of launch only.
    side = {}
    if args.compare_placements:
        for name, mode in (("naive", dbsp.MODE_NAIVE), ("balanced", dbsp.MODE_BALANCED), ("rounds", dbsp.MODE_ROUNDS)):
            plan = one_plan(mode)
            for _ in range(2):
                dbsp.sparse_attn_fwd(plan, q, k, v, o=o, lse=lse)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                dbsp.sparse_attn_fwd(plan, q, k, v, o=o, lse=lse)
            e1.record()
            torch.cuda.synchronize()
            rho_meas, n_cu = measured_rho(plan)
            st = plan.stats()
            side[name] = dict(kernel_ms=e0.elapsed_time(e1) / 3, rho_blocks=st["rho_plan"], rho_busy_per_cu=rho_meas, cus_seen=n_cu)
            plan.close()

    cost = None
    if args.fit_cost_model:
        # samples: one per partition and launch, all under balanced placements (the naive one runs at a
        # different speed per block: its compute units work on different heads and miss in L2).  Block
        # counts are spread by also planning the first half of the heads alone, item counts by the split length.
        L = max(2, nnz // (c["H"] * c["nQ"]))          # mean row length in blocks
        half = mask.copy()
        half[c["H"] // 2:] = 0
        sb, si, st_ = [], [], []
        for m_, mode, ml in ((mask, dbsp.MODE_BALANCED, -1), (mask, dbsp.MODE_BALANCED, L // 2), (mask, dbsp.MODE_ROUNDS, L),
                             (half, dbsp.MODE_BALANCED, -1), (half, dbsp.MODE_BALANCED, L // 2), (half, dbsp.MODE_ROUNDS, L)):
            plan = dbsp.plan_sparse_attn(m_, block, num_partitions=args.partitions, mode=mode, max_item_len=ml)
            for _ in range(2):
                dbsp.sparse_attn_fwd(plan, q, k, v, o=o, lse=lse)
            ticks, _ = plan.busy()
            sb.append(plan.array(dbsp.binding.PART_LOAD).copy())
            si.append(np.diff(plan.array(dbsp.binding.PART_PTR)).astype(np.int64))
            st_.append(ticks.astype(np.float64) / 100.0)            # 100 MHz ticks -> microseconds
            plan.close()
        sb, si, st_ = np.concatenate(sb), np.concatenate(si), np.concatenate(st_)
        keep = si > 0
        a_, c_, t0_, rms_ = dbsp.fit_cost_model(sb[keep], si[keep], st_[keep])
        cost = {"a_us_per_block": a_, "c_us_per_item": c_, "t0_us": t0_, "rms_us": rms_, "samples": int(keep.sum()),
                "item_cost_in_blocks": c_ / a_ if a_ > 0 else None, "mean_sample_us": float(st_[keep].mean())}

    # timed region: K steps of plan + forward
    plans = []
    static_plan = one_plan(dbsp.MODE_ROUNDS) if args.reuse_plan else None
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    plan_us = []

    def step(i, timed):
        plan = static_plan if static_plan is not None else one_plan(dbsp.MODE_ROUNDS)
        if timed:
            ev[i][0].record()
        dbsp.sparse_attn_fwd(plan, q, k, v, o=o, lse=lse)
        if timed:
            ev[i][1].record()
            plan_us.append(plan.stats(with_rho=False)["plan_usec"])
        if static_plan is None:
            plans.append(plan)
            if len(plans) > 2:          # released two steps later (freeing device memory waits for the device)
                plans.pop(0).close()

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    if args.calibrate and static_plan is None and plans:
        part_cost["v"] = plans[-1].calibrate()          # compute units differ by a few percent, systematically
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_s = t1 - t0
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    kern_avg = float(np.mean(kern_ms))
    last = static_plan if static_plan is not None else plans[-1]
    rho_busy, cus_seen = measured_rho(last)       # busy time per compute unit in the last timed launch
    hst = last.stats()
    planned = {"naive": hst["rho_naive"], "balanced": hst["rho_balanced"], "rounds": hst["rho_plan"]}
    if cost is not None:
        pred = cost["a_us_per_block"] * last.array(dbsp.binding.PART_LOAD) + \
            cost["c_us_per_item"] * np.diff(last.array(dbsp.binding.PART_PTR)) + cost["t0_us"]
        cost["predicted_slowest_partition_ms"] = float(pred.max()) / 1e3
        cost["measured_slowest_partition_ms"] = float(last.busy()[0].max()) / 100.0 / 1e3
    for p in plans:
        p.close()
    if static_plan is not None:
        static_plan.close()

    if args.traffic_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    value = flops * args.steps / total_s / 1e12
    kern_tflops = flops / (kern_avg * 1e-3) / 1e12
    default_launch = args.locality_groups == 8 and args.partitions == 0 and args.dynamic_tail == 40 and not args.zero_data
    traffic, traffic_src = recorded_traffic(cfg) if default_launch else (None, None)
    out = {
        "metric": "block-sparse attention effective TFLOPS over active blocks (4*b^2*d per active block pair)",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total_s * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic" if not args.zero_data else "synthetic, all-zero tensors (power experiment, not the benchmark)",
        "config": {"workload": f"config {cfg}: {c['name']} B={B} H={c['H']} Nq={c['Nq']} Nk={c['Nk']} d={d} block={block}, "
                               f"nnz={nnz} active blocks (density {nnz / mask.size:.3f})",
                   "step": "plan_sparse_attn + sparse_attn_fwd" if static_plan is None else "sparse_attn_fwd (plan reused)",
                   "partitions": hst["num_partitions"], "placement": "rounds", "locality_groups": max(1, args.locality_groups),
                   "dynamic_tail_permille": args.dynamic_tail},
        "pct_of_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "kernel_ms": kern_avg,
        "kernel_ms_min": float(np.min(kern_ms)),
        "kernel_ms_median": float(np.median(kern_ms)),
        "kernel_ms_p95": float(np.percentile(kern_ms, 95)),
        "plan_ms": float(np.mean(plan_us)) / 1e3 if plan_us else None,
        "plan_pct_of_kernel": (float(np.mean(plan_us)) / 1e3 / kern_avg * 100.0) if plan_us else None,
        "imbalance": {"rho_s_planned": planned, "rho_busy_per_cu": rho_busy, "cus_seen": cus_seen,
                      "placement_timed": "rounds",
                      "partition_cost": None if part_cost["v"] is None else {"min": int(part_cost["v"].min()), "max": int(part_cost["v"].max()),
                                                                          "unit": "1024 = mean time per block"},
                      **({"compare": side} if side else {})},
        "roofline": {"bound": "mfma", "achieved": kern_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": kern_tflops / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "dbsp_fwd_kernel", "flops_per_launch": flops,
                     "algorithmic_bytes_per_launch": algorithmic_bytes(mask, block, d, B),
                     "algorithmic_GB_per_s": algorithmic_bytes(mask, block, d, B) / (kern_avg * 1e-3) / 1e9,
                     **({"sustained_mfma_only": {**sustained, "frac_of_sustained": kern_tflops / sustained["mfma_tflops"]}}
                        if sustained else {})},
    }
    if cost is not None:
        out["cost_model"] = cost
    kw_timed = plan_kw(dbsp.MODE_ROUNDS)
    if not args.no_side_measurements:
        ld = low_density_heads(dbsp, torch, np, c, mask, q, k, v, o, lse, kw_timed)
        if ld is not None:
            out["low_density_heads"] = ld
    if (args.half_blocks or not args.no_side_measurements) and block == 128 and d == 128:
        out["half_blocks_64_tokens"] = pair_rows(dbsp, synth, torch, np, c, mask, q, k, v, o, lse, kw_timed)
    if args.speedup_sweep and cfg == 3:
        out["speedup_vs_imbalance"] = speedup_sweep(dbsp, synth, torch, np, q, k, v, o, lse, kw_timed)
    if args.placement_sweep:
        out["placement_sweep"] = placement_sweep(dbsp, torch, np, mask, block, q, k, v, o, lse)
    if args.extras:
        out["extras"] = extras(dbsp, synth, torch, np, cfg, c, mask, q, k, v, o, lse)
    if not args.no_side_measurements:
        del q, k, v, o, lse
        torch.cuda.empty_cache()
        kw_other = dict(kw_timed, num_partitions=0, partition_cost=None)
        out["other_configs"] = [other_config(dbsp, synth, torch, np, oc, kw_other) for oc in (2, 4, 5) if oc != cfg]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, c, mask, qb, kb, vb, budget_s=args.cpu_budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
