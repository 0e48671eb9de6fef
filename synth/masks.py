"""Seeded block-mask generators with the structure of video-DiT sparse attention masks.

The paper's masks (PAROAttention / SpargeAttn on Wan2.1 and CogVideoX1.5, evaluation
setup section) are not available; these synthetic recipes stand in for them.  A mask is
uint8 [H, nQ, nK]; nonzero means the (query block, key block) pair is computed.

All randomness comes from numpy PCG64 streams derived from `7000 + cfg` with
SeedSequence.spawn: stream h (h < H) drives head h, stream H drives per-config draws
(densities, head shuffles).
"""

from __future__ import annotations

import numpy as np

# cfg -> (B, H, d, block, nQ, nK)
CONFIGS = {
    1: dict(name="tiny", B=1, H=2, d=64, block=64, nQ=8, nK=8),
    2: dict(name="cogvideox5b-like", B=1, H=48, d=64, block=64, nQ=275, nK=275),
    3: dict(name="wan14b-like-480p", B=1, H=40, d=128, block=128, nQ=256, nK=256),
    4: dict(name="hunyuan-like-720p", B=1, H=24, d=128, block=128, nQ=928, nK=928),
    5: dict(name="device-share", B=1, H=10, d=128, block=128, nQ=128, nK=256),
}


def config_shape(cfg: int) -> dict:
    c = dict(CONFIGS[cfg])
    c["Nq"] = c["nQ"] * c["block"]
    c["Nk"] = c["nK"] * c["block"]
    return c


def _streams(cfg: int, H: int):
    ss = np.random.SeedSequence(7000 + cfg).spawn(H + 1)
    return [np.random.Generator(np.random.PCG64(s)) for s in ss]


def _fill_to_count(m: np.ndarray, target: int, rng) -> None:
    """Switch on uniformly chosen inactive blocks of one head until `target` are on."""
    have = int(m.sum())
    need = target - have
    if need <= 0:
        return
    flat = m.reshape(-1)
    off = np.flatnonzero(flat == 0)
    pick = rng.choice(off, size=min(need, off.size), replace=False)
    flat[pick] = 1


def _cfg1():
    c = CONFIGS[1]
    H, n = c["H"], c["nQ"]
    rngs = _streams(1, H)
    mask = np.zeros((H, n, n), dtype=np.uint8)
    for h, p in enumerate((0.5, 0.15)):
        m = (rngs[h].random((n, n)) < p).astype(np.uint8)
        m[np.arange(n), np.arange(n)] = 1
        mask[h] = m
    return mask


def _cfg2():
    c = CONFIGS[2]
    H, n = c["H"], c["nQ"]
    rngs = _streams(2, H)
    dens = rngs[H].beta(2.0, 6.0, size=H)
    I, J = np.indices((n, n))
    base = ((np.abs(I - J) <= 1) | (J < 2)).astype(np.uint8)
    mask = np.empty((H, n, n), dtype=np.uint8)
    for h in range(H):
        m = base.copy()
        _fill_to_count(m, int(round(float(dens[h]) * n * n)), rngs[h])
        mask[h] = m
    return mask


def _cfg3():
    c = CONFIGS[3]
    H, n = c["H"], c["nQ"]
    rngs = _streams(3, H)
    dens = rngs[H].uniform(0.05, 0.60, size=H)
    I, J = np.indices((n, n))
    band = np.zeros((n, n), dtype=bool)
    for kf in (-1, 0, 1):
        band |= np.abs(I - J - 16 * kf) <= 1
    mask = np.empty((H, n, n), dtype=np.uint8)
    for h in range(H):
        rng = rngs[h]
        m = band.astype(np.uint8)
        cols = rng.choice(n, size=4, replace=False)
        m[:, cols] = 1
        target = int(round(float(dens[h]) * n * n))
        have = int(m.sum())
        while have < target:
            corners = rng.integers(0, n, size=(256, 2))
            for r0, c0 in corners:
                blk = m[r0:r0 + 4, c0:c0 + 4]
                have += blk.size - int(blk.sum())
                blk[...] = 1
                if have >= target:
                    break
        mask[h] = m
    return mask


def _cfg4():
    c = CONFIGS[4]
    H, n = c["H"], c["nQ"]
    rngs = _streams(4, H)
    g = rngs[H]
    lo = g.uniform(0.05, 0.10, size=H // 2)
    hi = g.uniform(0.30, 0.50, size=H - H // 2)
    dens = np.concatenate([lo, hi])
    g.shuffle(dens)
    I, J = np.indices((n, n))
    base = ((np.abs(I - J) <= 2) | ((I // 32) == (J // 32))).astype(np.uint8)
    mask = np.empty((H, n, n), dtype=np.uint8)
    for h in range(H):
        m = base.copy()
        _fill_to_count(m, int(round(float(dens[h]) * n * n)), rngs[h])
        mask[h] = m
    return mask


def mask_sequence_cfg5(steps: int = 50):
    """Yield `steps` masks [10,128,256]; each step re-draws 20 % of the block positions."""
    c = CONFIGS[5]
    H, nQ, nK = c["H"], c["nQ"], c["nK"]
    rngs = _streams(5, H)
    dens = np.clip(rngs[H].lognormal(np.log(0.15), 0.8, size=H), 0.02, 0.9)
    diag = np.arange(nQ)
    mask = np.empty((H, nQ, nK), dtype=np.uint8)
    for h in range(H):
        m = (rngs[h].random((nQ, nK)) < dens[h]).astype(np.uint8)
        m[diag, diag] = 1
        mask[h] = m
    yield mask.copy()
    n_redraw = (nQ * nK) // 5
    for _ in range(1, steps):
        for h in range(H):
            rng = rngs[h]
            pos = rng.choice(nQ * nK, size=n_redraw, replace=False)
            val = (rng.random(n_redraw) < dens[h]).astype(np.uint8)
            flat = mask[h].reshape(-1)
            flat[pos] = val
            mask[h][diag, diag] = 1
        yield mask.copy()


def mask_for_config(cfg: int) -> np.ndarray:
    """Block mask uint8 [H, nQ, nK] of config `cfg` (config 5: the first step's mask)."""
    if cfg == 1:
        return _cfg1()
    if cfg == 2:
        return _cfg2()
    if cfg == 3:
        return _cfg3()
    if cfg == 4:
        return _cfg4()
    if cfg == 5:
        return next(mask_sequence_cfg5(1))
    raise ValueError(f"unknown config {cfg}")


def random_mask(H: int, nQ: int, nK: int, density: float, seed: int, keep_diag: bool = False) -> np.ndarray:
    """Plain Bernoulli(density) mask for randomised small test cases."""
    rng = np.random.Generator(np.random.PCG64(seed))
    m = (rng.random((H, nQ, nK)) < density).astype(np.uint8)
    if keep_diag:
        k = min(nQ, nK)
        m[:, np.arange(k), np.arange(k)] = 1
    return m


def imbalance_sweep_mask(rho_target: float, seed: int = 0) -> np.ndarray:
    """A mask of config 3's shape (40 heads, 256 x 256 blocks, mean density 0.3) whose per-head
    densities are spread so that a contiguous row-major split over 256 partitions has an
    imbalance ratio of about rho_target (between 1 and 3): a quarter of the heads get density
    0.3 * rho_target, the others share the rest evenly; inside a head the diagonal is on and the
    other blocks are uniformly random to the head's count.  (Stands in for the synthetic masks of
    the paper's speed-up-against-imbalance experiment, whose recipe the paper does not give.)"""
    c = CONFIGS[3]
    H, n = c["H"], c["nQ"]
    heavy = H // 4
    d_hi = min(0.95, 0.3 * float(rho_target))
    d_lo = max(0.01, (0.3 * H - d_hi * heavy) / (H - heavy))
    ss = np.random.SeedSequence([9100, int(seed), int(round(rho_target * 1000))]).spawn(H + 1)
    order = np.random.Generator(np.random.PCG64(ss[H])).permutation(H)       # which heads are the heavy ones
    mask = np.zeros((H, n, n), dtype=np.uint8)
    for k, h in enumerate(order):
        rng = np.random.Generator(np.random.PCG64(ss[h]))
        m = mask[h]
        m[np.arange(n), np.arange(n)] = 1
        _fill_to_count(m, int(round((d_hi if k < heavy else d_lo) * n * n)), rng)
    return mask


def refine_to_half_blocks(mask: np.ndarray, keep: float, seed: int = 0) -> np.ndarray:
    """A mask at half the block size: every active block becomes 2 x 2 blocks, each kept with
    probability `keep` (independently; a block may lose all four).  Stands in for masks built at
    64-token granularity (the paper's PAROAttention block size) on a workload whose recipe is
    stated at 128: keep = 1 is the same set of token pairs, lower values add fine-grained holes.
    The draw is one PCG64 stream seeded with 7100 + seed."""
    rng = np.random.Generator(np.random.PCG64(7100 + seed))
    fine = np.repeat(np.repeat(np.asarray(mask) != 0, 2, axis=1), 2, axis=2)
    if keep < 1.0:
        fine &= rng.random(fine.shape) < keep
    return fine.astype(np.uint8)
