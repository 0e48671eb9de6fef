"""Oracle: block-masked softmax attention, written out from its definition.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Definition followed: per head, O = P V with P = softmax(Q K^T / sqrt(d)) (Background,
"Visual Generative Models"), where block-wise sparse attention computes only the dense
blocks of a per-head block mask (Background, "Block-wise Sparse Attention"; Motivation:
each head owns one mask).  A skipped block contributes nothing to the softmax, which is
the same as a score of -inf there.

Readings where the paper is silent:
  * mask value 1 = compute the block, 0 = skip it;
  * LSE is the natural-log of the sum of exp(scaled score) over the active keys;
  * a query row whose mask row is all zero gives O = 0 and LSE = -inf;
  * the mask has no batch axis: every batch entry uses the same per-head mask.

Each query block is evaluated against the FULL key axis with inactive columns set to
-inf; nothing here uses compacted index lists, tiles, or running (online) statistics.
Arithmetic is float64 by default (pass dtype=np.float32 for a float32 evaluation).
"""

from __future__ import annotations

import numpy as np


def _row_block(qb, k, v, active_cols, scale, dtype):
    """One query block [b, d] against all keys [Nk, d]; active_cols: bool [Nk]."""
    s = (qb @ k.T) * dtype(scale)                       # scores, [b, Nk]
    s = np.where(active_cols[None, :], s, dtype(-np.inf))
    if not active_cols.any():
        return np.zeros((qb.shape[0], v.shape[1]), dtype=dtype), np.full(qb.shape[0], -np.inf, dtype=dtype)
    m = s.max(axis=1, keepdims=True)
    l = np.exp(s - m).sum(axis=1, keepdims=True)
    lse = m + np.log(l)
    p = np.exp(s - lse)                                 # softmax over active keys; exp(-inf) = 0
    return p @ v, lse[:, 0]


def masked_attention_rows(q, k, v, mask, block, rows, scale=None, dtype=np.float64):
    """Evaluate selected (batch, head, query-block) rows.

    q: [B,H,Nq,d]; k, v: [B,H,Nk,d] (any float dtype; converted to `dtype`);
    mask: [H,nQ,nK] (nonzero = active); rows: iterable of (b, h, I).
    Returns (O [len(rows), block, d], LSE [len(rows), block]) in `dtype`.
    """
    dtype = np.dtype(dtype).type
    B, H, Nq, d = q.shape
    Nk = k.shape[2]
    nQ, nK = Nq // block, Nk // block
    assert Nq == nQ * block and Nk == nK * block, "sequence lengths must be multiples of the block size"
    assert mask.shape == (H, nQ, nK)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    rows = list(rows)
    O = np.empty((len(rows), block, v.shape[-1]), dtype=dtype)
    L = np.empty((len(rows), block), dtype=dtype)
    for t, (b, h, I) in enumerate(rows):
        qb = np.asarray(q[b, h, I * block:(I + 1) * block], dtype=dtype)
        kk = np.asarray(k[b, h], dtype=dtype)
        vv = np.asarray(v[b, h], dtype=dtype)
        active_cols = np.repeat(mask[h, I] != 0, block)
        O[t], L[t] = _row_block(qb, kk, vv, active_cols, scale, dtype)
    return O, L


def masked_attention(q, k, v, mask, block, scale=None, dtype=np.float64):
    """All rows.  Returns (O [B,H,Nq,d], LSE [B,H,Nq]) in `dtype`."""
    B, H, Nq, d = q.shape
    nQ = Nq // block
    rows = [(b, h, I) for b in range(B) for h in range(H) for I in range(nQ)]
    O, L = masked_attention_rows(q, k, v, mask, block, rows, scale=scale, dtype=dtype)
    return O.reshape(B, H, Nq, v.shape[-1]), L.reshape(B, H, Nq)


def merge_partials(O_parts, LSE_parts):
    """Combine attention computed over disjoint key subsets (log-sum-exp identity).

    O_parts: [k, rows, d], LSE_parts: [k, rows].  LSE = log sum_k exp(LSE_k);
    O = sum_k exp(LSE_k - LSE) O_k.  Parts with LSE_k = -inf (empty subset) weigh 0.
    This is the identity Ring Attention uses to combine per-chunk partial attention
    (Background, "Sequence Parallelism").
    """
    O_parts = np.asarray(O_parts, dtype=np.float64)
    LSE_parts = np.asarray(LSE_parts, dtype=np.float64)
    m = LSE_parts.max(axis=0)
    safe_m = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(LSE_parts - safe_m[None])
    tot = w.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(tot > 0, safe_m + np.log(tot), -np.inf)
        wn = np.where(tot[None] > 0, w / tot[None], 0.0)
    O = (wn[:, :, None] * O_parts).sum(axis=0)
    return O, lse
