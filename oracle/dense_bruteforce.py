"""Textbook dense softmax attention, one query token at a time, float64.

TEST INFRASTRUCTURE ONLY.  Exists to pin `oracle.attention` (all-ones mask) to something
written separately: explicit loops over tokens, the softmax spelled as a ratio of
exponentials, no masking code at all.  O = softmax(Q K^T / sqrt(d)) V per head
(Background, "Visual Generative Models").
"""

from __future__ import annotations

import math

import numpy as np


def dense_attention(q, k, v, scale=None):
    """q [Nq,d], k,v [Nk,d] of one head -> (O [Nq,d], LSE [Nq]) in float64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Nq, d = q.shape
    Nk = k.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    O = np.zeros((Nq, v.shape[1]))
    LSE = np.zeros(Nq)
    for i in range(Nq):
        e = np.empty(Nk)
        for j in range(Nk):
            e[j] = math.exp(scale * float(np.dot(q[i], k[j])))   # inputs are O(1): no overflow
        z = float(e.sum())
        for j in range(Nk):
            O[i] += (e[j] / z) * v[j]
        LSE[i] = math.log(z)
    return O, LSE
