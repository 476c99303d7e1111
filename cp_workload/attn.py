"""Seeded synthetic attention matrices for the KV annotator: causal, every row sums to one.

Input generation only (no summed-area table, no scoring).  The shape follows what the paper's
annotator looks at (Sec. 4.2.1): a token attends mostly to nearby tokens and to tokens of its own
passage, and to a few "sink" tokens at the start of the prompt, so that some stretches are
self-contextualised and others lean on what precedes them."""
from __future__ import annotations

import numpy as np


def make_attention(n, seed=0xA77E0001, passage_mean=200, tau=24.0, sink=4, ld=None, chunk=512):
    """float32[n][ld] (ld = n rounded up to a multiple of 4 unless given); columns >= n are zero."""
    rng = np.random.default_rng(seed)
    ld = (n + 3) // 4 * 4 if ld is None else ld
    # passages: consecutive tokens share an id; attention inside the own passage gets a bonus
    ids = np.zeros(n, np.int64)
    i, p = 0, 0
    while i < n:
        ln = int(rng.geometric(1.0 / passage_mean))
        ids[i:i + ln] = p
        i += ln
        p += 1
    lean = rng.random(p) < 0.3  # some passages lean on earlier context instead of themselves
    out = np.zeros((n, ld), np.float32)
    cols = np.arange(n)
    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        rows = np.arange(r0, r1)[:, None]
        logit = rng.normal(0.0, 1.0, (r1 - r0, n))
        logit -= np.abs(rows - cols[None, :]) / tau
        same = ids[rows] == ids[None, cols]
        bonus = np.where(lean[ids[rows]], -1.0, 3.0)
        logit += same * bonus
        logit[:, :sink] += 2.0
        logit[cols[None, :] > rows] = -np.inf
        logit -= logit.max(axis=1, keepdims=True)
        e = np.exp(logit)
        out[r0:r1, :n] = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    return out


def make_mask(n, seed=0xA77E0002, run_mean=6.0, cover=0.05):
    """Sensitive runs (geometric length) covering about ``cover`` of the tokens."""
    rng = np.random.default_rng(seed)
    m = np.zeros(n, np.uint8)
    if cover <= 0.0:
        return m
    gap_mean = run_mean * (1.0 - cover) / cover
    i, sens = 0, False
    while i < n:
        ln = int(rng.geometric(1.0 / max(1.0, run_mean if sens else gap_mean)))
        if sens:
            m[i:i + ln] = 1
        i += ln
        sens = not sens
    return m
