"""Pins for the floating-anchor lookup (Sec. 4.2.2 Step 1: a window slides over the request and is
compared with the stored segments' prefix hashes; Step 2: O(1) substring hash from prefix hashes and
powers).  A hash-free brute-force model (token-by-token comparison) says which tokens must be served
from which slot."""
import numpy as np
import pytest

import oracle as O
from tests.bruteforce import BrutePool, runs

NONE = O.SLOT_NONE
M64 = (1 << 64) - 1


def _kv(n):
    return np.zeros((1, 2, n, 8), np.uint16)


L1 = lambda n: O.Layout(1, 1, 8, 16, 2 * n * 16, n * 16)  # noqa: E731
POOL1 = O.Layout(1, 1, 8, 32, 32, 16)


def _prompts(rng, R, T, vocab, p_sens):
    tok = rng.integers(0, vocab, R * T).astype(np.uint32)
    mask = (rng.random(R * T) < p_sens).astype(np.uint8)
    off = (np.arange(R + 1) * T).astype(np.uint32)
    return tok, mask, off


def brute_floating(bp, stored_runs, tok, mask, off, W):
    """Expected slot of every request token: run-start match first, else match from the latest
    floating anchor (a position after the run start where W tokens inside the run equal the first W
    tokens of a stored run of at least W tokens)."""
    prefixes = [r[:W] for r in stored_runs if len(r) >= W]
    out = [None] * len(tok)
    for _, a0, b0 in runs(tok, mask, off):
        run = [int(t) for t in tok[a0:b0]]
        anchors = [a for a in range(1, len(run) - W + 1) if any(run[a:a + W] == p for p in prefixes)]
        for i in range(len(run)):
            s = bp.find(run[: i + 1])
            if s is None:
                cand = [a for a in anchors if a <= i]
                if cand:
                    s = bp.find(run[cand[-1]: i + 1])
            out[a0 + i] = s
    return out


def test_run_offsets():
    mask = np.array([0, 0, 1, 0, 1, 1, 0, 0, 0], np.uint8)
    off = np.array([0, 4, 9], np.uint32)
    X = 0xFFFFFFFF
    assert list(O.run_offsets(mask, off)) == [0, 1, X, 0, X, X, 0, 1, 2]
    assert list(O.run_offsets(np.zeros(5, np.uint8), np.array([0, 2, 2, 5], np.uint32))) == [0, 1, 0, 1, 2]


def test_substring_key_equals_chain_hash_of_the_substring():
    """The key computed from an anchor is the plain chain hash the same tokens get as a run of their own."""
    rng = np.random.default_rng(0)
    W = 4
    seg = rng.integers(0, 32000, 40).astype(np.uint32)
    off1 = np.array([0, 40], np.uint32)
    h_seg = O.hash_segments(seg, np.zeros(40, np.uint8), off1)
    anchors = O.AnchorSet()
    O.insert_anchors(anchors, h_seg, O.run_offsets(np.zeros(40, np.uint8), off1), np.arange(40, dtype=np.uint32), W)
    assert len(anchors) == 1
    req = np.concatenate([rng.integers(0, 32000, 13).astype(np.uint32), seg, rng.integers(0, 32000, 5).astype(np.uint32)])
    m = np.zeros(len(req), np.uint8)
    off = np.array([0, len(req)], np.uint32)
    h = O.hash_segments(req, m, off)
    hf = O.hash_floating(anchors, h, O.run_offsets(m, off), W)
    assert (hf[:13] == O.HASH_NONE).all()  # no anchor before the segment starts
    assert np.array_equal(hf[13:53], h_seg)  # from the anchor on: exactly the segment's own keys
    # and written out from the definition: h[i] - h[a-1] * B^(i-a+1)
    i, a = 30, 13
    assert int(hf[i]) == (int(h[i]) - int(h[a - 1]) * pow(O.BASE, i - a + 1, 1 << 64)) & M64
    # a window that would leave the run never anchors: cut the request inside the segment's prefix
    m2 = m.copy()
    m2[15] = 1
    hf2 = O.hash_floating(anchors, O.hash_segments(req, m2, off), O.run_offsets(m2, off), W)
    assert (hf2 == O.HASH_NONE).all()


@pytest.mark.parametrize("seed,vocab,W", [(0, 2, 3), (1, 3, 2), (2, 3, 4), (3, 32000, 3), (4, 2, 1)])
def test_floating_lookup_against_brute_force(seed, vocab, W):
    rng = np.random.default_rng(seed)
    free = rng.permutation(3000).astype(np.uint32)
    ix, anchors, bp = O.Index(), O.AnchorSet(), BrutePool(free)
    pool = np.zeros((3000, 1, 2, 8), np.uint16)
    slot_pos = np.zeros(3000, np.int32)
    stored_runs = []
    used = 0
    for call in range(2):
        tok, mask, off = _prompts(rng, 3, 30, vocab, 0.15)
        if vocab == 32000:  # make donors and requests share material
            base_text = rng.integers(0, vocab, 60).astype(np.uint32)
            tok[10:50] = base_text[:40]
        h = O.hash_segments(tok, mask, off)
        ro = O.run_offsets(mask, off)
        so, n_new, _ = O.insert_kv(ix, h, off, free[used:], _kv(len(tok)), L1(len(tok)), pool, POOL1, slot_pos)
        used += n_new
        O.insert_anchors(anchors, h, ro, so, W)
        bp.insert(tok, mask, off)
        stored_runs += [[int(t) for t in tok[a:b]] for _, a, b in runs(tok, mask, off)]
        if vocab == 32000:
            keep = base_text
    tok, mask, off = _prompts(rng, 4, 40, vocab, 0.15)
    if vocab == 32000:
        tok[5:45] = keep[3:43]  # the shared text, but entered 3 tokens late: only a floating anchor can match it
    h = O.hash_segments(tok, mask, off)
    hf = O.hash_floating(anchors, h, O.run_offsets(mask, off), W)
    got = O.probe2(ix, h, hf)
    want = brute_floating(bp, stored_runs, tok, mask, off, W)
    want = np.array([NONE if s is None else s for s in want], np.uint32)
    assert np.array_equal(got, want)
    plain = O.probe(ix, h)
    assert ((plain != NONE) <= (got != NONE)).all()  # never fewer matches than run-start anchoring
    assert (got != NONE).sum() > (plain != NONE).sum()  # and here strictly more
    assert (got[mask == 1] == NONE).all()
