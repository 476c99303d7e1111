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


def brute_candidates(bp, stored_runs, run, W):
    """Hash-free: every candidate of one request run (a position after the run's first token where the
    next W tokens equal the first W tokens of a stored run), and for each the last token up to which
    the request goes on equalling stored text that starts there (token lists compared one by one)."""
    prefixes = [r[:W] for r in stored_runs if len(r) >= W]
    out = []
    for a in range(1, len(run) - W + 1):
        if not any(run[a:a + W] == p for p in prefixes):
            continue
        e = a + W - 1
        while e + 1 < len(run) and bp.find(run[a:e + 2]) is not None:
            e += 1
        out.append((a, e))
    return out


def brute_choice(cands):
    """Which candidates serve, and in which of the two streams: [(first token, last token, stream)].  A piece
    of covered text begins at the first candidate that no chosen text reaches; as long as a candidate that
    starts inside the covered text reaches beyond it, the one that reaches furthest (the earliest such) comes
    next; the chosen candidates of a piece alternate between the streams."""
    chosen, c = [], 0
    while c < len(cands):
        stream = 0
        while True:
            a, e = cands[c]
            chosen.append((a, e, stream))
            further = [d for d in range(c + 1, len(cands)) if cands[d][0] <= e and cands[d][1] > e]
            if not further:
                break
            far = max(cands[d][1] for d in further)
            c = min(d for d in further if cands[d][1] == far)
            stream ^= 1
        end = cands[c][1]
        while c < len(cands) and cands[c][0] <= end:
            c += 1
    for st in (0, 1):  # the texts inside one stream do not overlap
        segs = sorted((a, e) for a, e, s_ in chosen if s_ == st)
        assert all(segs[k][1] < segs[k + 1][0] for k in range(len(segs) - 1))
    return chosen


def brute_floating(bp, stored_runs, tok, mask, off, W):
    """Expected slot of every request token, from the tokens alone: the run-start match first; else the
    chosen candidate (brute_choice) of the first stream whose stored text covers the token, else that of
    the second stream.  Also returns, per token, whether ANY candidate's stored text (or
    the run-start match) covers it, every slot that would be a correct answer for it, and the largest
    number of candidates whose texts overlap at one token."""
    n = len(tok)
    out, covered, allowed, depth = [None] * n, [False] * n, [set() for _ in range(n)], 0
    for _, a0, b0 in runs(tok, mask, off):
        run = [int(t) for t in tok[a0:b0]]
        cands = brute_candidates(bp, stored_runs, run, W)  # (first token, last token) of every candidate's text
        chosen = brute_choice(cands)
        for i in range(len(run)):
            reach = [(a, e) for a, e in cands if a <= i <= e]  # all candidates whose text covers token i
            depth = max(depth, len(reach))
            s = bp.find(run[: i + 1])
            covered[a0 + i] = s is not None or bool(reach)
            allowed[a0 + i] = {x for x in [s] + [bp.find(run[a: i + 1]) for a, _ in reach] if x is not None}
            for st in (0, 1):
                if s is None:
                    seg = [(a, e) for a, e, s_ in chosen if s_ == st and a <= i <= e]
                    if seg:
                        s = bp.find(run[seg[0][0]: i + 1])
            out[a0 + i] = s
    return out, covered, allowed, depth


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
    ix = O.Index()
    O.insert_kv(ix, h_seg, off1, np.arange(40, dtype=np.uint32), _kv(40), L1(40), np.zeros((40, 1, 2, 8), np.uint16), POOL1,
                np.zeros(40, np.int32))
    hf, fo, hl, lo = O.hash_floating(anchors, ix, h, O.run_offsets(m, off), W)
    assert (hf[:13] == O.HASH_NONE).all() and (hl == O.HASH_NONE).all()  # one candidate: nothing for the second stream
    assert np.array_equal(hf[13:53], h_seg)  # from the candidate on: exactly the segment's own keys
    assert (hf[53:] == O.HASH_NONE).all()  # ... as far as the stored text reaches
    assert list(fo[13:16]) == [0, 1, 2] and (fo[53:] == 0xFFFFFFFF).all() and (lo == 0xFFFFFFFF).all()
    # and written out from the definition: h[i] - h[a-1] * B^(i-a+1)
    i, a = 30, 13
    assert int(hf[i]) == (int(h[i]) - int(h[a - 1]) * pow(O.BASE, i - a + 1, 1 << 64)) & M64
    # a window that would leave the run never anchors: cut the request inside the segment's prefix
    m2 = m.copy()
    m2[15] = 1
    hf2, _, hl2, _ = O.hash_floating(anchors, ix, O.hash_segments(req, m2, off), O.run_offsets(m2, off), W)
    assert (hf2 == O.HASH_NONE).all() and (hl2 == O.HASH_NONE).all()


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
    ro = O.run_offsets(mask, off)
    he, _, hl, _ = O.hash_floating(anchors, ix, h, ro, W)
    got = O.probe3(ix, h, he, hl)
    assert np.array_equal(got, O.merge_streams(O.match_streams(ix, tok, h, ro, anchors, W)))
    want, covered, allowed, depth = brute_floating(bp, stored_runs, tok, mask, off, W)
    want = np.array([NONE if s is None else s for s in want], np.uint32)
    # what does not depend on which candidate serves: exactly the tokens that the run-start match or some
    # candidate's stored text covers are served, however many candidates overlap, each from a slot that holds it
    assert np.array_equal(got != NONE, np.array(covered))
    assert all(int(g) in allowed[i] for i, g in enumerate(got) if g != NONE)
    assert np.array_equal(got, want)  # ... and the candidate is the chosen one
    if vocab <= 3 and W <= 3:
        assert depth >= 3  # these cases do have more than two candidates' texts overlapping at a token
    plain = O.probe(ix, h)
    assert ((plain != NONE) <= (got != NONE)).all()  # never fewer matches than run-start anchoring
    assert (got != NONE).sum() > (plain != NONE).sum()  # and here strictly more
    assert (got[mask == 1] == NONE).all()



def _store(ix, anchors, bp, stored_runs, free, used, tok, mask, off, W):
    h = O.hash_segments(tok, mask, off)
    n = len(tok)
    so, n_new, _ = O.insert_kv(ix, h, off, free[used:], _kv(n), L1(n), np.zeros((len(free), 1, 2, 8), np.uint16), POOL1,
                               np.zeros(len(free), np.int32))
    O.insert_anchors(anchors, h, O.run_offsets(mask, off), so, W)
    bp.insert(tok, mask, off)
    stored_runs += [[int(t) for t in tok[a:b]] for _, a, b in runs(tok, mask, off)]
    return used + n_new


def _lookup(ix, anchors, tok, mask, off, W):
    h = O.hash_segments(tok, mask, off)
    ro = O.run_offsets(mask, off)
    return O.merge_streams(O.match_streams(ix, tok, h, ro, anchors, W))


def test_an_earlier_candidate_is_not_lost_when_a_later_window_hits():
    """Two stored texts, one contained in the other ('abcdefgh' and 'defg'): every token of the longer one
    is served although a second candidate starts inside it; and two stored texts that overlap in the request
    ('XY' and 'YZ' against 'XYZ'): the part only the second one covers is served from the second."""
    W = 2
    free = np.arange(200, dtype=np.uint32)
    ix, anchors, bp, stored = O.Index(), O.AnchorSet(), BrutePool(free), []
    long_text = np.arange(100, 108, dtype=np.uint32)  # a b c d e f g h
    short = long_text[3:7]  # d e f g
    used = 0
    for t in (long_text, short):
        used = _store(ix, anchors, bp, stored, free, used, t, np.zeros(len(t), np.uint8), np.array([0, len(t)], np.uint32), W)
    req = np.concatenate([[7, 8], long_text, [9]]).astype(np.uint32)
    mask, off = np.zeros(len(req), np.uint8), np.array([0, len(req)], np.uint32)
    got = _lookup(ix, anchors, req, mask, off, W)
    want, covered, allowed, depth = brute_floating(bp, stored, req, mask, off, W)
    assert list(got) == [NONE if s is None else s for s in want]
    assert (got[2:10] != NONE).all() and got[10] == NONE and depth == 2  # 'h' included
    assert list(got[2:10]) == list(range(8))  # the longer text's own slots, in order
    # overlap: X Y stored, Y Z stored, request .. X Y Z ..
    ix, anchors, bp, stored = O.Index(), O.AnchorSet(), BrutePool(free), []
    X, Y, Z = np.arange(10, 14), np.arange(20, 25), np.arange(30, 33)
    used = 0
    for t in (np.concatenate([X, Y]), np.concatenate([Y, Z])):
        t = t.astype(np.uint32)
        used = _store(ix, anchors, bp, stored, free, used, t, np.zeros(len(t), np.uint8), np.array([0, len(t)], np.uint32), W)
    req = np.concatenate([[1], X, Y, Z, [2]]).astype(np.uint32)
    mask, off = np.zeros(len(req), np.uint8), np.array([0, len(req)], np.uint32)
    got = _lookup(ix, anchors, req, mask, off, W)
    want, covered, allowed, depth = brute_floating(bp, stored, req, mask, off, W)
    assert list(got) == [NONE if s is None else s for s in want] and depth == 2
    assert list(got[1:10]) == list(range(9))  # X Y from the first stored text
    assert list(got[10:13]) == [14, 15, 16]  # Z from the second, whose Y is a duplicate (slots 9..13 hold it)
    assert got[0] == NONE and got[13] == NONE


def test_window_of_one_token_loses_nothing_against_a_longer_window():
    """W = 1 makes every token that equals a stored run's first token a candidate; chance candidates inside
    or before a true one must not displace it."""
    rng = np.random.default_rng(11)
    free = rng.permutation(4000).astype(np.uint32)
    docs = [rng.integers(0, 50, int(n)).astype(np.uint32) for n in rng.integers(30, 60, 12)]  # small vocabulary: many chance hits
    served = {}
    for W in (1, 3):
        ix, anchors, bp, stored = O.Index(), O.AnchorSet(), BrutePool(free), []
        used = 0
        for d in docs:
            used = _store(ix, anchors, bp, stored, free, used, d, np.zeros(len(d), np.uint8), np.array([0, len(d)], np.uint32), W)
        r2 = np.random.default_rng(5)
        req = np.concatenate([np.concatenate([r2.integers(50, 99, int(r2.integers(3, 9))).astype(np.uint32), docs[k]])
                              for k in (3, 7, 1, 7)])
        mask, off = np.zeros(len(req), np.uint8), np.array([0, len(req)], np.uint32)
        got = _lookup(ix, anchors, req, mask, off, W)
        want, covered, allowed, depth = brute_floating(bp, stored, req, mask, off, W)
        assert list(got) == [NONE if s is None else s for s in want]
        assert np.array_equal(got != NONE, np.array(covered))
        served[W] = got != NONE
    assert (served[3] <= served[1]).all() and served[3].sum() >= sum(len(docs[k]) for k in (3, 7, 1, 7)) - 4 * 2
