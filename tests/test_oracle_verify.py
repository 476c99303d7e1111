"""Pins for exact verification (Sec. 4.2.2 Step 2: a hash match is a candidate that must be confirmed so
that no collision of the rolling hash produces a false match).

Ground truth is kept by the test itself, without any hash: the token string every slot was filled for.
A crafted collision of the mod-2^64 polynomial hash (two different 1024-token strings over two symbols
with the same hash for ANY odd base: the Thue-Morse construction) shows that the unverified lookup does
return a wrong slot and that the verified one does not."""
import numpy as np
import pytest

import oracle as O
from tests.bruteforce import BrutePool, runs

NONE = O.SLOT_NONE
X = 0xFFFFFFFF


def _kv(n):
    return np.zeros((1, 2, n, 8), np.uint16)


L1 = lambda n: O.Layout(1, 1, 8, 16, 2 * n * 16, n * 16)  # noqa: E731
POOL1 = O.Layout(1, 1, 8, 32, 32, 16)


def thue_morse_pair(k, x, y):
    """t and its complement, length 2^k, over the symbols x and y."""
    bits = [0]
    for _ in range(k):
        bits = bits + [1 - b for b in bits]
    t = np.array([x if b == 0 else y for b in bits], np.uint32)
    c = np.array([y if b == 0 else x for b in bits], np.uint32)
    return t, c


class Truth:
    """Pool driven through the oracle's insert, with the test's own record of what every slot holds."""

    def __init__(self, n_slots, seed=0, verified=True):
        rng = np.random.default_rng(seed)
        self.free = rng.permutation(n_slots).astype(np.uint32)
        self.ix = O.Index()
        self.text = O.Text(n_slots) if verified else None
        self.pool = np.zeros((n_slots, 1, 2, 8), np.uint16)
        self.slot_pos = np.zeros(n_slots, np.int32)
        self.used = 0
        self.truth = {}  # slot -> tuple of tokens (the run from its start through the storing token)

    def insert(self, tok, mask, off):
        h = O.hash_segments(tok, mask, off)
        ro = O.run_offsets(mask, off)
        before = self.used
        slot_out, n_new, _ = O.insert_kv(self.ix, h, off, self.free[self.used:], _kv(len(tok)), L1(len(tok)), self.pool,
                                         POOL1, self.slot_pos)
        self.used += n_new
        fresh = set(int(s) for s in self.free[before:self.used])
        for i in range(len(tok)):
            s = int(slot_out[i])
            if s in fresh and s not in self.truth:  # the first token that names a fresh slot filled it
                self.truth[s] = tuple(int(t) for t in tok[i - int(ro[i]): i + 1])
        if self.text is not None:
            slot_out = O.text_record(self.text, tok, ro, slot_out)
        return slot_out

    def lookup(self, tok, mask, off, verified=True):
        h = O.hash_segments(tok, mask, off)
        cand = O.probe(self.ix, h)
        if not verified:
            return cand
        return O.verify(self.text, tok, O.run_offsets(mask, off), cand)

    def unsound(self, tok, mask, off, slots):
        """Tokens served from a slot that was filled for a different text."""
        ro = O.run_offsets(mask, off)
        bad = []
        for i in np.flatnonzero(slots != NONE):
            want = tuple(int(t) for t in tok[i - int(ro[i]): i + 1])
            if self.truth.get(int(slots[i])) != want:
                bad.append(int(i))
        return bad


def test_thue_morse_strings_collide_for_this_hash():
    t, c = thue_morse_pair(10, 7, 11)
    assert len(t) == 1024 and (t != c).all()
    z, off = np.zeros(1024, np.uint8), np.array([0, 1024], np.uint32)
    ht, hc = O.hash_segments(t, z, off), O.hash_segments(c, z, off)
    assert ht[-1] == hc[-1]
    assert (ht[:-1] != hc[:-1]).all()  # only the full strings collide
    # the same from the definition, with Python integers
    B, M = O.BASE, 1 << 64
    assert sum((int(a) - int(b)) * pow(B, 1023 - j, M) for j, (a, b) in enumerate(zip(t, c))) % M == 0


def test_lookup_collision_is_rejected_only_with_verification():
    t, c = thue_morse_pair(10, 7, 11)
    tail = np.array([5, 6, 7], np.uint32)
    P = Truth(4096)
    donor = np.concatenate([t, tail])
    m, off = np.zeros(len(donor), np.uint8), np.array([0, len(donor)], np.uint32)
    so = P.insert(donor, m, off)
    assert (so != NONE).all() and P.used == len(donor)
    req = np.concatenate([c, tail])  # another text with the same hashes from token 1023 on
    plain = P.lookup(req, m, off, verified=False)
    assert (plain[:1023] == NONE).all() and (plain[1023:] != NONE).all()
    assert P.unsound(req, m, off, plain) == [1023, 1024, 1025, 1026]  # false matches without verification
    ver = P.lookup(req, m, off)
    assert (ver == NONE).all()
    # the stored text itself is still found, whole
    assert np.array_equal(P.lookup(donor, m, off), so)


def test_insert_collision_leaves_no_wrong_chain():
    t, c = thue_morse_pair(10, 7, 11)
    P = Truth(8192)
    a = np.concatenate([t, [5]]).astype(np.uint32)
    b = np.concatenate([c, [5, 9]]).astype(np.uint32)
    za, offa = np.zeros(len(a), np.uint8), np.array([0, len(a)], np.uint32)
    zb, offb = np.zeros(len(b), np.uint8), np.array([0, len(b)], np.uint32)
    sa = P.insert(a, za, offa)
    sb = P.insert(b, zb, offb)
    # b: tokens 0..1022 are new and stored; 1023 (same key as a's) and 1024 find a's entries: not b's text;
    # 1025 has a new key and takes a slot, but behind an unverified prefix: that slot must never match
    assert (sb[:1023] != NONE).all() and (sb[1023:] == NONE).all()
    assert P.used == len(a) + 1023 + 1
    la, lb = P.lookup(a, za, offa), P.lookup(b, zb, offb)
    assert np.array_equal(la, sa)
    assert np.array_equal(lb, sb)
    assert P.unsound(a, za, offa, la) == [] and P.unsound(b, zb, offb, lb) == []
    # the text whose hashes equal those of b's stored chain but which runs through a's slots: c..., then
    # "t + [5, 9]" has the key of b's token 1025 -> candidate is the slot filled for b's text: rejected
    q = np.concatenate([t, [5, 9]]).astype(np.uint32)
    lq = P.lookup(q, zb, offb)
    assert np.array_equal(lq[:1025], sa) and lq[1025] == NONE
    plain = P.lookup(q, zb, offb, verified=False)
    assert plain[1025] != NONE and P.unsound(q, zb, offb, plain) == [1025]


@pytest.mark.parametrize("seed,vocab", [(0, 2), (1, 3), (2, 32000)])
def test_without_collisions_verification_changes_nothing(seed, vocab):
    rng = np.random.default_rng(seed)
    P = Truth(4000, seed)
    bp = BrutePool(P.free)
    for _ in range(3):
        tok = rng.integers(0, vocab, 120).astype(np.uint32)
        mask = (rng.random(120) < 0.15).astype(np.uint8)
        off = np.array([0, 40, 40, 120], np.uint32)
        so = P.insert(tok, mask, off)
        want = np.array([NONE if s is None else s for s in bp.insert(tok, mask, off)], np.uint32)
        assert np.array_equal(so, want)
    tok = rng.integers(0, vocab, 200).astype(np.uint32)
    mask = (rng.random(200) < 0.1).astype(np.uint8)
    off = np.array([0, 100, 200], np.uint32)
    want = np.array([NONE if s is None else s for s in bp.probe(tok, mask, off)], np.uint32)
    assert np.array_equal(P.lookup(tok, mask, off), want)
    assert np.array_equal(P.lookup(tok, mask, off, verified=False), want)
    if vocab < 10:
        assert (want != NONE).sum() > 20
    assert P.unsound(tok, mask, off, want) == []


def test_verify_extends_from_segment_start_and_stops_at_first_failure():
    # hand-made candidates, no hashing at all: text store filled through text_record
    text = O.Text(16)
    tok = np.array([1, 2, 3, 4, 9, 1, 2], np.uint32)
    ro = np.array([0, 1, 2, 3, X, 0, 1], np.uint32)
    so = np.array([10, 11, 12, 13, NONE, 10, 11], np.uint32)  # the second run repeats the first's start
    assert np.array_equal(O.text_record(text, tok, ro, so), so)
    q = np.array([1, 2, 7, 4, 1, 2, 3], np.uint32)
    seg = np.array([0, 1, 2, 3, 0, 1, 2], np.uint32)
    cand = np.array([10, 11, 12, 13, 10, 11, 12], np.uint32)
    # token 2 differs (7 != 3): it and everything after it in that segment fail, also token 3 whose slot 13
    # holds "1 2 3 4", not "1 2 7 4"; the second segment is accepted whole
    assert list(O.verify(text, q, seg, cand)) == [10, 11, NONE, NONE, 10, 11, 12]
    # a candidate of the wrong length fails even when its last token is right: slot 12 holds three tokens
    assert list(O.verify(text, np.array([3], np.uint32), np.array([0], np.uint32), np.array([12], np.uint32))) == [NONE]
    # segment offsets that claim a longer history than the slot has
    assert list(O.verify(text, q[4:], np.array([X, 0, 1], np.uint32), np.array([10, 11, 12], np.uint32))) == [NONE] * 3
    # merge: fills only where the first stream found nothing
    first = np.array([NONE, 5, NONE], np.uint32)
    got = O.verify(text, q[4:], np.array([0, 1, 2], np.uint32), np.array([10, 11, 12], np.uint32), merge_into=first)
    assert list(got) == [10, 5, 12]


def test_floating_segments_are_verified_from_their_anchor():
    rng = np.random.default_rng(5)
    W = 4
    P = Truth(1024, 5)
    anchors = O.AnchorSet()
    seg = rng.integers(0, 32000, 30).astype(np.uint32)
    z, off = np.zeros(30, np.uint8), np.array([0, 30], np.uint32)
    so = P.insert(seg, z, off)
    O.insert_anchors(anchors, O.hash_segments(seg, z, off), O.run_offsets(z, off), so, W)
    req = np.concatenate([rng.integers(0, 32000, 7).astype(np.uint32), seg[:20], [123456], seg[21:]]).astype(np.uint32)
    m, roff = np.zeros(len(req), np.uint8), np.array([0, len(req)], np.uint32)
    h = O.hash_segments(req, m, roff)
    ro = O.run_offsets(m, roff)
    hf, fo, hl, lo = O.hash_floating(anchors, P.ix, h, ro, W)
    # the stored text reaches 20 tokens from the candidate; it is the only candidate, so the second stream is empty
    assert list(fo[:7]) == [X] * 7 and list(fo[7:27]) == list(range(20)) and list(fo[27:]) == [X] * (len(req) - 27)
    assert list(lo) == [X] * len(req) and (hl == O.HASH_NONE).all()
    a = O.verify(P.text, req, ro, O.probe(P.ix, h))
    assert (a == NONE).all()  # nothing matches from the run start
    b = O.verify(P.text, req, fo, O.probe(P.ix, hf), merge_into=a)
    assert np.array_equal(b[7:27], so[:20]) and (b[27:] == NONE).all() and (b[:7] == NONE).all()
    assert np.array_equal(O.verify(P.text, req, lo, O.probe(P.ix, hl), merge_into=b), b)
    streams = O.match_streams(P.ix, req, h, ro, anchors, W, P.text)
    assert np.array_equal(O.merge_streams(streams), b)
