"""Pins for the pool policies: minimum segment length and recompute marks (Sec. 4.2.1 "Optimization" and
Step 3), zero placeholders (Sec. 4.3.1 "Operational details") and least-recently-used eviction
(Sec. 4.3.5 "Lifecycle management").  Expected values come from hand examples and from independent
pure-Python models that use no hashing."""
from itertools import groupby

import numpy as np
import pytest

import oracle as O
from tests.bruteforce import runs

NONE = O.SLOT_NONE
X = NONE


def py_filter(slot, off, min_len, marks=None):
    """groupby formulation: stretches of matched tokens per request."""
    out = []
    for r in range(len(off) - 1):
        seg = [int(s) for s in slot[off[r]:off[r + 1]]]
        for matched, grp in groupby(seg, key=lambda s: s != NONE):
            grp = list(grp)
            if not matched or len(grp) < min_len:
                out += [NONE] * len(grp)
            else:
                out += [NONE if (marks is not None and marks[s]) else s for s in grp]
    return np.array(out, np.uint32)


def test_filter_hand_example():
    #            request 0                      | request 1
    slot = np.array([5, 6, X, 7, 8, 9, X, 1, 2, 3, 4, X, 2], np.uint32)
    off = np.array([0, 9, 13], np.uint32)
    # stretches: [5 6] [7 8 9] [1 2] | [3 4] [2]; the stretch "1 2 | 3 4" is cut by the request boundary
    assert list(O.filter_matches(slot, off, 3)) == [X, X, X, 7, 8, 9, X, X, X, X, X, X, X]
    assert list(O.filter_matches(slot, off, 2)) == [5, 6, X, 7, 8, 9, X, 1, 2, 3, 4, X, X]
    assert list(O.filter_matches(slot, off, 1)) == list(slot)
    assert list(O.filter_matches(slot, off, 0)) == list(slot)
    marks = np.zeros(10, np.uint8)
    marks[[8, 2]] = 1
    # a marked token still counts towards the length of its stretch, and is then dropped alone
    assert list(O.filter_matches(slot, off, 3, marks)) == [X, X, X, 7, X, 9, X, X, X, X, X, X, X]
    assert list(O.filter_matches(slot, off, 1, marks)) == [5, 6, X, 7, X, 9, X, 1, X, 3, 4, X, X]


@pytest.mark.parametrize("seed", range(4))
def test_filter_against_groupby_model(seed):
    rng = np.random.default_rng(seed)
    N = 500
    slot = rng.integers(0, 64, N).astype(np.uint32)
    slot[rng.random(N) < 0.2] = NONE
    cuts = np.sort(rng.choice(np.arange(1, N), 6, replace=False))
    off = np.concatenate([[0], cuts[:3], cuts[2:3], cuts[3:], [N]]).astype(np.uint32)  # one empty request
    marks = (rng.random(64) < 0.25).astype(np.uint8)
    for min_len in (1, 2, 5, 9, 1000):
        assert np.array_equal(O.filter_matches(slot, off, min_len), py_filter(slot, off, min_len))
        assert np.array_equal(O.filter_matches(slot, off, min_len, marks), py_filter(slot, off, min_len, marks))
    assert (O.filter_matches(slot, off, 1000) == NONE).all()


def test_marks_accumulate_and_ignore_tokens_without_slot():
    marks = np.zeros(8, np.uint8)
    O.mark_recompute(np.array([1, 2, X, 3, 99], np.uint32), np.array([1, 0, 1, 1, 1], np.uint8), marks)
    assert list(marks) == [0, 1, 0, 1, 0, 0, 0, 0]
    O.mark_recompute(np.array([1, 2], np.uint32), np.array([0, 1], np.uint8), marks)  # a later batch adds, never clears
    assert list(marks) == [0, 1, 1, 1, 0, 0, 0, 0]


def test_zero_placeholders():
    L, n, re = 2, 5, 8
    lay = O.Layout(L, 1, re, re * 2, 2 * n * re * 2, n * re * 2)
    dst = np.full((L, 2, n, re), 0xC0DE, np.uint16)
    O.fill_unmatched(np.array([3, X, X, 0, X], np.uint32), dst, lay)
    for t in range(n):
        assert (dst[:, :, t] == (0 if t in (1, 2, 4) else 0xC0DE)).all()


def py_threshold(stamps, now, needed, max_age):
    """Cohorts of equal (clipped) age, oldest first, until enough."""
    if needed == 0:
        return 0
    ages = {}
    for st in stamps:
        if st and st <= now:
            ages.setdefault(min(now - int(st), max_age - 1), []).append(st)
    total = 0
    for a in sorted(ages, reverse=True):
        total += len(ages[a])
        if total >= needed:
            return now - a + 1
    return now + 1


@pytest.mark.parametrize("seed", range(3))
def test_lru_threshold_against_cohort_model(seed):
    rng = np.random.default_rng(seed)
    now = 50
    stamps = rng.integers(0, now + 1, 300).astype(np.uint32)  # 0 = free
    for max_age in (4096, 16, 2):
        for needed in (0, 1, 5, 40, 150, 299, 10000):
            T = O.lru_threshold(stamps, now, needed, max_age)
            assert T == py_threshold(stamps, now, needed, max_age), (max_age, needed)
            n = int(((stamps != 0) & (stamps < T)).sum())
            if needed and T <= now:
                assert n >= needed
                # one cohort less would not be enough (or there is no younger boundary inside the window)
                if now - T + 2 <= max_age - 1:
                    assert int(((stamps != 0) & (stamps < T - 1)).sum()) < needed or T - 1 < 1
    assert O.lru_threshold(np.zeros(10, np.uint32), 5, 3) == 6  # nothing in use: "everything", which is nothing


def test_touch_only_raises():
    st = np.array([0, 3, 9, 0], np.uint32)
    O.touch(np.array([1, 2, 3, X, 77], np.uint32), 5, st)
    assert list(st) == [0, 5, 9, 5]


class PyLruPool:
    """Hash-free model: stored text (tuple of a run's tokens up to the token) -> slot, batch stamps."""

    def __init__(self, free):
        self.free = [int(s) for s in free]
        self.stored = {}
        self.stamp = {}

    def lookup(self, tok, mask, off, epoch):
        out = [NONE] * len(tok)
        for _, a, b in runs(tok, mask, off):
            for i in range(a, b):
                s = self.stored.get(tuple(int(t) for t in tok[a:i + 1]))
                if s is not None:
                    out[i] = s
                    self.stamp[s] = max(self.stamp[s], epoch)
        return out

    def insert(self, tok, mask, off, epoch):
        out = [NONE] * len(tok)
        for _, a, b in runs(tok, mask, off):
            for i in range(a, b):
                key = tuple(int(t) for t in tok[a:i + 1])
                s = self.stored.get(key)
                if s is None and self.free:
                    s = self.free.pop(0)
                    self.stored[key] = s
                    self.stamp[s] = 0
                if s is not None:
                    out[i] = s
                    self.stamp[s] = max(self.stamp[s], epoch)
        return out

    def evict(self, now, needed, max_age):
        T = py_threshold(list(self.stamp.values()), now, needed, max_age)
        gone = sorted(s for s, st in self.stamp.items() if st < T)
        self.stored = {k: s for k, s in self.stored.items() if self.stamp[s] >= T}
        for s in gone:
            del self.stamp[s]
        self.free += gone
        return gone


@pytest.mark.parametrize("seed,vocab", [(0, 3), (1, 4), (2, 32000)])
def test_lru_pool_lifecycle_against_hash_free_model(seed, vocab):
    rng = np.random.default_rng(seed)
    S = 160
    free = rng.permutation(S).astype(np.uint32)
    ix, model = O.Index(), PyLruPool(free)
    stamps = np.zeros(S, np.uint32)
    pool = np.zeros((S, 1, 2, 8), np.uint16)
    slot_pos = np.zeros(S, np.int32)
    free_list = free.copy()
    corpus = [rng.integers(0, vocab, 30).astype(np.uint32) for _ in range(6)]
    evictions = 0
    for epoch in range(1, 25):
        parts = [corpus[int(d)][: int(rng.integers(5, 31))] for d in rng.choice(6, 2, replace=False)]
        tok = np.concatenate(parts).astype(np.uint32)
        mask = (rng.random(len(tok)) < 0.1).astype(np.uint8)
        off = np.array([0, len(parts[0]), len(tok)], np.uint32)
        h = O.hash_segments(tok, mask, off)
        got = O.probe(ix, h)
        O.touch(got, epoch, stamps)
        assert list(got) == model.lookup(tok, mask, off, epoch)
        n_new_keys = len({int(x) for x, g in zip(h, got) if g == NONE and x != O.HASH_NONE})
        if n_new_keys > len(free_list):  # make room: least recently used first
            T = O.lru_threshold(stamps, epoch, n_new_keys - len(free_list), 8)
            freed = O.evict(ix, stamps, T)
            assert list(freed) == model.evict(epoch, n_new_keys - len(model.free), 8)
            free_list = np.concatenate([free_list, freed])
            evictions += 1
        kv = np.zeros((1, 2, len(tok), 8), np.uint16)
        lay = O.Layout(1, 1, 8, 16, 2 * len(tok) * 16, len(tok) * 16)
        so, n_new, fl = O.insert_kv(ix, h, off, free_list, kv, lay, pool, O.Layout(1, 1, 8, 32, 32, 16), slot_pos)
        free_list = free_list[n_new:]
        O.touch(so, epoch, stamps)
        assert list(so) == model.insert(tok, mask, off, epoch)
        assert len(free_list) == len(model.free) and sorted(model.stamp) == sorted(np.flatnonzero(stamps).tolist())
        # what is stored stays closed under "drop the last token": an ancestor is never older than its descendants
        for key, s in model.stored.items():
            if len(key) > 1:
                assert key[:-1] in model.stored and model.stamp[model.stored[key[:-1]]] >= model.stamp[s]
    assert evictions >= 2


@pytest.mark.parametrize("seed", range(12))
def test_two_key_streams_keep_stored_runs_prefix_closed_under_lru(seed):
    """With floating anchors a token can be served from the run-start stream while the floating stream,
    which serves a later token, also walked through that position.  Both streams' accepted slots must be
    stamped: then no stored text is ever newer than the text one token shorter, so evicting by age never
    takes the head of a run whose tail stays (which exact verification would then refuse to follow)."""
    rng = np.random.default_rng(40 + seed)
    vocab, W, S = 4, int(rng.integers(1, 6)), 200
    free = rng.permutation(S).astype(np.uint32)
    ix, text, anchors = O.Index(), O.Text(S), O.AnchorSet()
    stamps = np.zeros(S, np.uint32)
    pool, slot_pos = np.zeros((S, 1, 2, 8), np.uint16), np.zeros(S, np.int32)
    corpus = [rng.integers(0, vocab, 50).astype(np.uint32) for _ in range(5)]
    live = {}  # stored text -> slot, kept by the test

    def closed():
        return all(t[:-1] in live and stamps[live[t[:-1]]] >= stamps[s] for t, s in live.items() if len(t) > 1)

    for epoch in range(1, 16):
        parts = []
        for d in rng.choice(5, int(rng.integers(1, 4)), replace=False):
            lead = rng.integers(0, vocab, int(rng.integers(0, 5))).astype(np.uint32)
            a = int(rng.integers(0, 20))
            parts.append(np.concatenate([lead, corpus[d][a:a + int(rng.integers(1, 31))]]))
        tok = np.concatenate(parts).astype(np.uint32)
        mask = (rng.random(len(tok)) < 0.05).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum([len(x) for x in parts])]).astype(np.uint32)
        h, ro = O.hash_segments(tok, mask, off), O.run_offsets(mask, off)
        plain = O.probe(ix, h)
        for own in O.match_streams(ix, tok, h, ro, anchors, W, text):  # what every key stream accepted counts as used
            O.touch(own, epoch, stamps)
        assert closed(), ("lookup", epoch)
        new_keys = len({int(x) for x, g in zip(h, plain) if g == NONE and x != O.HASH_NONE})
        if new_keys > len(free):
            freed = O.evict(ix, stamps, O.lru_threshold(stamps, epoch, new_keys - len(free)), text, anchors=anchors)
            gone = set(freed.tolist())
            live = {t: s for t, s in live.items() if s not in gone}
            free = np.concatenate([free, freed])
            assert closed(), ("eviction", epoch)
            assert len(anchors) == sum(1 for t in live if len(t) == W)  # prefix hashes go with their runs
        kv = np.zeros((1, 2, len(tok), 8), np.uint16)
        lay = O.Layout(1, 1, 8, 16, 2 * len(tok) * 16, len(tok) * 16)
        so, n_new, _ = O.insert_kv(ix, h, off, free, kv, lay, pool, O.Layout(1, 1, 8, 32, 32, 16), slot_pos)
        fresh, free = set(free[:n_new].tolist()), free[n_new:]
        so = O.text_record(text, tok, ro, so)
        O.insert_anchors(anchors, h, ro, so, W)
        for _, a, b in runs(tok, mask, off):
            for i in range(a, b):
                if so[i] != NONE and int(so[i]) in fresh:
                    live[tuple(int(t) for t in tok[a:i + 1])] = int(so[i])
        O.touch(so, epoch, stamps)
        assert closed(), ("insert", epoch)
        assert len(anchors) == sum(1 for t in live if len(t) == W)  # one prefix hash per stored run of >= W tokens
        # everything the batch just stored or found is found again, whole
        again = O.verify(text, tok, ro, O.probe(ix, h))
        assert np.array_equal(again != NONE, so != NONE), epoch
