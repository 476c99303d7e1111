"""Pins for storing a text once (Sec. 4.3.5 "Lifecycle management": of duplicated segments, and of a
segment contained in another, one copy is kept).  A hash-free model over explicit token lists says which
tokens of a batch the pool already holds, which are stored, and as the continuation of which stored text."""
import numpy as np
import pytest

import oracle as O
from tests.bruteforce import BrutePool, runs
from tests.test_oracle_floating import brute_candidates, brute_choice

NONE = O.SLOT_NONE
L1 = lambda n: O.Layout(1, 1, 8, 16, 2 * n * 16, n * 16)  # noqa: E731
POOL1 = O.Layout(1, 1, 8, 32, 32, 16)


class TextPool(BrutePool):
    """BrutePool whose insert keeps one copy: texts are token tuples, compared element by element."""

    def __init__(self, free_slots, W):
        super().__init__(free_slots)
        self.W = W
        self.stored_runs = []  # every stored text that was a run's beginning when stored: the candidates' prefixes

    def serving(self, run, i, chosen):
        """(slot, start of the stored text that serves token i of the run), by the lookup's rule: the run-start
        match, else the serving candidate of the first stream that covers the token, else of the second."""
        s = self.find(run[: i + 1])
        if s is not None:
            return s, 0
        for stream in (0, 1):
            for a, e, st in chosen:
                if st == stream and a <= i <= e:
                    s = self.find(run[a: i + 1])
                    if s is not None:
                        return s, a
        return None, None

    def insert_once(self, tok, mask, off):
        out = [None] * len(tok)
        plan = []
        for _, a0, b0 in runs(tok, mask, off):  # what the pool holds is decided before anything is stored
            run = [int(t) for t in tok[a0:b0]]
            chosen = brute_choice(brute_candidates(self, self.stored_runs, run, self.W))
            c = 0
            for i in range(len(run)):
                s, start = self.serving(run, i, chosen)
                if s is not None:
                    c = start
                plan.append((a0 + i, s, run[c: i + 1]))
        new_runs = []
        for i, s, text in plan:
            if s is None:
                s = self.find(text)  # stored earlier in this batch under the same text
                if s is None and self.n_used < len(self.free):
                    s = self.free[self.n_used]
                    self.n_used += 1
                    self.stored.append((text, s))
                    if len(text) == self.W:
                        new_runs.append(text)
            out[i] = s
        # prefixes of length W of texts stored from their first token on
        self.stored_runs += [t for t in new_runs]
        return out


def oracle_insert_once(ix, anchors, tok, mask, off, free, used, pool, slot_pos, W, text=None):
    h, ro = O.hash_segments(tok, mask, off), O.run_offsets(mask, off)
    streams = O.match_streams(ix, tok, h, ro, anchors, W, text, with_offsets=True)
    ih, io, found = O.insert_keys(h, ro, streams)
    n = len(tok)
    so, n_new, fl = O.insert_kv_dedup(ix, ih, found, off, free[used:], np.zeros((1, 2, n, 8), np.uint16), L1(n), pool, POOL1,
                                      slot_pos)
    if text is not None:
        so = O.text_record_dedup(text, tok, io, found, so)
    O.insert_anchors(anchors, ih, io, so, W)
    return so, used + n_new, (ih, io, found)


def lookup(ix, anchors, tok, mask, off, W, text=None):
    h, ro = O.hash_segments(tok, mask, off), O.run_offsets(mask, off)
    return O.merge_streams(O.match_streams(ix, tok, h, ro, anchors, W, text))


@pytest.mark.parametrize("verify", [False, True])
def test_a_document_behind_different_leads_is_stored_once(verify):
    rng = np.random.default_rng(3)
    W, S = 4, 2000
    free = rng.permutation(S).astype(np.uint32)
    ix, anchors = O.Index(), O.AnchorSet()
    text = O.Text(S) if verify else None
    pool, slot_pos = np.zeros((S, 1, 2, 8), np.uint16), np.zeros(S, np.int32)
    doc = rng.integers(0, 32000, 120).astype(np.uint32)
    used = 0
    one = lambda t: (t.astype(np.uint32), np.zeros(len(t), np.uint8), np.array([0, len(t)], np.uint32))  # noqa: E731
    so, used, _ = oracle_insert_once(ix, anchors, *one(doc), free, used, pool, slot_pos, W, text)
    assert used == 120
    leads = [rng.integers(0, 32000, int(n)).astype(np.uint32) for n in (7, 31, 1, 16)]
    tails = [rng.integers(0, 32000, int(n)).astype(np.uint32) for n in (5, 0, 9, 3)]
    for lead, tail in zip(leads, tails):
        before = used
        so, used, (ih, io, found) = oracle_insert_once(ix, anchors, *one(np.concatenate([lead, doc, tail])), free, used, pool,
                                                       slot_pos, W, text)
        assert used - before == len(lead) + len(tail)  # the lead and what follows the document; the document not again
        assert np.array_equal(so[len(lead):len(lead) + 120], free[:120])  # served from the one stored copy
        assert list(io[:len(lead)]) == list(range(len(lead)))
        assert list(io[len(lead):]) == list(range(120 + len(tail)))  # the tail continues the document's stored text
    assert used == 120 + sum(map(len, leads)) + sum(map(len, tails)) and len(anchors) == 1 + sum(len(x) >= W for x in leads)
    # every prompt is found again whole, and so is "other text + document + a stored tail"
    for lead, tail in zip(leads, tails):
        assert (lookup(ix, anchors, *one(np.concatenate([lead, doc, tail])), W, text) != NONE).all()
    q = np.concatenate([rng.integers(0, 32000, 11).astype(np.uint32), doc, tails[2]])
    got = lookup(ix, anchors, *one(q), W, text)
    assert (got[:11] == NONE).all() and (got[11:] != NONE).all()


@pytest.mark.parametrize("seed,vocab,W,verify", [(0, 3, 2, False), (1, 2, 3, False), (2, 4, 1, False), (3, 3, 2, True),
                                                 (4, 32000, 3, True), (5, 5, 4, False)])
def test_insert_once_against_the_token_list_model(seed, vocab, W, verify):
    rng = np.random.default_rng(seed)
    S = 3000
    free = rng.permutation(S).astype(np.uint32)
    ix, anchors, tp = O.Index(), O.AnchorSet(), TextPool(free, W)
    text = O.Text(S) if verify else None
    pool, slot_pos = np.zeros((S, 1, 2, 8), np.uint16), np.zeros(S, np.int32)
    corpus = [rng.integers(0, vocab, int(n)).astype(np.uint32) for n in rng.integers(8, 30, 6)]
    used = 0
    for batch in range(5):
        parts = []
        for _ in range(3):
            d = corpus[int(rng.integers(0, 6))]
            a = int(rng.integers(0, 4))
            parts.append(np.concatenate([rng.integers(0, vocab, int(rng.integers(0, 6))).astype(np.uint32), d[a:],
                                         rng.integers(0, vocab, int(rng.integers(0, 4))).astype(np.uint32)]))
        tok = np.concatenate(parts).astype(np.uint32)
        mask = (rng.random(len(tok)) < 0.06).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum([len(p) for p in parts])]).astype(np.uint32)
        so, used, _ = oracle_insert_once(ix, anchors, tok, mask, off, free, used, pool, slot_pos, W, text)
        want = tp.insert_once(tok, mask, off)
        assert list(so) == [NONE if s is None else s for s in want], batch
        assert used == tp.n_used
        # stored texts stay closed under taking prefixes (the lookup's bisection and the eviction order rely on it)
        texts = {tuple(t) for t, _ in tp.stored}
        assert all(t[:-1] in texts for t in texts if len(t) > 1)
        assert len(ix) == len(tp.stored)
        # everything just stored or found is found again
        assert (lookup(ix, anchors, tok, mask, off, W, text)[mask == 0] != NONE).all()
    plain = sum(len(t) for t in corpus)
    assert used < 5 * 3 * 20  # far fewer tokens than were offered
    assert plain > 0


@pytest.mark.parametrize("verify", [False, True])
def test_a_batch_stored_request_by_request_keeps_one_copy_of_its_new_text(verify):
    """Texts of one call do not see each other: a text that is new to the pool and comes several times in one
    batch is stored once per lead.  Stored one request per call, the later requests find what the first stored.
    Both call patterns against the token-list model."""
    rng = np.random.default_rng(11)
    W, S = 4, 2000
    V = lambda n: rng.integers(0, 32000, int(n)).astype(np.uint32)  # noqa: E731
    doc = V(90)
    prompts = [np.concatenate([doc, V(6)]), np.concatenate([V(13), doc, V(4)]), np.concatenate([V(5), doc]),
               np.concatenate([V(21), doc, V(8)])]
    extra = [6, 13 + 4, 5, 21 + 8]  # tokens of each prompt outside the document

    def store(calls):
        free = rng.permutation(S).astype(np.uint32)
        ix, anchors, tp = O.Index(), O.AnchorSet(), TextPool(free, W)
        text = O.Text(S) if verify else None
        pool, slot_pos = np.zeros((S, 1, 2, 8), np.uint16), np.zeros(S, np.int32)
        used = 0
        for ps in calls:
            tok = np.concatenate(ps).astype(np.uint32)
            mask = np.zeros(len(tok), np.uint8)
            off = np.concatenate([[0], np.cumsum([len(p) for p in ps])]).astype(np.uint32)
            so, used, _ = oracle_insert_once(ix, anchors, tok, mask, off, free, used, pool, slot_pos, W, text)
            want = tp.insert_once(tok, mask, off)
            assert list(so) == [NONE if s is None else s for s in want]
            assert used == tp.n_used
        for p in prompts:  # either way every prompt is found again whole
            one = (p, np.zeros(len(p), np.uint8), np.array([0, len(p)], np.uint32))
            assert (lookup(ix, anchors, *one, W, text) != NONE).all()
        return used

    assert store([prompts]) == sum(map(len, prompts))  # one call: four copies of the document
    assert store([[p] for p in prompts]) == len(doc) + sum(extra)  # one request per call: one copy
