"""Pins for the oracle's insert / probe / span building: a hash-free brute-force
model on tiny inputs, and invariants that hold at any size (Sec. 3.3: only
non-sensitive tokens are shared; Sec. 4.3.5: one copy of a duplicate;
Sec. 4.3.1: unmatched positions are left alone)."""
import numpy as np
import pytest

import oracle as O
from cp_workload import gen
from oracle import harness as OH
from tests.bruteforce import BrutePool, runs

NONE = O.SLOT_NONE


def _rand_prompts(rng, R, T, vocab, p_sens):
    tok = rng.integers(0, vocab, R * T).astype(np.uint32)
    mask = (rng.random(R * T) < p_sens).astype(np.uint8)
    cuts = np.sort(rng.choice(np.arange(1, R * T), R - 1, replace=False)) if R > 1 else np.array([], int)
    off = np.concatenate([[0], cuts, [R * T]]).astype(np.uint32)
    return tok, mask, off


def _tiny_kv(n_tok, seed):
    # 1 layer, 1 head, head_dim 8: rows of 16 bytes, values = anything distinguishable
    rng = np.random.default_rng(seed)
    return rng.integers(0, 65535, (1, 2, n_tok, 8)).astype(np.uint16)


L1 = lambda n: O.Layout(1, 1, 8, 16, 2 * n * 16, n * 16)  # noqa: E731  layer-major buffer of n tokens
POOL1 = O.Layout(1, 1, 8, 32, 32, 16)  # token-major pool


def _as_u32(lst):
    return np.array([NONE if x is None else x for x in lst], np.uint32)


@pytest.mark.parametrize("seed,vocab,n_free", [(0, 3, 1000), (1, 2, 1000), (2, 4, 37), (3, 32000, 1000)])
def test_insert_and_probe_against_brute_force(seed, vocab, n_free):
    rng = np.random.default_rng(seed)
    free = rng.permutation(2000)[:n_free].astype(np.uint32)
    ix, bp = O.Index(), BrutePool(free)
    pool = np.zeros((2000, 1, 2, 8), np.uint16)
    slot_pos = np.full(2000, -1, np.int32)
    slot_tok = np.full(2000, NONE, np.uint32)
    used = 0
    for call in range(3):  # three insert calls: keys of earlier calls win over later ones
        tok, mask, off = _rand_prompts(rng, R=3, T=40, vocab=vocab, p_sens=0.2)
        h = O.hash_segments(tok, mask, off)
        src = _tiny_kv(len(tok), seed * 10 + call)
        slot_out, n_new, fl = O.insert_kv(ix, h, off, free[used:], src, L1(len(tok)), pool, POOL1, slot_pos,
                                          tok=tok, slot_tok=slot_tok)
        want = bp.insert(tok, mask, off)
        assert np.array_equal(slot_out, _as_u32(want))
        assert used + n_new == bp.n_used
        assert bool(fl & O.FLAG_POOL_FULL) == any(w is None and not m for w, m in zip(want, mask))
        # rows of newly stored tokens landed in their slots, position inside the request recorded
        new = set(int(s) for s in free[used : used + n_new])
        for i, s in enumerate(want):
            if s in new:
                new.discard(s)  # first occurrence is the owner
                r = int(np.searchsorted(off, i, side="right") - 1)
                assert slot_pos[s] == i - off[r] == bp.slot_pos[s]
                assert slot_tok[s] == tok[i]
                assert np.array_equal(pool[s, 0, 0], src[0, 0, i]) and np.array_equal(pool[s, 0, 1], src[0, 1, i])
        used += n_new
    assert len(ix) == bp.n_used
    # lookups with fresh prompts
    tok, mask, off = _rand_prompts(rng, R=4, T=50, vocab=vocab, p_sens=0.2)
    got = O.probe(ix, O.hash_segments(tok, mask, off))
    assert np.array_equal(got, _as_u32(bp.probe(tok, mask, off)))
    assert all(got[i] == NONE for i in range(len(tok)) if mask[i])  # a sensitive token is never served
    if vocab <= 4:
        assert (got != NONE).sum() > 20


def test_left_context_must_match_negative_case():
    # stored run: [x] + seg.  A request run that is just seg must not match (run-anchored reading).
    seg = [11, 12, 13, 14]
    ix = O.Index()
    dt = np.array([9] + seg, np.uint32)
    dm = np.zeros(5, np.uint8)
    off = np.array([0, 5], np.uint32)
    pool = np.zeros((8, 1, 2, 8), np.uint16)
    O.insert_kv(ix, O.hash_segments(dt, dm, off), off, np.arange(8, dtype=np.uint32), _tiny_kv(5, 0), L1(5), pool,
                POOL1, np.zeros(8, np.int32))
    rt = np.array(seg, np.uint32)
    assert (O.probe(ix, O.hash_segments(rt, np.zeros(4, np.uint8), np.array([0, 4], np.uint32))) == NONE).all()
    # whereas [x] + seg[:2] matches its 3 tokens, in the donor's slots
    rt = np.array([9] + seg[:2] + [99], np.uint32)
    got = O.probe(ix, O.hash_segments(rt, np.zeros(4, np.uint8), np.array([0, 4], np.uint32)))
    assert list(got) == [0, 1, 2, NONE]


def test_duplicate_insert_keeps_one_copy():
    rng = np.random.default_rng(5)
    tok, mask, off = _rand_prompts(rng, R=2, T=60, vocab=32000, p_sens=0.2)
    h = O.hash_segments(tok, mask, off)
    ix = O.Index()
    pool = np.zeros((500, 1, 2, 8), np.uint16)
    sp = np.zeros(500, np.int32)
    free = np.arange(500, dtype=np.uint32)
    s1, n1, _ = O.insert_kv(ix, h, off, free, _tiny_kv(120, 1), L1(120), pool, POOL1, sp)
    snap = pool.copy()
    s2, n2, _ = O.insert_kv(ix, h, off, free[n1:], _tiny_kv(120, 2), L1(120), pool, POOL1, sp)
    assert n1 == int((mask == 0).sum()) and n2 == 0
    assert np.array_equal(s1, s2) and np.array_equal(pool, snap)  # nothing rewritten
    # the same run twice inside one call: the first occurrence owns the slots
    t2 = np.concatenate([tok[:20], tok[:20]])
    m2 = np.concatenate([mask[:20], mask[:20]])
    m2[0] = m2[20] = 0
    o2 = np.array([0, 20, 40], np.uint32)
    ix2 = O.Index()
    s3, n3, _ = O.insert_kv(ix2, O.hash_segments(t2, m2, o2), o2, free, _tiny_kv(40, 3), L1(40), pool, POOL1, sp)
    assert np.array_equal(s3[:20], s3[20:]) and n3 == int((m2[:20] == 0).sum())
    assert list(s3[:20][m2[:20] == 0]) == list(range(n3))  # slots handed out in packed order


def _check_span_invariants(slot, off, src, dst, ln, n, slot_pos=None, delta=None):
    assert n == len(src)
    N = len(slot)
    # expanding the spans reproduces slot[]
    back = np.full(N, NONE, np.uint32)
    for s, d, l in zip(src, dst, ln):
        assert l >= 1
        assert (back[d : d + l] == NONE).all()  # disjoint
        back[d : d + l] = np.arange(s, s + l, dtype=np.uint32)
    assert np.array_equal(back, slot)
    assert (np.diff(dst.astype(np.int64)) > 0).all()  # (request, position) order
    req = np.searchsorted(off, dst, side="right") - 1
    for k in range(n):
        assert dst[k] + ln[k] <= off[req[k] + 1]  # a span never crosses a request boundary
        if slot_pos is not None:
            p = np.arange(dst[k], dst[k] + ln[k]) - off[req[k]]
            assert (p - slot_pos[src[k] : src[k] + ln[k]] == delta[k]).all()
    for k in range(n - 1):  # maximal: no two neighbours could be merged
        touching = dst[k] + ln[k] == dst[k + 1] and req[k] == req[k + 1] and src[k] + ln[k] == src[k + 1]
        if touching:
            assert slot_pos is not None and delta[k] != delta[k + 1]


def test_spans_invariants_random():
    rng = np.random.default_rng(6)
    for trial in range(20):
        N = int(rng.integers(1, 400))
        # runs of consecutive slots of random lengths, holes in between
        slot = np.full(N, NONE, np.uint32)
        i = 0
        while i < N:
            l = int(rng.integers(1, 12))
            if rng.random() < 0.6:
                s0 = int(rng.integers(0, 5000))
                slot[i : i + l] = np.arange(s0, s0 + min(l, N - i))
            i += l
        R = int(rng.integers(1, 5))
        off = np.concatenate([[0], np.sort(rng.integers(0, N + 1, R - 1)), [N]]).astype(np.uint32)
        src, dst, ln, delta, n, fl = O.build_spans(slot, off)
        assert fl == 0 and (delta == 0).all()
        _check_span_invariants(slot, off, src, dst, ln, n)
        assert ln.sum() == (slot != NONE).sum()
        slot_pos = rng.integers(-3, 4, 5100).astype(np.int32) + np.arange(5100, dtype=np.int32)
        src, dst, ln, delta, n, fl = O.build_spans(slot, off, slot_pos)
        _check_span_invariants(slot, off, src, dst, ln, n, slot_pos, delta)


def test_spans_hand_example():
    #        pos: 0  1  2   3    4   5  | 0   1
    slot = np.array([7, 8, 9, NONE, 10, 3, 4, 5], np.uint32)
    off = np.array([0, 6, 8], np.uint32)
    src, dst, ln, delta, n, fl = O.build_spans(slot, off)
    # 10 does not continue 9 (a hole between), 3 does not follow 10, and 4 starts request 1
    assert (list(src), list(dst), list(ln), n) == ([7, 10, 3, 4], [0, 4, 5, 6], [3, 1, 1, 2], 4)
    slot_pos = np.zeros(16, np.int32)
    slot_pos[[7, 8, 9]] = [0, 1, 5]  # slot 9 was cached at position 5: delta changes inside 7,8,9
    slot_pos[[4, 5]] = [10, 11]
    src, dst, ln, delta, n, fl = O.build_spans(slot, off, slot_pos)
    assert (list(src), list(dst), list(ln)) == ([7, 9, 10, 3, 4], [0, 2, 4, 5, 6], [2, 1, 1, 1, 2])
    assert list(delta) == [0, -3, 4, 5, -10]


def test_spans_overflow_keeps_first():
    slot = np.array([1, NONE, 3, NONE, 5, NONE, 7], np.uint32)
    off = np.array([0, 7], np.uint32)
    src, dst, ln, delta, n, fl = O.build_spans(slot, off, max_spans=2)
    assert n == 4 and fl == O.FLAG_SPANS_OVERFLOW
    assert (list(src), list(dst), list(ln)) == ([1, 3], [0, 2], [1, 1])


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("llama3-8b", {"scale": 1 / 16}), ("frag", {"scale": 1 / 64}),
                                     ("rope", {"scale": 1 / 32}), ("llama3-70b", {"scale": 1 / 64})])
def test_workload_invariants(name, kw):
    """Whole path on the five workloads (small scale, tiny KV rows): privacy invariant,
    soundness of every span against the stored token ids, structure of matches."""
    wl = gen.make(name, **kw)
    wl.shape = gen.KVShape(2, 1, 8)
    fl = []
    st = OH.prefill(wl, flags_out=fl)
    lk = OH.lookup(st)
    N = wl.n_tokens
    # nothing sensitive was stored or is served
    assert (st.donor_slot[wl.donor_mask == 1] == NONE).all()
    assert (lk.slot[wl.mask == 1] == NONE).all() and (lk.hash[wl.mask == 1] == O.HASH_NONE).all()
    assert len(st.index) == st.n_used == (st.slot_uid != 0xFFFFFFFFFFFFFFFF).sum()
    # every span is a common substring of the request and of what the pool stored, token by token
    covered = np.zeros(N, bool)
    for s, d, l in zip(lk.span_src, lk.span_dst, lk.span_len):
        assert (st.slot_tok[s : s + l] == wl.tok[d : d + l]).all()
        assert (wl.mask[d : d + l] == 0).all()
        covered[d : d + l] = True
    assert covered.sum() == (lk.slot != NONE).sum() > 0
    # within one run the matched flags read 1..1 0..0 (stored runs are prefix-closed)
    for _, a, b in runs(wl.tok, wl.mask, wl.off):
        m = (lk.slot[a:b] != NONE).astype(int)
        assert (np.diff(m) <= 0).all()
    # gathered bytes equal pool bytes (no rotation) / rows outside spans untouched
    re = wl.shape.row_bytes // 2
    if wl.rope_theta is None:
        for i in np.flatnonzero(covered)[:: max(1, covered.sum() // 200)]:
            assert np.array_equal(lk.dst[:, :, i], st.pool[lk.slot[i]])
    else:
        # reused pieces sit within max_shift of their cached place; only chance matches of a run's first
        # token(s) with an unrelated stored run fall outside
        assert (np.abs(lk.span_delta) <= wl.notes["max_shift"]).mean() > 0.9 and (lk.span_delta != 0).mean() > 0.7
        for i in np.flatnonzero(covered)[:: max(1, covered.sum() // 200)]:
            assert np.array_equal(lk.dst[:, 1, i], st.pool[lk.slot[i], :, 1])  # V is never rotated
    assert (lk.dst[:, :, ~covered] == 0xC0DE).all()
    # changing the ids of sensitive tokens changes no output bit (Sec. 3.3)
    tok2 = wl.tok.copy()
    tok2[wl.mask == 1] = (tok2[wl.mask == 1] + 1) % 32000
    lk2 = OH.lookup(st, tok=tok2)
    assert np.array_equal(lk2.slot, lk.slot) and np.array_equal(lk2.dst, lk.dst)
    assert lk.n_spans == len(lk.span_src)
    print(name, "tokens", N, "matched %.3f" % covered.mean(), "sensitive %.3f" % wl.mask.mean(), "spans", lk.n_spans,
          "pool used", st.n_used, "/", wl.pool_slots, "flags", fl)


def test_a_table_that_cannot_take_the_new_keys_stores_nothing():
    """Bounded table: a key holds an entry from the insert that first sees it (also when the pool had no slot for
    it, and after its slot is evicted) until the table is rebuilt; a batch whose new keys do not all fit sets
    TABLE_FULL and stores nothing, while keys stored before are still reported."""
    ix = O.Index()
    ix.rebuild(10)
    pool, slot_pos = np.zeros((64, 1, 2, 8), np.uint16), np.zeros(64, np.int32)
    lay = lambda n: O.Layout(1, 1, 8, 16, 2 * n * 16, n * 16)  # noqa: E731
    P = O.Layout(1, 1, 8, 32, 32, 16)
    free = np.arange(64, dtype=np.uint32)

    def ins(tok, free_slots):
        tok = np.asarray(tok, np.uint32)
        n = len(tok)
        h = O.hash_segments(tok, np.zeros(n, np.uint8), np.array([0, n], np.uint32))
        return O.insert_kv(ix, h, np.array([0, n], np.uint32), free_slots, np.zeros((1, 2, n, 8), np.uint16), lay(n), pool, P,
                           slot_pos)

    so, n_new, fl = ins([1, 2, 3, 4, 5, 6], free[:4])  # six keys, four slots: two keys keep an entry without a slot
    assert n_new == 4 and fl == O.FLAG_POOL_FULL and ix.entries == 6 and len(ix) == 4
    so, n_new, fl = ins([1, 2, 3, 9, 9, 9, 9, 9, 9], free[4:])  # 3 known + 6 new keys: 12 > 10
    assert fl == O.FLAG_TABLE_FULL and n_new == 0 and list(so[:3]) == [0, 1, 2] and (so[3:] == NONE).all()
    assert ix.entries == 6 and len(ix) == 4
    so, n_new, fl = ins([1, 2, 3, 4, 5, 6, 7, 8, 9, 10], free[4:])  # exactly fills the table: 6 entries + 4 new
    assert fl == 0 and n_new == 6 and ix.entries == 10 and len(ix) == 10  # 5 and 6 get their slots now
    so, n_new, fl = ins([7], free[10:])  # one more key does not fit any more
    assert fl == O.FLAG_TABLE_FULL and n_new == 0
    ix.rebuild(16)
    so, n_new, fl = ins([7], free[10:])
    assert fl == 0 and n_new == 1 and ix.entries == 11
