"""Pool policies on the GPU against the CPU oracle: minimum segment length and recompute marks
(Sec. 4.2.1 "Optimization", Step 3), zero placeholders (Sec. 4.3.1), least-recently-used eviction
(Sec. 4.3.5 "Lifecycle management").  Integer results bit for bit, buffers byte for byte."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen, kvgen
from oracle import harness as OH
from test_gpu_parity import G, compare_all  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu

NONE = O.SLOT_NONE


def _u8(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev)


@pytest.mark.parametrize("seed", [0, 1])
def test_filter_matches_random(G, seed):
    from paper_2605_23640_amd import binding as B
    rng = np.random.default_rng(seed)
    N, S = 5000, 300  # several scan tiles and a ragged tail
    slot = rng.integers(0, S, N).astype(np.uint32)
    slot[rng.random(N) < 0.12] = NONE
    cuts = np.sort(rng.choice(np.arange(1, N), 7, replace=False))
    off = np.concatenate([[0], cuts[:4], cuts[3:4], cuts[4:], [N]]).astype(np.uint32)  # with an empty request
    marks = (rng.random(S) < 0.25).astype(np.uint8)
    d_slot, d_off, d_marks = G.dev_i32(slot), G.dev_i32(off), _u8(marks, G.DEV)
    scratch = B.new_scratch(N, 0, G.DEV)
    out = torch.empty(N, dtype=torch.int32, device=G.DEV)
    for min_len in (0, 1, 2, 5, 9, 40, 100000):
        B.cp_filter_matches(d_slot, d_off, min_len, None, S, out, scratch)
        assert np.array_equal(G.host_u32(out), O.filter_matches(slot, off, min_len)), min_len
        B.cp_filter_matches(d_slot, d_off, min_len, d_marks, S, out, scratch)
        assert np.array_equal(G.host_u32(out), O.filter_matches(slot, off, min_len, marks)), min_len
    inplace = d_slot.clone()
    B.cp_filter_matches(inplace, d_off, 5, d_marks, S, inplace, scratch)
    assert np.array_equal(G.host_u32(inplace), O.filter_matches(slot, off, 5, marks))


def test_filter_matches_long_stretches_and_edges(G):
    from paper_2605_23640_amd import binding as B
    N = 4500
    scratch = B.new_scratch(N, 0, G.DEV)
    out = torch.empty(N, dtype=torch.int32, device=G.DEV)
    slot = np.arange(N, dtype=np.uint32)  # one stretch over more than four scan tiles ...
    for off in (np.array([0, N], np.uint32), np.array([0, 2047, 2049, N], np.uint32)):  # ... or cut by requests
        for min_len in (2, 2047, 2048, 2451, 2452, N, N + 1):
            B.cp_filter_matches(G.dev_i32(slot), G.dev_i32(off), min_len, None, 0, out, scratch)
            assert np.array_equal(G.host_u32(out), O.filter_matches(slot, off, min_len)), (off, min_len)
    none = np.full(N, NONE, np.uint32)
    B.cp_filter_matches(G.dev_i32(none), G.dev_i32(np.array([0, N], np.uint32)), 1, None, 0, out, scratch)
    assert (G.host_u32(out) == NONE).all()
    one = G.dev_i32(np.array([7], np.uint32))
    B.cp_filter_matches(one, G.dev_i32(np.array([0, 1], np.uint32)), 1, None, 0, out[:1], scratch)
    assert G.host_u32(out[:1])[0] == 7
    B.cp_filter_matches(one[:0], G.dev_i32(np.array([0, 0], np.uint32)), 1, None, 0, out[:0], scratch)  # N = 0


def test_marks_and_zero_placeholders(G):
    from paper_2605_23640_amd import binding as B
    rng = np.random.default_rng(3)
    N, S = 700, 64
    slot = rng.integers(0, S, N).astype(np.uint32)
    slot[rng.random(N) < 0.3] = NONE
    slot[5] = 1000  # a slot outside the pool is ignored by the marks
    rec = (rng.random(N) < 0.25).astype(np.uint8)
    want = np.zeros(S, np.uint8)
    want[3] = 1  # marks accumulate
    d_marks = _u8(want, G.DEV)
    O.mark_recompute(slot, rec, want)
    B.cp_mark_recompute(G.dev_i32(slot), _u8(rec, G.DEV), S, d_marks)
    assert np.array_equal(d_marks.cpu().numpy(), want)
    # zero rows for unmatched tokens, everything else untouched (three layers of 2 heads x 64: 256-byte rows)
    sh = gen.KVShape(3, 2, 64)
    lay = B.KVLayout.layer_major(sh.n_layers, sh.n_kv_heads, sh.head_dim, N)
    dst = G.poison_tensor(N * sh.tok_bytes)
    B.cp_fill_unmatched(G.dev_i32(slot), dst, lay)
    host = np.full((sh.n_layers, 2, N, sh.row_bytes // 2), kvgen.POISON16, np.uint16)
    O.fill_unmatched(slot, host, OH.buf_layout(sh, N))
    assert np.array_equal(G.dst_as_rows(dst, sh, N), host)
    assert (host[:, :, slot == NONE] == 0).all() and (host[:, :, slot != NONE] == kvgen.POISON16).all()


@pytest.mark.parametrize("seed", [0, 1])
def test_touch_and_lru_threshold(G, seed):
    from paper_2605_23640_amd import binding as B
    rng = np.random.default_rng(seed)
    S = 3000
    scratch = B.new_scratch(S, 0, G.DEV, S)
    thr = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    for now, lo in ((60, 0), (10000, 0), (10000, 9000)):  # the second has ages beyond the histogram's window
        stamps = rng.integers(lo, now + 1, S).astype(np.uint32)
        stamps[rng.random(S) < 0.2] = 0
        stamps[:3] = now + 5  # stamped "in the future": never chosen
        d = G.dev_i32(stamps)
        for needed in (0, 1, 17, 400, 1500, 2396, 2397, S, 5 * S):
            B.cp_lru_threshold(d, S, now, needed, thr, scratch)
            assert int(G.host_u32(thr)[0]) == O.lru_threshold(stamps, now, needed), (now, lo, needed)
    st = rng.integers(0, 50, S).astype(np.uint32)
    slot = rng.integers(0, S + 10, 4000).astype(np.uint32)
    slot[rng.random(4000) < 0.2] = NONE
    d = G.dev_i32(st)
    B.cp_touch(G.dev_i32(slot), 25, S, d)
    O.touch(slot, 25, st)
    assert np.array_equal(G.host_u32(d), st)


class Lifecycle:
    """The same multi-batch scenario driven through the GPU pool and through the oracle."""

    def __init__(self, G, S, shape, seed, verify, min_len=1, marks=False, zero_fill=False, anchor_window=None,
                 dedup=False):
        import paper_2605_23640_amd as cp
        self.G, self.cp, self.sh, self.S, self.seed = G, cp, shape, S, seed
        rng = np.random.default_rng(seed)
        free = rng.permutation(S).astype(np.uint32)
        self.pool = cp.KVPool(shape.n_layers, shape.n_kv_heads, shape.head_dim, S, 4 * S,
                              torch.from_numpy(free.view(np.int32)), device=G.DEV,
                              pool_tensor=G.poison_tensor(S * shape.tok_bytes), verify=verify, min_len=min_len,
                              recompute_marks=marks, zero_fill=zero_fill, lru=True, anchor_window=anchor_window,
                              dedup=dedup)
        self.dedup = dedup
        # oracle side
        self.W = anchor_window
        self.anchors = O.AnchorSet() if anchor_window is not None else None
        self.ix = O.Index()
        self.text = O.Text(S) if verify else None
        self.opool = np.full((S, shape.n_layers, 2, shape.row_bytes // 2), kvgen.POISON16, np.uint16)
        self.slot_pos = np.zeros(S, np.int32)
        self.stamps = np.zeros(S, np.uint32)
        self.marks = np.zeros(S, np.uint8) if marks else None
        self.free = free.copy()
        self.min_len, self.zero_fill = min_len, zero_fill
        self.evictions = 0
        self.flags = 0

    def batch(self, epoch, tok, mask, off, rec):
        G, cp, sh, S = self.G, self.cp, self.sh, self.S
        N = len(tok)
        self.pool.epoch = epoch
        d_tok, d_mask, d_off = G.dev_i32(tok), _u8(mask, G.DEV), G.dev_i32(off)
        buf = cp.LookupBuffers(N, N, G.DEV, n_pool_slots=S)
        dst = G.poison_tensor(N * sh.tok_bytes)
        self.pool.lookup(d_tok, d_mask, d_off, dst, buf)
        # oracle lookup
        h = O.hash_segments(tok, mask, off)
        ro = O.run_offsets(mask, off)
        plain = O.probe(self.ix, h)
        streams = O.match_streams(self.ix, tok, h, ro, self.anchors, self.W, self.text)
        for own in streams[1:]:  # slots a candidate stream walked through count as used, whichever stream serves
            O.touch(own, epoch, self.stamps)
        got = O.merge_streams(streams)
        O.touch(got, epoch, self.stamps)
        served = O.filter_matches(got, off, self.min_len, self.marks)
        src, dpos, ln, delta, n, fl = O.build_spans(served, off)
        odst = np.full((sh.n_layers, 2, N, sh.row_bytes // 2), kvgen.POISON16, np.uint16)
        O.gather_kv(self.opool, OH.pool_layout(sh), odst, OH.buf_layout(sh, N), src, dpos, ln)
        if self.zero_fill:
            O.fill_unmatched(served, odst, OH.buf_layout(sh, N))
        assert np.array_equal(G.host_u32(buf.slot), got), epoch
        if self.pool.filters:
            assert np.array_equal(G.host_u32(buf.served), served), epoch
        assert np.array_equal(G.dst_as_rows(dst, sh, N), odst), epoch
        # room for what this batch will store
        new_keys = len({int(x) for x, g in zip(h, plain) if g == NONE and x != O.HASH_NONE})
        if new_keys > len(self.free):
            T = O.lru_threshold(self.stamps, epoch, new_keys - len(self.free))
            freed = O.evict(self.ix, self.stamps, T, self.text, self.marks, self.anchors)
            self.ix.rebuild(0)  # the pool's evict() also moves the keys that still have a slot to a fresh table
            self.free = np.concatenate([self.free, freed])
            g_freed = self.pool.evict(new_keys - self.pool.n_free(), buf.scratch)
            assert int(G.host_u32(self.pool.threshold)[0]) == T
            assert np.array_equal(G.host_u32(g_freed), freed), epoch
            self.evictions += 1
        # insert the batch (its KV: generator rows with uids epoch * 2^20 + i)
        uid0 = epoch << 20
        kv = torch.empty(N * sh.tok_bytes, dtype=torch.uint8, device=G.DEV)
        kvgen.fill(G.stream_ptr(), C.c_void_p(kv.data_ptr()), G.gen_layout(self.pool.request_layout(N)), N, self.seed,
                   uid_base=uid0)
        sout = torch.empty(N, dtype=torch.int32, device=G.DEV)
        roff = torch.empty(N, dtype=torch.int32, device=G.DEV)
        n_g = self.pool.insert(d_tok, d_mask, d_off, kv, buf.hash, sout, buf.scratch, run_off_buf=roff,
                               recompute=_u8(rec, G.DEV) if self.marks is not None else None, buf=buf)
        okv = OH.gen_buffer(self.seed, sh, uid0, N)
        if self.dedup:  # every text once: what a lookup of the batch finds now (after the eviction) is left out
            streams = O.match_streams(self.ix, tok, h, ro, self.anchors, self.W, self.text, with_offsets=True)
            h, ro, found = O.insert_keys(h, ro, streams)  # from here on: the keys and offsets the batch is stored under
            so, n_new, fl = O.insert_kv_dedup(self.ix, h, found, off, self.free, okv, OH.buf_layout(sh, N), self.opool,
                                              OH.pool_layout(sh), self.slot_pos)
            assert np.array_equal(G.host_u64(buf.ins_hash), h), epoch
        else:
            so, n_new, fl = O.insert_kv(self.ix, h, off, self.free, okv, OH.buf_layout(sh, N), self.opool,
                                        OH.pool_layout(sh), self.slot_pos)
        self.free = self.free[n_new:]
        self.flags |= fl
        if self.text is not None:
            so = O.text_record_dedup(self.text, tok, ro, found, so) if self.dedup else O.text_record(self.text, tok, ro, so)
        if self.marks is not None:
            O.mark_recompute(so, rec, self.marks)
        if self.anchors is not None:
            O.insert_anchors(self.anchors, h, ro, so, self.W)
            assert int(self.pool.slot_anchor.sum().item()) == len(self.anchors), epoch
        O.touch(so, epoch, self.stamps)
        assert n_g == n_new and np.array_equal(G.host_u32(sout), so), epoch
        assert np.array_equal(G.host_u32(self.pool.slot_stamp), self.stamps), epoch
        if self.marks is not None:
            assert np.array_equal(self.pool.slot_recompute.cpu().numpy(), self.marks), epoch
        assert self.pool.n_free() == len(self.free) and int(self.pool.flags.item()) == self.flags
        from paper_2605_23640_amd import binding as B
        counts = torch.empty(2, dtype=torch.int32, device=G.DEV)
        B.cp_table_count(self.pool.table, counts)  # entries holding a key, of which with a slot
        assert tuple(G.host_u32(counts).tolist()) == (self.ix.entries, len(self.ix)), epoch


@pytest.mark.parametrize("verify,min_len,marks,zero_fill", [(False, 1, False, False), (True, 1, False, False),
                                                           (False, 4, True, True), (True, 3, True, True)])
def test_pool_lifecycle_with_eviction(G, verify, min_len, marks, zero_fill):
    rng = np.random.default_rng(11)
    sh = gen.KVShape(2, 2, 64)
    life = Lifecycle(G, 400, sh, 0xC0FFEE08, verify, min_len, marks, zero_fill)
    corpus = [rng.integers(0, 32000, 80).astype(np.uint32) for _ in range(8)]
    corpus_mask = [(rng.random(80) < 0.06).astype(np.uint8) for _ in range(8)]
    for epoch in range(1, 22):
        picks = rng.choice(8, 3, replace=False)
        cut = [int(rng.integers(20, 81)) for _ in picks]
        tok = np.concatenate([corpus[d][:c] for d, c in zip(picks, cut)]).astype(np.uint32)
        mask = np.concatenate([corpus_mask[d][:c] for d, c in zip(picks, cut)]).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum(cut)]).astype(np.uint32)
        rec = (rng.random(len(tok)) < 0.25).astype(np.uint8)
        life.batch(epoch, tok, mask, off, rec)
    assert life.evictions >= 2


@pytest.mark.parametrize("seed,vocab,W,verify", [(1, 3, 2, False), (2, 3, 2, True), (3, 4, 3, True), (4, 32000, 4, True),
                                                 (5, 2, 1, True), (6, 5, None, True)])
def test_pool_lifecycle_small_vocabulary_with_anchors(G, seed, vocab, W, verify):
    """Few distinct tokens: shared prefixes, duplicate runs inside a batch, chance anchors and evictions all
    occur often; floating anchors, verification, filter, marks and zero fill are on together."""
    rng = np.random.default_rng(seed)
    sh = gen.KVShape(1, 2, 64)
    life = Lifecycle(G, 300, sh, 0xC0FFEE09 + seed, verify, min_len=2, marks=True, zero_fill=True, anchor_window=W)
    corpus = [rng.integers(0, vocab, 60).astype(np.uint32) for _ in range(6)]
    for epoch in range(1, 26):
        parts = []
        for d in rng.choice(6, 3, replace=False):
            lead = rng.integers(0, vocab, int(rng.integers(0, 6))).astype(np.uint32)  # text in front of the shared one
            a = int(rng.integers(0, 20))
            parts.append(np.concatenate([lead, corpus[d][a:a + int(rng.integers(10, 41))]]))
        tok = np.concatenate(parts).astype(np.uint32)
        mask = (rng.random(len(tok)) < 0.08).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum([len(x) for x in parts])]).astype(np.uint32)
        rec = (rng.random(len(tok)) < 0.25).astype(np.uint8)
        life.batch(epoch, tok, mask, off, rec)
    assert life.evictions >= 1


def test_table_compact_after_eviction(G):
    from paper_2605_23640_amd import binding as B
    wl = gen.make("tiny")
    pool = G.make_pool(wl)
    pool.slot_stamp = torch.zeros(pool.n_slots, dtype=torch.int32, device=G.DEV)  # LRU stamps from the start
    st = G.prefill(wl, pool)
    # age half of the stored slots and evict them
    stamps = G.host_u32(pool.slot_stamp).copy()
    used = np.flatnonzero(stamps)
    stamps[used[::2]] = 5
    stamps[used[1::2]] = 9
    pool.slot_stamp.copy_(G.dev_i32(stamps))
    pool.epoch = 9
    scratch = B.new_scratch(wl.n_tokens, 0, G.DEV, pool.n_slots)
    freed = G.host_u32(pool.evict(len(used) // 2, scratch, compact=False))
    assert np.array_equal(freed, np.sort(used[::2]))
    hashes = torch.from_numpy(st.donor_hash.view(np.int64)).to(G.DEV)
    before = torch.empty(len(st.donor_hash), dtype=torch.int32, device=G.DEV)
    B.cp_probe(pool.table, hashes, before)
    b = G.host_u32(before)
    gone = np.isin(st.donor_slot, freed)
    assert (b[gone] == NONE).all() and np.array_equal(b[~gone], st.donor_slot[~gone])
    # the table still holds the evicted slots' keys; a compacted copy holds only the keys that have a slot
    counts = torch.empty(2, dtype=torch.int32, device=G.DEV)
    n_keys = len(np.unique(st.donor_hash[st.donor_hash != O.HASH_NONE]))
    n_live = len(np.unique(st.donor_slot[~gone & (st.donor_slot != NONE)]))
    B.cp_table_count(pool.table, counts)
    assert G.host_u32(counts).tolist() == [n_keys, n_live]
    fresh = B.Table(pool.table.capacity, G.DEV)
    B.cp_table_compact(pool.table, fresh, pool.flags)
    B.cp_table_count(fresh, counts)
    assert G.host_u32(counts).tolist() == [n_live, n_live] and n_live < n_keys
    after = torch.empty_like(before)
    B.cp_probe(fresh, hashes, after)
    assert np.array_equal(G.host_u32(after), b) and int(pool.flags.item()) == 0
    keys = G.host_u64(fresh.keys)
    assert (keys != O.HASH_NONE).sum() == len(np.unique(st.donor_slot[~gone & (st.donor_slot != NONE)]))
    # a table that is too small reports it
    tiny = B.Table(16, G.DEV)
    B.cp_table_compact(pool.table, tiny, pool.flags)
    assert int(pool.flags.item()) & B.FLAG_TABLE_FULL


@pytest.mark.parametrize("min_len,rho,zero_fill", [(16, 0.0, False), (1, 0.25, True), (24, 0.25, True)])
def test_policies_on_the_8b_shaped_workload(G, min_len, rho, zero_fill):
    wl = gen.make_docs("llama3-8b-small", 0xC0FFEE02, gen.KVShape(32, 8, 128), R=3, T=1371, prefix_len=300, n_docs=6,
                       doc_len=(150, 300), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096)
    rec = (wl.donor_u < rho).astype(np.uint8) if rho else None
    ost, olk, gst, glk = compare_all(G, wl, min_len=min_len, recompute=rec, zero_fill=zero_fill)
    matched, served = (olk.slot != NONE).sum(), (olk.served != NONE).sum()
    assert 0 < served < matched
    if zero_fill:
        rows = G.dst_as_rows(glk.dst, wl.shape, wl.n_tokens)
        assert (rows[:, :, olk.served == NONE] == 0).all()


def test_policies_with_rope_anchors_and_verification(G):
    wl = gen.make("float", scale=0.25)
    wl.shape = gen.KVShape(2, 8, 128)
    wl.rope_theta, wl.rope_style = 500000.0, 1
    rec = (wl.donor_u < 0.25).astype(np.uint8)
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=8, verify=True, min_len=12, recompute=rec, zero_fill=True)
    assert (olk.served != NONE).sum() > 100 and (glk.span_delta != 0).mean() > 0.5
