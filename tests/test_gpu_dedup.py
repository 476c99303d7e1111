"""Storing every text once (Sec. 4.3.5 "Lifecycle management") on the GPU against the CPU oracle: the keys a
batch is stored under, the slots, the pool's bytes and what later lookups are served, bit for bit."""
import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen, kvgen
from oracle import harness as OH
from test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

NONE = O.SLOT_NONE


def both(G, wl, W, verify, **policies):
    fl = []
    ost = OH.prefill(wl, flags_out=fl, anchor_window=W, verify=verify, dedup=True)
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=W, verify=verify, dedup=True, **policies))
    assert np.array_equal(gst.donor_hash, ost.donor_hash), "keys the batches were stored under"
    assert np.array_equal(gst.donor_slot, ost.donor_slot)
    assert sum(gst.n_inserted) == ost.n_used and gst.flags == fl[0]
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0  # every stored row, and nothing else
    live = ost.slot_uid != kvgen.UID_NONE
    assert np.array_equal(G.host_u32(gst.pool.slot_pos.view(torch.int32))[live].view(np.int32), ost.slot_pos[live])
    assert int(gst.pool.slot_anchor.sum().item()) == len(ost.anchors)  # one prefix hash per stored text of >= W tokens
    olk, glk = OH.lookup(ost), G.lookup(gst)
    for f in ("hash", "hash_float", "hash_late", "slot", "span_src", "span_dst", "span_len"):
        assert np.array_equal(getattr(glk, f), getattr(olk, f)), f
    assert np.array_equal(G.dst_as_rows(glk.dst, wl.shape, wl.n_tokens), olk.dst)
    return ost, gst, olk


@pytest.mark.parametrize("verify", [False, True])
def test_documents_behind_leads_are_stored_once(G, verify):
    rng = np.random.default_rng(21)
    V = lambda n: rng.integers(0, 32000, n).astype(np.uint32)  # noqa: E731
    docs = [V(int(n)) for n in (300, 170, 420)]
    leads = [V(int(n)) for n in (40, 7, 120, 1, 64, 33)]
    tails = [V(int(n)) for n in (10, 0, 25, 5, 0, 12)]
    donors = list(docs)  # first the documents alone, then prompts that quote them behind other text
    picks = [(0,), (1,), (2, 0), (0,), (1, 2), (2,)]
    for lead, tail, pk in zip(leads, tails, picks):
        donors.append(np.concatenate([lead] + [docs[d] for d in pk] + [tail]))
    reqs = [np.concatenate([V(9), docs[2], docs[0], tails[2], V(3)]), np.concatenate([leads[4], docs[1], docs[2], V(6)]),
            np.concatenate([V(2), docs[0], tails[3]])]
    wl = gen.from_prompts("stored-once", 0xC0FFEE31, gen.KVShape(2, 2, 64), donors, reqs, pool_slots=4096,
                          donor_batch_tokens=500)
    assert len(wl.donor_batches) >= 6
    ost, gst, olk = both(G, wl, 8, verify)
    # one copy of every document, the leads, and what follows a quoted document
    assert ost.n_used == sum(map(len, docs)) + sum(map(len, leads)) + sum(map(len, tails))
    o = wl.off
    assert (olk.slot[o[0] + 9:o[0] + 9 + 420 + 300 + 25] != NONE).all()  # docs 2, 0 and the tail stored behind them
    assert (olk.slot[o[1]:o[1] + 64 + 170 + 420] != NONE).all()
    # without it, the same donors take a slot for every token of every prompt
    plain = OH.prefill(wl, anchor_window=8, verify=verify)
    assert plain.n_used == sum(map(len, donors))
    plk = OH.lookup(plain)
    # ... and serve no token that the single copies do not serve (those serve a few more: text stored behind a
    # document continues the document's stored text, whatever the document is quoted behind)
    assert ((plk.slot != NONE) <= (olk.slot != NONE)).all() and (olk.slot != NONE).sum() > 1600


@pytest.mark.parametrize("seed,vocab,W,verify,base", [(1, 3, 2, False, None), (2, 4, 1, True, None), (3, 32000, 4, True, None),
                                                      (4, 2, 3, False, None), (5, 4, 2, True, 0x9E3779B97F4A7C15),
                                                      (6, 32000, 3, False, 10)])
def test_random_batches_stored_once(G, seed, vocab, W, verify, base):
    """(The last two cases hash with another base than the default one: the keys texts are continued under are
    substring keys, which take powers of the base.)"""
    rng = np.random.default_rng(seed)
    corpus = [rng.integers(0, vocab, int(n)).astype(np.uint32) for n in rng.integers(20, 90, 8)]

    def prompt():
        parts = []
        for _ in range(int(rng.integers(1, 4))):
            d = corpus[int(rng.integers(0, 8))]
            parts += [rng.integers(0, vocab, int(rng.integers(0, 9))).astype(np.uint32), d[int(rng.integers(0, 5)):]]
        return np.concatenate(parts + [rng.integers(0, vocab, int(rng.integers(0, 6))).astype(np.uint32)])

    donors = [prompt() for _ in range(14)]
    reqs = [prompt() for _ in range(5)]
    masks = lambda ps: [(rng.random(len(p)) < 0.04).astype(np.uint8) for p in ps]  # noqa: E731
    wl = gen.from_prompts("stored-once-random", 0xC0FFEE32 + seed, gen.KVShape(2, 2, 64), donors, reqs, pool_slots=2048,
                          donor_masks=masks(donors), request_masks=masks(reqs), donor_batch_tokens=260)
    wl.hash_base = base
    assert len(wl.donor_batches) >= 4
    ost, gst, olk = both(G, wl, W, verify)
    assert ost.n_used < 0.8 * len(wl.donor_tok)


@pytest.mark.parametrize("verify", [False, True])
def test_one_request_per_call_keeps_one_copy_of_a_batchs_new_text(G, verify):
    """Texts of one call do not see each other.  The same prompts in one call (four copies of their document, one
    per lead) and one request per call (one copy), each against the oracle."""
    rng = np.random.default_rng(13)
    V = lambda n: rng.integers(0, 32000, int(n)).astype(np.uint32)  # noqa: E731
    doc = V(700)
    donors = [np.concatenate([doc, V(40)]), np.concatenate([V(90), doc, V(30)]), np.concatenate([V(35), doc]),
              np.concatenate([V(150), doc, V(60)])]
    outside = 40 + 90 + 30 + 35 + 150 + 60
    reqs = [np.concatenate([V(12), doc, V(7)]), donors[3]]
    used = []
    for batch_tokens in (1 << 17, 800):  # everything in one call; one prompt per call
        wl = gen.from_prompts("one-per-call", 0xC0FFEE34, gen.KVShape(2, 2, 64), donors, reqs, pool_slots=8192,
                              donor_batch_tokens=batch_tokens)
        assert len(wl.donor_batches) == (1 if batch_tokens > 800 else 4)
        ost, gst, olk = both(G, wl, 8, verify)
        used.append(ost.n_used)
        assert (olk.slot[12:12 + 700] != NONE).all() and (olk.slot[wl.off[1]:] != NONE).all()
    assert used == [sum(map(len, donors)), 700 + outside]


def test_stored_once_with_a_full_pool_and_policies(G):
    """The free list runs out in the middle of a batch; LRU stamps, minimum length and zero fill are on."""
    rng = np.random.default_rng(9)
    V = lambda n: rng.integers(0, 32000, n).astype(np.uint32)  # noqa: E731
    doc = V(200)
    donors = [doc, np.concatenate([V(30), doc, V(40)]), np.concatenate([V(50), doc[:120], V(100)])]
    wl = gen.from_prompts("stored-once-full", 0xC0FFEE33, gen.KVShape(2, 2, 64), donors, [np.concatenate([V(5), doc, V(9)])],
                          pool_slots=512, donor_batch_tokens=300)
    wl.free_slots = wl.free_slots[:300]
    fl = []
    ost = OH.prefill(wl, flags_out=fl, anchor_window=4, dedup=True)
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=4, dedup=True, lru=True, min_len=16, zero_fill=True))
    assert fl[0] & O.FLAG_POOL_FULL and gst.flags == fl[0]
    assert np.array_equal(gst.donor_slot, ost.donor_slot) and sum(gst.n_inserted) == ost.n_used == 300
    olk, glk = OH.lookup(ost, min_len=16, zero_fill=True), G.lookup(gst)
    assert np.array_equal(glk.slot, olk.slot) and np.array_equal(glk.served, olk.served)
    assert np.array_equal(G.dst_as_rows(glk.dst, wl.shape, wl.n_tokens), olk.dst)


@pytest.mark.parametrize("block", range(3))
def test_random_life_cycles_with_evictions_stored_once(G, block):
    """Fifteen batches over vocabularies of two to six tokens through a pool that is too small for them, so that
    texts are found again, extended, evicted and stored anew; every output of every batch against the oracle."""
    from test_gpu_policies import Lifecycle

    evictions = 0
    for seed in range(block * 8, block * 8 + 8):
        rng = np.random.default_rng(77000 + seed)
        vocab = int(rng.choice([2, 3, 4, 6, 32000]))
        W = int(rng.choice([1, 2, 3, 5]))
        verify, min_len = bool(rng.integers(0, 2)), int(rng.integers(1, 6))
        marks, zf = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        S = int(rng.integers(80, 400))
        print("case", dict(seed=seed, vocab=vocab, W=W, verify=verify, min_len=min_len, marks=marks, zf=zf, S=S), flush=True)
        life = Lifecycle(G, S, gen.KVShape(1, 2, 64), 0xABE000 + seed, verify, min_len=min_len, marks=marks,
                         zero_fill=zf, anchor_window=W, dedup=True)
        corpus = [rng.integers(0, vocab, 50).astype(np.uint32) for _ in range(5)]
        for epoch in range(1, 16):
            parts = []
            for d in rng.choice(5, int(rng.integers(1, 4)), replace=False):
                lead = rng.integers(0, vocab, int(rng.integers(0, 5))).astype(np.uint32)
                a = int(rng.integers(0, 20))
                parts.append(np.concatenate([lead, corpus[d][a:a + int(rng.integers(1, 31))]]))
            if rng.random() < 0.2:
                parts.insert(int(rng.integers(0, len(parts) + 1)), np.zeros(0, np.uint32))  # an empty request
            tok = np.concatenate(parts).astype(np.uint32)
            mask = (rng.random(len(tok)) < rng.choice([0.0, 0.05, 0.3])).astype(np.uint8)
            off = np.concatenate([[0], np.cumsum([len(x) for x in parts])]).astype(np.uint32)
            life.batch(epoch, tok, mask, off, (rng.random(len(tok)) < 0.25).astype(np.uint8))
        evictions += life.evictions
    assert evictions > 0
