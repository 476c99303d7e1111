"""Parity at the full sizes of the benchmark configurations (Llama-3-8B shape,
fragmentation stress, RoPE-shift reuse, Llama-3-70B shape), in the launch
configuration bench.py times, and of one tensor-parallel rank's share of two of
them (one KV head per row).

Hashes, slots, spans, deltas and inserted slots are compared in full against
the CPU oracle (they do not depend on the KV shape, so the oracle runs them on
a one-layer stand-in pool).  KV bytes are checked everywhere on the device by
the generator's verify kernel: the oracle says which donor token owns each
slot and which slot serves each request token, the generator says what that
donor token's rows are, and every row of the pool and of the request buffers
must hold exactly that (or the untouched fill pattern).  Re-rotated keys are
compared on a seeded sample of tokens against the oracle's double-precision
rotation, one by one."""
import gc

import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen, kvgen
from oracle import harness as OH

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a ROCm device; there is no fallback path")
    from paper_2605_23640_amd import harness

    return harness


def bf16_ordinal(bits):
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def oracle_bookkeeping(wl):
    """Oracle prefill + lookup with a tiny stand-in KV shape (index, slots, spans only)."""
    import copy

    w = copy.copy(wl)
    w.shape = gen.KVShape(1, 1, 8)
    st = OH.prefill(w, src_provider=lambda t0, n: np.zeros((1, 2, n, 8), np.uint16))
    lk = OH.lookup(st, gather=False)
    return st, lk


def make_workload(name):
    """'llama3-70b' = the configuration; 'llama3-70b/1-head' = the same tokens, slots and spans with one KV head
    per row: what one rank of an 8-way tensor-parallel model holds (rows of 256 B, small tokens)."""
    base, _, share = name.partition("/")
    if not share:
        return gen.make(base)
    whole = gen.default_shape(base)
    return gen.make(base, shape=gen.KVShape(whole.n_layers, int(share.split("-")[0]), whole.head_dim))


@pytest.mark.parametrize("name", ["llama3-8b", "frag", "rope", "llama3-70b", "llama3-70b/1-head", "rope/1-head"])
def test_full_size(G, name):
    wl = make_workload(name)
    sh, N = wl.shape, wl.n_tokens
    print(f"\n[{name}] {wl.n_requests} requests x {N // wl.n_requests} tokens, pool "
          f"{wl.pool_slots * sh.tok_bytes / 2**30:.0f} GiB, request buffers {N * sh.tok_bytes / 2**30:.0f} GiB", flush=True)
    ost, olk = oracle_bookkeeping(wl)
    gst = G.prefill(wl)
    print(f"[{name}] prefilled {sum(gst.n_inserted)} tokens", flush=True)
    assert np.array_equal(gst.donor_hash, ost.donor_hash)
    assert np.array_equal(gst.donor_slot, ost.donor_slot)
    assert sum(gst.n_inserted) == ost.n_used and gst.flags == 0
    stored = ost.slot_uid != kvgen.UID_NONE
    assert np.array_equal(gst.pool.slot_pos.cpu().numpy()[stored], ost.slot_pos[stored])
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0  # the whole pool
    glk = G.lookup(gst)
    print(f"[{name}] lookup: {glk.n_spans} spans, {(glk.slot != O.SLOT_NONE).sum()} tokens served", flush=True)
    assert np.array_equal(glk.hash, olk.hash) and np.array_equal(glk.slot, olk.slot)
    assert glk.n_spans == olk.n_spans and glk.flags == 0
    for f in ("span_src", "span_dst", "span_len"):
        assert np.array_equal(getattr(glk, f), getattr(olk, f)), f
    served = olk.slot != O.SLOT_NONE
    assert (olk.slot[wl.mask == 1] == O.SLOT_NONE).all()  # no sensitive token is served
    # expected owner (donor token) of every request row; unmatched rows must still hold the fill pattern
    uid = np.full(N, kvgen.UID_NONE, np.uint64)
    uid[served] = ost.slot_uid[olk.slot[served]]
    lay = gst.pool.request_layout(N)
    if wl.rope_theta is None:
        assert G.verify_rows(glk.dst, lay, uid, wl.seed) == 0  # every row of the request buffers
    else:
        assert np.array_equal(glk.span_delta, olk.span_delta)
        delta = np.zeros(N, np.int32)
        for d, l, dl in zip(olk.span_dst, olk.span_len, olk.span_delta):
            delta[d:d + l] = dl
        rotated = served & (delta != 0)
        # V rows everywhere and K rows of unshifted tokens: exact generator bytes
        assert G.verify_rows(glk.dst, lay, uid, wl.seed, skip_k=rotated.astype(np.uint8)) == 0
        # K rows against the oracle's rotation on a stratified sample: one token of every re-rotated stretch of
        # every request (every reused run has a position delta of its own: some three thousand (request, delta)
        # pairs), at most 4000 of them, in the first, the middle and the last layer, every head
        rng = np.random.default_rng(wl.seed)
        req_of = np.searchsorted(wl.off, np.arange(N), side="right") - 1
        run_start = np.flatnonzero(rotated & ~np.concatenate([[False], rotated[:-1] & (delta[1:] == delta[:-1])
                                                               & (req_of[1:] == req_of[:-1])]))
        run_end = np.concatenate([run_start[1:], [N]])
        picks = []
        for a, b in zip(run_start, run_end):  # a stretch of one delta: tokens a .. (first token that differs)
            e = a
            while e < b and rotated[e] and delta[e] == delta[a] and req_of[e] == req_of[a]:
                e += 1
            picks.append(int(rng.integers(a, e)))
        picks = np.array(picks)
        if len(picks) > 4000:
            picks = np.sort(rng.choice(picks, 4000, replace=False))
        idx = picks
        n_pairs = len({(int(req_of[i]), int(delta[i])) for i in idx})
        layers = sorted({0, sh.n_layers // 2, sh.n_layers - 1})
        re = sh.row_bytes // 2
        view = glk.dst.view(torch.int16).view(sh.n_layers, 2, N, re)
        t_idx = torch.from_numpy(idx).to(G.DEV)
        got = np.stack([view[l, 0, t_idx, :].cpu().numpy().view(np.uint16) for l in layers])  # [layer][sample][re]
        src = kvgen.rows_for_tokens(wl.seed, uid[idx], sh.n_layers, re)[:, layers, 0, :]  # [sample][layer][re]
        D = sh.head_dim
        hist = np.zeros((len(layers), 3), np.int64)
        by_size = {}  # |delta| bucket -> histogram
        for s_, i in enumerate(idx):
            for li in range(len(layers)):
                for h in range(sh.n_kv_heads):
                    want = O.rope_head(src[s_, li, h * D:(h + 1) * D], int(delta[i]), wl.rope_theta, wl.rope_style)
                    d = np.abs(bf16_ordinal(got[li, s_, h * D:(h + 1) * D]) - bf16_ordinal(want))
                    b = np.bincount(np.minimum(d, 2), minlength=3)
                    hist[li] += b
                    key = min(int(abs(int(delta[i]))).bit_length(), 12)
                    by_size[key] = by_size.get(key, 0) + b
        print(f"[{name}] {len(idx)} sampled tokens, {n_pairs} (request, delta) pairs, requests {len(set(req_of[idx]))}, "
              f"deltas {int(delta[idx].min())} .. {int(delta[idx].max())}", flush=True)
        for li, l in enumerate(layers):
            print(f"[{name}]   layer {l}: bf16 distance {{0,1,>1}} {hist[li].tolist()}", flush=True)
        for k in sorted(by_size):
            print(f"[{name}]   |delta| < 2^{k}: {by_size[k].tolist()}", flush=True)
        assert len(idx) >= 2500 and n_pairs >= 2500 and len(set(req_of[idx])) == wl.n_requests
        assert hist[:, 2].sum() == 0  # every element within one bf16 step of the double-precision result
        assert hist[:, 1].sum() <= 1e-3 * hist.sum()
    del gst, glk
    gc.collect()
    torch.cuda.empty_cache()


def test_full_size_float_anchors_verified_policies(G):
    """The rows added beyond the base path at the 8B size: floating anchors (W = 16), exact
    verification, minimum stretch length, recompute marks, zero placeholders."""
    import copy

    W, min_len, rho = 16, 32, 0.25
    wl = gen.make("float")
    sh, N = wl.shape, wl.n_tokens
    rec = (wl.donor_u < rho).astype(np.uint8)
    w = copy.copy(wl)
    w.shape = gen.KVShape(1, 1, 8)
    ost = OH.prefill(w, src_provider=lambda t0, n: np.zeros((1, 2, n, 8), np.uint16), anchor_window=W, verify=True,
                     recompute=rec)
    olk = OH.lookup(ost, gather=False, min_len=min_len)
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=W, verify=True, min_len=min_len, recompute_marks=True,
                                    zero_fill=True), recompute=rec)
    print(f"\n[float] prefilled {sum(gst.n_inserted)} tokens", flush=True)
    assert np.array_equal(gst.donor_hash, ost.donor_hash) and np.array_equal(gst.donor_slot, ost.donor_slot)
    assert sum(gst.n_inserted) == ost.n_used and gst.flags == 0
    assert np.array_equal(gst.pool.slot_recompute.cpu().numpy(), ost.marks)
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0
    glk = G.lookup(gst)
    for f in ("hash", "hash_float", "hash_late", "run_off", "slot", "served", "span_src", "span_dst", "span_len"):
        assert np.array_equal(getattr(glk, f), getattr(olk, f)), f
    served = olk.served != O.SLOT_NONE
    matched = olk.slot != O.SLOT_NONE
    floating = matched & (O.probe(ost.index, olk.hash) == O.SLOT_NONE)
    print(f"[float] matched {matched.sum()} ({floating.sum()} through floating keys), served {served.sum()}, "
          f"{glk.n_spans} spans", flush=True)
    assert floating.sum() > 0.2 * N and 0.5 * matched.sum() < served.sum() < 0.8 * matched.sum()
    # served rows hold the owner's rows; every other row is zero
    uid = np.full(N, kvgen.UID_NONE, np.uint64)
    uid[served] = ost.slot_uid[olk.served[served]]
    lay = gst.pool.request_layout(N)
    view = glk.dst.view(torch.int16).view(sh.n_layers, 2, N, sh.row_bytes // 2)
    rest = torch.from_numpy(np.flatnonzero(~served)).to(G.DEV)
    for l in range(sh.n_layers):
        assert not bool(view[l][:, rest, :].any()), l
    # the verify kernel expects the fill pattern where no owner is named: put it back over the zero rows
    pat = int(np.array([kvgen.POISON16], np.uint16).view(np.int16)[0])
    for l in range(sh.n_layers):
        view[l][:, rest, :] = pat
    assert G.verify_rows(glk.dst, lay, uid, wl.seed) == 0
    del gst, glk, view
    gc.collect()
    torch.cuda.empty_cache()


def test_more_than_256_scan_tiles(G):
    """About 600,000 tokens in one batch: the ordered scans run over some 2,300 tiles, more than the two-launch form
    takes, so they use the three-launch form whose single-workgroup carry pass loops over several chunks of 256 tile
    totals (the configurations above stay within the two-launch form).
    Tiny KV rows; floating anchors, verification, minimum length and marks on, so every scan takes part."""
    from test_gpu_parity import compare_all

    rng = np.random.default_rng(0xC0FFEE0A)
    docs = [rng.integers(0, gen.VOCAB, 30000).astype(np.uint32) for _ in range(12)]
    dmask = [(rng.random(30000) < 0.02).astype(np.uint8) for _ in range(12)]
    parts_t, parts_m = [], []
    for r in range(50):
        pt, pm = [], []
        for d in rng.choice(12, 3, replace=False):
            a = int(rng.integers(0, 20000))
            ln = int(rng.integers(2000, 6000))
            lead = int(rng.integers(0, 30))
            pt += [rng.integers(0, gen.VOCAB, lead).astype(np.uint32), docs[d][a:a + ln]]
            pm += [np.zeros(lead, np.uint8), dmask[d][a:a + ln]]
        parts_t.append(np.concatenate(pt))
        parts_m.append(np.concatenate(pm))
    tok, mask = np.concatenate(parts_t), np.concatenate(parts_m)
    off = np.concatenate([[0], np.cumsum([len(p) for p in parts_t])]).astype(np.uint32)
    dtok, dm = np.concatenate(docs), np.concatenate(dmask)
    doff = (np.arange(13) * 30000).astype(np.uint32)
    S = 1 << 19
    wl = gen.Workload(name="many-tiles", seed=0xC0FFEE0A, shape=gen.KVShape(1, 1, 8), tok=tok, mask=mask, off=off,
                      donor_tok=dtok, donor_mask=dm, donor_off=doff, donor_batches=[(0, 12)], pool_slots=S,
                      free_slots=rng.permutation(S).astype(np.uint32), table_capacity=2 * S,
                      donor_u=rng.random(len(dtok), dtype=np.float32))
    assert wl.n_tokens > 256 * 1024 * 2 and len(dtok) > 256 * 1024
    rec = (wl.donor_u < 0.25).astype(np.uint8)
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=16, verify=True, min_len=24, recompute=rec, zero_fill=True)
    print(f"\n[many-tiles] {wl.n_tokens} tokens, {(olk.slot != O.SLOT_NONE).sum()} matched, "
          f"{(olk.served != O.SLOT_NONE).sum()} served, {olk.n_spans} spans", flush=True)
    assert (olk.served != O.SLOT_NONE).sum() > 100000


@pytest.mark.parametrize("all_rows", [False, True])
def test_pool_life_cycle_at_pool_scale(G, all_rows):
    """The pool of the 8B configuration (262,144 slots) through twelve batches of 16 x 4096 tokens drawn from a
    corpus larger than the pool: it fills up and least-recently-used batches are evicted several times.  Every
    output of every batch (slots, served slots, request buffers, stamps, marks, freed lists, thresholds, free
    list, flags) is compared with the oracle; KV rows are small so that the host can mirror the pool.
    ``all_rows``: floating anchors, exact verification, minimum length, recompute marks and zero fill on."""
    from test_gpu_policies import Lifecycle

    rng = np.random.default_rng(0xC0FFEE0B)
    S = 262144
    life = Lifecycle(G, S, gen.KVShape(1, 1, 64), 0xC0FFEE0B, verify=all_rows, min_len=32 if all_rows else 1,
                     marks=all_rows, zero_fill=all_rows, anchor_window=16 if all_rows else None)
    prefix = rng.integers(0, gen.VOCAB, 1024).astype(np.uint32)
    docs = [rng.integers(0, gen.VOCAB, int(rng.integers(512, 1025))).astype(np.uint32) for _ in range(450)]
    dmask = [(rng.random(len(d)) < 0.02).astype(np.uint8) for d in docs]
    drec = [(rng.random(len(d)) < 0.25).astype(np.uint8) for d in docs]  # marks travel with the text
    for epoch in range(1, 13):
        pt, pm, pr, lens = [], [], [], []
        recent = rng.choice(450, 120, replace=False)  # this batch's working set: some documents stay hot
        for r in range(16):
            lead = int(rng.integers(0, 40)) if all_rows else 0  # text in front of the first document
            t, m, c = [prefix, rng.integers(0, gen.VOCAB, lead).astype(np.uint32)], [np.zeros(1024 + lead, np.uint8)], \
                [np.zeros(1024 + lead, np.uint8)]
            for d in rng.choice(recent, 3, replace=False):
                t.append(docs[d]), m.append(dmask[d]), c.append(drec[d])
            n = sum(len(x) for x in t)
            t.append(rng.integers(0, gen.VOCAB, 4096 - n).astype(np.uint32))
            um = (rng.random(4096 - n) < 0.15).astype(np.uint8)
            um[0] = 1  # the user's text starts with a sensitive token: it never extends a document's run
            m.append(um), c.append(np.zeros(4096 - n, np.uint8))
            pt.append(np.concatenate(t)), pm.append(np.concatenate(m)), pr.append(np.concatenate(c)), lens.append(4096)
        tok, mask, rec = np.concatenate(pt).astype(np.uint32), np.concatenate(pm), np.concatenate(pr)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
        life.batch(epoch, tok, mask, off, rec)
        print("epoch", epoch, "free", len(life.free), "evictions", life.evictions, flush=True)
    assert life.evictions >= 2 and life.flags == 0
