"""Exact verification of matches (Sec. 4.2.2 Step 2) on the GPU against the CPU oracle, including
crafted collisions of the mod-2^64 rolling hash (a Thue-Morse pair: two different 1024-token strings
with equal hashes), at lookup time, at insert time across batches and inside one batch."""
import numpy as np
import pytest

import oracle as O
from cp_workload import gen
from oracle import harness as OH
from test_gpu_parity import G, compare_all  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu

NONE = O.SLOT_NONE


def thue_morse_pair(k, x, y):
    bits = [0]
    for _ in range(k):
        bits = bits + [1 - b for b in bits]
    return (np.array([x if b == 0 else y for b in bits], np.uint32),
            np.array([y if b == 0 else x for b in bits], np.uint32))


def workload(donors, batches, requests, pool_slots=8192, sens=()):
    """Prompts given as explicit token lists; no sensitive tokens unless listed as (request, position)."""
    def pack(parts):
        off = np.zeros(len(parts) + 1, np.uint32)
        off[1:] = np.cumsum([len(p) for p in parts])
        return np.concatenate(parts).astype(np.uint32), off
    dt, doff = pack(donors)
    rt, roff = pack(requests)
    rmask = np.zeros(len(rt), np.uint8)
    for r, p in sens:
        rmask[int(roff[r]) + p] = 1
    rng = np.random.default_rng(99)
    return gen.Workload(name="crafted", seed=0xC0FFEE07, shape=gen.KVShape(2, 2, 64), tok=rt, mask=rmask, off=roff,
                        donor_tok=dt, donor_mask=np.zeros(len(dt), np.uint8), donor_off=doff, donor_batches=batches,
                        pool_slots=pool_slots, free_slots=rng.permutation(pool_slots).astype(np.uint32),
                        table_capacity=2 * pool_slots)


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("llama3-8b", {"scale": 1 / 16}), ("frag", {"scale": 1 / 32})])
def test_no_collisions_same_result_as_without_verification(G, name, kw):
    wl = gen.make(name, **kw)
    wl.shape = gen.KVShape(2, 2, 64)
    ost, olk, gst, glk = compare_all(G, wl, verify=True)
    plain = OH.lookup(OH.prefill(wl), gather=False)
    assert np.array_equal(olk.slot, plain.slot)
    assert (glk.slot != NONE).mean() > 0.3


@pytest.mark.parametrize("W", [2, 16])
def test_float_workload_verified(G, W):
    wl = gen.make("float", scale=0.5)
    wl.shape = gen.KVShape(2, 2, 64)
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=W, verify=True)
    plain = OH.lookup(OH.prefill(wl, anchor_window=W), gather=False)
    # every confirmed match is one the unverified lookup also reports
    hit = olk.slot != NONE
    assert np.array_equal(olk.slot[hit], plain.slot[hit])
    assert hit.mean() > 0.6
    # a token the unverified lookup serves through the run-start key of a run that later changes to a
    # floating key is still served: the two key streams are confirmed independently
    assert hit.sum() >= 0.95 * (plain.slot != NONE).sum()


def test_rope_verified(G):
    wl = gen.make_rope(scale=1 / 16, shape=gen.KVShape(2, 8, 128))
    ost, olk, gst, glk = compare_all(G, wl, verify=True)
    assert (glk.span_delta != 0).mean() > 0.8


def test_collision_at_lookup(G):
    t, c = thue_morse_pair(10, 7, 11)
    tail = np.array([5, 6, 7], np.uint32)
    wl = workload([np.concatenate([t, tail])], [(0, 1)], [np.concatenate([c, tail]), np.concatenate([t, tail])])
    ost, olk, gst, glk = compare_all(G, wl, verify=True)
    assert (glk.slot[:1027] == NONE).all() and (glk.slot[1027:] != NONE).all()
    # without verification both sides serve the other text's rows from token 1023 on
    ost2, olk2, gst2, glk2 = compare_all(G, wl)
    assert (glk2.slot[1023:1027] != NONE).all()


def test_collision_at_insert_across_batches(G):
    t, c = thue_morse_pair(10, 7, 11)
    a, b = np.concatenate([t, [5]]), np.concatenate([c, [5, 9]])
    q = np.concatenate([t, [5, 9]])
    wl = workload([a, b], [(0, 1), (1, 2)], [a, b, q])
    ost, olk, gst, glk = compare_all(G, wl, verify=True)
    na, nb = len(a), len(b)
    assert (gst.donor_slot[:na] != NONE).all()
    assert (gst.donor_slot[na:na + 1023] != NONE).all() and (gst.donor_slot[na + 1023:] == NONE).all()
    assert sum(gst.n_inserted) == na + 1023 + 1  # b's last token took a slot that can never match
    s = glk.slot
    assert (s[:na] != NONE).all()
    assert (s[na:na + 1023] != NONE).all() and (s[na + 1023:na + nb] == NONE).all()
    assert (s[na + nb:na + nb + 1025] != NONE).all() and s[na + nb + 1025] == NONE


def test_collision_inside_one_batch(G):
    t, c = thue_morse_pair(10, 7, 11)
    a, b = np.concatenate([t, [5]]), np.concatenate([c, [5, 9]])
    wl = workload([a, b], [(0, 2)], [b, a])
    ost, olk, gst, glk = compare_all(G, wl, verify=True)
    na = len(a)
    assert (gst.donor_slot[na + 1023:] == NONE).all() and sum(gst.n_inserted) == na + 1023 + 1
    assert (glk.slot[1023:len(b)] == NONE).all() and (glk.slot[len(b):] != NONE).all()


def test_verify_chain_edge_cases(G):
    import torch

    from paper_2605_23640_amd import binding as B
    dev = G.DEV
    i32 = lambda a: G.dev_i32(np.asarray(a, np.uint32))  # noqa: E731
    X = 0xFFFFFFFF
    slot_tok = i32([0] * 16)
    slot_parent = i32([B.PARENT_POISON] * 16)
    # trie by hand: 10 <- 11 <- 12 <- 13 holds "1 2 3 4"
    for s, (tk, par) in {10: (1, X), 11: (2, 10), 12: (3, 11), 13: (4, 12)}.items():
        slot_tok[s], slot_parent[s] = tk, par - (1 << 32) if par > 0x7FFFFFFF else par
    scratch = B.new_scratch(8, 0, dev)
    out = torch.full((7,), 77, dtype=torch.int32, device=dev)
    q, seg, cand = i32([1, 2, 7, 4, 1, 2, 3]), i32([0, 1, 2, 3, 0, 1, 2]), i32([10, 11, 12, 13, 10, 11, 12])
    B.cp_verify_chain(q, seg, cand, slot_tok, slot_parent, 16, False, out, scratch)
    assert list(G.host_u32(out)) == [10, 11, X, X, 10, 11, 12]
    # candidate out of range, candidate NONE, parent NONE in mid-segment, offsets that do not count up
    B.cp_verify_chain(i32([1, 2, 3]), i32([0, 1, 2]), i32([10, 99, 12]), slot_tok, slot_parent, 16, False, out[:3], scratch)
    assert list(G.host_u32(out[:3])) == [10, X, X]
    B.cp_verify_chain(i32([1, 2, 3]), i32([0, 2, 3]), i32([10, 12, 13]), slot_tok, slot_parent, 16, False, out[:3], scratch)
    assert list(G.host_u32(out[:3])) == [10, X, X]
    B.cp_verify_chain(i32([2, 3]), i32([1, 2]), i32([11, 12]), slot_tok, slot_parent, 16, False, out[:2], scratch)
    assert list(G.host_u32(out[:2])) == [X, X]  # offset 1 at token 0: no predecessor
    # merge keeps what the first stream found
    first = i32([X, 5, X])
    B.cp_verify_chain(i32([1, 2, 3]), i32([0, 1, 2]), i32([10, 11, 12]), slot_tok, slot_parent, 16, True, first, scratch)
    assert list(G.host_u32(first)) == [10, 5, 12]
    # same array for cand and slot_out is refused; N = 0 is a no-op
    with pytest.raises(B.CpError):
        B.cp_verify_chain(q, seg, cand, slot_tok, slot_parent, 16, False, cand, scratch)
    B.cp_verify_chain(q[:0], seg[:0], cand[:0], slot_tok, slot_parent, 16, False, out[:0], scratch)


def test_three_streams_in_one_call_equal_the_calls_one_by_one(G):
    """cp_verify_streams against cp_probe + cp_verify_chain per stream and the merge, on a workload where all
    three streams find something and on random candidate slots (most of which must be rejected)."""
    import torch
    import paper_2605_23640_amd as cp
    B = cp.binding
    wl = gen.make("float", scale=0.125)  # documents stored alone, quoted behind other text
    wl.shape = gen.KVShape(1, 2, 64)
    st = G.prefill(wl, G.make_pool(wl, anchor_window=4, verify=True))
    pool, N = st.pool, wl.n_tokens
    tok, mask, off = G.dev_i32(wl.tok), torch.from_numpy(wl.mask.copy()).to(G.DEV), G.dev_i32(wl.off)
    buf = cp.LookupBuffers(N, N, G.DEV, n_pool_slots=pool.n_slots)
    B.cp_hash_probe(tok, mask, off, pool.table, buf.hash, buf.run_off, buf.cand, buf.scratch)
    B.cp_hash_floating(pool.table, pool.slot_anchor, pool.n_slots, buf.hash, buf.run_off, 4, buf.hash_float, buf.scratch,
                       off_a_out=buf.float_off, hash_b_out=buf.hash_late, off_b_out=buf.late_off)
    rng = np.random.default_rng(4)
    for junk in (False, True):
        cand0 = buf.cand.clone()
        if junk:  # a third of the run-start candidates replaced by arbitrary slots
            r = torch.from_numpy(rng.integers(0, pool.n_slots, N).astype(np.int32)).to(G.DEV)
            pick = torch.from_numpy(rng.random(N) < 0.33).to(G.DEV)
            cand0 = torch.where(pick, r, cand0)
        want_slot = torch.empty(N, dtype=torch.int32, device=G.DEV)
        want_own = [torch.empty(N, dtype=torch.int32, device=G.DEV) for _ in range(3)]
        tmp = torch.empty(N, dtype=torch.int32, device=G.DEV)
        for k, (key, seg) in enumerate(((None, buf.run_off), (buf.hash_float, buf.float_off), (buf.hash_late, buf.late_off))):
            c = cand0 if k == 0 else B.cp_probe(pool.table, key, tmp)
            B.cp_verify_chain(tok, seg, c, pool.slot_tok, pool.slot_parent, pool.n_slots, k > 0, want_slot, buf.scratch,
                              stream_out=want_own[k])
        got_slot = torch.empty(N, dtype=torch.int32, device=G.DEV)
        got_own = [torch.empty(N, dtype=torch.int32, device=G.DEV) for _ in range(3)]
        B.cp_verify_streams(pool.table, tok, buf.run_off, cand0, buf.hash_float, buf.float_off, buf.hash_late, buf.late_off,
                            pool.slot_tok, pool.slot_parent, pool.n_slots, got_slot, buf.scratch, stream_out=got_own)
        torch.cuda.synchronize()
        assert torch.equal(got_slot, want_slot) and all(torch.equal(g, w) for g, w in zip(got_own, want_own))
        served = [(G.host_u32(w) != NONE).sum() for w in want_own]
        assert all(x > 0 for x in served[:2]), served  # (stream b serves where two stored texts overlap: not here)
