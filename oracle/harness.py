"""Runs a synthetic workload through the CPU oracle: pool prefill from the donor
prompts, then the lookup path on the request batch.

TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark CPU-baseline leg).
Host buffers are laid out like the GPU side's so results compare directly:
the pool is token-major  uint16[slot][layer][K|V][row_elems], request / donor
buffers are layer-major  uint16[layer][K|V][token][row_elems].
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field

import numpy as np

import oracle as O
from cp_workload import kvgen


def pool_layout(shape) -> O.Layout:
    rb = shape.row_bytes
    return O.Layout(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.tok_bytes, 2 * rb, rb)


def buf_layout(shape, n_tok) -> O.Layout:
    rb = shape.row_bytes
    return O.Layout(shape.n_layers, shape.n_kv_heads, shape.head_dim, rb, 2 * n_tok * rb, n_tok * rb)


def gen_buffer(seed, shape, uid0, n_tok):
    """Layer-major buffer of n_tok tokens with uids uid0 .. uid0+n_tok-1 (host generator)."""
    re = shape.row_bytes // 2
    rows = kvgen.rows_for_tokens(seed, range(uid0, uid0 + n_tok), shape.n_layers, re)  # [t][l][kv][e]
    return np.ascontiguousarray(rows.transpose(1, 2, 0, 3))


@dataclass
class OracleState:
    wl: object
    index: O.Index
    pool: np.ndarray  # uint16[slots][L][2][row_elems]
    slot_pos: np.ndarray  # int32[slots]
    slot_tok: np.ndarray  # uint32[slots], audit: token id stored in the slot
    slot_uid: np.ndarray  # uint64[slots], audit: donor token (packed donor index) that filled the slot
    n_used: int = 0  # free-list entries consumed
    donor_hash: np.ndarray | None = None
    donor_slot: np.ndarray | None = None  # slot_out of every donor token
    times: dict = field(default_factory=dict)
    anchors: O.AnchorSet | None = None  # floating anchors: hashes of the stored runs' first W tokens
    anchor_window: int | None = None
    text: O.Text | None = None  # exact verification: the token string every slot was stored for
    marks: np.ndarray | None = None  # uint8 per slot: recompute marks


def prefill(wl, src_provider=None, pool=None, flags_out=None, anchor_window=None, verify=False,
            recompute=None, dedup=False, bounded_table=False) -> OracleState:
    """Insert the donor prompts batch by batch.  ``src_provider(first_tok, n_tok)``
    returns the layer-major KV buffer of a donor batch (default: host generator,
    uid = packed donor index).  With ``anchor_window`` = W the hash of every
    stored run's first W tokens is also recorded as a floating anchor; with
    ``verify`` the pool records every slot's text and reports only confirmed slots."""
    sh = wl.shape
    re = sh.row_bytes // 2
    if pool is None:
        pool = np.full((wl.pool_slots, sh.n_layers, 2, re), kvgen.POISON16, np.uint16)
    st = OracleState(
        wl=wl, index=O.Index(), pool=pool,
        slot_pos=np.full(wl.pool_slots, np.iinfo(np.int32).min, np.int32),
        slot_tok=np.full(wl.pool_slots, 0xFFFFFFFF, np.uint32),
        slot_uid=np.full(wl.pool_slots, kvgen.UID_NONE, np.uint64),
    )
    if bounded_table:  # the index as a table of the workload's capacity (in whole buckets of 16 entries)
        st.index.rebuild((int(wl.table_capacity) + 15) // 16 * 16)
    base = O.BASE if wl.hash_base is None else wl.hash_base
    st.donor_hash = O.hash_segments(wl.donor_tok, wl.donor_mask, wl.donor_off, base)
    if anchor_window is not None:
        st.anchors, st.anchor_window = O.AnchorSet(), int(anchor_window)
    if verify:
        st.text = O.Text(wl.pool_slots)
    if recompute is not None:  # uint8 per donor token: the annotator's recompute marks
        st.marks = np.zeros(wl.pool_slots, np.uint8)
    st.donor_slot = np.full(len(wl.donor_tok), O.SLOT_NONE, np.uint32)
    flags = 0
    for first, last in wl.donor_batches:
        t0, t1 = int(wl.donor_off[first]), int(wl.donor_off[last])
        n = t1 - t0
        src = src_provider(t0, n) if src_provider else gen_buffer(wl.seed, sh, t0, n)
        off = (wl.donor_off[first : last + 1] - wl.donor_off[first]).astype(np.uint32)
        before = st.n_used
        b_tok, b_mask, b_hash = wl.donor_tok[t0:t1], wl.donor_mask[t0:t1], st.donor_hash[t0:t1]
        b_roff = O.run_offsets(b_mask, off)
        if dedup:  # every text once: look the batch up first, leave out what the pool has (Sec. 4.3.5)
            streams = O.match_streams(st.index, b_tok, b_hash, b_roff, st.anchors, st.anchor_window, st.text,
                                      with_offsets=True, base=base)
            ins_hash, ins_off, found = O.insert_keys(b_hash, b_roff, streams, base)
            slot_out, n_new, fl = O.insert_kv_dedup(
                st.index, ins_hash, found, off, wl.free_slots[st.n_used :], src, buf_layout(sh, n), st.pool,
                pool_layout(sh), st.slot_pos, tok=b_tok, slot_tok=st.slot_tok)
            raw = slot_out
            if st.text is not None:
                slot_out = O.text_record_dedup(st.text, b_tok, ins_off, found, raw)
            st.donor_hash[t0:t1] = ins_hash
            b_hash, b_roff = ins_hash, ins_off
        else:
            slot_out, n_new, fl = O.insert_kv(
                st.index, b_hash, off, wl.free_slots[st.n_used :], src, buf_layout(sh, n), st.pool,
                pool_layout(sh), st.slot_pos, tok=b_tok, slot_tok=st.slot_tok)
            if st.text is not None:
                raw = slot_out
                slot_out = O.text_record(st.text, b_tok, b_roff, raw)
        if st.marks is not None:
            O.mark_recompute(slot_out, recompute[t0:t1], st.marks)
        if st.anchors is not None:
            O.insert_anchors(st.anchors, b_hash, b_roff, slot_out, st.anchor_window)
        st.donor_slot[t0:t1] = slot_out
        st.n_used += n_new
        flags |= fl
        # the tokens that took a new slot are exactly those whose slot is one handed out in this call
        new_slots = set(int(s) for s in wl.free_slots[before : st.n_used])
        seen = set()
        for i in range(n):
            s = int(raw[i]) if st.text is not None else int(slot_out[i])
            if s in new_slots and s not in seen:
                seen.add(s)
                st.slot_uid[s] = t0 + i
    if flags_out is not None:
        flags_out.append(flags)
    return st


@dataclass
class Lookup:
    hash: np.ndarray
    slot: np.ndarray
    span_src: np.ndarray
    span_dst: np.ndarray
    span_len: np.ndarray
    span_delta: np.ndarray
    n_spans: int
    flags: int
    dst: np.ndarray | None  # uint16[L][2][N][row_elems]
    times: dict
    hash_float: np.ndarray | None = None  # keys of candidate stream a (pools with floating anchors)
    run_off: np.ndarray | None = None
    served: np.ndarray | None = None  # slots after minimum length / recompute marks
    hash_late: np.ndarray | None = None  # keys of candidate stream b


def lookup(st: OracleState, tok=None, mask=None, off=None, gather=True, max_spans=None, min_len=1,
           zero_fill=False) -> Lookup:
    """Hash, probe, span building and gather for the request batch (timed per step)."""
    wl, sh = st.wl, st.wl.shape
    tok = wl.tok if tok is None else tok
    mask = wl.mask if mask is None else mask
    off = wl.off if off is None else off
    N = len(tok)
    re = sh.row_bytes // 2
    times = {}
    t = time.perf_counter()
    base = O.BASE if wl.hash_base is None else wl.hash_base
    h = O.hash_segments(tok, mask, off, base)
    times["hash"] = time.perf_counter() - t
    hf = hl = roff = None
    t = time.perf_counter()
    if st.text is None and st.anchors is None:
        slot = O.probe(st.index, h)
    else:
        roff = O.run_offsets(mask, off)
        if st.anchors is not None:
            hf, _, hl, _ = O.hash_floating(st.anchors, st.index, h, roff, st.anchor_window, base)
        slot = O.merge_streams(O.match_streams(st.index, tok, h, roff, st.anchors, st.anchor_window, st.text, base=base))
    times["probe"] = time.perf_counter() - t
    use_rope = wl.rope_theta is not None
    served = slot
    if min_len > 1 or st.marks is not None:
        t = time.perf_counter()
        served = O.filter_matches(slot, off, min_len, st.marks)
        times["filter"] = time.perf_counter() - t
    t = time.perf_counter()
    src, dst, ln, delta, n, fl = O.build_spans(served, off, st.slot_pos if use_rope else None, max_spans)
    times["spans"] = time.perf_counter() - t
    buf = None
    if gather:
        buf = np.full((sh.n_layers, 2, N, re), kvgen.POISON16, np.uint16)
        rope = O.Rope(wl.rope_theta, wl.rope_style) if use_rope else None
        t = time.perf_counter()
        O.gather_kv(st.pool, pool_layout(sh), buf, buf_layout(sh, N), src, dst, ln, delta if use_rope else None, rope)
        times["gather"] = time.perf_counter() - t
        if zero_fill:
            t = time.perf_counter()
            O.fill_unmatched(served, buf, buf_layout(sh, N))
            times["fill"] = time.perf_counter() - t
    return Lookup(h, slot, src, dst, ln, delta, n, fl, buf, times, hf, roff, served, hl)
