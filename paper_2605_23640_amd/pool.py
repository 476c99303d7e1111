"""A token-granular KV pool on one GPU: device memory (torch) plus the call
sequences of the two paths through libcacheprune.

    lookup :  cp_hash_segments -> cp_probe -> cp_build_spans -> cp_gather_kv
    insert :  cp_hash_segments -> cp_insert_kv

(the first two steps of the lookup are issued as one call, cp_hash_probe) and, for a pool with floating anchors
(window W),

    lookup :  cp_hash_runs -> cp_hash_floating -> cp_probe3 -> cp_build_spans -> cp_gather_kv
    insert :  cp_hash_runs -> cp_insert_kv -> cp_insert_anchors

and, for a pool that confirms every match exactly (``verify=True``),

    lookup :  cp_hash_probe (hashes, run offsets, candidates) -> cp_verify_chain -> cp_build_spans -> cp_gather_kv
              with floating anchors: cp_hash_probe -> cp_hash_floating -> cp_verify_streams (the three key
              streams probed and confirmed in one call) -> cp_build_spans -> cp_gather_kv
    insert :  cp_hash_runs -> cp_insert_kv_chain [-> cp_insert_anchors]

and, for a pool that stores every text once (``dedup=True``),

    insert :  the lookup's matching (every key stream's own finds) -> cp_insert_keys -> cp_insert_kv_dedup
              -> cp_insert_anchors

Policies hook in after the slots are known: cp_touch (LRU stamps), cp_filter_matches (minimum
length, recompute marks) before cp_build_spans, cp_fill_unmatched after the gather;
cp_mark_recompute / cp_touch after an insert; ``evict`` = cp_lru_threshold -> cp_evict.

Nothing here computes: tensors are allocated and handed to the C ABI.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


@dataclass
class LookupResult:
    hash: torch.Tensor  # int64[N]
    slot: torch.Tensor  # int32[N]
    span_src: torch.Tensor  # int32[max_spans]
    span_dst: torch.Tensor
    span_len: torch.Tensor
    span_delta: torch.Tensor
    span_off: torch.Tensor  # int32[max_spans + 1]
    n_spans: torch.Tensor  # int32[1], device
    served: torch.Tensor = None  # int32[N]: slot of the tokens that pass the pool's policies (slot itself without policies)


class LookupBuffers:
    """Reusable per-batch device arrays for the lookup path (N tokens, up to max_spans spans)."""

    def __init__(self, N, max_spans=None, device="cuda", n_pool_slots=0):
        self.N = N
        self.max_spans = N if max_spans is None else max_spans
        i32, i64 = torch.int32, torch.int64
        self.hash = torch.empty(N, dtype=i64, device=device)
        # floating anchors (if the pool uses them): keys of the two candidate streams (hash_float: stream a, hash_late: stream b)
        self.hash_float = torch.empty(N, dtype=i64, device=device)
        self.hash_late = torch.empty(N, dtype=i64, device=device)
        self.run_off = torch.empty(N, dtype=i32, device=device)
        self.float_off = torch.empty(N, dtype=i32, device=device)
        self.late_off = torch.empty(N, dtype=i32, device=device)
        self.cand = torch.empty(N, dtype=i32, device=device)  # unconfirmed slots (pools that verify)
        self.slot = torch.empty(N, dtype=i32, device=device)  # slot of every matched token
        # what each key stream alone found / accepted (run-start keys, candidate stream a, candidate stream b)
        self.stream_slot = [torch.empty(N, dtype=i32, device=device) for _ in range(3)]
        # storing every text once: key, offset in its stored text and "the pool has it" per token
        self.ins_hash = torch.empty(N, dtype=i64, device=device)
        self.ins_off = torch.empty(N, dtype=i32, device=device)
        self.found = torch.empty(N, dtype=i32, device=device)
        self.served = torch.empty(N, dtype=i32, device=device)  # ... of those that pass the pool's policies
        m = max(1, self.max_spans)
        self.span_src = torch.empty(m, dtype=i32, device=device)
        self.span_dst = torch.empty(m, dtype=i32, device=device)
        self.span_len = torch.empty(m, dtype=i32, device=device)
        self.span_delta = torch.empty(m, dtype=i32, device=device)
        self.span_off = torch.empty(m + 1, dtype=i32, device=device)
        self.n_spans = torch.zeros(1, dtype=i32, device=device)
        self.scratch = B.new_scratch(max(N, 1), self.max_spans, device, n_pool_slots)


class KVPool:
    """Pool of ``n_slots`` token slots (token-major rows), its hash table, the
    cached position of every slot and the free list (hand-out order)."""

    def __init__(self, n_layers, n_kv_heads, head_dim, n_slots, table_capacity, free_slots, rope=None,
                 device="cuda", pool_tensor=None, anchor_window=None, verify=False,
                 min_len=1, recompute_marks=False, zero_fill=False, lru=False, pool_layout="token",
                 gather_opts=None, insert_opts=None, dedup=False, hash_base=None):
        self.device = device
        # base of the chain hash (Sec. 4.2.2 draws it at random); None: the library's default
        self.hash_base = B.BASE if hash_base is None else int(hash_base)
        # launch options (binding.LaunchOpts or None = defaults) handed to every gather / insert of this pool
        self.gather_opts, self.insert_opts = gather_opts, insert_opts
        self.n_slots = int(n_slots)
        # store a text once: what a lookup of the batch finds (also behind other text, through the floating
        # anchors) is not stored again, and new tokens continue the stored text before them
        self.dedup = bool(dedup)
        assert not dedup or anchor_window is not None, "dedup needs floating anchors (anchor_window)"
        # "token": [slot][layer][K|V][head][dim], a token's rows are contiguous (the default);
        # "layer": [layer][K|V][slot][head][dim], every row of a token lies in another plane (for comparison)
        assert pool_layout in ("token", "layer")
        self.layout = (B.KVLayout.token_major(n_layers, n_kv_heads, head_dim) if pool_layout == "token"
                       else B.KVLayout.layer_major(n_layers, n_kv_heads, head_dim, self.n_slots))
        self.shape = (n_layers, n_kv_heads, head_dim)
        if pool_tensor is None:
            pool_tensor = torch.empty(self.n_slots * 2 * n_layers * n_kv_heads * head_dim * 2, dtype=torch.uint8,
                                      device=device)
        self.pool = pool_tensor
        self.table = B.Table((int(table_capacity) + B.TABLE_BUCKET - 1) // B.TABLE_BUCKET * B.TABLE_BUCKET, device)
        self.slot_pos = torch.zeros(self.n_slots, dtype=torch.int32, device=device)
        self.free_slots = free_slots.to(device=device, dtype=torch.int32).contiguous()
        self.n_used = 0  # free-list entries handed out so far (host copy)
        self.flags = torch.zeros(1, dtype=torch.int32, device=device)
        self.n_inserted = torch.zeros(1, dtype=torch.int32, device=device)
        self.rope = rope  # binding.Rope or None
        # floating anchors: window length W (None: run-start keys only) and one mark per slot; the keys of the
        # marked slots are the stored runs' prefix hashes
        self.anchor_window = anchor_window
        self.slot_anchor = None
        if anchor_window is not None:
            self.slot_anchor = torch.zeros(self.n_slots, dtype=torch.uint8, device=device)

        # exact verification: per slot, the token it was stored for and the slot of its predecessor in the run
        self.verify = bool(verify)
        self.slot_tok = self.slot_parent = None
        if self.verify:
            self.slot_tok = torch.zeros(self.n_slots, dtype=torch.int32, device=device)
            self.slot_parent = torch.full((self.n_slots,), B.PARENT_POISON - (1 << 32), dtype=torch.int32, device=device)
        # policies: minimum length of a reused stretch, per-slot recompute marks, zero placeholders for tokens
        # that are not served, least-recently-used eviction by batch number (epoch)
        self.min_len = int(min_len)
        self.slot_recompute = torch.zeros(self.n_slots, dtype=torch.uint8, device=device) if recompute_marks else None
        self.zero_fill = bool(zero_fill)
        self.slot_stamp = torch.zeros(self.n_slots, dtype=torch.int32, device=device) if lru else None
        self.epoch = 1
        self.threshold = torch.zeros(1, dtype=torch.int32, device=device)
        self.n_freed = torch.zeros(1, dtype=torch.int32, device=device)

    @property
    def filters(self):
        return self.min_len > 1 or self.slot_recompute is not None

    def n_free(self):
        return self.free_slots.numel() - self.n_used

    def evict(self, n_needed, scratch, stream=None, compact=True):
        """Free at least ``n_needed`` slots, least recently used batches first (whole batches
        at a time); the freed slots go to the end of the free list.  Reads one count back.
        With ``compact`` the live entries then move to a fresh table, so that the keys of
        evicted slots do not pile up and fill it."""
        assert self.slot_stamp is not None, "pool was created without lru=True"
        freed = torch.empty(self.n_slots, dtype=torch.int32, device=self.device)
        B.cp_lru_threshold(self.slot_stamp, self.n_slots, self.epoch, n_needed, self.threshold, scratch, stream=stream)
        B.cp_evict(self.table, self.slot_stamp, self.n_slots, self.threshold, freed, self.n_freed, self.slot_parent,
                   self.slot_recompute, self.slot_anchor, scratch, stream=stream)
        old = self.table
        if compact:
            fresh = B.Table(self.table.capacity, self.device, stream=stream)
            B.cp_table_compact(self.table, fresh, self.flags, stream=stream)
            self.table = fresh
        # the count is read on the host: wait for the stream the kernels were enqueued on (it need not
        # be torch's current one), which also keeps the old table's memory alive until they are done
        (torch.cuda.current_stream() if stream is None else stream).synchronize()
        del old
        n = int(self.n_freed.item())
        self.free_slots = torch.cat([self.free_slots[self.n_used:], freed[:n]])
        self.n_used = 0
        return freed[:n]

    def request_layout(self, n_tokens):
        L, H, D = self.shape
        return B.KVLayout.layer_major(L, H, D, n_tokens)

    def hash(self, tok, mask, off, out, scratch, stream=None):
        return B.cp_hash_segments(tok, mask, off, out, scratch, base=self.hash_base, stream=stream)

    def _match(self, tok, mask, off, buf: LookupBuffers, stream, per_stream, touch):
        """Hashes and slots of a batch: buf.slot = slot serving every token.  Returns the key streams as
        (offset of every token in its segment, that stream's own finds) in serving order; the finds are
        only filled in with ``per_stream`` (LRU stamps and storing-once need them).  ``touch``: stamp what
        the candidate streams found (the merged result is stamped by the caller)."""
        lru = touch and self.slot_stamp is not None
        if self.slot_anchor is None and not self.verify:
            B.cp_hash_probe(tok, mask, off, self.table, buf.hash, None, buf.slot, buf.scratch, base=self.hash_base,
                            stream=stream)
            return [(None, buf.slot)]
        if self.verify:  # the run-start stream's candidates come with the hashes
            B.cp_hash_probe(tok, mask, off, self.table, buf.hash, buf.run_off, buf.cand, buf.scratch,
                            base=self.hash_base, stream=stream)
        else:
            B.cp_hash_runs(tok, mask, off, buf.hash, buf.run_off, buf.scratch, base=self.hash_base, stream=stream)
        keys = [(buf.hash, buf.run_off)]
        if self.slot_anchor is not None:
            B.cp_hash_floating(self.table, self.slot_anchor, self.n_slots, buf.hash, buf.run_off, self.anchor_window,
                               buf.hash_float, buf.scratch, base=self.hash_base, stream=stream, off_a_out=buf.float_off,
                               hash_b_out=buf.hash_late, off_b_out=buf.late_off)
            keys += [(buf.hash_float, buf.float_off), (buf.hash_late, buf.late_off)]
        if self.verify and len(keys) == 3:  # the three streams confirmed in one pass
            B.cp_verify_streams(self.table, tok, buf.run_off, buf.cand, buf.hash_float, buf.float_off, buf.hash_late,
                                buf.late_off, self.slot_tok, self.slot_parent, self.n_slots, buf.slot, buf.scratch,
                                stream=stream, stream_out=buf.stream_slot if per_stream else (None, None, None))
        elif self.verify:
            B.cp_verify_chain(tok, buf.run_off, buf.cand, self.slot_tok, self.slot_parent, self.n_slots, False,
                              buf.slot, buf.scratch, stream=stream,
                              stream_out=buf.stream_slot[0] if per_stream else None)
        else:
            B.cp_probe3(self.table, buf.hash, buf.hash_float, buf.hash_late, buf.slot, stream=stream)
            if per_stream:
                for k, (key, _) in enumerate(keys):
                    B.cp_probe(self.table, key, buf.stream_slot[k], stream=stream)
        if lru:
            # where an earlier stream serves a token, a later one's slots still led to the tokens it does
            # serve: they count as used, or a stored run could lose its head to eviction
            for k in range(1, len(keys)):
                B.cp_touch(buf.stream_slot[k], self.epoch, self.n_slots, self.slot_stamp, stream=stream)
        return [(seg_off, buf.stream_slot[k]) for k, (_, seg_off) in enumerate(keys)]

    def lookup(self, tok, mask, off, dst, buf: LookupBuffers, gather=True, stream=None,
               gather_opts=None) -> LookupResult:
        """Serve a request batch: after the call the rows of every matched token of
        ``dst`` (layer-major, N tokens) hold the pooled KV.  No host synchronisation.
        ``gather_opts`` overrides the pool's launch options for this call."""
        N = tok.numel()
        self._match(tok, mask, off, buf, stream, per_stream=self.slot_stamp is not None, touch=True)
        if self.slot_stamp is not None:
            B.cp_touch(buf.slot, self.epoch, self.n_slots, self.slot_stamp, stream=stream)
        served = buf.slot  # buf.slot: every matched token; served: those that pass the policies
        if self.filters:
            served = B.cp_filter_matches(buf.slot, off, self.min_len, self.slot_recompute, self.n_slots, buf.served,
                                         buf.scratch, stream=stream)
        B.cp_build_spans(served, off, self.slot_pos if self.rope is not None else None, buf.max_spans, buf.span_src,
                         buf.span_dst, buf.span_len, buf.span_delta, buf.span_off, buf.n_spans, self.flags,
                         buf.scratch, stream=stream)
        if gather:
            B.cp_gather_kv(self.pool, self.layout, self.n_slots, dst, self.request_layout(N), N, buf.span_src,
                           buf.span_dst, buf.span_len, buf.span_delta if self.rope is not None else None,
                           buf.span_off, buf.n_spans, buf.max_spans, self.rope, self.flags, buf.scratch,
                           stream=stream, opts=self.gather_opts if gather_opts is None else gather_opts)
            if self.zero_fill:
                B.cp_fill_unmatched(served, dst, self.request_layout(N), stream=stream)
        return LookupResult(buf.hash, buf.slot, buf.span_src, buf.span_dst, buf.span_len, buf.span_delta,
                            buf.span_off, buf.n_spans, served)

    def insert(self, tok, mask, off, src, hash_buf, slot_out, scratch, hashes_ready=False, sync=True, stream=None,
               run_off_buf=None, recompute=None, insert_opts=None, buf: LookupBuffers = None):
        """Store the non-sensitive tokens of a batch that the pool does not hold yet,
        taking their KV rows from ``src`` (layer-major, N tokens).  With ``sync`` the
        host free-list cursor is advanced (one device-to-host read).  A pool with
        floating anchors or verification also needs ``run_off_buf`` (int32[N];
        filled here unless ``hashes_ready``).  ``recompute`` (uint8[N]): tokens the
        annotator marked for recomputation when their segment is reused."""
        N = tok.numel()
        if self.dedup:
            return self._insert_once(tok, mask, off, src, slot_out, sync, stream, recompute, insert_opts, buf)
        if self.slot_anchor is not None or self.verify:
            assert run_off_buf is not None, "a pool with floating anchors or verification needs run_off_buf"
            if not hashes_ready:
                B.cp_hash_runs(tok, mask, off, hash_buf, run_off_buf, scratch, base=self.hash_base, stream=stream)
        elif not hashes_ready:
            B.cp_hash_segments(tok, mask, off, hash_buf, scratch, base=self.hash_base, stream=stream)
        n_free = self.free_slots.numel() - self.n_used
        iopts = self.insert_opts if insert_opts is None else insert_opts
        if self.verify:
            B.cp_insert_kv_chain(self.table, hash_buf, tok, run_off_buf, off, self.free_slots[self.n_used:], n_free,
                                 src, self.request_layout(N), self.pool, self.layout, self.n_slots, self.slot_pos,
                                 self.slot_tok, self.slot_parent, slot_out, self.n_inserted, self.flags, scratch,
                                 stream=stream, opts=iopts)
        else:
            B.cp_insert_kv(self.table, hash_buf, off, self.free_slots[self.n_used:], n_free, src,
                           self.request_layout(N), self.pool, self.layout, self.n_slots, self.slot_pos, slot_out,
                           self.n_inserted, self.flags, scratch, stream=stream, opts=iopts)
        if self.slot_anchor is not None:  # a run's prefix hash is known from the moment its W-th token has a slot
            B.cp_insert_anchors(run_off_buf, slot_out, self.anchor_window, self.n_slots, self.slot_anchor, stream=stream)
        if recompute is not None:
            assert self.slot_recompute is not None, "pool was created without recompute_marks=True"
            B.cp_mark_recompute(slot_out, recompute, self.n_slots, self.slot_recompute, stream=stream)
        if self.slot_stamp is not None:
            B.cp_touch(slot_out, self.epoch, self.n_slots, self.slot_stamp, stream=stream)
        if sync:
            if stream is not None:  # the count comes from kernels on that stream, not torch's current one
                stream.synchronize()
            n = int(self.n_inserted.item())
            self.n_used += n
            return n
        return None

    def _insert_once(self, tok, mask, off, src, slot_out, sync, stream, recompute, insert_opts, buf):
        """insert() of a pool that stores every text once: the batch is looked up first (all key streams, no
        stamps), what the pool has is left out, and new tokens continue the stored text before them."""
        assert buf is not None and buf.N == tok.numel(), "a pool with dedup needs the batch's LookupBuffers"
        N = tok.numel()
        streams = self._match(tok, mask, off, buf, stream, per_stream=True, touch=False)
        B.cp_insert_keys(buf.hash, buf.run_off, streams, buf.ins_hash, buf.ins_off, buf.found, buf.scratch,
                         base=self.hash_base, stream=stream)
        n_free = self.free_slots.numel() - self.n_used
        B.cp_insert_kv_dedup(self.table, buf.ins_hash, buf.found, tok, buf.ins_off, off, self.free_slots[self.n_used:],
                             n_free, src, self.request_layout(N), self.pool, self.layout, self.n_slots, self.slot_pos,
                             self.slot_tok, self.slot_parent, slot_out, self.n_inserted, self.flags, buf.scratch,
                             stream=stream, opts=self.insert_opts if insert_opts is None else insert_opts)
        B.cp_insert_anchors(buf.ins_off, slot_out, self.anchor_window, self.n_slots, self.slot_anchor, stream=stream)
        if recompute is not None:
            assert self.slot_recompute is not None, "pool was created without recompute_marks=True"
            B.cp_mark_recompute(slot_out, recompute, self.n_slots, self.slot_recompute, stream=stream)
        if self.slot_stamp is not None:
            B.cp_touch(slot_out, self.epoch, self.n_slots, self.slot_stamp, stream=stream)
        if sync:
            if stream is not None:
                stream.synchronize()
            n = int(self.n_inserted.item())
            self.n_used += n
            return n
        return None
