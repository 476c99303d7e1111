"""Thin ctypes binding of libcacheprune.so: the same entry points as
``include/cacheprune.h``, taking torch CUDA(ROCm) tensors for device memory.

Argument marshalling only — every step of the path runs in the library's HIP
kernels.  There is no CPU fallback: if the library is not built or no GPU is
present, the calls raise.

Integer tensors use torch's signed dtypes of the same width (int32 for uint32,
int64 for uint64); the bit patterns are what the C ABI defines.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcacheprune.so")

HASH_NONE = 0xFFFFFFFFFFFFFFFF
SLOT_NONE = 0xFFFFFFFF
BASE = 0x100000001B3  # polynomial base of the chain hash
TABLE_BUCKET = 16

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP, ERR_SCRATCH, ERR_STATIC_LIMIT = 0, -1, -2, -3, -4, -5
STATIC_MAX_TOKENS, STATIC_MAX_SPANS, STATIC_MAX_SLOTS = 131072, 131072, 524288
FLAG_SPANS_OVERFLOW, FLAG_POOL_FULL, FLAG_TABLE_FULL, FLAG_BAD_INDEX = 1, 2, 4, 8

EXPORTS = [
    "cp_table_capacity_for", "cp_scratch_bytes", "cp_last_hip_error", "cp_table_init",
    "cp_hash_segments", "cp_probe", "cp_hash_probe", "cp_build_spans", "cp_gather_kv", "cp_gather_kv_static", "cp_insert_kv",
    "cp_event_create", "cp_event_elapsed_ms", "cp_event_destroy",
    "cp_hash_runs", "cp_insert_anchors", "cp_hash_floating", "cp_probe2", "cp_probe3",
    "cp_insert_kv_chain", "cp_verify_chain", "cp_verify_streams", "cp_insert_keys", "cp_insert_kv_dedup",
    "cp_filter_matches", "cp_mark_recompute", "cp_fill_unmatched", "cp_touch", "cp_lru_threshold", "cp_evict",
    "cp_table_compact", "cp_table_count", "cp_sat_scratch_bytes", "cp_sat_build", "cp_annotate",
]
PARENT_POISON = 0xFFFFFFFE
LRU_MAX_AGE = 4096


class CpError(RuntimeError):
    def __init__(self, fn, code):
        names = {-1: "CP_ERR_INVALID_ARG", -2: "CP_ERR_UNSUPPORTED", -3: "CP_ERR_HIP", -4: "CP_ERR_SCRATCH",
                 -5: "CP_ERR_STATIC_LIMIT (more than 131072 tokens or spans, or 524288 pool slots)"}
        extra = f" (hipError {lib().cp_last_hip_error()})" if code == ERR_HIP else ""
        super().__init__(f"{fn} failed: {names.get(code, code)}{extra}")
        self.code = code


class TableStruct(C.Structure):
    _fields_ = [("keys", C.c_void_p), ("vals", C.c_void_p), ("capacity", C.c_uint64)]


class KVLayout(C.Structure):
    """``cp_kv_layout``: row (t, layer, kv) at base + t*tok_stride + layer*layer_stride + kv*kv_stride."""

    _fields_ = [("n_layers", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("tok_stride", C.c_uint64), ("layer_stride", C.c_uint64), ("kv_stride", C.c_uint64)]

    @property
    def row_bytes(self):
        return self.n_kv_heads * self.head_dim * 2

    @staticmethod
    def token_major(n_layers, n_kv_heads, head_dim):
        """[slot][layer][K|V][head][dim]: all rows of a token contiguous."""
        rb = n_kv_heads * head_dim * 2
        return KVLayout(n_layers, n_kv_heads, head_dim, n_layers * 2 * rb, 2 * rb, rb)

    @staticmethod
    def layer_major(n_layers, n_kv_heads, head_dim, n_tokens):
        """[layer][K|V][token][head][dim]: per-layer K and V buffers."""
        rb = n_kv_heads * head_dim * 2
        return KVLayout(n_layers, n_kv_heads, head_dim, rb, 2 * n_tokens * rb, n_tokens * rb)


class Rope(C.Structure):
    _fields_ = [("theta", C.c_double), ("style", C.c_uint32)]


class LaunchOpts(C.Structure):
    """``cp_launch_opts``: per-call launch options of the row mover; zero = default everywhere."""

    _fields_ = [("read_sharing", C.c_uint32), ("blocks_per_cu", C.c_uint32), ("nontemporal", C.c_uint32),
                ("loads_in_flight", C.c_uint32), ("fanout", C.c_uint32), ("workgroups", C.c_uint32),
                ("reserved", C.c_uint32 * 2),
                ("start_event", C.c_void_p), ("stop_event", C.c_void_p)]

    def with_events(self, start, stop):
        """A copy that also asks for the two hipEvent_t handles to be recorded around the mover kernel."""
        o = LaunchOpts(self.read_sharing, self.blocks_per_cu, self.nontemporal, self.loads_in_flight, self.fanout,
                       self.workgroups)
        o.start_event, o.stop_event = start, stop
        return o


_lib = None


def lib():
    """Load libcacheprune.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with __graft_entry__.build() "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32, C.c_size_t
        L.cp_table_capacity_for.restype = u64
        L.cp_table_capacity_for.argtypes = [u64, C.c_double]
        L.cp_scratch_bytes.restype = sz
        L.cp_scratch_bytes.argtypes = [u32, u32, u32]
        L.cp_last_hip_error.restype = i32
        L.cp_table_init.restype = i32
        L.cp_table_init.argtypes = [vp, TableStruct]
        L.cp_hash_segments.restype = i32
        L.cp_hash_segments.argtypes = [vp, vp, vp, vp, u32, u32, u64, vp, vp, sz]
        L.cp_hash_probe.restype = i32
        L.cp_hash_probe.argtypes = [vp, vp, vp, vp, u32, u32, u64, TableStruct, vp, vp, vp, vp, sz]
        L.cp_probe.restype = i32
        L.cp_probe.argtypes = [vp, TableStruct, vp, u32, vp]
        L.cp_hash_runs.restype = i32
        L.cp_hash_runs.argtypes = [vp, vp, vp, vp, u32, u32, u64, vp, vp, vp, sz]
        L.cp_insert_anchors.restype = i32
        L.cp_insert_anchors.argtypes = [vp, vp, vp, u32, u32, u32, vp]
        L.cp_hash_floating.restype = i32
        L.cp_hash_floating.argtypes = [vp, TableStruct, vp, u32, vp, vp, u32, u64, u32, vp, vp, vp, vp, vp, sz]
        L.cp_insert_kv_chain.restype = i32
        L.cp_insert_kv_chain.argtypes = [vp, TableStruct, vp, vp, vp, vp, u32, u32, vp, u32, vp, KVLayout, vp, KVLayout,
                                         u32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_insert_keys.restype = i32
        L.cp_insert_keys.argtypes = [vp, vp, vp, u32, u64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz]
        L.cp_insert_kv_dedup.restype = i32
        L.cp_insert_kv_dedup.argtypes = [vp, TableStruct, vp, vp, vp, vp, vp, u32, u32, vp, u32, vp, KVLayout, vp, KVLayout,
                                         u32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_verify_chain.restype = i32
        L.cp_verify_chain.argtypes = [vp, vp, vp, vp, u32, vp, vp, u32, i32, vp, vp, vp, sz]
        L.cp_verify_streams.restype = i32
        L.cp_verify_streams.argtypes = [vp, TableStruct, vp, u32, vp, vp, vp, vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, sz]
        L.cp_filter_matches.restype = i32
        L.cp_filter_matches.argtypes = [vp, vp, vp, u32, u32, u32, vp, u32, vp, vp, sz]
        L.cp_mark_recompute.restype = i32
        L.cp_mark_recompute.argtypes = [vp, vp, vp, u32, u32, vp]
        L.cp_fill_unmatched.restype = i32
        L.cp_fill_unmatched.argtypes = [vp, vp, u32, vp, KVLayout]
        L.cp_touch.restype = i32
        L.cp_touch.argtypes = [vp, vp, u32, u32, u32, vp]
        L.cp_lru_threshold.restype = i32
        L.cp_lru_threshold.argtypes = [vp, vp, u32, u32, u32, vp, vp, sz]
        L.cp_evict.restype = i32
        L.cp_evict.argtypes = [vp, TableStruct, vp, u32, vp, vp, vp, vp, vp, vp, vp, sz]
        L.cp_table_compact.restype = i32
        L.cp_table_compact.argtypes = [vp, TableStruct, TableStruct, vp]
        L.cp_table_count.restype = i32
        L.cp_table_count.argtypes = [vp, TableStruct, vp]
        L.cp_sat_scratch_bytes.restype = sz
        L.cp_sat_scratch_bytes.argtypes = [u32]
        L.cp_sat_build.restype = i32
        L.cp_sat_build.argtypes = [vp, vp, u32, u64, vp, vp, vp, sz]
        L.cp_annotate.restype = i32
        L.cp_annotate.argtypes = [vp, vp, u32, vp, u32, u32, vp, vp, vp, vp, vp, vp, vp, sz]
        L.cp_probe2.restype = i32
        L.cp_probe2.argtypes = [vp, TableStruct, vp, vp, u32, vp]
        L.cp_probe3.restype = i32
        L.cp_probe3.argtypes = [vp, TableStruct, vp, vp, vp, u32, vp]
        L.cp_build_spans.restype = i32
        L.cp_build_spans.argtypes = [vp, vp, vp, u32, u32, vp, u32, vp, vp, vp, vp, vp, vp, vp, vp, sz]
        L.cp_gather_kv.restype = i32
        L.cp_gather_kv.argtypes = [vp, vp, KVLayout, u32, vp, KVLayout, u32, vp, vp, vp, vp, vp, vp, u32, vp, vp, vp, sz,
                                   vp]
        L.cp_gather_kv_static.restype = i32
        L.cp_gather_kv_static.argtypes = [vp, vp, KVLayout, u32, vp, KVLayout, u32, vp, vp, vp, vp, vp, vp, u32, vp, vp, vp]
        L.cp_insert_kv.restype = i32
        L.cp_insert_kv.argtypes = [vp, TableStruct, vp, vp, u32, u32, vp, u32, vp, KVLayout, vp, KVLayout, u32, vp, vp,
                                   vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(fn, rc):
    if rc != OK:
        raise CpError(fn, rc)


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("libcacheprune takes device tensors only")


def cp_table_capacity_for(n_keys, load_factor=0.5):
    return int(lib().cp_table_capacity_for(int(n_keys), float(load_factor)))


def cp_scratch_bytes(N, max_spans=0, n_pool_slots=0):
    return int(lib().cp_scratch_bytes(int(N), int(max_spans), int(n_pool_slots)))


def _opts(opts):
    return None if opts is None else C.byref(opts)


class HipEvents:
    """n timing hipEvents made by the library's own HIP runtime (cp_event_*)."""

    def __init__(self, n):
        L = lib()
        L.cp_event_create.restype = C.c_void_p
        L.cp_event_elapsed_ms.restype = C.c_float
        L.cp_event_elapsed_ms.argtypes = [C.c_void_p, C.c_void_p]
        L.cp_event_destroy.argtypes = [C.c_void_p]
        self.ev = []
        for _ in range(n):
            e = L.cp_event_create()
            if not e:
                raise RuntimeError("cp_event_create failed")
            self.ev.append(C.c_void_p(e))

    def elapsed_ms(self, a, b):
        ms = float(lib().cp_event_elapsed_ms(self.ev[a], self.ev[b]))
        if ms < 0:
            raise RuntimeError(f"cp_event_elapsed_ms failed (hipError {lib().cp_last_hip_error()})")
        return ms

    def close(self):
        for e in self.ev:
            lib().cp_event_destroy(e)
        self.ev = []


def new_scratch(N, max_spans, device="cuda", n_pool_slots=0):
    return torch.empty(cp_scratch_bytes(N, max_spans, n_pool_slots), dtype=torch.uint8, device=device)


class Table:
    """Device arrays of a ``cp_table`` (torch owns the memory)."""

    def __init__(self, capacity, device="cuda", stream=None):
        if capacity % TABLE_BUCKET:
            raise ValueError("capacity must be a multiple of 16")
        self.capacity = int(capacity)
        self.keys = torch.empty(self.capacity, dtype=torch.int64, device=device)
        self.vals = torch.empty(self.capacity, dtype=torch.int32, device=device)
        cp_table_init(self, stream)

    @property
    def struct(self):
        return TableStruct(self.keys.data_ptr(), self.vals.data_ptr(), self.capacity)


def cp_table_init(table: Table, stream=None):
    _check("cp_table_init", lib().cp_table_init(_stream(stream), table.struct))


def cp_hash_segments(tok, mask, off, hash_out, scratch, base=BASE, stream=None):
    """tok int32[N], mask uint8[N], off int32[R+1] -> hash_out int64[N]."""
    _need_cuda(tok, mask, off, hash_out, scratch)
    N, R = tok.numel(), off.numel() - 1
    assert mask.numel() == N and hash_out.numel() == N
    _check("cp_hash_segments", lib().cp_hash_segments(_stream(stream), _ptr(tok), _ptr(mask), _ptr(off), N, R, base,
                                                      _ptr(hash_out), _ptr(scratch), scratch.numel()))
    return hash_out


def cp_hash_probe(tok, mask, off, table: Table, hash_out, run_off_out, slot_out, scratch, base=BASE, stream=None):
    """cp_hash_segments / cp_hash_runs (``run_off_out`` may be None) and cp_probe in one pass."""
    _need_cuda(tok, mask, off, hash_out, run_off_out, slot_out, scratch)
    N, R = tok.numel(), off.numel() - 1
    assert mask.numel() == N and hash_out.numel() == N and slot_out.numel() == N
    assert run_off_out is None or run_off_out.numel() == N
    _check("cp_hash_probe", lib().cp_hash_probe(_stream(stream), _ptr(tok), _ptr(mask), _ptr(off), N, R, base,
                                                table.struct, _ptr(hash_out), _ptr(run_off_out), _ptr(slot_out),
                                                _ptr(scratch), scratch.numel()))
    return slot_out


def cp_hash_runs(tok, mask, off, hash_out, run_off_out, scratch, base=BASE, stream=None):
    """cp_hash_segments that also returns run_off int32[N] (tokens since the start of the run)."""
    _need_cuda(tok, mask, off, hash_out, run_off_out, scratch)
    N, R = tok.numel(), off.numel() - 1
    assert mask.numel() == N and hash_out.numel() == N and run_off_out.numel() == N
    _check("cp_hash_runs", lib().cp_hash_runs(_stream(stream), _ptr(tok), _ptr(mask), _ptr(off), N, R, base,
                                              _ptr(hash_out), _ptr(run_off_out), _ptr(scratch), scratch.numel()))
    return hash_out


def cp_insert_anchors(run_off, slot, W, n_pool_slots, slot_anchor, stream=None):
    _need_cuda(run_off, slot, slot_anchor)
    assert slot.numel() == run_off.numel() and slot_anchor.numel() >= n_pool_slots
    _check("cp_insert_anchors", lib().cp_insert_anchors(_stream(stream), _ptr(run_off), _ptr(slot), run_off.numel(),
                                                        int(W), n_pool_slots, _ptr(slot_anchor)))


def cp_hash_floating(table: Table, slot_anchor, n_pool_slots, hashes, run_off, W, hash_a_out, scratch, base=BASE,
                     stream=None, off_a_out=None, hash_b_out=None, off_b_out=None):
    _need_cuda(slot_anchor, hashes, run_off, hash_a_out, scratch, off_a_out, hash_b_out, off_b_out)
    N = hashes.numel()
    assert run_off.numel() == N and hash_a_out.numel() == N and slot_anchor.numel() >= n_pool_slots
    for t in (off_a_out, hash_b_out, off_b_out):
        assert t is None or t.numel() == N
    _check("cp_hash_floating", lib().cp_hash_floating(_stream(stream), table.struct, _ptr(slot_anchor), n_pool_slots,
                                                      _ptr(hashes), _ptr(run_off), N, base, int(W),
                                                      _ptr(hash_a_out), _ptr(off_a_out), _ptr(hash_b_out),
                                                      _ptr(off_b_out), _ptr(scratch), scratch.numel()))
    return hash_a_out


def cp_verify_streams(table: Table, tok, seg_off_0, cand_0, key_a, seg_off_a, key_b, seg_off_b, slot_tok, slot_parent,
                      n_pool_slots, slot_out, scratch, stream=None, stream_out=(None, None, None)):
    _need_cuda(tok, seg_off_0, cand_0, key_a, seg_off_a, key_b, seg_off_b, slot_tok, slot_parent, slot_out, scratch,
               *stream_out)
    N = tok.numel()
    for t in (seg_off_0, cand_0, key_a, seg_off_a, key_b, seg_off_b, slot_out):
        assert t.numel() == N
    assert slot_tok.numel() >= n_pool_slots and slot_parent.numel() >= n_pool_slots and len(stream_out) == 3
    _check("cp_verify_streams", lib().cp_verify_streams(
        _stream(stream), table.struct, _ptr(tok), N, _ptr(seg_off_0), _ptr(cand_0), _ptr(key_a), _ptr(seg_off_a),
        _ptr(key_b), _ptr(seg_off_b), _ptr(slot_tok), _ptr(slot_parent), n_pool_slots, _ptr(slot_out),
        _ptr(stream_out[0]), _ptr(stream_out[1]), _ptr(stream_out[2]), _ptr(scratch), scratch.numel()))
    return slot_out


def cp_verify_chain(tok, seg_off, cand, slot_tok, slot_parent, n_pool_slots, merge, slot_out, scratch, stream=None,
                    stream_out=None):
    _need_cuda(tok, seg_off, cand, slot_tok, slot_parent, slot_out, scratch, stream_out)
    N = tok.numel()
    assert seg_off.numel() == N and cand.numel() == N and slot_out.numel() == N
    assert slot_tok.numel() >= n_pool_slots and slot_parent.numel() >= n_pool_slots
    _check("cp_verify_chain", lib().cp_verify_chain(_stream(stream), _ptr(tok), _ptr(seg_off), _ptr(cand), N,
                                                    _ptr(slot_tok), _ptr(slot_parent), n_pool_slots, 1 if merge else 0,
                                                    _ptr(slot_out), _ptr(stream_out), _ptr(scratch), scratch.numel()))
    return slot_out


def cp_insert_kv_chain(table: Table, hashes, tok, run_off, off, free_slots, n_free, src, src_l: KVLayout, pool,
                       pool_l: KVLayout, n_pool_slots, slot_pos, slot_tok, slot_parent, slot_out, n_inserted,
                       status_flags, scratch, stream=None, opts: LaunchOpts | None = None):
    _need_cuda(hashes, tok, run_off, off, free_slots, src, pool, slot_pos, slot_tok, slot_parent, slot_out, n_inserted,
               status_flags, scratch)
    N, R = hashes.numel(), off.numel() - 1
    assert tok.numel() == N and run_off.numel() == N and slot_out.numel() == N
    assert free_slots is None or free_slots.numel() >= n_free
    assert slot_tok.numel() >= n_pool_slots and slot_parent.numel() >= n_pool_slots
    _check("cp_insert_kv_chain", lib().cp_insert_kv_chain(
        _stream(stream), table.struct, _ptr(hashes), _ptr(tok), _ptr(run_off), _ptr(off), N, R, _ptr(free_slots),
        n_free, _ptr(src), src_l, _ptr(pool), pool_l, n_pool_slots, _ptr(slot_pos), _ptr(slot_tok), _ptr(slot_parent),
        _ptr(slot_out), _ptr(n_inserted), _ptr(status_flags), _ptr(scratch), scratch.numel(), _opts(opts)))


def cp_insert_keys(hashes, run_off, streams, ins_hash_out, ins_off_out, found_out, scratch, base=BASE, stream=None):
    """``streams``: up to three (seg_off, slot) tensor pairs, one per lookup stream in serving order."""
    _need_cuda(hashes, run_off, ins_hash_out, ins_off_out, found_out, scratch, *[t for p in streams for t in p])
    N = hashes.numel()
    assert 1 <= len(streams) <= 3 and all(a.numel() == N and b.numel() == N for a, b in streams)
    assert ins_hash_out.numel() == N and ins_off_out.numel() == N and found_out.numel() == N
    ptrs = [_ptr(t) for p in streams for t in p] + [None] * (6 - 2 * len(streams))
    _check("cp_insert_keys", lib().cp_insert_keys(_stream(stream), _ptr(hashes), _ptr(run_off), N, base, *ptrs,
                                                  _ptr(ins_hash_out), _ptr(ins_off_out), _ptr(found_out), _ptr(scratch),
                                                  scratch.numel()))


def cp_insert_kv_dedup(table: Table, ins_hash, found, tok, ins_off, off, free_slots, n_free, src, src_l: KVLayout, pool,
                       pool_l: KVLayout, n_pool_slots, slot_pos, slot_tok, slot_parent, slot_out, n_inserted,
                       status_flags, scratch, stream=None, opts: LaunchOpts | None = None):
    _need_cuda(ins_hash, found, tok, ins_off, off, free_slots, src, pool, slot_pos, slot_tok, slot_parent, slot_out,
               n_inserted, status_flags, scratch)
    N, R = ins_hash.numel(), off.numel() - 1
    assert found.numel() == N and slot_out.numel() == N and (free_slots is None or free_slots.numel() >= n_free)
    _check("cp_insert_kv_dedup", lib().cp_insert_kv_dedup(
        _stream(stream), table.struct, _ptr(ins_hash), _ptr(found), _ptr(tok), _ptr(ins_off), _ptr(off), N, R,
        _ptr(free_slots), n_free, _ptr(src), src_l, _ptr(pool), pool_l, n_pool_slots, _ptr(slot_pos), _ptr(slot_tok),
        _ptr(slot_parent), _ptr(slot_out), _ptr(n_inserted), _ptr(status_flags), _ptr(scratch), scratch.numel(),
        _opts(opts)))


def cp_filter_matches(slot_in, off, min_len, slot_recompute, n_pool_slots, slot_out, scratch, stream=None):
    _need_cuda(slot_in, off, slot_recompute, slot_out, scratch)
    N, R = slot_in.numel(), off.numel() - 1
    assert slot_out.numel() == N and (slot_recompute is None or slot_recompute.numel() >= n_pool_slots)
    _check("cp_filter_matches", lib().cp_filter_matches(_stream(stream), _ptr(slot_in), _ptr(off), N, R, int(min_len),
                                                        _ptr(slot_recompute), n_pool_slots, _ptr(slot_out),
                                                        _ptr(scratch), scratch.numel()))
    return slot_out


def cp_mark_recompute(slot, recompute, n_pool_slots, slot_recompute, stream=None):
    _need_cuda(slot, recompute, slot_recompute)
    N = slot.numel()
    assert recompute.numel() == N and slot_recompute.numel() >= n_pool_slots
    _check("cp_mark_recompute", lib().cp_mark_recompute(_stream(stream), _ptr(slot), _ptr(recompute), N, n_pool_slots,
                                                        _ptr(slot_recompute)))


def cp_fill_unmatched(slot, dst, dst_l: KVLayout, stream=None):
    _need_cuda(slot, dst)
    _check("cp_fill_unmatched", lib().cp_fill_unmatched(_stream(stream), _ptr(slot), slot.numel(), _ptr(dst), dst_l))


def cp_touch(slot, epoch, n_pool_slots, slot_stamp, stream=None):
    _need_cuda(slot, slot_stamp)
    assert slot_stamp.numel() >= n_pool_slots
    _check("cp_touch", lib().cp_touch(_stream(stream), _ptr(slot), slot.numel(), int(epoch), n_pool_slots,
                                      _ptr(slot_stamp)))


def cp_lru_threshold(slot_stamp, n_pool_slots, epoch_now, n_needed, threshold_out, scratch, stream=None):
    _need_cuda(slot_stamp, threshold_out, scratch)
    assert slot_stamp.numel() >= n_pool_slots
    _check("cp_lru_threshold", lib().cp_lru_threshold(_stream(stream), _ptr(slot_stamp), n_pool_slots, int(epoch_now),
                                                      int(n_needed), _ptr(threshold_out), _ptr(scratch),
                                                      scratch.numel()))


def cp_evict(table: Table, slot_stamp, n_pool_slots, threshold, freed_slots, n_freed, slot_parent, slot_recompute,
             slot_anchor, scratch, stream=None):
    _need_cuda(slot_stamp, threshold, freed_slots, n_freed, slot_parent, slot_recompute, slot_anchor, scratch)
    assert slot_stamp.numel() >= n_pool_slots and freed_slots.numel() >= n_pool_slots
    _check("cp_evict", lib().cp_evict(_stream(stream), table.struct, _ptr(slot_stamp), n_pool_slots, _ptr(threshold),
                                      _ptr(freed_slots), _ptr(n_freed), _ptr(slot_parent), _ptr(slot_recompute),
                                      _ptr(slot_anchor), _ptr(scratch), scratch.numel()))


def cp_table_compact(src: Table, dst: Table, status_flags, stream=None):
    _need_cuda(status_flags)
    _check("cp_table_compact", lib().cp_table_compact(_stream(stream), src.struct, dst.struct, _ptr(status_flags)))


def cp_table_count(table: Table, counts_out, stream=None):
    """counts_out: int32[2] on the device <- (entries holding a key, of which with a slot)."""
    _need_cuda(counts_out)
    _check("cp_table_count", lib().cp_table_count(_stream(stream), table.struct, _ptr(counts_out)))


def new_sat_scratch(n, device="cuda"):
    return torch.empty(int(lib().cp_sat_scratch_bytes(int(n))), dtype=torch.uint8, device=device)


def cp_sat_build(attn, T, scratch, stream=None, mask=None):
    """attn float32[n][ld] -> T int64[n][n]; with ``mask`` (uint8[n]) only the part cp_annotate reads for it."""
    _need_cuda(attn, T, scratch, mask)
    assert mask is None or (mask.dtype == torch.uint8 and mask.numel() == attn.shape[0])
    n, ld = attn.shape[0], attn.stride(0)
    assert attn.dtype == torch.float32 and attn.stride(1) == 1 and T.dtype == torch.int64
    assert T.is_contiguous() and T.shape == (n, n)
    _check("cp_sat_build", lib().cp_sat_build(_stream(stream), _ptr(attn), n, ld, _ptr(mask), _ptr(T),
                                              _ptr(scratch), scratch.numel()))
    return T


def cp_annotate(T, mask, min_len, rho_percent, best_l, best_r, best_score, reusable, recompute, store_mask, scratch,
                stream=None):
    _need_cuda(T, mask, best_l, best_r, best_score, reusable, recompute, store_mask, scratch)
    n = T.shape[0]
    assert T.dtype == torch.int64 and T.is_contiguous() and T.shape == (n, n) and mask.numel() == n
    for t in (best_l, best_r, best_score, reusable, recompute):
        assert t.numel() == n
    _check("cp_annotate", lib().cp_annotate(_stream(stream), _ptr(T), n, _ptr(mask), int(min_len), int(rho_percent),
                                            _ptr(best_l), _ptr(best_r), _ptr(best_score), _ptr(reusable),
                                            _ptr(recompute), _ptr(store_mask), _ptr(scratch), scratch.numel()))


def cp_probe2(table: Table, hash_a, hash_b, slot_out, stream=None):
    _need_cuda(hash_a, hash_b, slot_out)
    N = hash_a.numel()
    assert hash_b.numel() == N and slot_out.numel() == N
    _check("cp_probe2", lib().cp_probe2(_stream(stream), table.struct, _ptr(hash_a), _ptr(hash_b), N, _ptr(slot_out)))
    return slot_out


def cp_probe3(table: Table, hash_a, hash_b, hash_c, slot_out, stream=None):
    _need_cuda(hash_a, hash_b, hash_c, slot_out)
    N = hash_a.numel()
    assert hash_b.numel() == N and hash_c.numel() == N and slot_out.numel() == N
    _check("cp_probe3", lib().cp_probe3(_stream(stream), table.struct, _ptr(hash_a), _ptr(hash_b), _ptr(hash_c), N,
                                        _ptr(slot_out)))
    return slot_out


def cp_probe(table: Table, hashes, slot_out, stream=None):
    _need_cuda(hashes, slot_out)
    N = hashes.numel()
    assert slot_out.numel() == N
    _check("cp_probe", lib().cp_probe(_stream(stream), table.struct, _ptr(hashes), N, _ptr(slot_out)))
    return slot_out


def cp_build_spans(slot, off, slot_pos, max_spans, span_src, span_dst, span_len, span_delta, span_off, n_spans,
                   status_flags, scratch, stream=None):
    _need_cuda(slot, off, slot_pos, span_src, span_dst, span_len, span_delta, span_off, n_spans, status_flags, scratch)
    N, R = slot.numel(), off.numel() - 1
    assert span_src.numel() >= max_spans and span_dst.numel() >= max_spans and span_len.numel() >= max_spans
    assert span_delta is None or span_delta.numel() >= max_spans
    assert span_off is None or span_off.numel() >= max_spans + 1
    _check("cp_build_spans", lib().cp_build_spans(
        _stream(stream), _ptr(slot), _ptr(off), N, R, _ptr(slot_pos), max_spans, _ptr(span_src), _ptr(span_dst),
        _ptr(span_len), _ptr(span_delta), _ptr(span_off), _ptr(n_spans), _ptr(status_flags), _ptr(scratch),
        scratch.numel()))


def cp_gather_kv(pool, pool_l: KVLayout, n_pool_slots, dst, dst_l: KVLayout, n_dst_tokens, span_src, span_dst,
                 span_len, span_delta, span_off, n_spans, max_spans, rope: Rope | None, status_flags, scratch,
                 stream=None, opts: LaunchOpts | None = None):
    _need_cuda(pool, dst, span_src, span_dst, span_len, span_delta, span_off, n_spans, status_flags, scratch)
    _check("cp_gather_kv", lib().cp_gather_kv(
        _stream(stream), _ptr(pool), pool_l, n_pool_slots, _ptr(dst), dst_l, n_dst_tokens, _ptr(span_src),
        _ptr(span_dst), _ptr(span_len), _ptr(span_delta), _ptr(span_off), _ptr(n_spans), max_spans,
        C.byref(rope) if rope is not None else None, _ptr(status_flags), _ptr(scratch),
        scratch.numel() if scratch is not None else 0, _opts(opts)))


def cp_gather_kv_static(pool, pool_l: KVLayout, n_pool_slots, dst, dst_l: KVLayout, n_dst_tokens, span_src, span_dst,
                        span_len, span_delta, span_off, n_spans, max_spans, rope: Rope | None, status_flags,
                        stream=None, opts: LaunchOpts | None = None):
    """cp_gather_kv without a scratch argument: the library's own device array is the working memory."""
    _need_cuda(pool, dst, span_src, span_dst, span_len, span_delta, span_off, n_spans, status_flags)
    _check("cp_gather_kv_static", lib().cp_gather_kv_static(
        _stream(stream), _ptr(pool), pool_l, n_pool_slots, _ptr(dst), dst_l, n_dst_tokens, _ptr(span_src),
        _ptr(span_dst), _ptr(span_len), _ptr(span_delta), _ptr(span_off), _ptr(n_spans), max_spans,
        C.byref(rope) if rope is not None else None, _ptr(status_flags), _opts(opts)))


def cp_insert_kv(table: Table, hashes, off, free_slots, n_free, src, src_l: KVLayout, pool, pool_l: KVLayout,
                 n_pool_slots, slot_pos, slot_out, n_inserted, status_flags, scratch, stream=None,
                 opts: LaunchOpts | None = None):
    _need_cuda(hashes, off, free_slots, src, pool, slot_pos, slot_out, n_inserted, status_flags, scratch)
    N, R = hashes.numel(), off.numel() - 1
    assert slot_out.numel() == N and (free_slots is None or free_slots.numel() >= n_free)
    _check("cp_insert_kv", lib().cp_insert_kv(
        _stream(stream), table.struct, _ptr(hashes), _ptr(off), N, R, _ptr(free_slots), n_free, _ptr(src), src_l,
        _ptr(pool), pool_l, n_pool_slots, _ptr(slot_pos), _ptr(slot_out), _ptr(n_inserted), _ptr(status_flags),
        _ptr(scratch), scratch.numel(), _opts(opts)))
