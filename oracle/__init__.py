"""ctypes front end of the CPU oracle (``cp_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product package never does.
Arrays are numpy arrays in host memory; every function returns new arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcp_oracle.so")

HASH_NONE = 0xFFFFFFFFFFFFFFFF
SLOT_NONE = 0xFFFFFFFF
FLAG_SPANS_OVERFLOW = 1
FLAG_POOL_FULL = 2
FLAG_TABLE_FULL = 4
BASE = 0x100000001B3


def build(force: bool = True) -> str:
    """Compile the oracle with g++ -O2 into ``libcp_oracle.so`` beside its source."""
    src = os.path.join(_HERE, "cp_oracle.cpp")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.run(
            ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB_PATH, src],
            check=True,
        )
    return _LIB_PATH


class Layout(C.Structure):
    """Mirror of ``cpo_layout`` (strides in bytes)."""

    _fields_ = [
        ("n_layers", C.c_uint32),
        ("n_kv_heads", C.c_uint32),
        ("head_dim", C.c_uint32),
        ("tok_stride", C.c_uint64),
        ("layer_stride", C.c_uint64),
        ("kv_stride", C.c_uint64),
    ]

    @property
    def row_bytes(self) -> int:
        return self.n_kv_heads * self.head_dim * 2


class Rope(C.Structure):
    _fields_ = [("theta", C.c_double), ("style", C.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = C.CDLL(_LIB_PATH)
        vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32
        L.cpo_index_new.restype = vp
        L.cpo_index_free.argtypes = [vp]
        L.cpo_index_size.restype = u64
        L.cpo_index_size.argtypes = [vp]
        L.cpo_index_rebuild.restype = None
        L.cpo_index_rebuild.argtypes = [vp, u64]
        L.cpo_index_entries.restype = u64
        L.cpo_index_entries.argtypes = [vp]
        L.cpo_hash_segments.argtypes = [vp, vp, vp, u32, u64, vp]
        L.cpo_probe.argtypes = [vp, vp, u32, vp]
        L.cpo_build_spans.restype = u32
        L.cpo_build_spans.argtypes = [vp, vp, u32, vp, u32, vp, vp, vp, vp, vp]
        L.cpo_gather_kv.argtypes = [vp, Layout, vp, Layout, vp, vp, vp, vp, u32, vp]
        L.cpo_insert_kv.restype = u32
        L.cpo_insert_kv.argtypes = [vp, vp, vp, u32, vp, u32, vp, Layout, vp, Layout, vp, vp, vp, vp, vp]
        L.cpo_anchor_set_new.restype = vp
        L.cpo_anchor_set_free.argtypes = [vp]
        L.cpo_anchor_set_size.restype = u64
        L.cpo_anchor_set_size.argtypes = [vp]
        L.cpo_run_offsets.argtypes = [vp, vp, u32, vp]
        L.cpo_insert_anchors.argtypes = [vp, vp, vp, vp, u32, u32]
        L.cpo_hash_floating.argtypes = [vp, vp, vp, vp, u32, u64, u32, vp, vp, vp, vp]
        L.cpo_insert_keys.restype = None
        L.cpo_insert_keys.argtypes = [vp, vp, vp, vp, u32, u32, u64, vp, vp, vp]
        L.cpo_insert_kv_dedup.restype = u32
        L.cpo_insert_kv_dedup.argtypes = [vp, vp, vp, vp, u32, vp, u32, vp, Layout, vp, Layout, vp, vp, vp, vp, vp]
        L.cpo_text_record_dedup.restype = None
        L.cpo_text_record_dedup.argtypes = [vp, vp, vp, vp, u32, vp]
        L.cpo_probe3.restype = None
        L.cpo_probe3.argtypes = [vp, vp, vp, vp, u32, vp]
        L.cpo_text_new.restype = vp
        L.cpo_text_new.argtypes = [u32]
        L.cpo_text_free.argtypes = [vp]
        L.cpo_text_record.argtypes = [vp, vp, vp, u32, vp]
        L.cpo_verify.argtypes = [vp, vp, vp, vp, u32, C.c_int, vp]
        L.cpo_filter_matches.argtypes = [vp, vp, u32, u32, vp, u32, vp]
        L.cpo_mark_recompute.argtypes = [vp, vp, u32, u32, vp]
        L.cpo_fill_unmatched.argtypes = [vp, u32, vp, Layout]
        L.cpo_touch.argtypes = [vp, u32, u32, u32, vp]
        L.cpo_lru_threshold.restype = u32
        L.cpo_lru_threshold.argtypes = [vp, u32, u32, u32, u32]
        L.cpo_evict.restype = u32
        L.cpo_evict.argtypes = [vp, vp, u32, u32, vp, vp, vp, vp]
        L.cpo_sat_build.argtypes = [vp, u32, u64, vp]
        L.cpo_sat_rect.restype = C.c_int64
        L.cpo_sat_rect.argtypes = [vp, u32, C.c_int64, C.c_int64, C.c_int64, C.c_int64]
        L.cpo_annotate.argtypes = [vp, u32, vp, u32, u32, vp, vp, vp, vp, vp]
        L.cpo_probe2.argtypes = [vp, vp, vp, u32, vp]
        L.cpo_bf16_to_double.restype = C.c_double
        L.cpo_bf16_to_double.argtypes = [C.c_uint16]
        L.cpo_double_to_bf16.restype = C.c_uint16
        L.cpo_double_to_bf16.argtypes = [C.c_double]
        L.cpo_rope_head.argtypes = [vp, vp, u32, i32, C.c_double, u32]
        L.cpo_rope_head_f64.argtypes = [vp, vp, u32, C.c_double, C.c_double, u32]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class Index:
    """The pool index (key -> slot)."""

    def __init__(self):
        self._h = C.c_void_p(lib().cpo_index_new())

    def __len__(self):
        return int(lib().cpo_index_size(self._h))

    def rebuild(self, capacity):
        """From now on a table of ``capacity`` entries that holds the keys with a slot (0 = unbounded)."""
        lib().cpo_index_rebuild(self._h, int(capacity))

    @property
    def entries(self):
        """Keys that hold a table entry (with or without a slot) since the last rebuild."""
        return int(lib().cpo_index_entries(self._h))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.cpo_index_free(self._h)
            self._h = None


class AnchorSet:
    """The stored runs' prefix hashes (floating-anchor lookup)."""

    def __init__(self):
        self._h = C.c_void_p(lib().cpo_anchor_set_new())

    def __len__(self):
        return int(lib().cpo_anchor_set_size(self._h))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.cpo_anchor_set_free(self._h)
            self._h = None


def run_offsets(mask, off):
    mask, off = _arr(mask, np.uint8), _arr(off, np.uint32)
    out = np.empty(mask.shape[0], np.uint32)
    lib().cpo_run_offsets(_p(mask), _p(off), len(off) - 1, _p(out))
    return out


def insert_anchors(anchors: AnchorSet, hashes, run_off, slot, W):
    """``slot``: what the insert of the same tokens reported; a run's prefix hash is kept while its W-th token is."""
    hashes, run_off, slot = _arr(hashes, np.uint64), _arr(run_off, np.uint32), _arr(slot, np.uint32)
    lib().cpo_insert_anchors(anchors._h, _p(hashes), _p(run_off), _p(slot), hashes.shape[0], int(W))


def hash_floating(anchors: AnchorSet, index: Index, hashes, run_off, W, base=BASE):
    """Keys and segment offsets of the two candidate streams: (hash_a, off_a, hash_b, off_b)."""
    hashes, run_off = _arr(hashes, np.uint64), _arr(run_off, np.uint32)
    n = hashes.shape[0]
    he, hl = np.empty(n, np.uint64), np.empty(n, np.uint64)
    eo, lo = np.empty(n, np.uint32), np.empty(n, np.uint32)
    lib().cpo_hash_floating(anchors._h, index._h, _p(hashes), _p(run_off), n, base, int(W), _p(he), _p(eo), _p(hl),
                            _p(lo))
    return he, eo, hl, lo


def match_streams(index: Index, tok, hashes, run_off, anchors: AnchorSet = None, W=None, text: "Text" = None,
                  with_offsets=False, base=BASE):
    """What every key stream of a lookup finds, in the order in which they serve a token: the run-start
    keys, then (pools with floating anchors) the keys of candidate stream a and of candidate stream b.
    With ``text`` each stream's slots are confirmed against the stored text along its own segments."""
    streams = [(hashes, run_off)]
    if anchors is not None:
        he, eo, hl, lo = hash_floating(anchors, index, hashes, run_off, W, base)
        streams += [(he, eo), (hl, lo)]
    out = []
    for keys, seg_off in streams:
        s = probe(index, keys)
        s = s if text is None else verify(text, tok, seg_off, s)
        out.append((seg_off, s) if with_offsets else s)
    return out


def merge_streams(streams):
    """A token is served from the first stream that has a slot for it."""
    out = np.array(streams[0], np.uint32, copy=True)
    for s in streams[1:]:
        out = np.where(out == SLOT_NONE, s, out).astype(np.uint32)
    return out


class Text:
    """The token string every pool slot was stored for (exact verification)."""

    def __init__(self, n_slots):
        self._h = lib().cpo_text_new(int(n_slots))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.cpo_text_free(self._h)
            self._h = None


def text_record(text: Text, tok, run_off, slot_out):
    """Record a batch after insert_kv; returns slot_out with unverified tokens set to NONE."""
    tok, run_off = _arr(tok, np.uint32), _arr(run_off, np.uint32)
    out = np.array(slot_out, dtype=np.uint32, copy=True)
    lib().cpo_text_record(text._h, _p(tok), _p(run_off), tok.shape[0], _p(out))
    return out


def verify(text: Text, tok, seg_off, cand, merge_into=None):
    tok, seg_off, cand = _arr(tok, np.uint32), _arr(seg_off, np.uint32), _arr(cand, np.uint32)
    out = np.empty(tok.shape[0], np.uint32) if merge_into is None else np.array(merge_into, np.uint32, copy=True)
    lib().cpo_verify(text._h, _p(tok), _p(seg_off), _p(cand), tok.shape[0], 0 if merge_into is None else 1, _p(out))
    return out


def probe2(index: Index, hash_a, hash_b):
    hash_a, hash_b = _arr(hash_a, np.uint64), _arr(hash_b, np.uint64)
    out = np.empty(hash_a.shape[0], np.uint32)
    lib().cpo_probe2(index._h, _p(hash_a), _p(hash_b), hash_a.shape[0], _p(out))
    return out


def probe3(index: Index, hash_a, hash_b=None, hash_c=None):
    hash_a = _arr(hash_a, np.uint64)
    hash_b = None if hash_b is None else _arr(hash_b, np.uint64)
    hash_c = None if hash_c is None else _arr(hash_c, np.uint64)
    out = np.empty(hash_a.shape[0], np.uint32)
    lib().cpo_probe3(index._h, _p(hash_a), None if hash_b is None else _p(hash_b), None if hash_c is None else _p(hash_c),
                     hash_a.shape[0], _p(out))
    return out


LRU_MAX_AGE = 4096  # ages of LRU_MAX_AGE - 1 epochs and more are evicted as one class


def filter_matches(slot, off, min_len, slot_recompute=None):
    slot, off = _arr(slot, np.uint32), _arr(off, np.uint32)
    out = np.empty(slot.shape[0], np.uint32)
    n_slots = 0 if slot_recompute is None else slot_recompute.shape[0]
    lib().cpo_filter_matches(_p(slot), _p(off), len(off) - 1, int(min_len),
                             None if slot_recompute is None else _p(slot_recompute), n_slots, _p(out))
    return out


def mark_recompute(slot, recompute, slot_recompute):
    """In place on slot_recompute (uint8[n_slots])."""
    slot, recompute = _arr(slot, np.uint32), _arr(recompute, np.uint8)
    assert slot_recompute.dtype == np.uint8 and slot_recompute.flags.c_contiguous
    lib().cpo_mark_recompute(_p(slot), _p(recompute), slot.shape[0], slot_recompute.shape[0], _p(slot_recompute))


def fill_unmatched(slot, dst, dst_l: Layout):
    slot = _arr(slot, np.uint32)
    assert dst.flags.c_contiguous
    lib().cpo_fill_unmatched(_p(slot), slot.shape[0], _p(dst), dst_l)


def touch(slot, epoch, slot_stamp):
    """In place on slot_stamp (uint32[n_slots])."""
    slot = _arr(slot, np.uint32)
    assert slot_stamp.dtype == np.uint32 and slot_stamp.flags.c_contiguous
    lib().cpo_touch(_p(slot), slot.shape[0], int(epoch), slot_stamp.shape[0], _p(slot_stamp))


def lru_threshold(slot_stamp, epoch_now, n_needed, max_age=LRU_MAX_AGE):
    assert slot_stamp.dtype == np.uint32 and slot_stamp.flags.c_contiguous
    return int(lib().cpo_lru_threshold(_p(slot_stamp), slot_stamp.shape[0], int(epoch_now), int(n_needed), int(max_age)))


def evict(index: Index, slot_stamp, threshold, text: "Text | None" = None, slot_recompute=None,
          anchors: "AnchorSet | None" = None):
    """Frees slots in place; returns the freed slots (ascending)."""
    assert slot_stamp.dtype == np.uint32 and slot_stamp.flags.c_contiguous
    freed = np.empty(slot_stamp.shape[0], np.uint32)
    n = lib().cpo_evict(index._h, _p(slot_stamp), slot_stamp.shape[0], int(threshold), _p(freed),
                        None if text is None else text._h, None if slot_recompute is None else _p(slot_recompute),
                        None if anchors is None else anchors._h)
    return freed[:n].copy()


def sat_build(attn):
    """attn: float32[n][ld] (ld >= n) -> int64[n][n] summed-area table of the fixed-point weights."""
    attn = np.ascontiguousarray(attn, np.float32)
    n, ld = attn.shape[0], attn.shape[1]
    T = np.empty((n, n), np.int64)
    lib().cpo_sat_build(_p(attn), n, ld, _p(T))
    return T


def sat_rect(T, x1, x2, y1, y2):
    return int(lib().cpo_sat_rect(_p(T), T.shape[0], int(x1), int(x2), int(y1), int(y2)))


def annotate(T, mask, min_len=1, rho_percent=25):
    """Returns (best_l, best_r, best_score, reusable, recompute), one entry per token."""
    mask = _arr(mask, np.uint8)
    n = T.shape[0]
    assert T.dtype == np.int64 and T.flags.c_contiguous and mask.shape[0] == n
    bl, br = np.empty(n, np.uint32), np.empty(n, np.uint32)
    bs = np.empty(n, np.int64)
    reus, rec = np.empty(n, np.uint8), np.empty(n, np.uint8)
    lib().cpo_annotate(_p(T), n, _p(mask), int(min_len), int(rho_percent), _p(bl), _p(br), _p(bs), _p(reus), _p(rec))
    return bl, br, bs, reus, rec


def hash_segments(tok, mask, off, base=BASE):
    tok, mask, off = _arr(tok, np.uint32), _arr(mask, np.uint8), _arr(off, np.uint32)
    out = np.empty(tok.shape[0], dtype=np.uint64)
    lib().cpo_hash_segments(_p(tok), _p(mask), _p(off), len(off) - 1, base, _p(out))
    return out


def probe(index: Index, hashes):
    hashes = _arr(hashes, np.uint64)
    out = np.empty(hashes.shape[0], dtype=np.uint32)
    lib().cpo_probe(index._h, _p(hashes), hashes.shape[0], _p(out))
    return out


def build_spans(slot, off, slot_pos=None, max_spans=None):
    """Returns (src, dst, len, delta, n_spans_found, flags); arrays hold min(n, max_spans)."""
    slot, off = _arr(slot, np.uint32), _arr(off, np.uint32)
    if slot_pos is not None:
        slot_pos = _arr(slot_pos, np.int32)
    if max_spans is None:
        max_spans = max(1, slot.shape[0])
    src = np.zeros(max_spans, np.uint32)
    dst = np.zeros(max_spans, np.uint32)
    ln = np.zeros(max_spans, np.uint32)
    delta = np.zeros(max_spans, np.int32)
    flags = np.zeros(1, np.uint32)
    n = lib().cpo_build_spans(_p(slot), _p(off), len(off) - 1, _p(slot_pos), max_spans, _p(src), _p(dst),
                              _p(ln), _p(delta), _p(flags))
    k = min(n, max_spans)
    return src[:k], dst[:k], ln[:k], delta[:k], int(n), int(flags[0])


def gather_kv(pool, pool_l: Layout, dst, dst_l: Layout, src, dstpos, ln, delta=None, rope: Rope | None = None):
    """Copies in place into ``dst`` (a writable uint8/uint16 numpy buffer)."""
    src, dstpos, ln = _arr(src, np.uint32), _arr(dstpos, np.uint32), _arr(ln, np.uint32)
    if delta is not None:
        delta = _arr(delta, np.int32)
    lib().cpo_gather_kv(_p(pool), pool_l, _p(dst), dst_l, _p(src), _p(dstpos), _p(ln), _p(delta), len(src),
                        C.byref(rope) if rope is not None else None)


def insert_kv(index: Index, hashes, off, free_slots, src, src_l: Layout, pool, pool_l: Layout, slot_pos,
              tok=None, slot_tok=None):
    """Returns (slot_out, n_inserted, flags).  ``pool``, ``slot_pos`` (and ``slot_tok``) are updated in place."""
    hashes, off, free_slots = _arr(hashes, np.uint64), _arr(off, np.uint32), _arr(free_slots, np.uint32)
    assert slot_pos.dtype == np.int32 and slot_pos.flags.c_contiguous
    if tok is not None:
        tok = _arr(tok, np.uint32)
        assert slot_tok is not None and slot_tok.dtype == np.uint32
    slot_out = np.empty(hashes.shape[0], np.uint32)
    flags = np.zeros(1, np.uint32)
    n = lib().cpo_insert_kv(index._h, _p(hashes), _p(off), len(off) - 1, _p(free_slots), len(free_slots), _p(src),
                            src_l, _p(pool), pool_l, _p(slot_pos), _p(slot_out), _p(flags), _p(tok), _p(slot_tok))
    return slot_out, int(n), int(flags[0])


def insert_keys(hashes, run_off, streams, base=BASE):
    """``streams``: list of (seg_off, slot) per lookup stream, in serving order.  Returns (ins_hash, ins_off, found)."""
    hashes, run_off = _arr(hashes, np.uint64), _arr(run_off, np.uint32)
    n, k = hashes.shape[0], len(streams)
    segs = [_arr(so, np.uint32) for so, _ in streams]
    slots = [_arr(sl, np.uint32) for _, sl in streams]
    seg_p = (C.c_void_p * k)(*[a.ctypes.data for a in segs])
    slot_p = (C.c_void_p * k)(*[a.ctypes.data for a in slots])
    ih, io, fo = np.empty(n, np.uint64), np.empty(n, np.uint32), np.empty(n, np.uint32)
    lib().cpo_insert_keys(_p(hashes), _p(run_off), seg_p, slot_p, k, n, base, _p(ih), _p(io), _p(fo))
    return ih, io, fo


def insert_kv_dedup(index: Index, ins_hash, found, off, free_slots, src, src_l: Layout, pool, pool_l: Layout, slot_pos,
                    tok=None, slot_tok=None):
    """insert_kv under the keys of ``insert_keys``, leaving out the tokens that were found."""
    ins_hash, found = _arr(ins_hash, np.uint64), _arr(found, np.uint32)
    off, free_slots = _arr(off, np.uint32), _arr(free_slots, np.uint32)
    assert slot_pos.dtype == np.int32 and slot_pos.flags.c_contiguous
    if tok is not None:
        tok = _arr(tok, np.uint32)
        assert slot_tok is not None and slot_tok.dtype == np.uint32
    slot_out = np.empty(ins_hash.shape[0], np.uint32)
    flags = np.zeros(1, np.uint32)
    n = lib().cpo_insert_kv_dedup(index._h, _p(ins_hash), _p(found), _p(off), len(off) - 1, _p(free_slots),
                                  len(free_slots), _p(src), src_l, _p(pool), pool_l, _p(slot_pos), _p(slot_out),
                                  _p(flags), _p(tok), _p(slot_tok))
    return slot_out, int(n), int(flags[0])


def text_record_dedup(text: "Text", tok, ins_off, found, slot_out):
    tok, ins_off, found = _arr(tok, np.uint32), _arr(ins_off, np.uint32), _arr(found, np.uint32)
    out = np.array(slot_out, dtype=np.uint32, copy=True)
    lib().cpo_text_record_dedup(text._h, _p(tok), _p(ins_off), _p(found), tok.shape[0], _p(out))
    return out


def bf16_to_double(bits: int) -> float:
    return float(lib().cpo_bf16_to_double(int(bits)))


def double_to_bf16(x: float) -> int:
    return int(lib().cpo_double_to_bf16(float(x)))


def rope_head(x_bits, delta: int, theta: float, style: int = 0):
    x_bits = _arr(x_bits, np.uint16)
    out = np.empty_like(x_bits)
    lib().cpo_rope_head(_p(x_bits), _p(out), x_bits.shape[0], int(delta), float(theta), int(style))
    return out


def rope_head_f64(x, delta: float, theta: float, style: int = 0):
    x = _arr(x, np.float64)
    out = np.empty_like(x)
    lib().cpo_rope_head_f64(_p(x), _p(out), x.shape[0], float(delta), float(theta), int(style))
    return out
