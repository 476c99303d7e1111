"""Counter-based generator of synthetic KV values (bf16, roughly N(0,1)).

Every element is a pure function of (seed, token uid, layer, K|V, element
index), computed with integers only, so the host (numpy, below) and the device
(``kvgen.hip``: fill and verify kernels for tests and benchmarks) produce the
same bits and any row can be re-derived without keeping a buffer around.

This is input generation and test tooling: none of the method's arithmetic
lives here, and neither the oracle nor the GPU library includes this code.

Definition (all 64-bit, wrapping):
    row_id = (uid * n_layers + layer) * 2 + kv
    z  = seed + row_id * C1 + pair * C2         (pair = element index // 2)
    z ^= z >> 32; z *= M; z ^= z >> 32; z *= M; z ^= z >> 32
    element 2*pair   uses the low  32 bits of z, element 2*pair+1 the high 32
    s = sum of the 4 bytes of those 32 bits        (0 .. 1020, mean 510, sd 147.8)
    x = float32(s - 510) * SCALE                   (one float multiply; SCALE = float 0x3BDDB47B ~ 1/147.8)
    value = x rounded to bf16, round-to-nearest-even on the float's bits
A token whose uid is ``UID_NONE`` gets the poison pattern in every element.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

C1 = 0x9E3779B97F4A7C15
C2 = 0xD1B54A32D192ED03
M = 0xD6E8FEB86659FD93
UID_NONE = 0xFFFFFFFFFFFFFFFF
SCALE = np.array([0x3BDDB47B], np.uint32).view(np.float32)[0]  # float nearest to 1 / 147.8
POISON16 = 0xC0DE  # bf16 bit pattern written where no value may appear

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcp_kvgen.so")


def row(seed: int, uid: int, layer: int, kv: int, n_layers: int, row_elems: int) -> np.ndarray:
    """One row as uint16[row_elems] (bf16 bit patterns), computed on the host."""
    if uid == UID_NONE:
        return np.full(row_elems, POISON16, np.uint16)
    with np.errstate(over="ignore"):
        row_id = np.uint64((((uid * n_layers) + layer) * 2 + kv) & 0xFFFFFFFFFFFFFFFF)
        pair = np.arange(row_elems // 2, dtype=np.uint64)
        z = np.uint64(seed) + row_id * np.uint64(C1) + pair * np.uint64(C2)
        z ^= z >> np.uint64(32)
        z *= np.uint64(M)
        z ^= z >> np.uint64(32)
        z *= np.uint64(M)
        z ^= z >> np.uint64(32)
    words = np.empty(row_elems, np.uint32)
    words[0::2] = (z & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    words[1::2] = (z >> np.uint64(32)).astype(np.uint32)
    s = (words & 0xFF) + ((words >> 8) & 0xFF) + ((words >> 16) & 0xFF) + (words >> 24)
    x = (s.astype(np.int32) - 510).astype(np.float32) * SCALE
    u = x.view(np.uint32)
    u = u + np.uint32(0x7FFF) + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def rows_for_tokens(seed, uids, n_layers, row_elems):
    """uint16[len(uids), n_layers, 2, row_elems] on the host (same definition as ``row``,
    vectorised over rows; meant for up to a few hundred MB)."""
    uids = np.asarray(list(uids) if not isinstance(uids, np.ndarray) else uids, dtype=np.uint64)
    n = len(uids)
    out = np.empty((n, n_layers, 2, row_elems), np.uint16)
    if n == 0:
        return out
    flat = out.reshape(n * n_layers * 2, row_elems)
    lkv = np.arange(n_layers * 2, dtype=np.uint64)  # layer * 2 + kv
    pair = np.arange(row_elems // 2, dtype=np.uint64)
    step = max(1, (1 << 22) // max(1, row_elems))  # rows per chunk
    with np.errstate(over="ignore"):
        row_id = ((uids[:, None] * np.uint64(n_layers * 2)) + lkv[None, :]).reshape(-1)
        for r0 in range(0, len(row_id), step):
            rid = row_id[r0 : r0 + step]
            z = np.uint64(seed) + rid[:, None] * np.uint64(C1) + pair[None, :] * np.uint64(C2)
            z ^= z >> np.uint64(32)
            z *= np.uint64(M)
            z ^= z >> np.uint64(32)
            z *= np.uint64(M)
            z ^= z >> np.uint64(32)
            words = np.empty((len(rid), row_elems), np.uint32)
            words[:, 0::2] = (z & np.uint64(0xFFFFFFFF)).astype(np.uint32)
            words[:, 1::2] = (z >> np.uint64(32)).astype(np.uint32)
            s = (words & 0xFF) + ((words >> 8) & 0xFF) + ((words >> 16) & 0xFF) + (words >> 24)
            x = (s.astype(np.int32) - 510).astype(np.float32) * SCALE
            u = x.view(np.uint32)
            u = u + np.uint32(0x7FFF) + ((u >> 16) & 1)
            flat[r0 : r0 + step] = (u >> 16).astype(np.uint16)
    poison = uids == np.uint64(UID_NONE)
    if poison.any():
        out[poison] = POISON16
    return out


# ---------------------------------------------------------------------------
# device side (tests and benchmarks only)


class GenLayout(C.Structure):
    """Byte address of row (t, l, kv) = base + t*tok_stride + l*layer_stride + kv*kv_stride."""

    _fields_ = [
        ("n_layers", C.c_uint32),
        ("row_elems", C.c_uint32),
        ("tok_stride", C.c_uint64),
        ("layer_stride", C.c_uint64),
        ("kv_stride", C.c_uint64),
    ]


def build(force: bool = True) -> str:
    """hipcc kvgen.hip -> libcp_kvgen.so beside it.  Packed-FP32 arithmetic is switched off for the
    device code; the host pass notes once per option that it does not know that feature, and any
    other compiler output fails the build."""
    src = os.path.join(_HERE, "kvgen.hip")
    if force or not os.path.exists(_LIB_PATH):
        note = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
        p = subprocess.run(
            ["hipcc", "--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-Wall", "-Werror", "-Xclang",
             "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", _LIB_PATH, src],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        said = [ln for ln in p.stdout.splitlines() if ln.strip() and ln.strip() != note]
        if p.returncode != 0 or said:
            raise RuntimeError(f"hipcc kvgen.hip (exit {p.returncode}):\n" + "\n".join(said))
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is not built; run __graft_entry__.build() first")
        L = C.CDLL(_LIB_PATH)
        vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
        L.kvgen_fill.restype = C.c_int
        L.kvgen_fill.argtypes = [vp, vp, GenLayout, vp, u64, u32, u64]
        L.kvgen_verify.restype = C.c_int
        L.kvgen_verify.argtypes = [vp, vp, GenLayout, vp, vp, u32, u64, vp]
        L.kvgen_stream.restype = C.c_int
        L.kvgen_stream.argtypes = [vp, C.c_int, vp, vp, u64, vp]
        _lib = L
    return _lib


def fill(stream, base_ptr, layout: GenLayout, n_tok, seed, uid_ptr=None, uid_base=0):
    """Fill rows of tokens 0..n_tok-1 of a device buffer.  Token t has uid
    ``uid_ptr[t]`` (device uint64 array) or ``uid_base + t``."""
    rc = lib().kvgen_fill(stream, base_ptr, layout, uid_ptr, uid_base, n_tok, seed)
    if rc != 0:
        raise RuntimeError(f"kvgen_fill failed: hipError {rc}")


def verify(stream, base_ptr, layout: GenLayout, uid_ptr, n_tok, seed, n_bad_ptr, skip_k_ptr=None):
    """Adds to ``*n_bad_ptr`` (device uint64) the number of 16-bit elements of
    tokens 0..n_tok-1 that differ from the generator's value for ``uid_ptr[t]``
    (poison for UID_NONE).  K rows of tokens with ``skip_k_ptr[t] != 0`` are not
    checked."""
    rc = lib().kvgen_verify(stream, base_ptr, layout, uid_ptr, skip_k_ptr, n_tok, seed, n_bad_ptr)
    if rc != 0:
        raise RuntimeError(f"kvgen_verify failed: hipError {rc}")


def stream(stream, mode, a_ptr, b_ptr, n_bytes, sink_ptr):
    """Plain streaming kernel over a contiguous device buffer: mode "read" (a), "write" (b) or "copy" (a -> b);
    ``n_bytes`` a multiple of 128 KiB.  For bandwidth ceilings and profiler-counter calibration."""
    rc = lib().kvgen_stream(stream, {"read": 0, "write": 1, "copy": 2}[mode], a_ptr, b_ptr, n_bytes, sink_ptr)
    if rc != 0:
        raise RuntimeError(f"kvgen_stream failed: hipError {rc}")
