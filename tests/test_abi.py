"""The C-ABI library loads without a GPU and exports every function that
include/cacheprune.h declares; host-only helpers behave as documented."""
import ctypes
import os
import re

import paper_2605_23640_amd as cp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cacheprune.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"cp_hash_segments", "cp_probe", "cp_build_spans", "cp_gather_kv", "cp_insert_kv"} <= set(names)
    lib = ctypes.CDLL(cp.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in cacheprune.h but not exported"
    assert sorted(cp.binding.EXPORTS) == names  # the binding knows the same list


def test_host_helpers():
    assert cp.cp_table_capacity_for(131072, 0.85) == 154208  # ceil(131072 / 0.85) rounded up to a bucket multiple
    assert cp.cp_table_capacity_for(100, 0.5) == 208 and cp.cp_table_capacity_for(16, 1.0) == 32
    assert cp.cp_table_capacity_for(0, 0.5) == 16
    a, b = cp.cp_scratch_bytes(1000, 1000, 0), cp.cp_scratch_bytes(2000, 1000, 0)
    assert 0 < a < b < cp.cp_scratch_bytes(2000, 1000, 4096)
    assert cp.binding.lib().cp_last_hip_error() == 0


def test_binding_refuses_host_tensors():
    import pytest
    import torch

    t = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(ValueError):
        cp.cp_hash_segments(t, t.view(torch.uint8)[:4], t[:2], torch.zeros(4, dtype=torch.int64), t.view(torch.uint8))


def test_argument_errors_are_found_on_the_host():
    """Bad arguments are rejected before anything is enqueued, so this runs without a GPU.  Pointers here
    are made-up aligned addresses that the library must not (and, failing first, does not) touch."""
    B = cp.binding
    L = B.lib()
    P, Q, S = 0x10000, 0x20000, 0x30000  # "device pointers", 64 KiB aligned
    big = 1 << 30
    tab = B.TableStruct(P, Q, 1024)
    lay = B.KVLayout.token_major(2, 2, 64)
    INV, UNS, SCR = B.ERR_INVALID_ARG, B.ERR_UNSUPPORTED, B.ERR_SCRATCH
    # empty batches are no-ops
    assert L.cp_hash_segments(None, None, None, None, 0, 0, B.BASE, None, None, 0) == B.OK
    assert L.cp_probe(None, tab, None, 0, None) == B.OK
    assert L.cp_verify_chain(None, None, None, None, 0, None, None, 0, 0, None, None, None, 0) == B.OK
    assert L.cp_filter_matches(None, None, None, 0, 0, 1, None, 0, None, None, 0) == B.OK
    assert L.cp_sat_build(None, None, 0, 0, None, None, None, 0) == B.OK
    # null or inconsistent arguments
    assert L.cp_hash_segments(None, None, Q, S, 4, 1, B.BASE, P, S, big) == INV
    assert L.cp_hash_segments(None, P, Q, S, 4, 0, B.BASE, P, S, big) == INV  # no requests
    assert L.cp_hash_runs(None, P, Q, S, 4, 1, B.BASE, P, None, S, big) == INV  # run_off missing
    assert L.cp_hash_segments(None, P, Q, S, 4, 1, B.BASE, P, S, 1) == SCR  # scratch too small
    assert L.cp_hash_segments(None, P, Q, S, 4, 1, B.BASE, P, S + 8, big) == INV  # scratch misaligned
    assert L.cp_probe(None, B.TableStruct(None, Q, 1024), P, 4, Q) == INV
    assert L.cp_probe(None, B.TableStruct(P, Q, 1000), P, 4, Q) == INV  # capacity not a multiple of 16
    assert L.cp_probe(None, B.TableStruct(P + 8, Q, 1024), P, 4, Q) == INV  # keys misaligned
    assert L.cp_probe2(None, tab, P, None, 4, Q) == INV
    assert L.cp_insert_anchors(None, Q, Q, 4, 0, 16, S) == INV  # W = 0
    assert L.cp_insert_anchors(None, Q, Q, 4, 2, 16, None) == INV  # no mark array
    assert L.cp_hash_floating(None, tab, S, 16, P, Q, 4, B.BASE, 0, P, None, None, None, S, big) == INV  # W = 0
    assert L.cp_hash_floating(None, tab, None, 16, P, Q, 4, B.BASE, 2, P, None, None, None, S, big) == INV  # no mark array
    assert L.cp_probe3(None, tab, P, P, None, 4, Q) == INV
    assert L.cp_build_spans(None, None, Q, 4, 1, None, 4, P, P, P, None, None, Q, Q, S, big) == INV
    assert L.cp_insert_kv(None, tab, P, Q, 4, 1, S, 4, None, lay, P, lay, 16, P, Q, S, S, S, big, None) == INV
    assert L.cp_insert_kv_chain(None, tab, P, Q, Q, Q, 4, 1, S, 4, P, lay, P, lay, 16, P, None, None, Q, S, S, S,
                                big, None) == INV
    assert L.cp_verify_chain(None, P, P, Q, 4, P, P, 16, 0, Q, None, S, big) == INV  # cand and slot_out are one array
    vs = lambda **kw: L.cp_verify_streams(*[kw.get(k, v) for k, v in dict(  # noqa: E731
        stream=None, table=tab, tok=P, N=4, seg0=P, cand0=Q, key_a=P, seg_a=P, key_b=P, seg_b=P, slot_tok=P, slot_parent=P,
        n_slots=16, slot_out=S, so0=None, soa=None, sob=None, scratch=S, bytes=big).items()])
    assert vs(N=0) == B.OK
    assert vs(key_b=None) == INV and vs(cand0=S) == INV  # a stream's keys missing; cand_0 and slot_out are one array
    assert vs(table=B.TableStruct(P, Q, 1000)) == INV and vs(bytes=16) == SCR and vs(n_slots=1 << 31) == UNS
    assert L.cp_filter_matches(None, None, Q, 4, 1, 1, None, 0, P, S, big) == INV
    assert L.cp_mark_recompute(None, P, None, 4, 16, Q) == INV
    assert L.cp_fill_unmatched(None, None, 4, P, lay) == INV
    assert L.cp_fill_unmatched(None, P, 4, Q, B.KVLayout(2, 2, 3, 96, 24, 12)) == UNS  # rows of 12 bytes
    assert L.cp_touch(None, P, 4, 0, 16, Q) == INV  # epoch 0 means "free"
    assert L.cp_lru_threshold(None, None, 16, 5, 1, P, S, big) == INV
    assert L.cp_evict(None, tab, None, 16, P, Q, S, None, None, None, S, big) == INV
    assert L.cp_table_compact(None, tab, tab, S) == INV  # source and destination share memory
    assert L.cp_table_count(None, tab, None) == INV and L.cp_table_count(None, B.TableStruct(P, Q, 1000), S) == INV
    assert L.cp_sat_build(None, P, 100, 64, None, Q, S, big) == INV  # row stride shorter than a row
    assert L.cp_sat_build(None, P, (1 << 20) + 1, 1 << 21, None, Q, S, big) == UNS
    assert L.cp_sat_build(None, P, 100, 100, None, Q, S, 16) == SCR
    assert L.cp_annotate(None, P, 100, Q, 1, 101, P, P, P, Q, Q, None, S, big) == INV  # rho above 100 %
    # launch options outside their documented ranges
    gather = lambda o: L.cp_gather_kv(None, P, lay, 16, Q, lay, 4, S, S, S, None, None, S, 4, None, S, S, big,  # noqa: E731
                                      ctypes.byref(o))
    assert gather(B.LaunchOpts(read_sharing=3)) == INV
    assert gather(B.LaunchOpts(loads_in_flight=5)) == INV
    assert gather(B.LaunchOpts(fanout=17)) == INV
    assert gather(B.LaunchOpts(start_event=P)) == INV  # one event without the other
    o = B.LaunchOpts()
    o.reserved[1] = 1
    assert gather(o) == INV
    assert L.cp_insert_kv(None, tab, P, Q, 4, 1, S, 4, P, lay, P, lay, 16, P, Q, S, S, S, big,
                          ctypes.byref(B.LaunchOpts(nontemporal=5))) == INV
    assert L.cp_sat_scratch_bytes(10000) > (157 * 10112 + 79 * 10048) * 8  # tile carries of a 10,000-token request


def test_header_and_library_from_plain_c(tmp_path):
    """include/cacheprune.h is a C header: it compiles as C99 on its own, and a C program that passes the
    structs by value gets the documented answers from the host-side checks (no GPU involved)."""
    import os
    import subprocess

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c",
                    os.path.join(inc, "cacheprune.h")], check=True)
    lib = cp.binding.lib()._name
    exe = str(tmp_path / "abi_c_check")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", inc, "-o", exe,
                    os.path.join(root, "tests", "abi_c_check.c"), lib, "-Wl,-rpath," + os.path.dirname(lib),
                    "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0 and run.stdout.strip() == "abi ok", (run.returncode, run.stdout, run.stderr)
