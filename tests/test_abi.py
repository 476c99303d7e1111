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
