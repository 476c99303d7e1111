"""Floating-anchor lookup (Sec. 4.2.2, Steps 1-2) on the GPU against the CPU
oracle: run offsets, floating keys, slots, spans and gathered rows bit for bit."""
import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen
from test_gpu_parity import G, compare_all  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu

NONE = O.SLOT_NONE


def small_float(shape=gen.KVShape(2, 2, 64), scale=0.5):
    wl = gen.make("float", scale=scale)
    wl.shape = shape
    return wl


@pytest.mark.parametrize("W", [1, 3, 16, 64])
def test_float_workload(G, W):
    wl = small_float()
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=W)
    start_only = O.probe(ost.index, olk.hash)
    gained = (olk.slot != NONE).sum() - (start_only != NONE).sum()
    print(f"W={W}: hits {np.mean(olk.slot != NONE):.3f}, of which through floating keys {gained / len(olk.slot):.3f}")
    assert gained > 0.3 * len(olk.slot)  # most of this workload is reachable through an anchor only
    assert (olk.hash_float != O.HASH_NONE).sum() >= gained


def test_window_longer_than_every_run(G):
    wl = small_float(scale=0.125)
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=100000)
    assert (olk.hash_float == O.HASH_NONE).all()
    assert np.array_equal(olk.slot, O.probe(ost.index, olk.hash))


def test_anchors_change_nothing_where_runs_align(G):
    # prefix-aligned documents: every stored run also starts a run in the requests
    wl = gen.make("tiny")
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=4)
    assert (glk.slot != NONE).mean() > 0.5


def test_rope_with_anchors(G):
    wl = small_float(shape=gen.KVShape(2, 8, 128), scale=0.25)
    wl.rope_theta, wl.rope_style = 500000.0, 0
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=8)
    assert (glk.span_delta != 0).mean() > 0.5


def test_anchor_table_full_is_flagged(G):
    from paper_2605_23640_amd import binding as B

    wl = small_float(scale=0.5)
    pool = G.make_pool(wl, anchor_window=2, anchor_capacity=16)  # one bucket: 16 anchors at most
    gst = G.prefill(wl, pool)
    assert gst.flags & B.FLAG_TABLE_FULL
    # what did get in still serves lookups consistently: every hit names a slot holding that token's key
    glk = G.lookup(gst)
    hit = glk.slot != NONE
    stored = dict(zip(gst.donor_hash.tolist(), gst.donor_slot.tolist()))
    for i in np.flatnonzero(hit)[:2000]:
        s = int(glk.slot[i])
        assert stored.get(int(glk.hash[i])) == s or stored.get(int(glk.hash_float[i])) == s
