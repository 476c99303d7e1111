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


HITS = {}


@pytest.mark.parametrize("W", [1, 3, 16, 64])
def test_float_workload(G, W):
    wl = small_float()
    ost, olk, gst, glk = compare_all(G, wl, anchor_window=W)
    start_only = O.probe(ost.index, olk.hash)
    gained = (olk.slot != NONE).sum() - (start_only != NONE).sum()
    print(f"W={W}: hits {np.mean(olk.slot != NONE):.3f}, of which through floating keys {gained / len(olk.slot):.3f}")
    assert gained > 0.3 * len(olk.slot)  # most of this workload is reachable through an anchor only
    assert ((olk.hash_float != O.HASH_NONE) | (olk.hash_late != O.HASH_NONE)).sum() >= gained
    HITS[W] = glk.slot != NONE
    if W == 3:  # a one-token window makes many chance candidates; none of them may cost a match
        assert (HITS[3] <= HITS[1]).all(), "W = 1 serves fewer tokens than W = 3"


def test_overlapping_and_nested_candidates(G):
    """Stored texts that contain one another or overlap inside a request: a later window hit must not cost what
    an earlier candidate covers (every token of 'abcdefgh' with 'defg' also stored), and the part only the later
    one covers is served from it ('XY' + 'YZ' against 'XYZ').  Hand-built donors, checked against the oracle."""
    rng = np.random.default_rng(77)
    V = lambda n: rng.integers(0, 32000, n).astype(np.uint32)  # noqa: E731
    long_text, X, Y, Z = V(40), V(12), V(15), V(9)
    donors = [long_text, long_text[10:25], np.concatenate([X, Y]), np.concatenate([Y, Z])]
    reqs = [np.concatenate([V(5), long_text, V(3)]), np.concatenate([V(2), X, Y, Z, V(4)]),
            np.concatenate([V(1), long_text[10:40], V(2), Y, Z])]
    wl = gen.from_prompts("overlap", 0xC0FFEE21, gen.KVShape(2, 2, 64), donors, reqs, pool_slots=512)
    for W in (1, 2, 4):
        ost, olk, gst, glk = compare_all(G, wl, anchor_window=W)
        o = wl.off
        assert (glk.slot[o[0] + 5:o[0] + 45] != NONE).all()  # all of the long text, its last tokens included
        assert (glk.slot[o[1] + 2:o[1] + 2 + 12 + 15 + 9] != NONE).all()  # X Y Z whole
        # the third request enters the long text at its 11th token: only the shorter stored text starts there
        assert (glk.slot[o[2] + 1:o[2] + 16] != NONE).all() and (glk.slot[o[2] + 16:o[2] + 31] == NONE).all()
        assert (glk.slot[o[2] + 33:o[2] + 33 + 24] != NONE).all()  # Y Z behind other text
    compare_all(G, wl, anchor_window=2, verify=True)


def test_a_staircase_of_overlapping_texts_is_served_whole(G):
    """Seven stored texts, each 25 tokens of one 85-token sequence, ten tokens apart: up to three of them cover
    a token of a request that quotes the sequence.  Every token from the first text's start on is served, the
    chosen texts alternate between the two candidate streams, and verification confirms each on its own."""
    rng = np.random.default_rng(78)
    V = lambda n: rng.integers(0, 32000, n).astype(np.uint32)  # noqa: E731
    seq = V(85)
    donors = [seq[k:k + 25] for k in range(0, 61, 10)]
    reqs = [np.concatenate([V(4), seq, V(3)]), np.concatenate([V(2), seq[10:70]]), np.concatenate([seq[5:80], V(6)])]
    wl = gen.from_prompts("staircase", 0xC0FFEE22, gen.KVShape(2, 2, 64), donors, reqs, pool_slots=512)
    for W, verify in ((1, False), (3, False), (8, True)):
        ost, olk, gst, glk = compare_all(G, wl, anchor_window=W, verify=verify)
        o = wl.off
        assert (glk.slot[o[0] + 4:o[0] + 4 + 85] != NONE).all() and (glk.slot[o[0] + 89:o[0] + 92] == NONE).all()
        assert (glk.slot[o[1] + 2:o[1] + 62] != NONE).all()
        # the third request starts inside the first stored text: served from the second text's start (token 10) on
        assert (glk.slot[o[2]:o[2] + 5] == NONE).all() and (glk.slot[o[2] + 5:o[2] + 75] != NONE).all()
        both = (olk.hash_float != O.HASH_NONE) & (olk.hash_late != O.HASH_NONE)
        assert both.sum() >= 3 * 15  # where consecutive chosen texts overlap, a token has a key in either stream


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


@pytest.mark.parametrize("n_free", [None, 300])
def test_a_prefix_hash_lives_with_its_token(G, n_free):
    """The set of stored prefix hashes is the set of slots that hold a run's W-th token: one mark per
    such slot and no other, also when the pool runs full and some W-th tokens get no slot."""
    from oracle import harness as OH

    W = 5
    wl = small_float(scale=0.5)
    if n_free is not None:
        wl.free_slots = wl.free_slots[:n_free]
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=W))
    ost = OH.prefill(wl, anchor_window=W)
    assert np.array_equal(gst.donor_slot, ost.donor_slot)
    ro = O.run_offsets(wl.donor_mask, wl.donor_off)
    want = np.unique(ost.donor_slot[(ro == W - 1) & (ost.donor_slot != NONE)])
    assert len(want) == len(ost.anchors) and len(want) > 0
    got = np.flatnonzero(gst.pool.slot_anchor.cpu().numpy())
    assert np.array_equal(got, want)
    if n_free is not None:
        assert ((ro == W - 1) & (ost.donor_slot == NONE) & (wl.donor_mask == 0)).any()  # some runs lost their W-th token
    glk, olk = G.lookup(gst), OH.lookup(ost)
    assert np.array_equal(glk.hash_float, olk.hash_float) and np.array_equal(glk.slot, olk.slot)
