"""The privacy invariant on the GPU path (Sec. 3.3 / 4.2.1: sensitive tokens are never shared): nothing
the library produces may depend on WHICH tokens the sensitive positions hold.  Two runs that differ
only in the ids of the sensitive tokens (donors and requests) must agree in every output bit, and no
sensitive position may be hashed, stored, matched or written."""
import copy

import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen, kvgen
from test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu
NONE = O.SLOT_NONE


def run(G, wl, kw, rec):
    st = G.prefill(wl, G.make_pool(wl, **kw), recompute=rec)
    lk = G.lookup(st)
    return st, lk


@pytest.mark.parametrize("name,scale,kw", [
    ("llama3-8b", 1 / 8, {}),
    ("frag", 1 / 32, {"verify": True}),
    ("float", 1 / 2, {"anchor_window": 8, "verify": True, "min_len": 6, "recompute_marks": True, "zero_fill": True,
                      "lru": True}),
])
def test_sensitive_token_ids_do_not_matter(G, name, scale, kw):
    wl = gen.make(name, scale=scale)
    wl.shape = gen.KVShape(2, 2, 64)
    rec = (wl.donor_u < 0.25).astype(np.uint8) if kw.get("recompute_marks") else None
    other = copy.copy(wl)
    rng = np.random.default_rng(77)
    other.tok, other.donor_tok = wl.tok.copy(), wl.donor_tok.copy()
    other.tok[wl.mask == 1] = rng.integers(0, gen.VOCAB, int(wl.mask.sum()))
    other.donor_tok[wl.donor_mask == 1] = rng.integers(0, gen.VOCAB, int(wl.donor_mask.sum()))
    assert wl.mask.sum() > 20 and (other.tok != wl.tok).sum() > 10
    sa, la = run(G, wl, kw, rec)
    sb, lb = run(G, other, kw, rec)
    # nothing sensitive is hashed, stored or served
    assert (la.hash[wl.mask == 1] == O.HASH_NONE).all() and (la.slot[wl.mask == 1] == NONE).all()
    assert (sa.donor_hash[wl.donor_mask == 1] == O.HASH_NONE).all() and (sa.donor_slot[wl.donor_mask == 1] == NONE).all()
    rows = G.dst_as_rows(la.dst, wl.shape, wl.n_tokens)
    untouched = 0 if kw.get("zero_fill") else kvgen.POISON16
    assert (rows[:, :, wl.mask == 1] == untouched).all()
    # and every output is the same in both runs
    for f in ("hash", "slot", "served", "span_src", "span_dst", "span_len", "span_off", "n_spans", "flags"):
        a, b = getattr(la, f), getattr(lb, f)
        assert np.array_equal(a, b), f
    for f in ("hash_float", "hash_late", "run_off"):
        if getattr(la, f) is not None:
            assert np.array_equal(getattr(la, f), getattr(lb, f)), f
    assert torch.equal(la.dst, lb.dst) and torch.equal(sa.pool.pool, sb.pool.pool)
    assert np.array_equal(sa.donor_hash, sb.donor_hash) and np.array_equal(sa.donor_slot, sb.donor_slot)
    assert torch.equal(sa.pool.slot_pos, sb.pool.slot_pos)
    for f in ("slot_tok", "slot_parent", "slot_recompute", "slot_stamp", "slot_anchor"):
        if getattr(sa.pool, f) is not None:
            assert torch.equal(getattr(sa.pool, f), getattr(sb.pool, f)), f
    assert np.array_equal(np.sort(G.host_u64(sa.pool.table.keys)), np.sort(G.host_u64(sb.pool.table.keys)))
