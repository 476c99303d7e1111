"""Input generators: determinism, stated structure of the five workloads, and
agreement of the two host forms of the KV value generator."""
import numpy as np

from cp_workload import gen, kvgen


def test_kvgen_vectorised_equals_rowwise_and_looks_normal():
    uids = np.array([0, 1, 7, 123456789, kvgen.UID_NONE], np.uint64)
    rows = kvgen.rows_for_tokens(42, uids, 3, 64)
    for t, u in enumerate(uids):
        for l in range(3):
            for kv in range(2):
                assert np.array_equal(rows[t, l, kv], kvgen.row(42, int(u), l, kv, 3, 64))
    assert (rows[4] == kvgen.POISON16).all()
    big = kvgen.rows_for_tokens(1, np.arange(64), 4, 256)
    x = (big.astype(np.uint32) << 16).view(np.float32)
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02 and np.abs(x).max() < 3.6
    assert len(np.unique(big)) > 500  # values differ across tokens, layers, K/V and elements
    assert not np.array_equal(big[0, 0, 0], big[0, 0, 1]) and not np.array_equal(big[0, 0, 0], big[1, 0, 0])


def test_workloads_are_deterministic_and_well_formed():
    for name, kw in [("tiny", {}), ("llama3-8b", {"scale": 1 / 16}), ("frag", {"scale": 1 / 32}),
                     ("rope", {"scale": 1 / 16}), ("llama3-70b", {"scale": 1 / 32})]:
        a, b = gen.make(name, **kw), gen.make(name, **kw)
        for f in ("tok", "mask", "off", "donor_tok", "donor_mask", "donor_off", "free_slots"):
            assert np.array_equal(getattr(a, f), getattr(b, f)), (name, f)
        assert a.off[0] == 0 and a.off[-1] == len(a.tok) == len(a.mask) and (np.diff(a.off.astype(np.int64)) >= 0).all()
        assert a.donor_off[-1] == len(a.donor_tok) and a.tok.max() < gen.VOCAB
        assert sorted(a.free_slots.tolist()) == list(range(a.pool_slots))  # a permutation of the slots
        assert a.donor_batches[0][0] == 0 and a.donor_batches[-1][1] == len(a.donor_off) - 1
        assert all(x[1] == y[0] for x, y in zip(a.donor_batches, a.donor_batches[1:]))


def test_full_size_shapes_match_the_stated_configurations():
    t = gen.make("tiny")
    assert (t.n_requests, t.n_tokens, t.pool_slots, t.shape.tok_bytes) == (1, 512, 4096, 1024)
    assert len(t.donor_off) - 1 == 8 and 0.12 < t.mask.mean() < 0.28
    a = gen.make("llama3-8b")
    assert (a.n_requests, a.n_tokens, a.pool_slots, a.shape.tok_bytes) == (16, 65536, 262144, 128 * 1024)
    assert (a.mask[:1024] == 0).all() and 0.09 < a.mask.mean() < 0.15  # 15 % of the non-system tokens
    f = gen.make("frag")
    assert (f.n_requests, f.n_tokens, f.pool_slots) == (64, 131072, 131072)
    assert abs(f.mask.mean() - 0.40) < 0.02 and abs(f.pool_slots / f.table_capacity - 0.85) < 1e-3
    r = gen.make("rope")
    assert (r.n_requests, r.n_tokens, r.rope_theta) == (16, 131072, 500000.0)
    assert r.notes["max_shift"] == 512 and r.notes["reused_runs"] > 2000 and abs(r.mask.mean() - 0.25) < 0.02
    b = gen.make("llama3-70b")
    assert (b.n_requests, b.n_tokens, b.pool_slots, b.shape.tok_bytes) == (4, 131072, 393216, 320 * 1024)
    assert b.pool_slots * b.shape.tok_bytes == 120 * 2**30 and 0.06 < b.mask.mean() < 0.11


def test_float_workload_and_recompute_draws():
    f = gen.make("float", scale=0.25)
    g = gen.make("float", scale=0.25)
    assert np.array_equal(f.tok, g.tok) and np.array_equal(f.donor_u, g.donor_u)
    assert (f.n_requests, f.n_tokens) == (4, 4096) and len(f.donor_off) - 1 == 16
    # documents are stored on their own; in the requests they sit behind text of the request's own
    first_doc = f.donor_tok[f.donor_off[0]:f.donor_off[1]]
    assert not any(np.array_equal(f.tok[o:o + 8], first_doc[:8]) for o in f.off[:-1])  # no request starts with a document
    # the recompute draw travels with the text: the shared prefix of the 8B-shaped donors carries one draw
    a = gen.make("llama3-8b", scale=1 / 16)
    p = 64  # prefix length at this scale
    assert np.array_equal(a.donor_tok[:p], a.donor_tok[a.donor_off[1]:a.donor_off[1] + p])
    assert np.array_equal(a.donor_u[:p], a.donor_u[a.donor_off[1]:a.donor_off[1] + p])
    assert a.donor_u.dtype == np.float32 and 0.2 < (f.donor_u < 0.25).mean() < 0.3  # float: no repeated text
    sub = gen.subsample(a, 1)
    assert len(sub.donor_u) == len(sub.donor_tok)


def test_attention_generator():
    from cp_workload import attn as AT
    a, b = AT.make_attention(300), AT.make_attention(300)
    assert np.array_equal(a, b) and a.shape == (300, 300) and a.dtype == np.float32
    assert (np.triu(a, 1) == 0).all() and np.allclose(a.sum(axis=1), 1.0, atol=1e-5) and (a >= 0).all()
    assert a[:, :4].sum() > 4 * a[:, 4:8].sum() * 0.5  # the sink tokens draw visible weight
    assert AT.make_attention(10, ld=16).shape == (10, 16)
    m = AT.make_mask(20000, run_mean=8.0, cover=0.01)
    assert 0.004 < m.mean() < 0.02 and AT.make_mask(50, cover=0.0).sum() == 0
    assert 0.4 < AT.make_mask(5000, run_mean=1.0, cover=0.6).mean() < 0.8
