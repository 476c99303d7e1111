"""Parity of libcacheprune (HIP, through the C ABI) against the CPU oracle on the
same seeded inputs: hashes, slots, spans, inserted slots and copied rows bit for
bit; re-rotated keys within one bf16 step."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen, kvgen
from oracle import harness as OH
from tests.exact_rope import exact_rotation

pytestmark = pytest.mark.gpu

NONE = O.SLOT_NONE


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a ROCm device; there is no fallback path")
    from paper_2605_23640_amd import harness as gpu_run

    return gpu_run


def bf16_ordinal(bits):
    """Map bf16 bit patterns to integers that are consecutive for adjacent values."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def compare_all(G, wl, max_ulp_sample=None, anchor_window=None, verify=False, min_len=1,
                recompute=None, zero_fill=False, pool_layout="token"):
    """Run prefill + lookup on both sides and compare everything."""
    fl = []
    ost = OH.prefill(wl, flags_out=fl, anchor_window=anchor_window, verify=verify, recompute=recompute)
    olk = OH.lookup(ost, min_len=min_len, zero_fill=zero_fill)
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=anchor_window, verify=verify,
                                    min_len=min_len, recompute_marks=recompute is not None, zero_fill=zero_fill,
                                    pool_layout=pool_layout),
                    recompute=recompute)
    glk = G.lookup(gst)
    assert np.array_equal(glk.served, olk.served)
    if recompute is not None:
        assert np.array_equal(gst.pool.slot_recompute.cpu().numpy(), ost.marks)
    if anchor_window is not None:
        assert np.array_equal(glk.run_off, olk.run_off)
        assert np.array_equal(glk.hash_float, olk.hash_float)
        assert np.array_equal(glk.hash_late, olk.hash_late)
    N = wl.n_tokens
    assert np.array_equal(gst.donor_hash, ost.donor_hash)
    assert np.array_equal(gst.donor_slot, ost.donor_slot)
    assert sum(gst.n_inserted) == ost.n_used and gst.flags == fl[0]
    assert np.array_equal(G.host_u32(gst.pool.slot_pos.view(torch.int32))[ost.slot_uid != kvgen.UID_NONE].view(np.int32),
                          ost.slot_pos[ost.slot_uid != kvgen.UID_NONE])
    # the pool itself: every stored slot holds its donor token's rows, every other slot is untouched
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0
    assert np.array_equal(glk.hash, olk.hash)
    assert np.array_equal(glk.slot, olk.slot)
    assert glk.n_spans == olk.n_spans and glk.flags == olk.flags
    for f in ("span_src", "span_dst", "span_len"):
        assert np.array_equal(getattr(glk, f), getattr(olk, f)), f
    if wl.rope_theta is not None:
        assert np.array_equal(glk.span_delta, olk.span_delta)
    assert np.array_equal(glk.span_off, np.concatenate([[0], np.cumsum(olk.span_len)]).astype(np.uint32))
    got = G.dst_as_rows(glk.dst, wl.shape, N)
    if wl.rope_theta is None:
        assert np.array_equal(got, olk.dst)
    else:
        assert np.array_equal(got[:, 1], olk.dst[:, 1])  # V rows: bit exact
        d = np.abs(bf16_ordinal(got[:, 0]) - bf16_ordinal(olk.dst[:, 0]))
        hist = np.bincount(np.minimum(d, 2).ravel(), minlength=3)
        print("bf16 ordinal distance of re-rotated keys {0,1,>1}:", hist.tolist())
        assert hist[2] == 0  # within one bf16 step of the double-precision result, every element
        assert hist[1] <= 1e-3 * hist.sum()
    return ost, olk, gst, glk


def test_tiny_config(G):
    wl = gen.make("tiny")
    ost, olk, gst, glk = compare_all(G, wl)
    assert glk.n_spans > 100 and (glk.slot != NONE).mean() > 0.5


def test_llama8b_shape_small(G):
    # true row shape (32 layers x 8 heads x 128), a few thousand tokens: several scan tiles + ragged tail
    wl = gen.make_docs("llama3-8b-small", 0xC0FFEE02, gen.KVShape(32, 8, 128), R=3, T=1371, prefix_len=300, n_docs=6,
                       doc_len=(150, 300), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096)
    compare_all(G, wl)


def test_layer_major_pool_whole_path(G):
    """The pool's layout is the caller's choice (three strides): insert, lookup and re-rotation with one plane per
    (layer, K|V) instead of contiguous tokens give the same slots, spans and rows."""
    wl = gen.make_docs("llama3-8b-small", 0xC0FFEE02, gen.KVShape(32, 8, 128), R=3, T=1371, prefix_len=300, n_docs=6,
                       doc_len=(150, 300), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096)
    compare_all(G, wl, pool_layout="layer")
    compare_all(G, gen.make_rope(scale=1 / 32, shape=gen.KVShape(3, 2, 128)), pool_layout="layer", anchor_window=8,
                verify=True)


def test_llama70b_shape_small(G):
    wl = gen.make_docs("llama3-70b-small", 0xC0FFEE05, gen.KVShape(80, 8, 128), R=2, T=700, prefix_len=200, n_docs=5,
                       doc_len=(60, 120), docs_per_request=4, run_mean=12.0, cover=0.10, pool_slots=1024,
                       donor_batch_tokens=700)
    assert len(wl.donor_batches) > 1
    compare_all(G, wl)


def test_frag_small_high_load(G):
    wl = gen.make_frag(scale=1 / 32, shape=gen.KVShape(4, 8, 128))
    assert abs(wl.pool_slots / wl.table_capacity - 0.85) < 0.01
    ost, olk, gst, glk = compare_all(G, wl)
    assert gst.pool.n_used == wl.pool_slots  # the pool is exactly full


@pytest.mark.parametrize("style", [0, 1])
def test_rope_small(G, style):
    wl = gen.make_rope(scale=1 / 16, shape=gen.KVShape(3, 8, 128))
    wl.rope_style = style
    ost, olk, gst, glk = compare_all(G, wl)
    assert (glk.span_delta != 0).mean() > 0.8


def test_rope_small_head_dim_64_and_large_shifts(G):
    wl = gen.make_rope(scale=1 / 4, shape=gen.KVShape(1, 2, 64), max_shift=4 * 4096)  # deltas anywhere in the 2048-token prompts
    ost, olk, gst, glk = compare_all(G, wl)
    assert np.abs(glk.span_delta).max() > 1000


@pytest.mark.parametrize("base", [0x9E3779B97F4A7C15, 3, 10])
def test_other_bases_of_the_chain_hash(G, base):
    """The base is an argument of every hashing call (Sec. 4.2.2 draws it at random).  A 64-bit odd base, a tiny
    one, and the even base of the paper's decimal example, whose powers vanish mod 2^64 after 64 tokens so that
    long runs collide in crowds: keys, slots and served bytes still equal the oracle's, with and without
    floating anchors and confirmation of matches (storing every text once: test_gpu_dedup.py)."""
    wl = gen.make_float(scale=1 / 4, shape=gen.KVShape(2, 2, 64))
    wl.hash_base = base
    compare_all(G, wl)
    compare_all(G, wl, anchor_window=8)
    compare_all(G, wl, anchor_window=8, verify=True)
    wl.rope_theta, wl.rope_style = 500000.0, 0
    compare_all(G, wl, anchor_window=16, verify=True, min_len=4)


@pytest.mark.parametrize("shape", [(1, 64, 128), (2, 40, 128), (1, 16, 512), (70, 1, 32)])
def test_rows_longer_than_a_step_of_the_mover_and_many_layers(G, shape):
    """Rows of 16 KiB, 10 KiB and 16 KiB: a step of the mover's 256 lanes covers a quarter of a row or less, so a
    lane changes column from step to step and (second shape) row boundaries fall inside a step.  And 140 rows of
    64 bytes.  Copying and rotating."""
    sh = gen.KVShape(*shape)
    compare_all(G, gen.make_docs("long-rows", 0xC0FFEEA0 + shape[1], sh, R=3, T=500, prefix_len=80, n_docs=5,
                                 doc_len=(40, 120), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=2048))
    wl = gen.make_rope(seed=0xC0FFEEB0 + shape[1], scale=1 / 16, shape=sh)
    ost, olk, gst, glk = compare_all(G, wl)
    assert (glk.span_delta[:glk.n_spans] != 0).mean() > 0.5


@pytest.mark.parametrize("shape", [(2, 1, 256), (1, 2, 512), (2, 3, 256), (1, 1, 512)])
def test_rope_with_heads_of_256_and_512_elements(G, shape):
    """The widest heads the rotating gather takes: a head's two halves then lie 16 or 32 lanes apart, and the
    cos/sin values of one destination fill a quarter or half of the workgroup's table, so that a slot read by
    many requests is served in passes of 8 or 4 destinations.  Both pairing styles, both pool layouts."""
    sh = gen.KVShape(*shape)
    for style, layout in ((0, "token"), (1, "layer")):
        wl = gen.make_rope(seed=0xC0FFEE80 + shape[1] + shape[2], scale=1 / 16, shape=sh)
        wl.rope_style = style
        ost, olk, gst, glk = compare_all(G, wl, pool_layout=layout)
        assert (glk.span_delta != 0).mean() > 0.8
        # one stored text read by twelve requests, each of which has it at another position: chains of twelve
        # destinations with twelve different rotations
        rng = np.random.default_rng(shape[2])
        doc = rng.integers(0, 32000, 640).astype(np.uint32)  # more slots than the mover has workgroups: chains stay chains
        behind = lambda k: (np.concatenate([np.ones(k), doc]).astype(np.uint32),  # noqa: E731  (k sensitive tokens in front)
                            np.concatenate([np.ones(k), np.zeros(len(doc))]).astype(np.uint8))
        reqs = [behind(k) for k in (0, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233)]
        wl = gen.from_prompts("wide-heads", 0xC0FFEE90 + shape[2], sh, [behind(1)[0]], [r[0] for r in reqs], pool_slots=1024,
                              donor_masks=[behind(1)[1]], request_masks=[r[1] for r in reqs])
        wl.rope_theta, wl.rope_style = 500000.0, style
        ost, olk, gst, glk = compare_all(G, wl, pool_layout=layout)
        assert (glk.slot != NONE).sum() == 12 * 640 and len(set(glk.span_delta[:glk.n_spans].tolist())) == 12


@pytest.mark.parametrize("shape", [(2, 3, 64), (3, 5, 128), (1, 6, 16), (2, 7, 32), (1, 12, 64)])
def test_head_counts_that_are_not_powers_of_two(G, shape):
    """Rows of 24, 80, 12, 28 and 96 sixteen-byte vectors: a step of the mover's 256 lanes then ends in the
    middle of a row, and a wavefront holds K and V rows side by side.  Copying and rotating gathers, both
    pool layouts."""
    sh = gen.KVShape(*shape)
    compare_all(G, gen.make_docs("odd-heads", 0xC0FFEE40 + shape[1], sh, R=3, T=700, prefix_len=100, n_docs=6,
                                 doc_len=(60, 200), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096))
    for style, layout in ((0, "token"), (1, "layer")):
        wl = gen.make_rope(seed=0xC0FFEE50 + shape[1], scale=1 / 16, shape=sh)
        wl.rope_style = style
        ost, olk, gst, glk = compare_all(G, wl, pool_layout=layout)
        assert (glk.span_delta != 0).mean() > 0.8


@pytest.mark.parametrize("shape", [(32, 1, 128), (5, 2, 128), (3, 1, 128), (7, 4, 128)])
def test_short_rows_of_a_tensor_parallel_share(G, shape):
    """One or a few KV heads per GPU, as on a rank of a tensor-parallel model: rows of 256 B to 1 KiB and small
    tokens.  The mover then takes several tokens per visit to its work counter (in strides, with a ragged last
    group), and a rotating gather deals the K rows and the V rows of a step to different wavefronts, also where
    the last step of a token holds fewer rows than a full one (5, 3 and 7 layers)."""
    sh = gen.KVShape(*shape)
    ost, olk, gst, glk = compare_all(G, gen.make_docs("tp-share", 0xC0FFEE70 + shape[0], sh, R=6, T=1500, prefix_len=200,
                                                      n_docs=8, doc_len=(100, 300), docs_per_request=4, run_mean=8.0,
                                                      cover=0.15, pool_slots=8192))
    assert (glk.slot != NONE).sum() > 3000  # several groups of tickets
    for style, layout in ((0, "token"), (1, "layer")):
        wl = gen.make_rope(seed=0xC0FFEE60 + shape[0], scale=1 / 4, shape=sh)
        wl.rope_style = style
        ost, olk, gst, glk = compare_all(G, wl, pool_layout=layout)
        assert (glk.span_delta != 0).sum() > 1500


@pytest.mark.parametrize("shape", [(2, 2, 64), (4, 8, 128)])
def test_thousands_of_destinations_read_a_few_slots(G, shape):
    """Read sharing at its extremes.  Five thousand one-token requests for the same stored token: fewer chains
    than workgroups, so the mover drops the links and moves every token on its own.  Then six hundred stored
    tokens asked for ten times each: chains of ten, walked by the workgroup that takes them.  Copying and
    rotating (the stored tokens sit behind a sensitive token, one position further on than in the requests)."""
    sh = gen.KVShape(*shape)
    rng = np.random.default_rng(3)
    lead = lambda t: np.concatenate([[1], t]).astype(np.uint32)  # noqa: E731  (a sensitive token in front)
    lead_mask = lambda t: np.concatenate([[1], np.zeros(len(t))]).astype(np.uint8)  # noqa: E731
    one = [np.array([7, 9, 11], np.uint32)]
    many = [np.array([t], np.uint32) for t in rng.permutation(32000)[:600]]
    for donors, reqs in ((one, [np.array([7], np.uint32)] * 5000 + [np.array([7, 9], np.uint32)] * 50),
                         (many, [many[i % 600] for i in range(6000)])):
        wl = gen.from_prompts("few-slots", 5, sh, [lead(d) for d in donors], reqs, pool_slots=1024,
                              donor_masks=[lead_mask(d) for d in donors])
        ost, olk, gst, glk = compare_all(G, wl)
        assert (glk.slot != NONE).all() and len(np.unique(glk.slot)) <= 600
        wl.rope_theta, wl.rope_style = 500000.0, 0
        ost, olk, gst, glk = compare_all(G, wl)
        assert (glk.span_delta[:glk.n_spans] == -1).all()


def test_contiguous_slots_give_long_spans(G):
    wl = gen.make_docs("contig", 7, gen.KVShape(4, 2, 64), R=4, T=1500, prefix_len=400, n_docs=5, doc_len=(200, 400),
                       docs_per_request=3, run_mean=8.0, cover=0.10, pool_slots=4096)
    wl.free_slots = np.arange(wl.pool_slots, dtype=np.uint32)  # slots handed out in order
    ost, olk, gst, glk = compare_all(G, wl)
    assert glk.span_len.max() >= 100 and glk.n_spans < (glk.slot != NONE).sum() / 4


def test_edge_cases_lookup(G):
    wl = gen.make("tiny")
    ost = OH.prefill(wl)
    gst = G.prefill(wl)
    cases = {
        "empty batch": (np.zeros(0, np.uint32), np.zeros(0, np.uint8), np.array([0], np.uint32)),
        "empty requests": (wl.tok[:5], wl.mask[:5], np.array([0, 0, 5, 5], np.uint32)),
        "single token": (wl.donor_tok[6:7], np.zeros(1, np.uint8), np.array([0, 1], np.uint32)),
        "all sensitive": (wl.tok[:100], np.ones(100, np.uint8), np.array([0, 50, 100], np.uint32)),
        "one-token requests": (wl.tok[:64], wl.mask[:64], np.arange(65, dtype=np.uint32)),
        "donor replay": (wl.donor_tok[:1500], wl.donor_mask[:1500], np.array([0, 512, 1024, 1500], np.uint32)),
    }
    for name, (tok, mask, off) in cases.items():
        o = OH.lookup(ost, tok=tok, mask=mask, off=off)
        g = G.lookup(gst, tok=tok, mask=mask, off=off)
        assert np.array_equal(g.hash, o.hash) and np.array_equal(g.slot, o.slot), name
        assert g.n_spans == o.n_spans and np.array_equal(g.span_src, o.span_src), name
        assert np.array_equal(g.span_dst, o.span_dst) and np.array_equal(g.span_len, o.span_len), name
        if len(tok):
            assert np.array_equal(G.dst_as_rows(g.dst, wl.shape, len(tok)), o.dst), name
    # span capacity: only the first max_spans spans are kept, gathered, and the overflow is flagged
    o = OH.lookup(ost, max_spans=37)
    g = G.lookup(gst, max_spans=37)
    assert o.flags == g.flags == O.FLAG_SPANS_OVERFLOW and g.n_spans == 37 and o.n_spans > 37
    assert np.array_equal(g.span_src, o.span_src) and np.array_equal(g.span_len, o.span_len)
    assert np.array_equal(G.dst_as_rows(g.dst, wl.shape, wl.n_tokens), o.dst)


def test_pool_full_and_repeat_insert(G):
    wl = gen.make("tiny")
    n_free = 700  # fewer slots than the donors need
    fl = []
    wl2 = gen.make("tiny")
    wl2.free_slots = wl.free_slots[:n_free]
    ost = OH.prefill(wl2, flags_out=fl)
    gst = G.prefill(wl, G.make_pool(wl, n_free=n_free))
    assert fl[0] == O.FLAG_POOL_FULL == gst.flags and ost.n_used == n_free == sum(gst.n_inserted)
    assert np.array_equal(gst.donor_slot, ost.donor_slot)
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0
    o, g = OH.lookup(ost), G.lookup(gst)
    assert np.array_equal(g.slot, o.slot) and np.array_equal(G.dst_as_rows(g.dst, wl.shape, wl.n_tokens), o.dst)
    # inserting everything again stores nothing and reports the same slots
    gst2 = G.prefill(wl, gst.pool)
    assert sum(gst2.n_inserted) == 0 and np.array_equal(gst2.donor_slot, ost.donor_slot)


def test_insert_is_deterministic(G):
    wl = gen.make_frag(scale=1 / 64, shape=gen.KVShape(1, 1, 8))
    ref = OH.prefill(wl).donor_slot
    for _ in range(10):
        assert np.array_equal(G.prefill(wl).donor_slot, ref)


def test_layer_major_pool_gather(G):
    """The gather takes any strides: same spans out of a layer-major pool."""
    import ctypes as C

    import paper_2605_23640_amd as cp

    rng = np.random.default_rng(3)
    L, H, D, S, N = 3, 2, 64, 300, 200
    rb = H * D * 2
    pool = rng.integers(0, 65536, (L, 2, S, H * D)).astype(np.uint16)
    src = np.array([10, 250, 40], np.uint32)
    dst = np.array([0, 50, 199], np.uint32)
    ln = np.array([30, 50, 1], np.uint32)
    want = np.full((L, 2, N, H * D), kvgen.POISON16, np.uint16)
    O.gather_kv(pool, O.Layout(L, H, D, rb, 2 * S * rb, S * rb), want, O.Layout(L, H, D, rb, 2 * N * rb, N * rb), src,
                dst, ln)
    dpool = torch.from_numpy(pool.view(np.int16)).to(G.DEV)
    out = G.poison_tensor(N * L * 2 * rb)
    flags = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    n_sp = torch.tensor([3], dtype=torch.int32, device=G.DEV)
    scratch = cp.binding.new_scratch(N, 8, G.DEV, S)
    cp.cp_gather_kv(dpool, cp.binding.KVLayout.layer_major(L, H, D, S), S, out, cp.binding.KVLayout.layer_major(L, H, D, N),
                    N, G.dev_i32(src), G.dev_i32(dst), G.dev_i32(ln), None, None, n_sp, 8, None, flags, scratch)
    torch.cuda.synchronize()
    assert np.array_equal(G.dst_as_rows(out, gen.KVShape(L, H, D), N), want) and int(flags.item()) == 0
    # a span that points outside the pool is skipped and flagged, nothing else is disturbed
    out2 = G.poison_tensor(N * L * 2 * rb)
    bad_src = np.array([10, 290, 40], np.uint32)  # 290 + 50 > 300 slots
    cp.cp_gather_kv(dpool, cp.binding.KVLayout.layer_major(L, H, D, S), S, out2,
                    cp.binding.KVLayout.layer_major(L, H, D, N), N, G.dev_i32(bad_src), G.dev_i32(dst), G.dev_i32(ln),
                    None, None, n_sp, 8, None, flags, scratch)
    torch.cuda.synchronize()
    assert int(flags.item()) == cp.binding.FLAG_BAD_INDEX
    got = G.dst_as_rows(out2, gen.KVShape(L, H, D), N)
    assert np.array_equal(got[:, :, :50], want[:, :, :50]) and np.array_equal(got[:, :, 199], want[:, :, 199])
    assert np.array_equal(got[:, :, 50:60], pool[:, :, 290:300]) and (got[:, :, 60:100] == kvgen.POISON16).all()


def test_argument_errors_are_reported_not_launched(G):
    import paper_2605_23640_amd as cp

    t = torch.zeros(64, dtype=torch.int32, device=G.DEV)
    h = torch.zeros(64, dtype=torch.int64, device=G.DEV)
    small = torch.zeros(256, dtype=torch.uint8, device=G.DEV)
    with pytest.raises(cp.binding.CpError) as e:
        cp.cp_hash_segments(t, t.view(torch.uint8)[:64], t[:2], h, small[:16])
    assert e.value.code == cp.binding.ERR_SCRATCH
    tab = cp.binding.Table(64, G.DEV)
    tab.capacity = 40  # not a multiple of the bucket size
    with pytest.raises(cp.binding.CpError) as e:
        cp.cp_probe(tab, h, t)
    assert e.value.code == cp.binding.ERR_INVALID_ARG


def test_verify_kernel_counts_real_differences(G):
    """The device-side checker used at full size: agrees with the host generator and reports what differs."""
    import ctypes as C

    import paper_2605_23640_amd as cp

    L, H, D, n = 3, 2, 64, 37
    lay = cp.binding.KVLayout.layer_major(L, H, D, n)
    buf = torch.empty(n * L * 2 * H * D * 2, dtype=torch.uint8, device=G.DEV)
    kvgen.fill(G.stream_ptr(), C.c_void_p(buf.data_ptr()), G.gen_layout(lay), n, 99, uid_base=1000)
    host = kvgen.rows_for_tokens(99, np.arange(1000, 1000 + n), L, H * D).transpose(1, 2, 0, 3)
    assert np.array_equal(G.dst_as_rows(buf, gen.KVShape(L, H, D), n), host)  # device fill == host definition
    uids = np.arange(1000, 1000 + n, dtype=np.uint64)
    assert G.verify_rows(buf, lay, uids, 99) == 0
    wrong = uids.copy()
    wrong[5] += 1  # one token expected to be another one: (nearly) all its elements differ
    bad = G.verify_rows(buf, lay, wrong, 99)
    assert 0.9 * L * 2 * H * D < bad <= L * 2 * H * D
    assert G.verify_rows(buf, lay, uids, 98) > 0.9 * n * L * 2 * H * D  # another seed: everything differs
    buf.view(torch.int16)[7] += 1  # a single flipped element is seen
    assert G.verify_rows(buf, lay, uids, 99) == 1


def test_two_pools_on_two_streams_with_different_launch_options(G):
    """Every call takes the caller's stream and its own launch options: two pools' lookups, issued at the same
    time on two streams with different options for the row mover, give what each gives alone on the default
    stream with the default options (the library keeps no state between calls; each pool has its own scratch)."""
    import paper_2605_23640_amd as cp

    wl = gen.make_docs("streams", 0xC0FFEE0E, gen.KVShape(4, 2, 64), R=3, T=900, prefix_len=200, n_docs=6,
                       doc_len=(100, 200), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096)
    st_a = G.prefill(wl, G.make_pool(wl, anchor_window=8, verify=True, min_len=4))
    st_b = G.prefill(wl, G.make_pool(wl))
    want_a, want_b = G.lookup(st_a), G.lookup(st_b)  # default stream, the pools' own options
    N, sh = wl.n_tokens, wl.shape
    tok, mask, off = G.dev_i32(wl.tok), torch.from_numpy(wl.mask.copy()).to(G.DEV), G.dev_i32(wl.off)
    bufs = [cp.LookupBuffers(N, N, G.DEV, n_pool_slots=st.pool.n_slots) for st in (st_a, st_b)]
    dsts = [G.poison_tensor(N * sh.tok_bytes) for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]  # default priority
    opts = [cp.binding.LaunchOpts(read_sharing=1, loads_in_flight=4, workgroups=64, fanout=2),
            cp.binding.LaunchOpts(read_sharing=2, nontemporal=4, loads_in_flight=8, blocks_per_cu=2)]
    torch.cuda.synchronize()
    for _ in range(3):  # interleaved launches on the two streams
        for st, buf, dst, s, o in zip((st_a, st_b), bufs, dsts, streams, opts):
            st.pool.lookup(tok, mask, off, dst, buf, stream=s, gather_opts=o)
    for s in streams:
        s.synchronize()
    for want, buf, dst, st in zip((want_a, want_b), bufs, dsts, (st_a, st_b)):
        assert np.array_equal(G.host_u32(buf.slot), want.slot)
        assert np.array_equal(G.host_u32(buf.served if st.pool.filters else buf.slot), want.served)
        assert np.array_equal(G.dst_as_rows(dst, sh, N), G.dst_as_rows(want.dst, sh, N))
        assert int(st.pool.flags.item()) == 0


def test_insert_and_evict_on_a_stream_that_is_not_the_current_one(G):
    """insert() and evict() read a count back on the host: they must wait for the stream their kernels ran on.
    The same life cycle (store, look up, evict, store more) on a side stream and on the default stream leaves
    the same slots, free list and pool bytes."""
    import paper_2605_23640_amd as cp

    wl = gen.make_docs("side-stream", 0xC0FFEE0F, gen.KVShape(2, 2, 64), R=4, T=600, prefix_len=100, n_docs=8,
                       doc_len=(80, 160), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=2048)
    sh = wl.shape

    def life_cycle(side):
        pool = G.make_pool(wl, lru=True)
        stream = torch.cuda.Stream() if side else None
        out = []
        with torch.cuda.stream(torch.cuda.default_stream()):  # the current stream stays the default one
            for first, last in ((0, 2), (2, 4)):
                t0, t1 = int(wl.off[first]), int(wl.off[last])
                n = t1 - t0
                src = torch.empty(n * sh.tok_bytes, dtype=torch.uint8, device=G.DEV)
                kvgen.fill(G.stream_ptr(), C.c_void_p(src.data_ptr()), G.gen_layout(pool.request_layout(n)), n, wl.seed,
                           uid_base=t0)
                tok, mask = G.dev_i32(wl.tok[t0:t1]), torch.from_numpy(wl.mask[t0:t1].copy()).to(G.DEV)
                off = G.dev_i32((wl.off[first:last + 1] - wl.off[first]).astype(np.uint32))
                hbuf = torch.empty(n, dtype=torch.int64, device=G.DEV)
                sout = torch.empty(n, dtype=torch.int32, device=G.DEV)
                scratch = cp.binding.new_scratch(n, 0, G.DEV, pool.n_slots)
                buf = cp.LookupBuffers(n, n, G.DEV, n_pool_slots=pool.n_slots)
                dst = G.poison_tensor(n * sh.tok_bytes)
                torch.cuda.synchronize()  # inputs were prepared on the default stream
                pool.epoch += 1
                pool.lookup(tok, mask, off, dst, buf, stream=stream)
                stored = pool.insert(tok, mask, off, src, hbuf, sout, scratch, stream=stream)
                freed = pool.evict(200, scratch, stream=stream) if first == 0 else None
                torch.cuda.synchronize()
                out.append((stored, G.host_u32(sout).copy(), G.host_u32(buf.slot).copy(),
                            None if freed is None else G.host_u32(freed).copy(), pool.n_used,
                            G.host_u32(pool.free_slots).copy(), dst.cpu().numpy().copy()))
        return out, pool.pool.cpu().numpy()

    (want, want_pool), (got, got_pool) = life_cycle(False), life_cycle(True)
    assert want[0][0] > 0 and len(want[0][3]) >= 200 and want[1][0] > 0
    for w, g in zip(want, got):
        assert w[0] == g[0] and w[4] == g[4]
        for x, y in zip(w[1:4] + w[5:], g[1:4] + g[5:]):
            assert (x is None and y is None) or np.array_equal(x, y)
    assert np.array_equal(want_pool, got_pool)


def test_hash_and_probe_in_one_pass_equal_the_two_calls(G):
    """cp_hash_probe against cp_hash_segments / cp_hash_runs followed by cp_probe, on a table at load 0.85
    (walks over several buckets) and on batches that take the scan's one-, two- and three-launch form."""
    import paper_2605_23640_amd as cp

    wl = gen.make_frag(scale=1 / 32, shape=gen.KVShape(2, 2, 64))
    st = G.prefill(wl)
    rng = np.random.default_rng(5)
    for n_rep in (1, 3, 140):  # 4096 tokens per copy of the batch
        tok = np.tile(wl.tok, n_rep)[: 4096 * n_rep if n_rep > 1 else 700]
        mask = np.tile(wl.mask, n_rep)[: len(tok)]
        off = np.unique(np.concatenate([[0, len(tok)], rng.integers(0, len(tok), 7)])).astype(np.uint32)
        d_tok, d_mask, d_off = G.dev_i32(tok), torch.from_numpy(mask.copy()).to(G.DEV), G.dev_i32(off)
        N = len(tok)
        scratch = cp.binding.new_scratch(N, 0, G.DEV)
        h1, h2 = (torch.empty(N, dtype=torch.int64, device=G.DEV) for _ in range(2))
        r1, r2, s1, s2 = (torch.empty(N, dtype=torch.int32, device=G.DEV) for _ in range(4))
        cp.cp_hash_runs(d_tok, d_mask, d_off, h1, r1, scratch)
        cp.cp_probe(st.pool.table, h1, s1)
        cp.cp_hash_probe(d_tok, d_mask, d_off, st.pool.table, h2, r2, s2, scratch)
        torch.cuda.synchronize()
        assert torch.equal(h1, h2) and torch.equal(r1, r2) and torch.equal(s1, s2), N
        assert np.array_equal(G.host_u64(h1), O.hash_segments(tok, mask, off))
        assert (G.host_u32(s1) != NONE).mean() > 0.3


def test_table_overflow_stores_nothing_and_a_rebuilt_table_goes_on(G):
    """A batch whose new keys do not fit the table sets TABLE_FULL and stores nothing, whatever the order in which
    its tokens reached the table; after the table has been rebuilt into a larger one the same batch is stored."""
    import paper_2605_23640_amd as cp

    rng = np.random.default_rng(12)
    V = lambda n: rng.integers(0, 32000, n).astype(np.uint32)  # noqa: E731
    a, b, c = V(70), V(90), V(30)
    donors = [a, np.concatenate([a[:40], b]), c]  # 70 keys fit 96 entries; the second batch brings 90 more; the third 30
    wl = gen.from_prompts("table-overflow", 0xC0FFEE41, gen.KVShape(2, 2, 64), donors, [np.concatenate([a, V(3), c])],
                          pool_slots=512, donor_batch_tokens=100)
    wl.table_capacity = 96
    assert len(wl.donor_batches) == 3
    fl = []
    ost = OH.prefill(wl, flags_out=fl, bounded_table=True)
    gst = G.prefill(wl)
    assert gst.pool.table.capacity == 96
    assert fl[0] == O.FLAG_TABLE_FULL and gst.flags == fl[0]
    assert np.array_equal(gst.donor_slot, ost.donor_slot) and gst.n_inserted == [70, 0, 0] and ost.n_used == 70
    o = wl.donor_off
    assert (ost.donor_slot[o[1]:o[1] + 40] != NONE).all() and (ost.donor_slot[o[1] + 40:] == NONE).all()
    assert G.verify_rows(gst.pool.pool, gst.pool.layout, ost.slot_uid, wl.seed) == 0
    pool = gst.pool
    counts = torch.empty(2, dtype=torch.int32, device=G.DEV)

    def table_counts():  # (entries holding a key, of which with a slot)
        cp.cp_table_count(pool.table, counts)
        return tuple(G.host_u32(counts).tolist())

    used, live = table_counts()  # which keys of the failed batches took the last entries is not specified
    assert live == len(ost.index) == 70 and ost.index.entries == 70 <= used <= 96
    # rebuild into a larger table and store the two batches again
    fresh = cp.binding.Table(512, G.DEV)
    cp.cp_table_compact(pool.table, fresh, pool.flags)
    pool.table = fresh
    pool.flags.zero_()
    ost.index.rebuild(512)
    for d in (1, 2):
        t0, t1 = int(o[d]), int(o[d + 1])
        n = t1 - t0
        tok, mask, off = wl.donor_tok[t0:t1], wl.donor_mask[t0:t1], np.array([0, n], np.uint32)
        src = torch.empty(n * wl.shape.tok_bytes, dtype=torch.uint8, device=G.DEV)
        kvgen.fill(G.stream_ptr(), C.c_void_p(src.data_ptr()), G.gen_layout(pool.request_layout(n)), n, wl.seed, uid_base=t0)
        hbuf = torch.empty(n, dtype=torch.int64, device=G.DEV)
        sout = torch.empty(n, dtype=torch.int32, device=G.DEV)
        got_n = pool.insert(G.dev_i32(tok), torch.from_numpy(mask.copy()).to(G.DEV), G.dev_i32(off), src, hbuf, sout,
                            cp.binding.new_scratch(n, 0, G.DEV))
        so, n_new, f2 = O.insert_kv(ost.index, O.hash_segments(tok, mask, off), off, wl.free_slots[ost.n_used:],
                                    OH.gen_buffer(wl.seed, wl.shape, t0, n), OH.buf_layout(wl.shape, n), ost.pool,
                                    OH.pool_layout(wl.shape), ost.slot_pos)
        ost.n_used += n_new
        assert f2 == 0 and int(pool.flags.item()) == 0 and got_n == n_new == (90 if d == 1 else 30)
        assert np.array_equal(G.host_u32(sout), so)
        assert table_counts() == (ost.index.entries, len(ost.index))
    assert table_counts() == (190, 190)
    glk, olk = G.lookup(gst), OH.lookup(ost)
    assert np.array_equal(glk.slot, olk.slot) and (glk.slot != NONE).sum() == 70  # (the request has c behind other text)


def test_rope_deltas_up_to_the_whole_int32_range(G):
    """Position deltas of any size: every digit level of the kernel's cos/sin tables, INT_MAX, INT_MIN + 1 and
    INT_MIN (whose magnitude does not fit an int32), element by element against an 80-digit reference (the
    double-precision oracle's own angle delta * frequency is rounded to 2^-22 rad at such sizes, so it is
    compared with the same reference, one step more loosely)."""
    import paper_2605_23640_amd as cp

    sh = gen.KVShape(2, 2, 128)
    theta = 500000.0
    deltas = np.array([1, -1, 127, 128, -16383, 16384, -2097151, 1 << 21, (1 << 28) + 12345, -(1 << 30), 1 << 30,
                       2**31 - 1, -(2**31) + 1, -(2**31)], np.int64).astype(np.int32)
    n = len(deltas)
    pool_l = cp.binding.KVLayout.token_major(sh.n_layers, sh.n_kv_heads, sh.head_dim)
    dst_l = cp.binding.KVLayout.layer_major(sh.n_layers, sh.n_kv_heads, sh.head_dim, n)
    pool = torch.empty(n * sh.tok_bytes, dtype=torch.uint8, device=G.DEV)
    kvgen.fill(G.stream_ptr(), C.c_void_p(pool.data_ptr()), G.gen_layout(pool_l), n, 77, uid_base=500)
    dst = G.poison_tensor(n * sh.tok_bytes)
    ar = torch.arange(n, dtype=torch.int32, device=G.DEV)
    ones = torch.ones(n, dtype=torch.int32, device=G.DEV)
    flags = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    n_spans = torch.tensor([n], dtype=torch.int32, device=G.DEV)
    cp.cp_gather_kv(pool, pool_l, n, dst, dst_l, n, ar, ar, ones, torch.from_numpy(deltas).to(G.DEV), None, n_spans, n,
                    cp.binding.Rope(theta, 0), flags, cp.binding.new_scratch(n, n, G.DEV, n))
    torch.cuda.synchronize()
    assert int(flags.item()) == 0
    got = G.dst_as_rows(dst, sh, n)  # [L][2][n][row]
    src = kvgen.rows_for_tokens(77, np.arange(500, 500 + n, dtype=np.uint64), sh.n_layers, sh.row_bytes // 2)
    assert np.array_equal(got[:, 1], src[:, :, 1].transpose(1, 0, 2))  # V rows: bit exact
    D = sh.head_dim
    worst_gpu = worst_oracle = 0
    for t, dl in enumerate(deltas):
        for l in range(sh.n_layers):
            for h in range(sh.n_kv_heads):
                x = src[t, l, 0, h * D:(h + 1) * D]
                want = exact_rotation(x, int(dl), theta, D)
                worst_gpu = max(worst_gpu, int(np.abs(bf16_ordinal(got[l, 0, t, h * D:(h + 1) * D]) - bf16_ordinal(want)).max()))
                worst_oracle = max(worst_oracle, int(np.abs(bf16_ordinal(O.rope_head(x, int(dl), theta, 0)) - bf16_ordinal(want)).max()))
    print(f"bf16 distance from the 80-digit rotation: GPU <= {worst_gpu}, double-precision oracle <= {worst_oracle}")
    assert worst_gpu <= 1 and worst_oracle <= 2
