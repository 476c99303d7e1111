"""cp_gather_kv_static (the gather whose working memory is an array inside the library's device
code, for callers that cannot allocate) against cp_gather_kv on the same spans: every byte of the
request buffers equal, on two calls in a row, the second with a smaller input — the shared array
still holds the first call's descriptors, chain heads and tables then."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_23640_amd as cp
from cp_workload import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a ROCm device; there is no fallback path")
    from paper_2605_23640_amd import harness as gpu_run

    return gpu_run


def both_gathers(G, st, n_requests):
    """Look the first n_requests requests up, then gather their spans once through each entry point."""
    wl = st.wl
    N = int(wl.off[n_requests])
    lk = G.lookup(st, tok=wl.tok[:N], mask=wl.mask[:N], off=wl.off[:n_requests + 1], gather=False)
    assert lk.n_spans > 0
    pool = st.pool
    dev = lambda a: G.dev_i32(a)  # noqa: E731
    src, dstp, ln = dev(lk.span_src), dev(lk.span_dst), dev(lk.span_len)
    delta = dev(lk.span_delta) if pool.rope is not None else None
    n_spans = torch.tensor([lk.n_spans], dtype=torch.int32, device=G.DEV)
    lay = pool.request_layout(N)
    out = []
    for static in (False, True):
        dst = G.poison_tensor(N * wl.shape.tok_bytes)
        pool.flags.zero_()
        if static:
            cp.cp_gather_kv_static(pool.pool, pool.layout, pool.n_slots, dst, lay, N, src, dstp, ln, delta, None,
                                   n_spans, lk.n_spans, pool.rope, pool.flags)
        else:
            scratch = cp.binding.new_scratch(N, lk.n_spans, G.DEV, pool.n_slots)
            cp.cp_gather_kv(pool.pool, pool.layout, pool.n_slots, dst, lay, N, src, dstp, ln, delta, None, n_spans,
                            lk.n_spans, pool.rope, pool.flags, scratch)
        torch.cuda.synchronize()
        assert int(pool.flags.item()) == 0
        out.append(dst)
    served = int(lk.span_len.sum())
    assert torch.equal(out[0], out[1]), f"{n_requests} requests: the two entry points wrote different bytes"
    assert not torch.equal(out[1], G.poison_tensor(out[1].numel())), "nothing was gathered"
    return served


@pytest.mark.parametrize("kind", ["copy", "rope"])
def test_static_scratch_gather_equals_the_gather_with_caller_scratch(G, kind):
    if kind == "copy":
        wl = gen.make_docs("static-scratch", 0xC0FFEE11, gen.KVShape(4, 2, 64), R=4, T=700, prefix_len=150, n_docs=6,
                           doc_len=(80, 160), docs_per_request=3, run_mean=8.0, cover=0.15, pool_slots=4096)
    else:
        wl = gen.make_rope(scale=1 / 32, shape=gen.KVShape(3, 2, 128))
    st = G.prefill(wl)
    big = both_gathers(G, st, wl.n_requests)
    small = both_gathers(G, st, 1)  # a smaller input next: what the first call left in the array must not show
    assert 0 < small < big
    again = both_gathers(G, st, wl.n_requests)
    assert again == big


def test_static_scratch_gather_limits_are_errors():
    """Sizes above the array's capacity are refused on the host, before anything is enqueued (no GPU needed
    for that, but the library is only loaded where one is)."""
    B = cp.binding
    L = B.lib()
    P, Q, S = 0x10000, 0x20000, 0x30000
    lay = B.KVLayout.token_major(2, 2, 64)
    call = lambda slots, toks, spans: L.cp_gather_kv_static(None, P, lay, slots, Q, lay, toks, S, S, S, None, None, S,  # noqa: E731
                                                            spans, None, S, None)
    assert call(B.STATIC_MAX_SLOTS + 1, 16, 16) == B.ERR_STATIC_LIMIT
    assert call(16, B.STATIC_MAX_TOKENS + 1, 16) == B.ERR_STATIC_LIMIT
    assert call(16, 16, B.STATIC_MAX_SPANS + 1) == B.ERR_STATIC_LIMIT
    assert call(16, 0, 16) == B.OK  # nothing to do
    assert ctypes.sizeof(B.LaunchOpts) == 48
