"""The library allocates nothing, never synchronises and enqueues kernels only, so a whole step
(lookup with gather, then insert) can be recorded into a HIP graph and replayed.  Every replay must
reproduce the eager result."""
import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import gen
from test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kw", [{}, {"anchor_window": 8, "verify": True, "min_len": 4, "zero_fill": True, "lru": True}])
def test_step_replays_from_a_graph(G, kw):
    import paper_2605_23640_amd as cp
    wl = gen.make("float", scale=0.25)
    wl.shape = gen.KVShape(2, 2, 64)
    st = G.prefill(wl, G.make_pool(wl, **kw))
    pool, sh, N = st.pool, wl.shape, wl.n_tokens
    tok, mask, off = G.dev_i32(wl.tok), torch.from_numpy(wl.mask.copy()).to(G.DEV), G.dev_i32(wl.off)
    buf = cp.LookupBuffers(N, N, G.DEV, n_pool_slots=pool.n_slots)
    dst = G.poison_tensor(N * sh.tok_bytes)
    slot_out = torch.empty(N, dtype=torch.int32, device=G.DEV)
    ins_scratch = cp.binding.new_scratch(N, 0, G.DEV)
    keys0, vals0 = pool.table.keys.clone(), pool.table.vals.clone()
    pool0 = pool.pool.clone()
    anchors0 = pool.slot_anchor.clone() if pool.slot_anchor is not None else None

    def step():
        pool.lookup(tok, mask, off, dst, buf)
        pool.insert(tok, mask, off, dst, buf.hash, slot_out, ins_scratch, sync=False, run_off_buf=buf.run_off)

    def restore():
        pool.table.keys.copy_(keys0)
        pool.table.vals.copy_(vals0)
        pool.pool.copy_(pool0)
        if anchors0 is not None:
            pool.slot_anchor.copy_(anchors0)
        dst.copy_(G.poison_tensor(N * sh.tok_bytes))
        slot_out.fill_(-7)

    step()  # eager reference
    torch.cuda.synchronize()
    want = {"dst": dst.clone(), "slot": buf.slot.clone(), "served": buf.served.clone(), "out": slot_out.clone(),
            "n": int(pool.n_inserted.item()), "pool": pool.pool.clone(), "keys": pool.table.keys.clone()}
    assert want["n"] > 0 and (G.host_u32(want["slot"]) != O.SLOT_NONE).mean() > 0.15
    restore()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    restore()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for replay in range(4):
        restore()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dst, want["dst"]), replay
        assert torch.equal(buf.slot, want["slot"]) and torch.equal(slot_out, want["out"]), replay
        if pool.filters:
            assert torch.equal(buf.served, want["served"]), replay
        assert int(pool.n_inserted.item()) == want["n"] and torch.equal(pool.pool, want["pool"]), replay
        # the arrangement of table entries may differ from run to run, the set of keys may not
        assert np.array_equal(np.sort(G.host_u64(pool.table.keys)), np.sort(G.host_u64(want["keys"]))), replay
        buf.slot.random_(0, 5)  # eager work between replays
        torch.cuda.synchronize()
