#!/usr/bin/env python3
"""Benchmark of the CachePrune KV sharing path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama3-8b]

One *step* is one pass of the whole hot path over one request batch of the
workload, all inputs resident in HBM:

    lookup : cp_hash_segments -> cp_probe -> cp_build_spans -> cp_gather_kv
    insert : cp_insert_kv of the same batch (hashes from the lookup), taking the
             KV rows of the tokens the pool does not hold yet from the request
             buffers
    reset  : the table's key/value arrays are copied back from a snapshot
             (device to device, a few MiB) so that every step meets the same
             pool state; this copy is inside the timed region.

Prints ONE JSON line.  `value` is the KV bytes moved per second by the whole
step (gather and insert, read + write); `roofline` prices the gather kernel
alone against the HBM peak; `cpu_baseline` is the CPU oracle timed on this
host on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published peak HBM3E bandwidth
# HBM bytes of one gather launch as the profiler's counters saw them: rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE runs of this command (defaults, per workload), each scaled by what the same counter
# reads for a plain streaming kernel of known size.  They are copied from the summaries under profiles/
# (gather_rows_kernel_<workload>.txt; annotator_<n>.txt): measurements of an earlier run of the same
# code, not of this run, and the bench line says so next to them.
PROFILED_TRAFFIC = {"llama3-8b": 9036137124, "rope": 9681278928, "llama3-70b": 58311324550, "frag": 17228238218,
                    "annotator-10000-full": 896676416, "annotator-10000": 347912128}
PROFILED_FETCH = {"llama3-8b": 3093454910, "rope": 4436765597, "llama3-70b": 25345741631, "frag": 7416232637}
# scatter_rows_kernel of the default step (scatter_rows_kernel_<workload>.txt and the gather files): (fetched, written)
PROFILED_SCATTER = {"llama3-8b": (1687323882, 1686578150), "rope": (7662540819, 7659772570),
                    "llama3-70b": (6636802933, 6635752960)}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def host_info():
    """CPU model and logical CPU count of the machine the oracle is timed on."""
    model = None
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"cpu": model, "logical_cpus": os.cpu_count(), "oracle_threads": 1}


def cpu_baseline(wl, n_requests, G, torch, np, anchor_window=None, verify=False, min_len=1, recompute=0.0,
                 zero_fill=False):
    """The CPU oracle, as it stands, on the first ``n_requests`` requests of the workload."""
    import oracle as O
    from cp_workload import gen
    from oracle import harness as OH

    sw = gen.subsample(wl, n_requests, pool_slots=1 << 17)
    sh = sw.shape
    n_d = len(sw.donor_tok)
    re = sh.row_bytes // 2
    # donor KV: written by the generator's device kernel, then copied to the host
    dev = torch.empty(n_d * sh.tok_bytes, dtype=torch.uint8, device=G.DEV)
    lay = G.cp.binding.KVLayout.layer_major(sh.n_layers, sh.n_kv_heads, sh.head_dim, n_d)
    from cp_workload import kvgen
    kvgen.fill(G.stream_ptr(), C.c_void_p(dev.data_ptr()), G.gen_layout(lay), n_d, sw.seed, uid_base=0)
    torch.cuda.synchronize()
    host_src = dev.view(torch.int16).cpu().numpy().view(np.uint16).reshape(sh.n_layers, 2, n_d, re)
    del dev
    pool = np.empty((sw.pool_slots, sh.n_layers, 2, re), np.uint16)  # untouched pages stay virtual
    st = OH.prefill(sw, src_provider=lambda t0, n: np.ascontiguousarray(host_src[:, :, t0:t0 + n]), pool=pool,
                    anchor_window=anchor_window, verify=verify,
                    recompute=None if recompute <= 0.0 else (sw.donor_u < recompute).astype(np.uint8))
    del host_src
    lk = OH.lookup(st, min_len=min_len, zero_fill=zero_fill)  # hash, probe, spans, gather: timed inside
    N = sw.n_tokens
    slot_pos = st.slot_pos
    t = time.perf_counter()
    slot_out, n_new, _ = O.insert_kv(st.index, lk.hash, sw.off, sw.free_slots[st.n_used:], lk.dst, OH.buf_layout(sh, N),
                                     st.pool, OH.pool_layout(sh), slot_pos)
    if st.text is not None:
        O.text_record(st.text, sw.tok, lk.run_off, slot_out)
    t_ins = time.perf_counter() - t
    matched = int((lk.served != O.SLOT_NONE).sum())
    t_total = sum(lk.times.values()) + t_ins
    moved = 2.0 * sh.tok_bytes * (matched + n_new)
    return {
        "value": moved / t_total / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {n_requests} of {wl.n_requests} requests ({N} tokens, {matched} reused, {n_new} stored), "
                  f"same step (lookup + insert), pool of {sw.pool_slots} slots with the donors those requests use",
        "reused_tokens_per_s": matched / t_total,
        "seconds": {**{k: round(v, 4) for k, v in lk.times.items()}, "insert": round(t_ins, 4)},
        "host": host_info(),
    }


def annotator_bench(args):
    """Side benchmark (not the headline metric): the KV annotator on one n x n attention matrix."""
    import numpy as np
    import torch

    import oracle as O
    from cp_workload import attn as AT
    from paper_2605_23640_amd import binding as B
    from paper_2605_23640_amd import harness as G

    n, K = args.annotator, args.steps
    t0 = time.time()
    a = AT.make_attention(n)
    mask = AT.make_mask(n, run_mean=8.0, cover=0.01)  # few, short sensitive runs: segments of ~800 tokens
    log(f"[bench] attention matrix {n} x {n} generated ({time.time() - t0:.1f}s)")
    d_a, d_mask = torch.from_numpy(a).to(G.DEV), torch.from_numpy(mask).to(G.DEV)
    T = torch.empty((n, n), dtype=torch.int64, device=G.DEV)
    scratch = B.new_sat_scratch(n, G.DEV)
    i32 = lambda: torch.empty(n, dtype=torch.int32, device=G.DEV)  # noqa: E731
    u8 = lambda: torch.empty(n, dtype=torch.uint8, device=G.DEV)  # noqa: E731
    bl, br, bs, reus, rec, sm = i32(), i32(), torch.empty(n, dtype=torch.int64, device=G.DEV), u8(), u8(), u8()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * K)]

    def step(k=None):
        if k is not None:
            ev[3 * k].record()
        B.cp_sat_build(d_a, T, scratch, mask=None if args.full_table else d_mask)
        if k is not None:
            ev[3 * k + 1].record()
        B.cp_annotate(T, d_mask, args.min_len if args.min_len > 1 else 128, 25, bl, br, bs, reus, rec, sm, scratch)
        if k is not None:
            ev[3 * k + 2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(K):
        step(k)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t_start) / K * 1e3
    sat_ms = float(np.mean([ev[3 * k].elapsed_time(ev[3 * k + 1]) for k in range(K)]))
    ann_ms = float(np.mean([ev[3 * k + 1].elapsed_time(ev[3 * k + 2]) for k in range(K)]))
    # algorithmic: every weight on or below the diagonal read once (4 B), its table entry written once (8 B);
    # when the build knows the mask, a table entry is owed only where a search can look (rows of a coarse
    # segment [a, b] x columns a-1 .. row, plus the diagonal), and the weights under those entries are read again
    tri = n * (n + 1) / 2
    if args.full_table:
        entries = tri
        sat_bytes = 12.0 * tri
    else:
        entries, i = float(int(mask.sum())), 0  # diagonal entries of the sensitive rows
        while i < n:
            if mask[i]:
                i += 1
                continue
            j = i
            while j + 1 < n and not mask[j + 1]:
                j += 1
            ln = j - i + 1
            entries += ln * (ln + 1) / 2 + (ln if i > 0 else 0)
            i = j + 1
        sat_bytes = 4.0 * tri + 12.0 * entries
    out = {
        "metric": "KV annotator: attention matrix entries per second (summed-area table + segment search + marks)",
        "value": n * n / (ms * 1e-3), "unit": "entries/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 weights as 2^-32 fixed point, int64 sums", "data": "synthetic",
        "config": {"workload": f"one request of {n} tokens, {int(mask.sum())} sensitive, min_len "
                               f"{args.min_len if args.min_len > 1 else 128}, rho 25 %",
                   "reusable_tokens": int(reus.sum().item()), "recompute_tokens": int(rec.sum().item()),
                   "table": "whole lower triangle" if args.full_table else "only where a search can look",
                   "table_entries_owed": int(entries), "lower_triangle_entries": int(tri)},
        "sat_build_ms": sat_ms, "annotate_ms": ann_ms,
        "roofline": {"kernel": "cp_sat_build (3 launches)" if args.full_table else "cp_sat_build (3 launches, mask known)",
                     "bound": "hbm", "achieved": sat_bytes / (sat_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": sat_bytes / (sat_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": PROFILED_TRAFFIC.get(f"annotator-{n}" + ("-full" if args.full_table else "")),
                     "traffic_source": f"profiles/annotator_{n}.txt (rocprofv3 counters of an earlier run, not of this run)"},
    }
    if args.cpu_requests > 0:
        t = time.perf_counter()
        oT = O.sat_build(a)
        t_sat = time.perf_counter() - t
        t = time.perf_counter()
        want = O.annotate(oT, mask, args.min_len if args.min_len > 1 else 128, 25)
        t_ann = time.perf_counter() - t
        # (a table built for the mask is compared through the decisions it leads to; the tests compare its entries)
        same = (not args.full_table or bool(np.array_equal(np.tril(T.cpu().numpy()), np.tril(oT)))) and all(
            np.array_equal(g.cpu().numpy().view(w.dtype), w) for g, w in zip((bl, br, bs, reus, rec), want))
        out["cpu_baseline"] = {"value": n * n / (t_sat + t_ann), "unit": "entries/s", "cores": 1, "kind": "oracle",
                               "sample": "the same matrix, whole", "seconds": {"sat": round(t_sat, 3),
                                                                                "annotate": round(t_ann, 3)},
                               "gpu_result_identical": same, "host": host_info()}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3-8b", choices=["tiny", "llama3-8b", "frag", "rope", "llama3-70b", "float"])
    ap.add_argument("--anchor-window", type=int, default=None,
                    help="W: look stored runs up through floating anchors as well (default: run-start keys only)")
    ap.add_argument("--verify", action="store_true",
                    help="confirm every match exactly against the pool's per-slot (token, parent) records")
    ap.add_argument("--min-len", type=int, default=1, help="drop matched stretches shorter than this many tokens")
    ap.add_argument("--recompute", type=float, default=0.0,
                    help="fraction of the stored tokens marked for recomputation (seeded, uniform): not served")
    ap.add_argument("--zero-fill", action="store_true", help="write zero rows for every token that is not served")
    ap.add_argument("--lru", action="store_true", help="keep last-use stamps for eviction")
    ap.add_argument("--dedup", action="store_true",
                    help="store every text once: what a lookup of a batch finds (also behind other text) is not stored again "
                         "(needs --anchor-window)")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="KV heads held by this GPU (0 = the workload's own): the share of a tensor-parallel rank")
    ap.add_argument("--free-list", default="random", choices=["random", "sequential"],
                    help="order in which pool slots are handed out (the configurations say random)")
    ap.add_argument("--pool-layout", default="token", choices=["token", "layer"],
                    help="token: a token's rows are contiguous in the pool (default); layer: one plane per (layer, K|V)")
    ap.add_argument("--full-table", action="store_true",
                    help="with --annotator: build the whole summed-area table, not only the part the mask leaves to search")
    ap.add_argument("--annotator", type=int, default=0, metavar="N",
                    help="side benchmark: run the KV annotator on one N x N attention matrix instead of the KV path")
    ap.add_argument("--cpu-requests", type=int, default=16, help="requests in the CPU-oracle sample (0 = skip)")
    # launch options of the row mover (cp_launch_opts; 0 = the library's default)
    ap.add_argument("--read-sharing", type=int, default=0, help="1 = tokens reading one slot share the read, 2 = not")
    ap.add_argument("--blocks-per-cu", type=int, default=0, help="resident workgroups per compute unit")
    ap.add_argument("--nontemporal", type=int, default=0, help="1 + (bit 0: non-temporal loads, bit 1: stores)")
    ap.add_argument("--loads-in-flight", type=int, default=0, help="16-byte loads per lane before the first store")
    ap.add_argument("--fanout", type=int, default=0, help="destinations written per pass over a shared slot")
    ap.add_argument("--workgroups", type=int, default=0, help="grid size of the row mover (overrides --blocks-per-cu)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side measurements (gather without read sharing, plain copy): used under the profiler")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain fill and one plain read kernel of known size (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU: the HIP path has no fallback")
    import paper_2605_23640_amd as cp
    from cp_workload import gen
    from paper_2605_23640_amd import harness as G

    if args.annotator:
        return annotator_bench(args)

    opts = cp.binding.LaunchOpts(args.read_sharing, args.blocks_per_cu, args.nontemporal, args.loads_in_flight,
                                 args.fanout, args.workgroups)

    t0 = time.time()
    if args.kv_heads:  # one rank's share under tensor parallelism: the same tokens and slots, fewer heads per row
        whole = gen.default_shape(args.workload)
        wl = gen.make(args.workload, shape=gen.KVShape(whole.n_layers, args.kv_heads, whole.head_dim))
    else:
        wl = gen.make(args.workload)
    if args.free_list == "sequential":  # slots handed out in ascending order: matched runs become long spans
        wl.free_slots = np.arange(wl.pool_slots, dtype=np.uint32)
    sh = wl.shape
    N = wl.n_tokens
    log(f"[bench] workload {wl.name}: {wl.n_requests} requests, {N} tokens, {sh.tok_bytes // 1024} KiB/token, "
        f"pool {wl.pool_slots} slots = {wl.pool_slots * sh.tok_bytes / 2**30:.1f} GiB")
    rec = None
    if args.recompute > 0.0:
        assert wl.donor_u is not None, "this workload draws no recompute marks"
        rec = (wl.donor_u < args.recompute).astype(np.uint8)
    gst = G.prefill(wl, G.make_pool(wl, anchor_window=args.anchor_window, verify=args.verify, min_len=args.min_len,
                                    recompute_marks=rec is not None, zero_fill=args.zero_fill, lru=args.lru,
                                    pool_layout=args.pool_layout, gather_opts=opts, insert_opts=opts, dedup=args.dedup),
                    recompute=rec)
    pool = gst.pool
    log(f"[bench] pool prefilled: {pool.n_used} tokens stored ({time.time() - t0:.1f}s)")

    tok, mask, off = G.dev_i32(wl.tok), torch.from_numpy(wl.mask.copy()).to(G.DEV), G.dev_i32(wl.off)
    buf = cp.LookupBuffers(N, N, G.DEV, n_pool_slots=pool.n_slots)
    dst = G.poison_tensor(N * sh.tok_bytes)
    slot_out = torch.empty(N, dtype=torch.int32, device=G.DEV)
    ins_scratch = cp.binding.new_scratch(N, 0, G.DEV)
    ins_buf = cp.LookupBuffers(N, 0, G.DEV) if args.dedup else None  # the lookup that precedes a storing-once insert
    keys0, vals0 = pool.table.keys.clone(), pool.table.vals.clone()
    if pool.slot_anchor is not None:
        anchor0 = pool.slot_anchor.clone()
    K = args.steps
    # hipEvent pairs that the library records around its two row-mover kernels (gather, scatter), on the launch stream
    hev = cp.binding.HipEvents(4 * K + 2)
    ev_ins = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]

    def step(k=None):
        pool.lookup(tok, mask, off, dst, buf,
                    gather_opts=None if k is None else opts.with_events(hev.ev[4 * k], hev.ev[4 * k + 1]))
        if k is not None:
            ev_ins[k][0].record()
        pool.insert(tok, mask, off, dst, buf.hash, slot_out, ins_scratch, hashes_ready=True, sync=False,
                    run_off_buf=buf.run_off, buf=ins_buf,
                    insert_opts=None if k is None else opts.with_events(hev.ev[4 * k + 2], hev.ev[4 * k + 3]))
        if k is not None:
            ev_ins[k][1].record()
        pool.table.keys.copy_(keys0, non_blocking=True)
        pool.table.vals.copy_(vals0, non_blocking=True)
        if pool.slot_anchor is not None:
            pool.slot_anchor.copy_(anchor0, non_blocking=True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(K):
        step(k)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start

    n_spans = int(buf.n_spans.item())
    matched = int(buf.span_off[n_spans].item())
    inserted = int(pool.n_inserted.item())
    flags = int(pool.flags.item())
    slots = G.host_u32(buf.served if pool.filters else buf.slot)
    unique_src = int(len(np.unique(slots[slots != 0xFFFFFFFF])))
    gather_ms = float(np.mean([hev.elapsed_ms(4 * k, 4 * k + 1) for k in range(K)]))
    insert_ms = float(np.mean([a.elapsed_time(b) for a, b in ev_ins]))  # the whole cp_insert_kv call
    scatter_ms = float(np.mean([hev.elapsed_ms(4 * k + 2, 4 * k + 3) for k in range(K)])) if inserted else None
    ms_per_step = t_total / K * 1e3
    gather_bytes = 2.0 * sh.tok_bytes * matched  # algorithmic: every reused row read once and written once
    step_bytes = 2.0 * sh.tok_bytes * (matched + inserted)
    gather_gbps = gather_bytes / (gather_ms * 1e-3) / 1e9
    min_hbm_bytes = sh.tok_bytes * (matched + unique_src)
    min_hbm_gbps = min_hbm_bytes / (gather_ms * 1e-3) / 1e9

    def gather_alone(o, reps=5):
        """cp_gather_kv alone on the spans of the last step; returns ms of its mover kernel."""
        ms = []
        o = o.with_events(hev.ev[4 * K], hev.ev[4 * K + 1])
        for r in range(reps + 1):
            cp.cp_gather_kv(pool.pool, pool.layout, pool.n_slots, dst, pool.request_layout(N), N, buf.span_src,
                            buf.span_dst, buf.span_len, buf.span_delta if pool.rope is not None else None,
                            buf.span_off, buf.n_spans, buf.max_spans, pool.rope, pool.flags, buf.scratch, opts=o)
            torch.cuda.synchronize()
            if r:
                ms.append(hev.elapsed_ms(4 * K, 4 * K + 1))
        return float(np.mean(ms))

    # the same gather with every token reading its own copy of the source rows (no sharing of reads)
    own_read_ms = None
    if not args.no_extras:
        own = opts.with_events(None, None)
        own.read_sharing = 2
        own_read_ms = gather_alone(own)

    # the retriever's share alone: hashing, table lookups, (verification, filters,) span building; no KV moved
    front_ms = None
    if not args.no_extras:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pool.lookup(tok, mask, off, dst, buf, gather=False)
        e0.record()
        for _ in range(K):
            pool.lookup(tok, mask, off, dst, buf, gather=False)
        e1.record()
        torch.cuda.synchronize()
        front_ms = e0.elapsed_time(e1) / K

    # the same step replayed from a HIP graph (lookup + insert recorded once; the table resets stay eager)
    graph_ms = None
    if not args.no_extras:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            pool.lookup(tok, mask, off, dst, buf)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            pool.lookup(tok, mask, off, dst, buf)
            pool.insert(tok, mask, off, dst, buf.hash, slot_out, ins_scratch, hashes_ready=True, sync=False,
                        run_off_buf=buf.run_off, buf=ins_buf)

        def restore_tables():
            pool.table.keys.copy_(keys0, non_blocking=True)
            pool.table.vals.copy_(vals0, non_blocking=True)
            if pool.slot_anchor is not None:
                pool.slot_anchor.copy_(anchor0, non_blocking=True)

        restore_tables()
        for _ in range(2):
            graph.replay()
            restore_tables()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for _ in range(K):
            graph.replay()
            restore_tables()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t_g) / K * 1e3
        assert int(buf.n_spans.item()) == n_spans and int(pool.n_inserted.item()) == inserted
        del graph

    # what this GPU reaches for plain contiguous streams (16-byte accesses over the request buffers: read all
    # of it, write all of it, copy its first half to its second), and torch's device-to-device copy
    ceilings = None
    if not args.no_extras:
        from cp_workload import kvgen
        sink = torch.zeros(64, dtype=torch.int32, device=G.DEV)
        span = (dst.numel() // 2) // 131072 * 131072  # bytes of one half, whole 128 KiB chunks
        a_ptr, b_ptr = C.c_void_p(dst.data_ptr()), C.c_void_p(dst.data_ptr() + span)

        def timed(fn, reps=5):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e-3

        sp, snk = G.stream_ptr(), C.c_void_p(sink.data_ptr())
        t_r = timed(lambda: kvgen.stream(sp, "read", a_ptr, None, 2 * span, snk))
        t_w = timed(lambda: kvgen.stream(sp, "write", None, a_ptr, 2 * span, snk))
        t_c = timed(lambda: kvgen.stream(sp, "copy", a_ptr, b_ptr, span, snk))
        half = dst[:span], dst[span:2 * span]
        t_t = timed(lambda: half[1].copy_(half[0]))
        ceilings = {"read_GBps": 2 * span / t_r / 1e9, "write_GBps": 2 * span / t_w / 1e9,
                    "copy_GBps_read_plus_write": 2 * span / t_c / 1e9, "torch_d2d_copy_GBps_read_plus_write": 2 * span / t_t / 1e9,
                    "bytes": 2 * span, "kernels": "cp_workload/kvgen.hip stream_{read,write,copy}_kernel"}

    # the stored counter readings belong to the gather of the default options
    same_gather = (args.anchor_window is None and args.min_len <= 1 and args.recompute == 0 and not args.dedup
                   and args.pool_layout == "token" and args.free_list == "random" and not args.kv_heads)
    out = {
        "metric": "KV gather GB/s (% of HBM peak) + reused tokens/sec, Llama-3-8B KV shape",
        "value": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64 hashes, bf16 rows moved bit-exact" + (", f64 key rotation" if pool.rope is not None else ""),
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: {wl.n_requests} requests x {N // wl.n_requests} tokens, "
                        f"{sh.n_layers} layers x {sh.n_kv_heads} KV heads x {sh.head_dim} bf16 "
                        f"({sh.tok_bytes // 1024} KiB/token), pool {wl.pool_slots} slots "
                        f"({wl.pool_slots * sh.tok_bytes / 2**30:.0f} GiB) {args.pool_layout}-major, slots in {args.free_list} order",
            "step": "hash+probe+spans+gather, insert of the batch's new tokens, table reset",
            "anchor_window": args.anchor_window, "verify": args.verify, "min_len": args.min_len,
            "recompute_fraction": args.recompute, "zero_fill": args.zero_fill, "lru_stamps": args.lru,
            "store_once": args.dedup, "pool_tokens_after_prefill": pool.n_used,
            "pool_layout": args.pool_layout, "free_list": args.free_list,
            "tokens": N, "reused_tokens": matched, "hit_fraction": matched / N, "spans": n_spans,
            "distinct_source_slots": unique_src, "stored_tokens_per_step": inserted, "status_flags": flags,
        },
        "reused_tokens_per_s": matched / (ms_per_step * 1e-3),  # over the whole step, insert included
        # over the lookup alone (hash, probe, spans, gather on one stream) and over the gather's mover kernel alone
        "reused_tokens_per_s_lookup": None if front_ms is None else matched / ((front_ms + gather_ms) * 1e-3),
        "reused_tokens_per_s_gather": matched / (gather_ms * 1e-3),
        "insert_GBps": 2.0 * sh.tok_bytes * inserted / (insert_ms * 1e-3) / 1e9 if insert_ms > 0 else None,
        "gather_GBps": gather_gbps,
        "gather_pct_of_hbm_peak": 100.0 * gather_gbps / HBM_PEAK_GBPS,
        "gather_ms": gather_ms, "insert_ms": insert_ms, "scatter_kernel_ms": scatter_ms,
        "front_and_reset_ms": ms_per_step - gather_ms - insert_ms,
        "ms_per_step_from_hip_graph": graph_ms,
        "retrieval_front_end_ms": front_ms,
        "retrieval_front_end_ms_per_10k_tokens": None if front_ms is None else front_ms * 1e4 / N,
        "gather_GBps_without_read_sharing": None if own_read_ms is None else gather_bytes / (own_read_ms * 1e-3) / 1e9,
        "streaming_ceilings": ceilings,
        "roofline": {
            "kernel": "gather_rows_kernel (cp_gather_kv)", "bound": "hbm",
            # algorithmic bytes (every reused row read once and written once) / kernel time
            "achieved": gather_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gather_gbps / HBM_PEAK_GBPS,
            # bytes that must cross HBM in this run when every distinct source row is read once (rows
            # written + distinct rows read, counted from this run's slots) / this run's kernel time
            "hbm_bytes_min": min_hbm_bytes, "hbm_achieved": min_hbm_gbps, "hbm_frac": min_hbm_gbps / HBM_PEAK_GBPS,
            # the same kernel with every token reading for itself: algorithmic bytes = bytes crossing HBM
            "frac_without_read_sharing": (None if own_read_ms is None
                                          else gather_bytes / (own_read_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS),
            "traffic": PROFILED_TRAFFIC.get(wl.name) if same_gather else None,
            "traffic_source": (f"profiles/gather_rows_kernel_{wl.name}.txt: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier "
                               "run of this command, not of this run" if same_gather and wl.name in PROFILED_TRAFFIC else None),
            # of the bytes the profiler saw the kernel fetch, the part that are pool rows some request
            # asked for (every distinct source row once); the rest is descriptors, lists, re-fetches
            "fetched_bytes_landing_in_output": (sh.tok_bytes * unique_src / PROFILED_FETCH[wl.name]
                                                if wl.name in PROFILED_FETCH and same_gather else None),
            # bytes the requests asked for (one row set per reused token) over bytes fetched: above 1 where
            # several requests are served from one fetch of a shared slot
            "useful_over_fetched": (sh.tok_bytes * matched / PROFILED_FETCH[wl.name]
                                    if wl.name in PROFILED_FETCH and same_gather else None),
        },
        # the scatter half of cp_insert_kv: every stored token's rows read from the request buffers and
        # written to its pool slot, nothing shared
        "roofline_insert": None if not scatter_ms else {
            "kernel": "scatter_rows_kernel (cp_insert_kv)", "bound": "hbm",
            "achieved": 2.0 * sh.tok_bytes * inserted / (scatter_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": 2.0 * sh.tok_bytes * inserted / (scatter_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "tokens_stored": inserted, "kernel_ms": scatter_ms, "whole_call_ms": insert_ms,
            "traffic": sum(PROFILED_SCATTER[wl.name]) if wl.name in PROFILED_SCATTER and same_gather else None,
            "traffic_source": (f"profiles/scatter_rows_kernel_{wl.name}.txt: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this command, not of this run"
                               if wl.name in PROFILED_SCATTER and same_gather else None),
        },
    }
    hev.close()
    if args.calibrate:
        # kernels of known traffic for scaling the profiler's byte counters: the generator's fill
        # writes, and its verify reads, every byte of the request buffers exactly once
        from cp_workload import kvgen
        lay = pool.request_layout(N)
        kvgen.fill(G.stream_ptr(), C.c_void_p(dst.data_ptr()), G.gen_layout(lay), N, wl.seed, uid_base=0)
        bad = G.verify_rows(dst, lay, np.arange(N, dtype=np.uint64), wl.seed)
        torch.cuda.synchronize()
        snk = torch.zeros(64, dtype=torch.int32, device=G.DEV)
        whole = dst.numel() // 131072 * 131072
        kvgen.stream(G.stream_ptr(), "read", C.c_void_p(dst.data_ptr()), None, whole, C.c_void_p(snk.data_ptr()))
        kvgen.stream(G.stream_ptr(), "write", None, C.c_void_p(dst.data_ptr()), whole, C.c_void_p(snk.data_ptr()))
        torch.cuda.synchronize()
        out["calibration"] = {"fill_kernel_bytes_written": N * sh.tok_bytes, "verify_kernel_bytes_read": N * sh.tok_bytes,
                              "stream_read_kernel_bytes_read": whole, "stream_write_kernel_bytes_written": whole,
                              "verify_mismatches": bad, "gather_bytes_written": sh.tok_bytes * matched,
                              "gather_bytes_read_algorithmic": sh.tok_bytes * matched,
                              "gather_bytes_read_distinct": sh.tok_bytes * unique_src}
    if args.cpu_requests > 0:
        del dst
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_requests, G, torch, np, args.anchor_window, args.verify,
                                           args.min_len, args.recompute, args.zero_fill)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
