"""Seeded synthetic workloads: token ids, sensitivity masks, request offsets,
donor prompts for pool prefill, free lists and table sizes.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
hashing, no table, no span logic, no rotation) and serves the CPU oracle and
the GPU library alike.  Everything is host-side numpy; KV values come from
``cp_workload.kvgen``.

The five named workloads follow the five benchmark configurations (tiny,
Llama-3-8B shape, fragmentation stress, RoPE-shift reuse, Llama-3-70B shape).
They stand in for the paper's RAG-style prompts (Sec. 3.2: a long shared
system/template part, retrieved passages reused across requests, a short
unique user part, sensitive tokens a small fraction arranged in short runs);
no dataset item is reproduced.  ``scale`` shrinks a workload for tests while
keeping its structure.
"""
from __future__ import annotations

import inspect
from dataclasses import dataclass, field

import numpy as np

VOCAB = 32000


@dataclass(frozen=True)
class KVShape:
    n_layers: int
    n_kv_heads: int
    head_dim: int

    @property
    def row_bytes(self) -> int:  # one (token, layer, K|V) row, bf16
        return self.n_kv_heads * self.head_dim * 2

    @property
    def tok_bytes(self) -> int:  # all rows of one token
        return self.n_layers * 2 * self.row_bytes


@dataclass
class Workload:
    name: str
    seed: int
    shape: KVShape
    # request batch (the lookup side), R requests packed back to back
    tok: np.ndarray  # uint32[N]
    mask: np.ndarray  # uint8[N], 1 = sensitive
    off: np.ndarray  # uint32[R+1]
    # donor prompts (pool prefill), inserted in order, possibly in several batches
    donor_tok: np.ndarray
    donor_mask: np.ndarray
    donor_off: np.ndarray
    donor_batches: list  # list of (first_donor, last_donor_exclusive)
    pool_slots: int
    free_slots: np.ndarray  # uint32 permutation of the pool's slots: hand-out order
    table_capacity: int
    rope_theta: float | None = None  # None: no key re-rotation in this workload
    rope_style: int = 0
    notes: dict = field(default_factory=dict)
    # base of the chain hash for this workload (None: the library's default); Sec. 4.2.2 draws it at random
    hash_base: int | None = None
    # one uniform number per donor token, equal wherever donors share text (it travels with the prefix and with
    # each document): "marked for recomputation at rate rho" = donor_u < rho.  None: not drawn for this workload.
    donor_u: np.ndarray | None = None

    @property
    def n_tokens(self) -> int:
        return int(self.off[-1])

    @property
    def n_requests(self) -> int:
        return len(self.off) - 1


# --------------------------------------------------------------------------
# small helpers


def _tokens(rng, n):
    return rng.integers(0, VOCAB, size=int(n), dtype=np.uint32)


def _geom(rng, mean):
    """Geometric length >= 1 with the given mean."""
    if mean <= 1.0:
        return 1
    return int(rng.geometric(1.0 / mean))


def _mask_process(rng, n, run_mean, cover, start_sensitive=False):
    """Alternating non-sensitive gaps / sensitive runs, both geometric, so that a
    fraction ``cover`` of the tokens is sensitive in expectation."""
    m = np.zeros(int(n), np.uint8)
    if cover <= 0.0 or n == 0:
        return m
    gap_mean = run_mean * (1.0 - cover) / cover
    i = 0
    sens = start_sensitive
    while i < n:
        ln = _geom(rng, run_mean if sens else gap_mean)
        if sens:
            m[i : i + ln] = 1
        i += ln
        sens = not sens
    return m


def _pack(parts_tok, parts_mask):
    off = np.zeros(len(parts_tok) + 1, np.uint32)
    off[1:] = np.cumsum([len(p) for p in parts_tok])
    if len(parts_tok) == 0:
        return np.zeros(0, np.uint32), np.zeros(0, np.uint8), off
    return (
        np.concatenate(parts_tok).astype(np.uint32),
        np.concatenate(parts_mask).astype(np.uint8),
        off,
    )


def _batches(donor_off, max_tokens):
    """Split donors into consecutive batches of at most ``max_tokens`` tokens."""
    out, first, n = [], 0, len(donor_off) - 1
    for d in range(n):
        if d > first and int(donor_off[d + 1]) - int(donor_off[first]) > max_tokens:
            out.append((first, d))
            first = d
    if n > first:
        out.append((first, n))
    return out


# --------------------------------------------------------------------------
# workload 1: tiny


def make_tiny(seed=0xC0FFEE01, T=512, n_donors=8, pool_slots=4096, shape=KVShape(2, 2, 64)):
    rng = np.random.default_rng(seed)
    tok = _tokens(rng, T)
    mask = _mask_process(rng, T, run_mean=6.0, cover=0.20)
    # the request's non-sensitive segments
    segs, i = [], 0
    while i < T:
        if mask[i]:
            i += 1
            continue
        j = i
        while j < T and not mask[j]:
            j += 1
        segs.append(tok[i:j].copy())
        i = j
    d_tok, d_mask = [], []
    for d in range(n_donors):
        pt, pm = [], []
        n = 0
        order = rng.permutation(len(segs))
        for si in order:
            seg = segs[si]
            sep = _geom(rng, 6.0)
            pt.append(_tokens(rng, sep))
            pm.append(np.ones(sep, np.uint8))
            if rng.random() < 0.5:
                u = rng.random()
                if u < 0.25 and len(seg) > 1:  # a proper prefix, then different text
                    k = int(rng.integers(1, len(seg)))
                    piece = np.concatenate([seg[:k], _tokens(rng, len(seg) - k)])
                elif u < 0.5:  # the whole segment and more
                    piece = np.concatenate([seg, _tokens(rng, _geom(rng, 8.0))])
                else:
                    piece = seg.copy()
            else:
                piece = _tokens(rng, len(seg))
            if d == 0 and si == order[0]:
                # negative case: the segment preceded by one extra non-sensitive token
                piece = np.concatenate([_tokens(rng, 1), seg])
            pt.append(piece)
            pm.append(np.zeros(len(piece), np.uint8))
            n += sep + len(piece)
            if n >= T:
                break
        t = np.concatenate(pt)[:T]
        m = np.concatenate(pm)[:T]
        if len(t) < T:
            pad = T - len(t)
            t = np.concatenate([t, _tokens(rng, pad)])
            m = np.concatenate([m, np.ones(pad, np.uint8)])
        d_tok.append(t)
        d_mask.append(m)
    dt, dm, doff = _pack(d_tok, d_mask)
    return Workload(
        name="tiny", seed=seed, shape=shape,
        tok=tok, mask=mask, off=np.array([0, T], np.uint32),
        donor_tok=dt, donor_mask=dm, donor_off=doff, donor_batches=[(0, n_donors)],
        pool_slots=pool_slots, free_slots=rng.permutation(pool_slots).astype(np.uint32),
        table_capacity=2 * pool_slots,
    )


# --------------------------------------------------------------------------
# workloads 2 and 5: shared system prefix + documents from a corpus + user text


def make_docs(name, seed, shape, R, T, prefix_len, n_docs, doc_len, docs_per_request, run_mean, cover,
              pool_slots, table_capacity=None, donor_batch_tokens=1 << 17, lead_len=None):
    """Requests = shared prefix [+ a unique non-sensitive lead of lead_len=(lo, hi) tokens] + documents + the
    user's own text; donors = prefix + one document each."""
    rng = np.random.default_rng(seed)
    prefix = _tokens(rng, prefix_len)
    docs, dmasks = [], []
    for _ in range(n_docs):
        ln = int(rng.integers(doc_len[0], doc_len[1] + 1))
        docs.append(_tokens(rng, ln))
        dmasks.append(_mask_process(rng, ln, run_mean, cover))  # the mask travels with the document
    r_tok, r_mask, picks = [], [], []
    for _ in range(R):
        chosen = rng.choice(n_docs, size=min(docs_per_request, n_docs), replace=False)
        pt, pm, n = [prefix], [np.zeros(prefix_len, np.uint8)], prefix_len
        used = []
        if lead_len is not None:  # text of this request alone, in the same run as the document after it
            ln = int(rng.integers(lead_len[0], lead_len[1] + 1))
            pt.append(_tokens(rng, ln))
            pm.append(np.zeros(ln, np.uint8))
            n += ln
        for d in chosen:
            room = T - n
            if room <= 0:
                break
            ln = min(len(docs[d]), room)
            pt.append(docs[d][:ln])
            pm.append(dmasks[d][:ln])
            n += ln
            used.append(int(d))
        if n < T:  # the user's own text: never in the pool
            pt.append(_tokens(rng, T - n))
            pm.append(_mask_process(rng, T - n, run_mean, cover))
        r_tok.append(np.concatenate(pt)[:T])
        r_mask.append(np.concatenate(pm)[:T])
        picks.append(used)
    tok, mask, off = _pack(r_tok, r_mask)
    d_tok = [np.concatenate([prefix, docs[d]]) for d in range(n_docs)]
    d_mask = [np.concatenate([np.zeros(prefix_len, np.uint8), dmasks[d]]) for d in range(n_docs)]
    dt, dm, doff = _pack(d_tok, d_mask)
    if table_capacity is None:
        table_capacity = 2 * pool_slots
    urng = np.random.default_rng(seed ^ 0x5EC0)  # a stream of its own: the prompts above do not depend on it
    prefix_u = urng.random(prefix_len, dtype=np.float32)
    doc_u = [urng.random(len(d), dtype=np.float32) for d in docs]
    donor_u = np.concatenate([np.concatenate([prefix_u, doc_u[d]]) for d in range(n_docs)])
    return Workload(
        name=name, seed=seed, shape=shape, tok=tok, mask=mask, off=off,
        donor_tok=dt, donor_mask=dm, donor_off=doff, donor_batches=_batches(doff, donor_batch_tokens),
        pool_slots=pool_slots, free_slots=rng.permutation(pool_slots).astype(np.uint32),
        table_capacity=table_capacity, notes={"picks": picks}, donor_u=donor_u,
    )


def from_prompts(name, seed, shape, donors, requests, pool_slots, donor_masks=None, request_masks=None,
                 donor_batch_tokens=1 << 17):
    """A workload from explicit token lists: ``donors`` are stored one after the other, in batches of at most
    ``donor_batch_tokens`` tokens; ``requests`` are looked up.  Masks default to "nothing sensitive".  For
    hand-built test cases."""
    rng = np.random.default_rng(seed)
    as_u32 = lambda xs: [np.asarray(x, np.uint32) for x in xs]  # noqa: E731
    zeros = lambda xs: [np.zeros(len(x), np.uint8) for x in xs]  # noqa: E731
    donors, requests = as_u32(donors), as_u32(requests)
    dt, dm, doff = _pack(donors, donor_masks or zeros(donors))
    tok, mask, off = _pack(requests, request_masks or zeros(requests))
    return Workload(name=name, seed=seed, shape=shape, tok=tok, mask=mask, off=off, donor_tok=dt, donor_mask=dm,
                    donor_off=doff, donor_batches=_batches(doff, donor_batch_tokens), pool_slots=pool_slots,
                    free_slots=rng.permutation(pool_slots).astype(np.uint32), table_capacity=2 * pool_slots)


def make_llama8b(seed=0xC0FFEE02, scale=1.0, shape=KVShape(32, 8, 128)):
    s = scale
    return make_docs("llama3-8b", seed, shape, R=max(2, round(16 * s)), T=max(64, round(4096 * s)),
                     prefix_len=max(8, round(1024 * s)), n_docs=max(4, round(64 * s)),
                     doc_len=(max(4, round(512 * s)), max(8, round(1024 * s))), docs_per_request=3,
                     run_mean=8.0, cover=0.15, pool_slots=max(256, round(262144 * s)))


def make_llama70b(seed=0xC0FFEE05, scale=1.0, shape=KVShape(80, 8, 128)):
    s = scale
    return make_docs("llama3-70b", seed, shape, R=max(2, round(4 * min(1.0, s * 4))), T=max(64, round(32768 * s)),
                     prefix_len=max(8, round(4096 * s)), n_docs=max(4, round(256 * s)),
                     doc_len=(max(4, round(1024 * s)), max(8, round(2048 * s))), docs_per_request=16,
                     run_mean=12.0, cover=0.10, pool_slots=max(256, round(393216 * s)),
                     donor_batch_tokens=max(1024, round(65536 * min(1.0, s * 4))))


def make_float(seed=0xC0FFEE06, scale=1.0, shape=KVShape(32, 8, 128)):
    """Documents stored on their own (their runs start at the document's first token) and
    retrieved into requests behind text that differs per request: the part of a document up to
    its first sensitive token continues the run of whatever precedes it, so only a floating
    anchor (Sec. 4.2.2 Step 1) finds it; later runs match by their run-start keys as well."""
    s = scale
    return make_docs("float", seed, shape, R=max(2, round(16 * s)), T=max(64, round(4096 * s)),
                     prefix_len=0, n_docs=max(4, round(64 * s)),
                     doc_len=(max(4, round(512 * s)), max(8, round(1024 * s))), docs_per_request=4,
                     run_mean=8.0, cover=0.02, pool_slots=max(256, round(262144 * s)),
                     lead_len=(max(1, round(16 * s)), max(2, round(256 * s))))


# --------------------------------------------------------------------------
# workload 3: fragmentation stress


def make_frag(seed=0xC0FFEE03, scale=1.0, shape=KVShape(32, 8, 128), load=0.85, miss_frac=0.05):
    rng = np.random.default_rng(seed)
    R, T = max(2, round(64 * scale)), max(64, round(2048 * scale))
    pool_slots = max(256, round(131072 * scale))
    # Span corpus: runs of 1..16 tokens, each stored as a whole run (a sensitive
    # token before it).  Two runs that begin with the same tokens share keys, so
    # count distinct run prefixes (token tuples, no hashing) until the pool is
    # exactly full.
    seen = set()
    spans = []
    while len(seen) < pool_slots:
        ln = int(rng.integers(1, 17))
        sp = _tokens(rng, ln)
        t = tuple(int(x) for x in sp)
        new = [t[: k + 1] for k in range(ln) if t[: k + 1] not in seen]
        if len(seen) + len(new) > pool_slots:  # cut the last run so the count lands exactly
            keep = pool_slots - len(seen)
            # prefixes are added shortest first, so keeping the first `keep` new ones keeps a prefix
            new = new[:keep]
            sp = sp[: len(new[-1])]
        seen.update(new)
        spans.append(sp)
    # donors: [sensitive separator][span][sensitive separator][span]..., ~T tokens each
    d_tok, d_mask, cur_t, cur_m, n = [], [], [], [], 0
    for sp in spans:
        sep = int(rng.integers(1, 9))
        cur_t += [_tokens(rng, sep), sp]
        cur_m += [np.ones(sep, np.uint8), np.zeros(len(sp), np.uint8)]
        n += sep + len(sp)
        if n >= T:
            d_tok.append(np.concatenate(cur_t))
            d_mask.append(np.concatenate(cur_m))
            cur_t, cur_m, n = [], [], 0
    if cur_t:
        d_tok.append(np.concatenate(cur_t))
        d_mask.append(np.concatenate(cur_m))
    dt, dm, doff = _pack(d_tok, d_mask)
    # requests: reusable spans (uniform 1..16) between sensitive runs (uniform 1..8).
    # With those lengths alone 4.5/13 = 34.6 % of the tokens would be sensitive; a
    # fraction q of the reusable spans is turned sensitive as well so that the
    # coverage is 40 % while reusable spans keep their length distribution.
    q = (0.40 * 13.0 - 4.5) / 8.5
    r_tok, r_mask = [], []
    for _ in range(R):
        pt, pm, n = [], [], 0
        while n < T:
            sep = int(rng.integers(1, 9))
            pt.append(_tokens(rng, sep))
            pm.append(np.ones(sep, np.uint8))
            if rng.random() < miss_frac:
                sp = _tokens(rng, int(rng.integers(1, 17)))
            else:
                sp = spans[int(rng.integers(0, len(spans)))]
            pt.append(sp)
            pm.append(np.full(len(sp), 1 if rng.random() < q else 0, np.uint8))
            n += sep + len(sp)
        r_tok.append(np.concatenate(pt)[:T])
        r_mask.append(np.concatenate(pm)[:T])
    tok, mask, off = _pack(r_tok, r_mask)
    capacity = int(np.ceil(pool_slots / load))
    return Workload(
        name="frag", seed=seed, shape=shape, tok=tok, mask=mask, off=off,
        donor_tok=dt, donor_mask=dm, donor_off=doff, donor_batches=_batches(doff, 1 << 16),
        pool_slots=pool_slots, free_slots=rng.permutation(pool_slots).astype(np.uint32),
        table_capacity=capacity, notes={"n_spans_corpus": len(spans)},
    )


# --------------------------------------------------------------------------
# workload 4: reuse at shifted positions (key re-rotation)


def _stretches(mask):
    """Maximal non-sensitive stretches [a, b) of one prompt's mask."""
    m = np.concatenate([[1], mask, [1]]).astype(np.int8)
    d = np.diff(m)
    return list(zip(np.flatnonzero(d == -1).tolist(), np.flatnonzero(d == 1).tolist()))


def make_rope(seed=0xC0FFEE04, scale=1.0, shape=KVShape(32, 8, 128), theta=500000.0, max_shift=512, fresh=0.3):
    """Every reused span sits in the request at its cached position plus a delta of its own, drawn
    uniformly from [-max_shift, max_shift].

    Donor prompts and requests have the same length and the same sensitive-run process (geometric runs
    of mean 8 covering 25 %).  A request is its own text except that a fraction 1 - ``fresh`` of its
    non-sensitive stretches begin with a stored run: for a stretch that starts at position a, a delta is
    drawn and the stretch takes the tokens of a donor run that starts at position a - delta (the first of
    up to sixteen draws for which a donor has a run starting exactly there), as far as the shorter of the
    two goes; what is left of the stretch is the request's own text.  A run starts right behind a
    sensitive token (or at position 0) in donor and request alike, so the copied tokens match from
    their first token on, at a position delta that no other span of the batch shares except by chance.
    Different requests, and different stretches of one request, may copy the same donor run."""
    rng = np.random.default_rng(seed)
    s = scale
    ms = max(2, round(max_shift * s))
    R, T = max(2, round(16 * s)), max(32, round(8192 * s))
    n_donors = max(8, round(28 * s))
    pool_slots = max(256, round(262144 * s))
    run_mean, cover = 8.0, 0.25
    d_tok = [_tokens(rng, T) for _ in range(n_donors)]
    d_mask = [_mask_process(rng, T, run_mean, cover) for _ in range(n_donors)]
    runs_at = {}  # position -> [(donor, length)] of the stored runs that start there
    for d in range(n_donors):
        for a, b in _stretches(d_mask[d]):
            runs_at.setdefault(a, []).append((d, b - a))
    r_tok, r_mask, n_reused_runs = [], [], 0
    for _ in range(R):
        m = _mask_process(rng, T, run_mean, cover)
        t = _tokens(rng, T)
        for a, b in _stretches(m):
            if rng.random() < fresh:
                continue
            for _attempt in range(16):
                q = a - int(rng.integers(-ms, ms + 1))
                cands = runs_at.get(q)
                if cands:
                    break
            else:
                continue
            long_enough = [c for c in cands if c[1] >= b - a]
            d, ln = long_enough[int(rng.integers(0, len(long_enough)))] if long_enough else max(cands, key=lambda c: c[1])
            n = min(b - a, ln)
            t[a:a + n] = d_tok[d][q:q + n]
            n_reused_runs += 1
        r_tok.append(t)
        r_mask.append(m)
    tok, mask, off = _pack(r_tok, r_mask)
    dt, dm, doff = _pack(d_tok, d_mask)
    return Workload(
        name="rope", seed=seed, shape=shape, tok=tok, mask=mask, off=off,
        donor_tok=dt, donor_mask=dm, donor_off=doff, donor_batches=_batches(doff, 1 << 17),
        pool_slots=pool_slots, free_slots=rng.permutation(pool_slots).astype(np.uint32),
        table_capacity=2 * pool_slots, rope_theta=theta, rope_style=0,
        notes={"max_shift": ms, "reused_runs": n_reused_runs},
    )


def subsample(wl: Workload, n_requests: int, pool_slots: int | None = None) -> Workload:
    """A bounded sample of a workload: its first ``n_requests`` requests and, when the
    workload records which documents each request uses, only the donor prompts of those
    documents.  The pool may be shrunk (same bytes per token, fewer slots); donors stay in
    their original order and form one insert batch."""
    n_requests = min(n_requests, wl.n_requests)
    e = int(wl.off[n_requests])
    picks = wl.notes.get("picks")
    n_donors = len(wl.donor_off) - 1
    keep = sorted({d for p in picks[:n_requests] for d in p}) if picks is not None else list(range(n_donors))
    dt = [wl.donor_tok[wl.donor_off[d]:wl.donor_off[d + 1]] for d in keep]
    dm = [wl.donor_mask[wl.donor_off[d]:wl.donor_off[d + 1]] for d in keep]
    dtok, dmask, doff = _pack(dt, dm)
    slots = wl.pool_slots if pool_slots is None else pool_slots
    assert slots >= len(dtok), "sample pool too small for its donors"
    rng = np.random.default_rng(wl.seed ^ 0x5A5A)
    free = wl.free_slots if slots == wl.pool_slots else rng.permutation(slots).astype(np.uint32)
    return Workload(
        name=f"{wl.name}[first {n_requests} requests]", seed=wl.seed, shape=wl.shape,
        tok=wl.tok[:e].copy(), mask=wl.mask[:e].copy(), off=wl.off[:n_requests + 1].copy(),
        donor_tok=dtok, donor_mask=dmask, donor_off=doff, donor_batches=[(0, len(keep))],
        pool_slots=slots, free_slots=free,
        table_capacity=wl.table_capacity if slots == wl.pool_slots else 2 * slots,
        rope_theta=wl.rope_theta, rope_style=wl.rope_style, notes={"donors_kept": keep},
        donor_u=None if wl.donor_u is None else
        np.concatenate([wl.donor_u[wl.donor_off[d]:wl.donor_off[d + 1]] for d in keep]),
    )


WORKLOADS = {
    "tiny": lambda scale=1.0, **kw: make_tiny(**kw),
    "llama3-8b": make_llama8b,
    "frag": make_frag,
    "rope": make_rope,
    "llama3-70b": make_llama70b,
    "float": make_float,
}


def make(name, **kw) -> Workload:
    return WORKLOADS[name](**kw)


def default_shape(name) -> KVShape:
    """The KV shape a workload is built with unless ``shape=`` says otherwise."""
    f = make_tiny if name == "tiny" else WORKLOADS[name]
    return inspect.signature(f).parameters["shape"].default
