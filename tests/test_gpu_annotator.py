"""The KV annotator on the GPU (Sec. 4.2.1 Steps 1-3) against the CPU oracle: the summed-area table
and every decision bit for bit (the arithmetic is integer on both sides)."""
import numpy as np
import pytest
import torch

import oracle as O
from cp_workload import attn as AT
from test_gpu_parity import G  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu
X = 0xFFFFFFFF


UNWRITTEN = -7777777


def gpu_annotate(G, a, mask, min_len, rho, masked=False):
    """``masked``: the table build is told the mask and writes only what a search can read."""
    from paper_2605_23640_amd import binding as B
    n = a.shape[0]
    d_a = torch.from_numpy(a).to(G.DEV)
    T = torch.full((n, n), UNWRITTEN, dtype=torch.int64, device=G.DEV)
    scratch = B.new_sat_scratch(n, G.DEV)
    B.cp_sat_build(d_a, T, scratch, mask=torch.from_numpy(mask).to(G.DEV) if masked else None)
    i32 = lambda: torch.empty(n, dtype=torch.int32, device=G.DEV)  # noqa: E731
    u8 = lambda: torch.empty(n, dtype=torch.uint8, device=G.DEV)  # noqa: E731
    bl, br, bs, reus, rec, sm = i32(), i32(), torch.empty(n, dtype=torch.int64, device=G.DEV), u8(), u8(), u8()
    B.cp_annotate(T, torch.from_numpy(mask).to(G.DEV), min_len, rho, bl, br, bs, reus, rec, sm, scratch)
    torch.cuda.synchronize()
    return (T.cpu().numpy(), G.host_u32(bl), G.host_u32(br), bs.cpu().numpy(), reus.cpu().numpy(), rec.cpu().numpy(),
            sm.cpu().numpy())


def check(G, a, mask, min_len, rho):
    T, bl, br, bs, reus, rec, sm = gpu_annotate(G, a, mask, min_len, rho)
    oT = O.sat_build(a)
    n = len(mask)
    assert np.array_equal(np.tril(T), np.tril(oT))  # what the library promises: every j <= i
    assert np.array_equal(np.triu(oT, 1), np.triu(np.repeat(np.diag(oT)[:, None], n, axis=1), 1))  # T[i][j>i] = T[i][i]
    want = O.annotate(oT, mask, min_len, rho)
    for g, w, name in zip((bl, br, bs, reus, rec), want, ("best_l", "best_r", "best_score", "reusable", "recompute")):
        assert np.array_equal(g, w), name
    assert np.array_equal(sm, 1 - reus)
    # the same with a table build that knows the mask: identical decisions, and the table is right wherever a
    # search may look (rows of a segment [a, b] x columns a-1 .. row, and the diagonal)
    T2, *outs2 = gpu_annotate(G, a, mask, min_len, rho, masked=True)
    for g, w, name in zip(outs2, (bl, br, bs, reus, rec, sm), ("best_l", "best_r", "best_score", "reusable", "recompute", "store")):
        assert np.array_equal(g, w), ("masked build", name)
    need = np.eye(n, dtype=bool)
    i = 0
    while i < n:
        if mask[i]:
            i += 1
            continue
        j = i
        while j + 1 < n and not mask[j + 1]:
            j += 1
        need[i:j + 1, max(i - 1, 0):j + 1] = True
        i = j + 1
    need &= np.tri(n, dtype=bool)
    assert np.array_equal(T2[need], oT[need])
    return want


@pytest.mark.parametrize("n,min_len,rho", [(1, 1, 25), (7, 1, 50), (64, 4, 25), (65, 1, 25), (200, 16, 25),
                                           (333, 1, 100), (700, 128, 25), (1000, 32, 0)])
def test_annotator_small(G, n, min_len, rho):
    a = AT.make_attention(n, seed=n, passage_mean=max(3, n // 8), tau=max(2.0, n / 40))
    mask = AT.make_mask(n, seed=n + 1, run_mean=2.0, cover=0.06)
    bl, br, bs, reus, rec = check(G, a, mask, min_len, rho)
    if n >= 200 and min_len <= 32:
        assert reus.sum() > 0 and (rho == 0 or rec.sum() > 0)


def test_annotator_full_size(G):
    """n = 10,000 (the size the side benchmark runs): 400 MB of weights, an 800 MB table."""
    n = 10000
    a = AT.make_attention(n)
    mask = AT.make_mask(n, run_mean=8.0, cover=0.01)
    bl, br, bs, reus, rec = check(G, a, mask, 128, 25)
    assert reus.sum() > 0.8 * n and abs(int(rec.sum()) - int(reus.sum()) // 4) < 20
    T2 = gpu_annotate(G, a, mask, 128, 25, masked=True)[0]
    assert (np.tril(T2) == UNWRITTEN).mean() > 0.3  # with a dozen segments most of the triangle is never asked for
    one = np.zeros(n, np.uint8)  # a single segment: every (l, r) pair is a candidate
    bl, br, bs, reus, rec = check(G, a, one, 128, 25)
    assert bl[0] != X


def test_annotator_table_beyond_4_gib(G):
    """n = 24,000: the table holds 4.6 GB, byte offsets no longer fit 32 bits; compared in row blocks."""
    from paper_2605_23640_amd import binding as B
    n = 24000
    a = AT.make_attention(n, seed=3)
    mask = AT.make_mask(n, seed=4, run_mean=8.0, cover=0.01)
    d_a = torch.from_numpy(a).to(G.DEV)
    T = torch.empty((n, n), dtype=torch.int64, device=G.DEV)
    scratch = B.new_sat_scratch(n, G.DEV)
    B.cp_sat_build(d_a, T, scratch)
    i32 = lambda: torch.empty(n, dtype=torch.int32, device=G.DEV)  # noqa: E731
    u8 = lambda: torch.empty(n, dtype=torch.uint8, device=G.DEV)  # noqa: E731
    bl, br, bs, reus, rec, sm = i32(), i32(), torch.empty(n, dtype=torch.int64, device=G.DEV), u8(), u8(), u8()
    B.cp_annotate(T, torch.from_numpy(mask).to(G.DEV), 128, 25, bl, br, bs, reus, rec, sm, scratch)
    torch.cuda.synchronize()
    oT = O.sat_build(a)
    cols = np.arange(n)[None, :]
    for r0 in range(0, n, 2000):
        rows = np.arange(r0, r0 + 2000)[:, None]
        g, w = T[r0:r0 + 2000].cpu().numpy(), oT[r0:r0 + 2000]
        assert not ((g != w) & (cols <= rows)).any(), r0
    want = O.annotate(oT, mask, 128, 25)
    got = (G.host_u32(bl), G.host_u32(br), bs.cpu().numpy(), reus.cpu().numpy(), rec.cpu().numpy())
    for g, w, name in zip(got, want, ("best_l", "best_r", "best_score", "reusable", "recompute")):
        assert np.array_equal(g, w), name
    assert want[3].sum() > 0.8 * n


def test_annotator_edge_inputs(G):
    n = 130
    z = np.zeros(n, np.uint8)
    eye = np.zeros((n, 132), np.float32)
    eye[np.arange(n), np.arange(n)] = 1
    bl, br, bs, reus, rec = check(G, eye, z, 1, 30)
    assert bl[0] == 0 and br[0] == n - 1 and reus.all() and list(np.flatnonzero(rec)) == list(range(39))
    first = np.zeros((n, 132), np.float32)
    first[:, 0] = 1
    m = z.copy()
    m[0] = 1
    bl, br, bs, reus, rec = check(G, first, m, 1, 0)
    assert bl[1] == 1 and br[1] == 1 and not reus.any()  # the best substring fails Intra > Inter: nothing reusable
    check(G, first, m, 70, 10)  # ties over many candidates: the first window of 70 tokens
    bl, br, bs, reus, rec = check(G, np.zeros((n, 132), np.float32), z, 2, 50)  # all scores tie at zero
    assert bl[0] == 0 and br[0] == 1 and not reus.any() and not rec.any()
    both = eye.copy()  # one segment passes the criterion, the next one (attending to token 0 only) does not
    both[70:, :] = 0
    both[70:, 0] = 1
    cut = z.copy()
    cut[69] = 1
    bl, br, bs, reus, rec = check(G, both, cut, 1, 50)
    assert reus[:69].all() and not reus[69:].any() and bs[70] < 0
    check(G, eye, np.ones(n, np.uint8), 1, 25)  # everything sensitive
    junk = AT.make_attention(n, seed=5)
    junk[3, 1], junk[9, 2], junk[11, 4], junk[12, 5], junk[13, 6] = np.nan, np.inf, -3e9, 262144.0, 262145.0
    junk[2, 100] = 0.7  # above the diagonal
    junk[20, 7], junk[20, 8] = 2.0 ** -33, 3 * 2.0 ** -33
    mk = AT.make_mask(n, seed=6, run_mean=2.0, cover=0.1)
    check(G, junk, mk, 3, 25)
    # a row stride larger than n
    wide = np.zeros((n, 200), np.float32)
    wide[:, :132] = AT.make_attention(n, seed=8)
    wide[:, 140:] = 5.0  # padding the library must never read as weights
    check(G, wide, mk, 1, 25)
    # a row stride that is no multiple of four floats: the library falls back to scalar loads
    odd = np.zeros((n, 133), np.float32)
    odd[:, :132] = AT.make_attention(n, seed=9)
    check(G, odd, mk, 2, 25)


def test_annotator_feeds_the_pool(G):
    """store_mask and recompute go straight into hashing / insert / marks: only the chosen substrings are stored."""
    import paper_2605_23640_amd as cp
    from cp_workload import gen
    from paper_2605_23640_amd import binding as B
    n = 600
    rng = np.random.default_rng(4)
    a = AT.make_attention(n, seed=21, passage_mean=80)
    mask = AT.make_mask(n, seed=22, run_mean=3.0, cover=0.05)
    T, bl, br, bs, reus, rec, sm = gpu_annotate(G, a, mask, 8, 25)
    tok = rng.integers(0, 32000, n).astype(np.uint32)
    sh = gen.KVShape(2, 2, 64)
    S = 1024
    pool = cp.KVPool(sh.n_layers, sh.n_kv_heads, sh.head_dim, S, 2 * S, torch.arange(S, dtype=torch.int32),
                     device=G.DEV, pool_tensor=G.poison_tensor(S * sh.tok_bytes), recompute_marks=True)
    d_tok, d_off = G.dev_i32(tok), G.dev_i32(np.array([0, n], np.uint32))
    d_sm, d_rec = torch.from_numpy(sm).to(G.DEV), torch.from_numpy(rec).to(G.DEV)
    src = G.poison_tensor(n * sh.tok_bytes)
    hbuf = torch.empty(n, dtype=torch.int64, device=G.DEV)
    sout = torch.empty(n, dtype=torch.int32, device=G.DEV)
    stored = pool.insert(d_tok, d_sm, d_off, src, hbuf, sout, B.new_scratch(n, 0, G.DEV), recompute=d_rec)
    assert stored == int(reus.sum())
    so = G.host_u32(sout)
    assert ((so != X) == (reus == 1)).all()
    marks = pool.slot_recompute.cpu().numpy()
    assert marks.sum() == rec.sum() and set(np.flatnonzero(marks)) == set(so[rec == 1].tolist())
