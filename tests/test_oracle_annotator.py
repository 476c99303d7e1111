"""Pins for the KV annotator's oracle (Sec. 4.2.1: summed-area table, optimal substring per coarse
segment, recompute marks): closed forms, numpy cumulative sums, and brute force straight from the
definitions of IntraAttn / InterAttn (double sums over the raw matrix) on small inputs."""
import numpy as np
import pytest

import oracle as O
from cp_workload import attn as AT

X = 0xFFFFFFFF
S = 1 << 32


def q_matrix(a):
    """The fixed-point image, written independently with numpy."""
    n = a.shape[0]
    q = np.rint(a[:, :n].astype(np.float64) * S)
    q[~np.isfinite(q)] = 0
    q[np.abs(a[:, :n].astype(np.float64)) > 2.0 ** 18] = 0
    return np.tril(q).astype(np.int64)


def test_quantiser_and_table_against_cumsum():
    a = AT.make_attention(150, ld=152)
    a[5, 3] = np.nan
    a[6, 2] = np.inf
    a[7, 1] = 3e7  # beyond the accepted range
    a[9, 4] = 2.0 ** -33  # exactly half a unit: ties go to even (0)
    a[9, 5] = 3 * 2.0 ** -33  # 1.5 units -> 2
    a[2, 100] = 0.5  # above the diagonal: ignored
    T = O.sat_build(a)
    with np.errstate(invalid="ignore"):
        q = q_matrix(np.nan_to_num(a, nan=0.0, posinf=0.0))
    q[7, 1] = 0
    assert q[9, 4] == 0 and q[9, 5] == 2 and q[2, 100] == 0
    assert np.array_equal(T, np.cumsum(np.cumsum(q, axis=0), axis=1))
    rng = np.random.default_rng(0)
    for _ in range(200):
        x1, x2 = sorted(rng.integers(0, 150, 2))
        y1, y2 = sorted(rng.integers(0, 150, 2))
        assert O.sat_rect(T, x1, x2, y1, y2) == int(q[x1:x2 + 1, y1:y2 + 1].sum())
    assert O.sat_rect(T, 3, 2, 0, 5) == 0 and O.sat_rect(T, 0, 5, 4, 3) == 0  # empty ranges
    # rows of a softmax sum to one: the last column is i + 1 up to rounding of the entries
    b = AT.make_attention(64)
    Tb = O.sat_build(b)
    assert np.abs(Tb[:, -1] / S - np.arange(1, 65)).max() < 1e-4


def brute(qm, mask, min_len, rho):
    """Everything from the definitions: IntraAttn(l,r) = sum_i sum_{j=l..i}, InterAttn = sum_i sum_{j<l}."""
    n = len(mask)
    bl, br = np.full(n, X, np.uint32), np.full(n, X, np.uint32)
    bs = np.zeros(n, np.int64)
    reus, rec = np.zeros(n, np.uint8), np.zeros(n, np.uint8)
    a = 0
    while a < n:
        if mask[a]:
            a += 1
            continue
        b = a
        while b + 1 < n and not mask[b + 1]:
            b += 1
        best = None
        for l in range(a, b + 1):
            for r in range(l, b + 1):
                if r - l + 1 < max(1, min_len):
                    continue
                intra = sum(int(qm[i, j]) for i in range(l, r + 1) for j in range(l, i + 1))
                inter = sum(int(qm[i, j]) for i in range(l, r + 1) for j in range(0, l))
                if best is None or intra - inter > best[0]:
                    best = (intra - inter, l, r)
        if best is not None:
            sc, l, r = best
            bl[a:b + 1], br[a:b + 1], bs[a:b + 1] = l, r, sc
        if best is not None and best[0] > 0:  # reuse criterion: IntraAttn(l, r) > InterAttn(l, r)
            reus[l:r + 1] = 1
            d = [sum(int(qm[i, j]) for j in range(0, l)) - sum(int(qm[i, j]) for j in range(l, i + 1))
                 for i in range(l, r + 1)]
            order = sorted(range(r - l + 1), key=lambda k: (-d[k], k))
            for k in order[: (r - l + 1) * rho // 100]:
                rec[l + k] = 1
        a = b + 1
    return bl, br, bs, reus, rec


@pytest.mark.parametrize("seed,min_len,rho", [(0, 1, 25), (1, 3, 50), (2, 6, 25), (3, 1, 100), (4, 2, 0)])
def test_annotate_against_definitions(seed, min_len, rho):
    n = 36
    a = AT.make_attention(n, seed=seed, passage_mean=7, tau=3.0, sink=1)
    mask = AT.make_mask(n, seed=seed + 10, run_mean=1.5, cover=0.2)
    T = O.sat_build(a)
    got = O.annotate(T, mask, min_len, rho)
    want = brute(q_matrix(a), mask, min_len, rho)
    for g, w, name in zip(got, want, ("best_l", "best_r", "best_score", "reusable", "recompute")):
        assert np.array_equal(g, w), name
    assert (got[3][mask == 1] == 0).all() and (got[4] <= got[3]).all()


def test_annotate_closed_forms():
    n = 10
    z = np.zeros(n, np.uint8)
    # every token attends to itself only: intra = length, inter = 0 -> the whole segment wins
    eye = np.eye(n, dtype=np.float32)
    bl, br, bs, reus, rec = O.annotate(O.sat_build(eye), z, 1, 30)
    assert (bl == 0).all() and (br == n - 1).all() and (bs == n * S).all() and reus.all()
    assert list(np.flatnonzero(rec)) == [0, 1, 2]  # all tokens tie at -1: the earliest three of ten at 30 %
    # every token attends to token 0 only.  With token 0 in the segment the whole segment wins ...
    first = np.zeros((n, n), np.float32)
    first[:, 0] = 1
    bl, br, bs, _, _ = O.annotate(O.sat_build(first), z, 1, 0)
    assert bl[0] == 0 and br[0] == n - 1 and bs[0] == n * S
    # ... with token 0 sensitive everything else only looks outside: score = -length, the first single token wins
    m = z.copy()
    m[0] = 1
    bl, br, bs, reus, _ = O.annotate(O.sat_build(first), m, 1, 0)
    assert bl[0] == X and bl[1] == 1 and br[1] == 1 and bs[1] == -S
    assert not reus.any()  # ... but fails the reuse criterion (inter-attention exceeds intra-attention): nothing to store
    # the minimum length then forces the first window of that length
    bl, br, bs, _, _ = O.annotate(O.sat_build(first), m, 4, 0)
    assert bl[1] == 1 and br[1] == 4 and bs[1] == -4 * S
    # a segment shorter than the minimum yields nothing; segments are independent
    m2 = np.array([0, 0, 1, 0, 0, 0, 0, 1, 0, 0], np.uint8)
    bl, br, bs, reus, _ = O.annotate(O.sat_build(eye), m2, 3, 0)
    assert list(bl) == [X, X, X, 3, 3, 3, 3, X, X, X] and list(br[3:7]) == [6] * 4 and list(reus) == [0, 0, 0, 1, 1, 1, 1, 0, 0, 0]
    # all-zero attention: every score ties at 0, the first candidate wins
    bl, br, bs, reus, rec = O.annotate(O.sat_build(np.zeros((n, n), np.float32)), z, 2, 50)
    assert bl[0] == 0 and br[0] == 1 and bs[0] == 0
    assert not reus.any() and not rec.any()  # intra-attention must exceed inter-attention, not equal it
    # a segment is judged by its own best substring: one passes the criterion, the other does not
    two = np.zeros((n, n), np.float32)
    two[np.arange(4), np.arange(4)] = 1  # tokens 0..3 attend to themselves
    two[5:, 0] = 1                       # tokens 5..9 attend to token 0, outside their segment
    m3 = z.copy()
    m3[4] = 1
    bl, br, bs, reus, rec = O.annotate(O.sat_build(two), m3, 1, 50)
    assert list(reus) == [1, 1, 1, 1, 0, 0, 0, 0, 0, 0] and bs[0] == 4 * S and bs[5] == -S and rec.sum() == 2


def test_generator_shapes():
    a = AT.make_attention(101)
    assert a.shape == (101, 104) and a.dtype == np.float32 and (np.triu(a[:, :101], 1) == 0).all()
    assert np.allclose(a[:, :101].sum(axis=1), 1.0, atol=1e-5) and (a[:, 101:] == 0).all()
    m = AT.make_mask(5000)
    assert 0.02 < m.mean() < 0.1
