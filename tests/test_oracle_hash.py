"""Pins for the oracle's chain hash (polynomial rolling hash of Sec. 4.2.2,
segmented by sensitive tokens as in Sec. 4.2.1)."""
import numpy as np

import oracle as O
from tests.bruteforce import runs

M64 = (1 << 64) - 1
B = O.BASE


def H(tok, mask=None, off=None, base=B):
    tok = np.asarray(tok, np.uint32)
    mask = np.zeros(len(tok), np.uint8) if mask is None else np.asarray(mask, np.uint8)
    off = np.array([0, len(tok)], np.uint32) if off is None else np.asarray(off, np.uint32)
    return [int(x) for x in O.hash_segments(tok, mask, off, base)]


def test_decimal_worked_example():
    # With base 10 the hash of a run is the decimal number whose digits are tok+1.
    assert H([1, 2, 3], base=10) == [2, 23, 234]
    # a sensitive token cuts the number; the chain restarts after it
    assert H([1, 2, 3, 4, 5], mask=[0, 0, 1, 0, 0], base=10) == [2, 23, O.HASH_NONE, 5, 56]
    # so does a request boundary
    assert H([1, 2, 3, 4], off=[0, 2, 4], base=10) == [2, 23, 4, 45]
    # token id 0 still contributes (digit 1): [0] and [0, 0] differ
    assert H([0, 0], base=10) == [1, 11]


def test_closed_forms_default_base():
    assert H([7]) == [8]
    assert H([31999, 0]) == [32000, (32000 * B + 1) & M64]
    t = [5, 17, 31999, 0, 12345]
    want = sum((t[m] + 1) * pow(B, len(t) - 1 - m) for m in range(len(t))) & M64  # the polynomial, term by term
    assert H(t)[-1] == want


def test_wraps_mod_2_64():
    rng = np.random.default_rng(1)
    t = rng.integers(0, 32000, 40)
    exact = sum((int(t[m]) + 1) * B ** (len(t) - 1 - m) for m in range(len(t)))
    assert exact > M64  # really overflows
    assert H(t)[-1] == exact % (1 << 64)


def test_none_value_is_remapped():
    # run [0, 5] with base 2^64 - 7 gives  1 * base + 6 = 2^64 - 1 = NONE  ->  NONE - 1
    assert H([0, 5], base=(1 << 64) - 7) == [1, O.HASH_NONE - 1]


def test_substring_identity_against_unsegmented_prefix_hashes():
    """Sec. 4.2.2 "full verification": hash(a..i) = P[i] - P[a-1] * base^(i-a+1)."""
    rng = np.random.default_rng(2)
    n = 300
    tok = rng.integers(0, 32000, n).astype(np.uint32)
    mask = (rng.random(n) < 0.15).astype(np.uint8)
    off = np.array([0, 97, 98, 211, n], np.uint32)
    seg = H(tok, mask, off)
    P = [0] + H(tok)  # P[k] = hash of tok[0..k-1], no segmentation
    n_checked = 0
    for _, a, b in runs(tok, mask, off):
        for i in range(a, b):
            assert seg[i] == (P[i + 1] - P[a] * pow(B, i - a + 1, 1 << 64)) & M64
            n_checked += 1
    assert n_checked == int((mask == 0).sum())
    assert all(seg[i] == O.HASH_NONE for i in range(n) if mask[i])


def test_sensitive_ids_do_not_matter():
    rng = np.random.default_rng(3)
    n = 500
    tok = rng.integers(0, 32000, n).astype(np.uint32)
    mask = (rng.random(n) < 0.3).astype(np.uint8)
    off = np.array([0, 200, n], np.uint32)
    tok2 = tok.copy()
    tok2[mask == 1] = rng.integers(0, 32000, int(mask.sum()))
    assert H(tok, mask, off) == H(tok2, mask, off)


def test_equal_hash_iff_equal_run_prefix_small_vocab():
    rng = np.random.default_rng(4)
    n = 400
    tok = rng.integers(0, 3, n).astype(np.uint32)  # tiny vocabulary: many equal prefixes
    mask = (rng.random(n) < 0.25).astype(np.uint8)
    off = np.array([0, 150, 151, n], np.uint32)
    h = H(tok, mask, off)
    pref = {}
    for _, a, b in runs(tok, mask, off):
        for i in range(a, b):
            pref[i] = tuple(int(x) for x in tok[a : i + 1])
    idx = sorted(pref)
    n_equal = 0
    for x in idx:
        for y in idx:
            assert (h[x] == h[y]) == (pref[x] == pref[y])
            n_equal += x != y and pref[x] == pref[y]
    assert n_equal > 100  # the case "equal prefixes at different places" was really exercised


def test_empty_and_degenerate():
    assert H([]) == []
    assert H([], off=[0, 0, 0]) == []
    assert H([9, 9], mask=[1, 1]) == [O.HASH_NONE, O.HASH_NONE]
    assert H([3], off=[0, 0, 1, 1]) == [4]
