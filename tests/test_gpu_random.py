"""Seeded random scenarios, GPU against the oracle: option combinations nobody wrote a test for
(vocabularies of two to six tokens so that prefixes, duplicates and chance anchors collide all the
time; empty requests; evictions; ties in the annotator).  Everything is compared as in the tests
these reuse: bit for bit."""
import numpy as np
import pytest

from cp_workload import attn as AT
from cp_workload import gen
from test_gpu_annotator import check
from test_gpu_parity import G  # noqa: F401  (fixture)
from test_gpu_policies import Lifecycle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(4))
def test_random_pool_lifecycles_small(G, block):
    for seed in range(block * 10, block * 10 + 10):
        rng = np.random.default_rng(1000 + seed)
        vocab = int(rng.choice([2, 3, 4, 6, 32000]))
        W = [None, 1, 2, 3, 5][int(rng.integers(0, 5))]
        verify, min_len = bool(rng.integers(0, 2)), int(rng.integers(1, 6))
        marks, zf = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        S = int(rng.integers(80, 400))
        print("case", dict(seed=seed, vocab=vocab, W=W, verify=verify, min_len=min_len, marks=marks, zf=zf, S=S), flush=True)
        life = Lifecycle(G, S, gen.KVShape(1, 2, 64), 0xABC000 + seed, verify, min_len=min_len, marks=marks,
                         zero_fill=zf, anchor_window=W)
        corpus = [rng.integers(0, vocab, 50).astype(np.uint32) for _ in range(5)]
        for epoch in range(1, 16):
            parts = []
            for d in rng.choice(5, int(rng.integers(1, 4)), replace=False):
                lead = rng.integers(0, vocab, int(rng.integers(0, 5))).astype(np.uint32)
                a = int(rng.integers(0, 20))
                parts.append(np.concatenate([lead, corpus[d][a:a + int(rng.integers(1, 31))]]))
            if rng.random() < 0.2:
                parts.insert(int(rng.integers(0, len(parts) + 1)), np.zeros(0, np.uint32))  # an empty request
            tok = np.concatenate(parts).astype(np.uint32)
            mask = (rng.random(len(tok)) < rng.choice([0.0, 0.05, 0.3])).astype(np.uint8)
            off = np.concatenate([[0], np.cumsum([len(x) for x in parts])]).astype(np.uint32)
            life.batch(epoch, tok, mask, off, (rng.random(len(tok)) < 0.25).astype(np.uint8))


@pytest.mark.parametrize("block", range(2))
def test_random_pool_lifecycles_several_scan_tiles(G, block):
    for seed in range(block * 6, block * 6 + 6):
        rng = np.random.default_rng(5000 + seed)
        vocab = int(rng.choice([2, 3, 5, 32000]))
        W = [None, 1, 3, 16, 64][int(rng.integers(0, 5))]
        verify, min_len = bool(rng.integers(0, 2)), int(rng.choice([1, 2, 8, 40]))
        marks, zf = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        S = int(rng.integers(3000, 9000))
        print("case", dict(seed=seed, vocab=vocab, W=W, verify=verify, min_len=min_len, marks=marks, zf=zf, S=S), flush=True)
        life = Lifecycle(G, S, gen.KVShape(1, 1, 64), 0xABD000 + seed, verify, min_len=min_len, marks=marks,
                         zero_fill=zf, anchor_window=W)
        corpus = [rng.integers(0, vocab, 1500).astype(np.uint32) for _ in range(5)]
        for epoch in range(1, 9):
            parts = []
            for d in rng.choice(5, int(rng.integers(2, 5)), replace=False):
                lead = rng.integers(0, vocab, int(rng.integers(0, 40))).astype(np.uint32)
                a = int(rng.integers(0, 500))
                parts.append(np.concatenate([lead, corpus[d][a:a + int(rng.integers(1, 1000))]]))
            tok = np.concatenate(parts).astype(np.uint32)
            mask = (rng.random(len(tok)) < rng.choice([0.0, 0.01, 0.1])).astype(np.uint8)
            off = np.concatenate([[0], np.cumsum([len(x) for x in parts])]).astype(np.uint32)
            life.batch(epoch, tok, mask, off, (rng.random(len(tok)) < 0.25).astype(np.uint8))
        assert life.evictions >= 1


@pytest.mark.parametrize("block", range(3))
def test_random_annotator_inputs(G, block):
    for seed in range(block * 15, block * 15 + 15):
        rng = np.random.default_rng(9000 + seed)
        n = int(rng.integers(1, 700))
        a = AT.make_attention(n, seed=seed, passage_mean=int(rng.integers(2, 80)), tau=float(rng.uniform(1, 30)),
                              ld=n + int(rng.integers(0, 9)))
        if rng.random() < 0.3:  # coarse weights: many exact ties between substrings and between tokens
            a = (np.round(a * 8) / 8).astype(np.float32)
        mask = AT.make_mask(n, seed=seed, run_mean=float(rng.uniform(1, 5)), cover=float(rng.choice([0.0, 0.02, 0.2, 0.6])))
        min_len, rho = int(rng.choice([0, 1, 2, 7, 64, 130])), int(rng.choice([0, 10, 25, 50, 100]))
        print("case", seed, n, a.shape[1], min_len, rho, int(mask.sum()), flush=True)
        check(G, a, mask, min_len, rho)
