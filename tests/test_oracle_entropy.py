"""Pins of the oracle's entropy-coding part (Sec. 3.1, last paragraph) against what the mathematics and the
paper fix: Kraft's equality, the noiseless-coding bounds, exact lengths for dyadic laws, optimality by brute
force over every complete prefix code of small alphabets, and the two figures the paper prints for b = 4."""
import itertools
import math

import numpy as np
import pytest

from oracle import turboquant_oracle as o


def _best_by_enumeration(p):
    """Smallest expected length over every length vector with Kraft sum exactly 1."""
    K = len(p)
    best = math.inf
    for L in itertools.product(range(1, K), repeat=K):
        if sum(2.0 ** -l for l in L) == 1.0:
            best = min(best, sum(pi * l for pi, l in zip(p, L)))
    return best


def test_dyadic_and_uniform_laws_have_exact_lengths():
    assert list(o.huffman_lengths([0.5, 0.25, 0.125, 0.125])) == [1, 2, 3, 3]
    assert list(o.huffman_lengths([0.125, 0.5, 0.125, 0.25])) == [3, 1, 3, 2]
    for b in (1, 2, 3, 4):
        assert list(o.huffman_lengths(np.full(1 << b, 2.0 ** -b))) == [b] * (1 << b)
    assert list(o.huffman_lengths([1.0])) == [0]


@pytest.mark.parametrize("seed", range(6))
def test_lengths_are_optimal_and_complete(seed):
    rng = np.random.default_rng(seed)
    K = 3 + seed % 4
    p = rng.dirichlet(np.ones(K) * (0.3 + seed))
    L = o.huffman_lengths(p)
    assert sum(2.0 ** -int(l) for l in L) == 1.0  # Kraft with equality: a complete code
    mean = float((p * L).sum())
    assert abs(mean - _best_by_enumeration(p)) < 1e-12
    H = o.index_entropy(p)
    assert H - 1e-12 <= mean < H + 1


def test_canonical_codewords_are_prefix_free_and_round_trip():
    rng = np.random.default_rng(3)
    p = rng.dirichlet(np.ones(16) * 0.5)
    L = o.huffman_lengths(p)
    C = o.canonical_codewords(L)
    words = [format(int(c), "b").zfill(int(l)) for c, l in zip(C, L)]
    for a, b in itertools.permutations(words, 2):
        assert not b.startswith(a)
    idx = rng.integers(0, 16, size=(7, 64))
    bits, starts = o.prefix_encode(idx, L, C)
    assert len(bits) == int(L[idx].sum()) and starts[3] == int(L[idx[:3]].sum())
    assert np.array_equal(o.prefix_decode(bits, L, C, 7, 64), idx)


def test_paper_figures_for_four_bits(paper):
    """Entropy of the b = 4 index distribution "approximately 3.8"; an optimal prefix code reduces the average
    bit-width "by 5 %" (both to the printed precision); smaller gains at smaller b."""
    savings = {}
    for b in (1, 2, 3, 4):
        c, _, _ = o.lloyd_max_codebook(1536, b)
        p = o.bucket_masses(c, 1536)
        assert abs(p.sum() - 1) < 1e-12
        L = o.huffman_lengths(p)
        savings[b] = 1 - float((p * L).sum()) / b
        if b == 4:
            assert abs(o.index_entropy(p) - paper["entropy_b4"]) < 0.05
    assert abs(savings[4] - paper["prefix_saving_b4"]) < 0.005
    assert savings[1] == 0 and savings[2] < savings[3] < savings[4]
