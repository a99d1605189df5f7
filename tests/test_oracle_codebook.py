"""Pins for the oracle's Huffman codebook (Section 3.1.2; built once per layer from the code histogram, Section 3).

Expected values: hand-derived cases in tests/golden/huffman_ties.txt, the Kraft equality, brute-force optimal
prefix-code cost on tiny alphabets, textbook special cases, and the entropy bounds.
"""
import itertools
import math
import pathlib

import numpy as np
import pytest

GOLDEN = pathlib.Path(__file__).parent / "golden" / "huffman_ties.txt"


def _cases():
    out = []
    for line in GOLDEN.read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        counts, lens, codes = [p.split() for p in line.split("|")]
        out.append(([int(c) for c in counts], [int(x) for x in lens], codes))
    return out


def _hist(counts):
    h = np.zeros(256, np.uint64)
    h[: len(counts)] = counts
    return h


@pytest.mark.parametrize("counts,lens,codes", _cases())
def test_hand_derived_cases(oracle, counts, lens, codes):
    ln, cd, halv = oracle.build_codebook(_hist(counts), len(counts), 12)
    assert halv == 0
    assert list(ln[: len(counts)]) == lens
    assert [format(int(cd[s]), "b").zfill(int(ln[s])) for s in range(len(counts))] == codes
    assert not ln[len(counts):].any()


def _kraft_units(ln, max_len=16):
    return sum(1 << (max_len - int(l)) for l in ln if l)


def _complete_length_multisets(n, max_depth):
    """All non-decreasing length sequences of n code words with Kraft sum exactly 1."""
    out = []

    def rec(prefix, remaining_units, depth_min):
        k = n - len(prefix)
        if k == 0:
            if remaining_units == 0:
                out.append(tuple(prefix))
            return
        for L in range(depth_min, max_depth + 1):
            u = 1 << (max_depth - L)
            if u * k < remaining_units:  # even k words this short cannot fill the rest
                break
            if u > remaining_units:
                continue
            rec(prefix + [L], remaining_units - u, L)

    rec([], 1 << max_depth, 1)
    return out


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7, 8])
def test_cost_is_brute_force_optimal_on_tiny_alphabets(oracle, n):
    rng = np.random.default_rng(100 + n)
    shapes = _complete_length_multisets(n, n - 1 if n > 2 else 1)
    assert shapes
    for trial in range(40):
        counts = rng.integers(1, 30, n) if trial % 2 else rng.integers(1, 4, n)
        ln, cd, _ = oracle.build_codebook(_hist(counts), n, 12)
        cost = int(sum(int(c) * int(l) for c, l in zip(counts, ln[:n])))
        assert _kraft_units(ln) == 1 << 16
        desc = sorted((int(c) for c in counts), reverse=True)
        best = min(sum(c * l for c, l in zip(desc, shape)) for shape in shapes)
        assert cost == best, (counts, ln[:n])


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_cost_is_optimal_over_every_length_assignment(oracle, n):
    # no appeal to sorting: enumerate every assignment of lengths 1..n-1 that satisfies the Kraft inequality
    rng = np.random.default_rng(200 + n)
    md = max(1, n - 1)
    feasible = [a for a in itertools.product(range(1, md + 1), repeat=n) if sum(2.0 ** -l for l in a) <= 1.0]
    for _ in range(25):
        counts = rng.integers(1, 20, n)
        ln, _, _ = oracle.build_codebook(_hist(counts), n, 12)
        cost = sum(int(c) * int(l) for c, l in zip(counts, ln[:n]))
        assert cost == min(sum(int(c) * l for c, l in zip(counts, a)) for a in feasible)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7, 8])
def test_uniform_power_of_two_alphabet_is_fixed_length(oracle, k):
    n = 1 << k
    ln, cd, _ = oracle.build_codebook(_hist([9] * n), n, 12)
    assert list(ln[:n]) == [k] * n
    assert list(cd[:n]) == list(range(n))  # canonical codes of equal length count up in symbol order


def test_geometric_counts_give_the_unary_like_code(oracle):
    counts = [1, 1] + [1 << i for i in range(1, 11)]  # 1,1,2,4,...,1024 -> lengths 11,11,10,...,1
    n = len(counts)
    ln, _, halv = oracle.build_codebook(_hist(counts), n, 12)
    assert halv == 0
    assert list(ln[:n]) == [n - 1, n - 1] + list(range(n - 2, 0, -1))


def _entropy_bits(counts):
    c = np.asarray(counts, np.float64)
    p = c / c.sum()
    return float(-(p * np.log2(p)).sum())


def test_cost_within_one_bit_of_entropy_on_gaussian_like_histograms(oracle):
    rng = np.random.default_rng(7)
    for nsym in (26, 51, 101):
        x = np.clip(np.rint(rng.normal((nsym - 1) / 2, nsym / 6, 200000)), 0, nsym - 1).astype(np.int64)
        counts = np.bincount(x, minlength=nsym)
        ln, cd, _ = oracle.build_codebook(_hist(counts), nsym, 12)
        f = np.maximum(counts, 1)
        avg = float((f * ln[:nsym]).sum() / f.sum())
        H = _entropy_bits(f)
        assert H <= avg + 1e-12 and avg < H + 1.0
        assert _kraft_units(ln) == 1 << 16
        assert all(ln[:nsym] > 0) and not ln[nsym:].any()


def _heap_huffman_cost(f):
    import heapq
    h = [int(x) for x in f]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def test_length_limit(oracle):
    # Fibonacci-like counts force a 40-deep tree; the limit must hold, Kraft must stay an equality, and the code
    # must still be an optimal code for the counts after the stated number of halvings
    counts = [1, 1]
    while len(counts) < 40:
        counts.append(counts[-1] + counts[-2])
    n = len(counts)
    for max_len in (8, 10, 12, 16):
        ln, cd, halv = oracle.build_codebook(_hist(counts), n, max_len)
        assert halv > 0
        assert int(ln.max()) <= max_len
        assert _kraft_units(ln) == 1 << 16
        f = np.array(counts, dtype=object)
        for _ in range(halv):
            f = np.array([max(1, (int(v) + 1) >> 1) for v in f], dtype=object)
        assert sum(int(a) * int(b) for a, b in zip(f, ln[:n])) == _heap_huffman_cost(f)


def test_every_admissible_limit_on_random_histograms(oracle):
    # peaked histograms of the workloads' alphabet sizes under every limit from the fixed-length width up to 12: the
    # limit holds, Kraft stays an equality, a more frequent level never gets a longer word, and the lengths are an
    # optimal code for the counts after the reported number of halvings (checked against a heap Huffman written here)
    rng = np.random.default_rng(77)
    for nsym in (6, 8, 21, 26, 51, 101, 126):
        for trial in range(3):
            centre, width = rng.uniform(0, nsym), rng.uniform(0.5, nsym / 3)
            counts = np.rint(1e6 * np.exp(-0.5 * ((np.arange(nsym) - centre) / width) ** 2)).astype(np.int64)
            counts[rng.integers(0, nsym, 3)] = 0   # some levels unseen at prefill
            for max_len in range(max(1, math.ceil(math.log2(nsym))), 13):
                ln, cd, halv = oracle.build_codebook(_hist(counts), nsym, max_len)
                assert 1 <= int(ln[:nsym].min()) and int(ln.max()) <= max_len and not ln[nsym:].any()
                assert _kraft_units(ln) == 1 << 16
                f = np.array([max(1, int(v)) for v in counts], dtype=object)
                for _ in range(halv):
                    f = np.array([max(1, (int(v) + 1) >> 1) for v in f], dtype=object)
                assert sum(int(a) * int(b) for a, b in zip(f, ln[:nsym])) == _heap_huffman_cost(f)
                order = np.argsort(-f.astype(np.float64), kind="stable")
                lens_by_freq = [int(ln[i]) for i in order]
                freqs = [int(f[i]) for i in order]
                for a in range(nsym - 1):
                    if freqs[a] > freqs[a + 1]:
                        assert lens_by_freq[a] <= min(lens_by_freq[a + 1:])


def test_unseen_levels_still_get_codes(oracle):
    # the codebook is built once at prefill and reused for later blocks: every level below n_sym must be encodable
    counts = [0] * 51
    counts[25] = 1000
    ln, cd, _ = oracle.build_codebook(_hist(counts), 51, 12)
    assert all(ln[:51] > 0) and not ln[51:].any()
    assert ln[25] == 1
    assert _kraft_units(ln) == 1 << 16


def test_canonical_codes_are_prefix_free_and_ordered(oracle):
    rng = np.random.default_rng(9)
    for nsym in (2, 3, 26, 51, 101, 256):
        counts = rng.integers(0, 1000, nsym) ** 2
        ln, cd, _ = oracle.build_codebook(_hist(counts), nsym, 12)
        words = [format(int(cd[s]), "b").zfill(int(ln[s])) for s in range(nsym)]
        assert all(len(w) == ln[s] for s, w in enumerate(words))
        for a, b in itertools.permutations(range(nsym), 2):
            assert not words[b].startswith(words[a])
        order = sorted(range(nsym), key=lambda s: (int(ln[s]), s))
        # left-aligned code values strictly increase along (length, symbol) order
        aligned = [int(cd[s]) << (16 - int(ln[s])) for s in order]
        assert all(x < y for x, y in zip(aligned, aligned[1:]))
        assert aligned[0] == 0


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.build_codebook(_hist([1, 1]), 1, 12)
    with pytest.raises(ValueError):
        oracle.build_codebook(_hist([1, 1]), 2, 40)
    assert math.isclose(_entropy_bits([1, 1]), 1.0)
