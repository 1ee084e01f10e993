"""Pins for the oracle's Huffman-coded levels (Sec. 5, "Efficient Encoding": a Huffman code for the level indices,
built from a sample and then kept).  The paper fixes nothing beyond that; pinned here by examples worked by hand
(tests/golden/huffman_examples.txt), Kraft's equality, optimality against brute force over all length assignments,
prefix-freeness, the bit-length identity and the round trip, sync entries checked by decoding from them."""
import itertools
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def golden(kind):
    rows = []
    for line in open(os.path.join(HERE, "golden", "huffman_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [x.strip() for x in line.split("|")]
        if f[0] == kind:
            rows.append(f[1:])
    return rows


@pytest.mark.parametrize("s,hist,lengths,codes", golden("L"))
def test_hand_built_codes(s, hist, lengths, codes):
    s = int(s)
    got = oracle.huffman_lengths([int(x) for x in hist.split()], s)
    assert [int(x) for x in got] == [int(x) for x in lengths.split()]
    assert oracle.huffman_codes(got, s) == codes.split()


@pytest.mark.parametrize("s,lengths,bucket,levels,bits", golden("E"))
def test_hand_coded_bit_strings(s, lengths, bucket, levels, bits):
    s, bucket = int(s), int(bucket)
    lengths = [int(x) for x in lengths.split()]
    flat = [int(x) for part in levels.split("/") for x in part.split()]
    q = np.array([abs(x) | (0x80 if x < 0 else 0) for x in flat], dtype=np.uint8)
    bo, words, _ = oracle.encode_huffman(q, bucket, s, lengths)
    want = ["".join(part.split()) for part in bits.split("/")]
    for b, w in enumerate(want):
        start = (int(bo[b]) + 31) // 32 * 32
        assert int(bo[b + 1]) - start == len(w)
        assert oracle.words_to_bits(words, start, int(bo[b + 1])) == w
    np.testing.assert_array_equal(oracle.decode_huffman(bo, words, q.size, bucket, s, lengths), q)


def kraft(lengths):
    return sum(2.0 ** -int(l) for l in lengths)


@pytest.mark.parametrize("s", [1, 2, 3, 5, 9, 14])
def test_kraft_equality_and_prefix_freeness(s):
    rng = np.random.default_rng(s)
    for trial in range(30):
        hist = (rng.random(s + 2) ** 6 * 10 ** rng.integers(0, 9)).astype(np.uint64)
        lengths = oracle.huffman_lengths(hist, s)
        assert kraft(lengths) == 1.0 and lengths.min() >= 1 and lengths.max() <= s + 1
        codes = oracle.huffman_codes(lengths, s)
        for a, b in itertools.permutations(codes, 2):
            assert not b.startswith(a)
        w = hist + 1                          # a heavier symbol never has a longer codeword
        for i in range(s + 2):
            for j in range(s + 2):
                if w[i] > w[j]:
                    assert lengths[i] <= lengths[j]


@pytest.mark.parametrize("s", [1, 2, 3])
def test_optimal_against_brute_force(s):
    """Minimum of sum (hist+1) * length over every length assignment that satisfies Kraft's inequality."""
    rng = np.random.default_rng(10 + s)
    n = s + 2
    feasible = [c for c in itertools.product(range(1, n), repeat=n) if kraft(c) <= 1.0]
    for trial in range(40):
        hist = rng.integers(0, 50, size=n).astype(np.uint64)
        w = (hist + 1).astype(np.int64)
        best = min(int(np.dot(w, c)) for c in feasible)
        assert int(np.dot(w, oracle.huffman_lengths(hist, s).astype(np.int64))) == best


@pytest.mark.parametrize("bucket,s,S,d", [(1000, 3, 256, 4321), (8192, 3, 512, 20000), (512, 6, 64, 5000), (7, 14, 0, 100),
                                          (2048, 4, 1024, 5000)])
def test_round_trip_lengths_and_sync(bucket, s, S, d):
    rng = np.random.default_rng(bucket + s)
    q = np.where(rng.random(d) < 0.15, rng.integers(1, s + 2, d), 0).astype(np.uint8)
    q |= np.where((q > 0) & (rng.random(d) < 0.5), 0x80, 0).astype(np.uint8)
    lengths = oracle.huffman_lengths(oracle.level_histogram_of(q[: d // 3], s), s)    # the code comes from a sample
    codes = oracle.huffman_codes(lengths, s)
    bo, words, sync = oracle.encode_huffman(q, bucket, s, lengths, S)
    np.testing.assert_array_equal(oracle.decode_huffman(bo, words, d, bucket, s, lengths), q)
    nb, ns = oracle.num_buckets(d, bucket), oracle.num_sync_huffman(bucket, S)
    lev = (q & 0x7F).astype(np.int64)
    per_coord = lengths.astype(np.int64)[lev] + (lev > 0)
    for b in range(nb):
        lo, hi = b * bucket, min(d, (b + 1) * bucket)
        start = (int(bo[b]) + 31) // 32 * 32
        assert int(bo[b + 1]) - start == int(per_coord[lo:hi].sum())          # bit length identity
        assert b == 0 or start - int(bo[b]) < 32                              # word alignment, nothing else between
        for g in range(1, ns + 1):
            first = lo + g * S
            off = int(sync[b * ns + g - 1])
            assert off == int(per_coord[lo:min(first, hi)].sum())            # where coordinate g*S starts
            if first < hi:                                                    # and decoding from there finds it
                bits = oracle.words_to_bits(words, start + off, min(start + off + 16, int(bo[b + 1])))
                level = int(lev[first])
                assert bits.startswith(codes[level])


def test_unseen_levels_still_have_codes_and_bad_input_is_rejected():
    s = 3
    lengths = oracle.huffman_lengths([1000, 0, 0, 0, 0], s)       # the sample saw only zeros
    q = np.array([4, 0x84, 1, 0, 2, 3], dtype=np.uint8)
    bo, words, _ = oracle.encode_huffman(q, 6, s, lengths)
    np.testing.assert_array_equal(oracle.decode_huffman(bo, words, 6, 6, s, lengths), q)
    with pytest.raises(ValueError):
        oracle.huffman_codes([1, 1, 2, 3, 3], s)                  # not a complete code
    with pytest.raises(RuntimeError):
        oracle.encode_huffman(np.array([5], dtype=np.uint8), 4, s, lengths)      # level above s + 1
    with pytest.raises(ValueError):
        oracle.decode_huffman(bo, words[:-1] if words.size > 1 else np.zeros(1, np.uint32), 6, 6, s,
                              oracle.huffman_lengths([0, 1000, 0, 0, 0], s))     # the wrong code: runs off the end
