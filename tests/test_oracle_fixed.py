"""Pins for the oracle's fixed-width coding (Sec. 5: the "4-bit"/"8-bit" variants; 3 bits in Table 1).  The paper
fixes only the width; the layout is this project's and is pinned by examples packed by hand
(tests/golden/fixed_examples.txt), the size formula, single-code bit positions and unpack(pack(q)) == q."""
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "fixed_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        b, bucket, s, levels, words = [x.strip() for x in line.split("|")]
        buckets = [[int(t) for t in part.split()] for part in levels.split("/")]
        rows.append((int(b), int(bucket), int(s), buckets, [int(w, 16) for w in words.split()]))
    return rows


@pytest.mark.parametrize("b,bucket,s,buckets,words", golden())
def test_hand_packed_examples(b, bucket, s, buckets, words):
    flat = [x for part in buckets for x in part]
    assert all(len(part) == bucket for part in buckets[:-1]) and len(buckets[-1]) <= bucket
    q = np.array([abs(x) | (0x80 if x < 0 else 0) for x in flat], dtype=np.uint8)
    packed = oracle.pack_fixed(q, bucket, s, b)
    assert [int(w) for w in packed] == words
    np.testing.assert_array_equal(oracle.unpack_fixed(packed, q.size, bucket, s, b), q)


def test_size_formula_and_rejections():
    assert oracle.fixed_words(8192, 8192, 4) == 1024
    assert oracle.fixed_words(8193, 8192, 4) == 2048                 # the short bucket has a whole field too
    assert oracle.fixed_words(100, 12, 3) == 9 * 2                   # ceil(36 / 32) = 2 words per bucket
    q = np.array([1, 2, 3, 0], dtype=np.uint8)
    with pytest.raises(ValueError):
        oracle.pack_fixed(q, 4, 3, 3)                                # s + 2 = 5 levels need 3 level bits: b >= 4
    with pytest.raises(ValueError):
        oracle.pack_fixed(np.array([5], dtype=np.uint8), 4, 2, 4)    # level index above s + 1
    with pytest.raises(ValueError):
        oracle.pack_fixed(np.array([0x80], dtype=np.uint8), 4, 2, 4) # a zero carries no sign
    with pytest.raises(ValueError):
        oracle.unpack_fixed(np.array([0x80000000], dtype=np.uint32), 1, 4, 2, 4)   # code 1000: "-0"


@pytest.mark.parametrize("b,s", [(3, 2), (4, 3), (4, 6), (5, 10), (8, 14), (8, 3), (6, 1)])
def test_single_codes_sit_where_the_layout_says(b, s):
    """One nonzero coordinate at a time: its code occupies bits [i*b, i*b+b) of its bucket's field, MSB first."""
    bucket, d = 37, 100
    wpb = (bucket * b + 31) // 32
    for i in (0, 1, 10, 36, 37, 73, 99):
        for level, neg in ((1, 0), (s + 1, 1)):
            q = np.zeros(d, dtype=np.uint8)
            q[i] = level | (neg << 7)
            packed = oracle.pack_fixed(q, bucket, s, b)
            assert packed.size == ((d + bucket - 1) // bucket) * wpb
            code = (neg << (b - 1)) | level
            bits = "".join(format(int(w), "032b") for w in packed)
            start = (i // bucket) * wpb * 32 + (i % bucket) * b
            assert bits[start:start + b] == format(code, "0%db" % b)
            assert bits.count("1") == bin(code).count("1")


@pytest.mark.parametrize("b,s,bucket,d", [(3, 2, 1000, 4321), (4, 3, 8192, 20000), (4, 6, 512, 5000), (8, 14, 7, 100),
                                          (5, 9, 33, 1000), (3, 1, 64, 300)])
def test_round_trip_and_average(b, s, bucket, d):
    rng = np.random.default_rng(b * 100 + s)
    K = 3
    norms_list, packed_list, dense = [], [], np.zeros(d)
    for _ in range(K):
        q = np.where(rng.random(d) < 0.6, rng.integers(1, s + 2, d), 0).astype(np.uint8)
        q |= np.where((q > 0) & (rng.random(d) < 0.5), 0x80, 0).astype(np.uint8)
        packed = oracle.pack_fixed(q, bucket, s, b)
        np.testing.assert_array_equal(oracle.unpack_fixed(packed, d, bucket, s, b), q)
        norms = (10.0 ** rng.uniform(-2, 2, size=oracle.num_buckets(d, bucket))).astype(np.float32)
        norms_list.append(norms)
        packed_list.append(packed)
        lv = np.where(q & 0x7F, np.ldexp(1.0, (q & 0x7F).astype(np.int64) - 1 - s), 0.0)
        dense += np.repeat(norms.astype(np.float64), bucket)[:d] * np.where(q & 0x80, -1.0, 1.0) * lv
    out = oracle.unpack_average_fixed(norms_list, packed_list, d, bucket, s, b, 1.0 / K)
    np.testing.assert_allclose(out, dense / K, rtol=1e-15, atol=0)
