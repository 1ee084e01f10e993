"""Pins for the oracle's Elias recursive coding, ENCODE and DECODE (App. A).

Expected values are hand-worked from Alg. 2 and the ENCODE description (text
fixtures under tests/golden/), or are properties the paper states: unique
decodability, shorter codes for smaller values, |ERC(N)| growth (App. A items 1-3),
sum of gaps <= d (App. C), Thm 2's code-length bound, DECODE(ENCODE(x)) = x, and
the aggregate of Alg. 1 computed densely.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------------- ERC

def test_erc_hand_worked_codewords():
    for row in read_rows("erc_codewords.txt"):
        n, code = row.split()
        assert oracle.erc_encode(int(n)) == code, n
        assert oracle.erc_decode(code) == (int(n), len(code))


def test_erc_hand_worked_lengths():
    for row in read_rows("erc_lengths.txt"):
        lo, hi, length = map(int, row.split())
        for n in {lo, lo + 1, (lo + hi) // 2, hi - 1, hi}:
            if lo <= n <= hi:
                assert oracle.erc_length(n) == length, n


def test_erc_rejects_non_positive():
    with pytest.raises(ValueError):
        oracle.erc_encode(0)


def test_erc_roundtrip_prefix_free_and_monotone():
    codes = [oracle.erc_encode(n) for n in range(1, 70001)]
    for n, c in enumerate(codes, start=1):
        # decoding needs no knowledge of N's range and stops exactly at the code's end,
        # also when more bits follow (App. A item 3)
        assert oracle.erc_decode(c + "1011") == (n, len(c))
    lens = [len(c) for c in codes]
    assert all(a <= b for a, b in zip(lens, lens[1:]))          # shorter codes for smaller values
    srt = sorted(codes)
    assert all(not b.startswith(a) for a, b in zip(srt, srt[1:]))  # prefix-free
    for n in [2 ** k for k in range(17, 32)] + [2 ** 32 - 1, 2 ** 31 + 12345]:
        c = oracle.erc_encode(n)
        assert oracle.erc_decode(c) == (n, len(c))
        # App. A item 1: |ERC(N)| <= (1 + o(1)) log N + 1; an explicit form of the o(1) term
        lg = math.log2(n)
        assert len(c) <= lg + 2 * math.log2(lg + 1) + 5
    with pytest.raises(ValueError):
        oracle.erc_decode("1110")        # truncated code


# -------------------------------------------------------------------- ENCODE

def signed_levels_to_q(vals):
    return np.array([(abs(x) | (0x80 if x < 0 else 0)) for x in vals], dtype=np.uint8)


def test_encode_hand_worked_examples():
    for row in read_rows("encode_examples.txt"):
        s, vals, bits = [x.strip() for x in row.split("|")]
        q = signed_levels_to_q([int(x) for x in vals.split()])
        bits = "" if bits == "-" else bits
        bit_off, words, _ = oracle.encode(q, q.size, int(s))
        assert bit_off.tolist() == [0, len(bits)]
        assert oracle.words_to_bits(words, 0, len(bits)) == bits
        assert words.size == (len(bits) + 31) // 32
        # pad bits are zero
        assert oracle.words_to_bits(words, len(bits), 32 * words.size) == "0" * (32 * words.size - len(bits))
        np.testing.assert_array_equal(oracle.decode_levels(bit_off, words, q.size, q.size, int(s)), q)


def test_encode_two_buckets_alignment_and_offsets():
    # bucket 0: "110001010001110" (15 bits), bucket 1 starts at bit 32, bucket 2 empty,
    # bucket 3 short (3 coords): gap 2 -> 100, -, level 1 -> 0
    q = signed_levels_to_q([0, 0, 1, 0, 0, 0, -3, 0,
                            0, 0, 0, 0, 0, 0, 0, 4,
                            0, 0, 0, 0, 0, 0, 0, 0,
                            0, -1, 0])
    bit_off, words, _ = oracle.encode(q, 8, 3)
    b1 = "1110000" + "0" + "101000"          # gap 8, +, ERC(4)
    b3 = "100" + "1" + "0"
    assert bit_off.tolist() == [0, 15, 32 + len(b1), 64, 64 + len(b3)]
    assert oracle.words_to_bits(words, 0, 15) == "110001010001110"
    assert oracle.words_to_bits(words, 32, 32 + len(b1)) == b1
    assert oracle.words_to_bits(words, 64, 64 + len(b3)) == b3
    assert words.size == 3
    np.testing.assert_array_equal(oracle.decode_levels(bit_off, words, q.size, 8, 3), q)


def test_encode_bit_count_formula_and_gap_sum():
    """Length of a bucket = sum over nonzeros of |ERC(gap)| + 1 + |ERC(j)| (App. C parts
    R and E), with sum of gaps <= bucket size."""
    rng = np.random.default_rng(1)
    bucket, s = 512, 3
    q = np.where(rng.random(5 * bucket - 100) < 0.2, rng.integers(1, s + 2, 5 * bucket - 100), 0).astype(np.uint8)
    q |= np.where((q > 0) & (rng.random(q.size) < 0.5), 0x80, 0).astype(np.uint8)
    bit_off, words, _ = oracle.encode(q, bucket, s)
    for b in range(5):
        seg = q[b * bucket:(b + 1) * bucket]
        nz = np.flatnonzero(seg & 0x7F)
        gaps = np.diff(np.concatenate(([-1], nz)))
        assert gaps.sum() <= seg.size and (gaps >= 1).all()
        bits = sum(oracle.erc_length(int(g)) + 1 + oracle.erc_length(int(seg[i] & 0x7F)) for g, i in zip(gaps, nz))
        start = (int(bit_off[b]) + 31) // 32 * 32
        assert int(bit_off[b + 1]) - start == bits
    assert words.size == (int(bit_off[-1]) + 31) // 32


def test_encode_capacity_and_bad_level():
    q = np.full(64, 4, np.uint8)
    with pytest.raises(RuntimeError):
        oracle.encode(q, 64, 3, words_cap=2)
    with pytest.raises(RuntimeError):
        oracle.encode(np.full(8, 5, np.uint8), 8, 3)      # level index above s+1
    assert oracle.max_words(64, 64, 3) * 32 >= 64 * 8


@pytest.mark.parametrize("bucket,s,stride", [(8192, 3, 512), (16384, 7, 1024), (512, 3, 512), (1000, 2, 256), (8192, 4, 0)])
def test_roundtrip_and_sync_entries(bucket, s, stride):
    rng = np.random.default_rng(bucket + s)
    d = 3 * bucket + bucket // 3
    dens = np.repeat(rng.choice([0.0, 0.002, 0.07, 0.5, 1.0], size=(d + 255) // 256), 256)[:d]
    q = np.where(rng.random(d) < dens, rng.integers(1, s + 2, d), 0).astype(np.uint8)
    q |= np.where((q > 0) & (rng.random(d) < 0.5), 0x80, 0).astype(np.uint8)
    q[bucket - 1] = 0x81                      # nonzero in the last place of bucket 0
    bit_off, words, sync = oracle.encode(q, bucket, s, stride)
    np.testing.assert_array_equal(oracle.decode_levels(bit_off, words, d, bucket, s), q)
    ns = oracle.num_sync(bucket, stride)
    assert sync.size == ns * oracle.num_buckets(d, bucket)
    # every sync entry holds the offset of the first record at or after its boundary: decoding from
    # there, with the first gap replaced by the recorded position, reproduces that record
    for b in range(oracle.num_buckets(d, bucket)):
        seg = q[b * bucket:(b + 1) * bucket]
        start = (int(bit_off[b]) + 31) // 32 * 32
        nzall = np.flatnonzero(seg & 0x7F)
        for g in range(1, ns + 1):
            e = int(sync[b * ns + g - 1])
            after = nzall[nzall >= g * stride]
            off = e & 0x1FFFFF
            if after.size == 0:
                assert e == (int(bit_off[b + 1]) - start) | oracle.SYNC_EMPTY
                continue
            first = int(after[0])
            if first < (g + 1) * stride:
                assert (e >> 31) == 0 and ((e >> 21) & 0x3FF) == first - g * stride
            else:
                assert (e >> 31) == 1 and ((e >> 21) & 0x3FF) == 0
            bits = oracle.words_to_bits(words, start + off, int(bit_off[b + 1]))
            gap, p = oracle.erc_decode(bits)
            prev = nzall[nzall < first]
            assert gap == first - (int(prev[-1]) if prev.size else -1)
            assert bits[p] == ("1" if seg[first] & 0x80 else "0")
            assert oracle.erc_decode(bits, p + 1)[0] == (seg[first] & 0x7F)


def test_decode_rejects_malformed_streams():
    q = signed_levels_to_q([0, 0, 1, 0, 0, 0, -3, 0])
    bit_off, words, _ = oracle.encode(q, 8, 3)
    bad = bit_off.copy(); bad[1] -= 2                      # record cut short
    with pytest.raises(ValueError):
        oracle.decode_levels(bad, words, 8, 8, 3)
    with pytest.raises(ValueError):                        # index runs past the bucket
        oracle.decode_levels(bit_off, words, 6, 6, 3)
    with pytest.raises(ValueError):                        # level index 3 > s+1 for s = 1
        oracle.decode_levels(bit_off, words, 8, 8, 1)


# ------------------------------------------------------- code length, Thm 2

@pytest.mark.parametrize("kind", ["gauss", "constant"])
def test_code_length_bound_theorem2(kind):
    """bucket 8192, s = 3: 2^(2s) + 2^s sqrt(d) <= d/e holds, so the mean of
    32 + payload bits stays below N_Q (o(1) terms taken as 0, logs base 2)."""
    d, s = 8192, 3
    n = 2 ** (2 * s) + 2 ** s * math.sqrt(d)
    assert n <= d / math.e
    NQ = 32 - 1 + 3 * n + n * math.log2(d / n) + n * math.log2(math.log2(8 * (2 ** (2 * s) + d) / n))
    rng = np.random.default_rng(5)
    v = rng.standard_normal(d).astype(np.float32) if kind == "gauss" else np.full(d, 0.3, np.float32)
    nrm = oracle.bucket_norms(v, d).astype(np.float32)
    lens = []
    for seed in range(100):
        q = oracle.quantize(v, d, s, seed, nrm)
        bit_off, _, _ = oracle.encode(q, d, s)
        lens.append(32 + int(bit_off[1]))
    assert np.mean(lens) <= NQ
    assert np.mean(lens) >= 0.3 * NQ        # the bound is not vacuous for these inputs


# --------------------------------------------------- DECODE + aggregate, Alg. 1

def test_decode_average_equals_dense_mean():
    rng = np.random.default_rng(9)
    d, bucket, s, K = 5000, 512, 3, 5
    norms, offs, words, dense = [], [], [], np.zeros(d)
    for k in range(K):
        v = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 0)).astype(np.float32)
        nrm = oracle.bucket_norms(v, bucket).astype(np.float32)
        q = oracle.quantize(v, bucket, s, k, nrm)
        bo, w, _ = oracle.encode(q, bucket, s)
        norms.append(nrm); offs.append(bo); words.append(w)
        # Def. 1 written out per coordinate, without the codec
        j = (q & 0x7F).astype(int)
        h = np.where(j > 0, 2.0 ** (j - 1 - s), 0.0)
        dense += np.repeat(nrm.astype(np.float64), bucket)[:d] * np.where(q & 0x80, -1.0, 1.0) * h
    out = oracle.decode_average(norms, offs, words, d, bucket, s, 1.0 / K)
    np.testing.assert_allclose(out, dense / K, rtol=1e-15, atol=0)
    prior = rng.standard_normal(d)
    out2 = oracle.decode_average(norms, offs, words, d, bucket, s, 0.25, prior=prior)
    np.testing.assert_allclose(out2, prior + 0.25 * dense, rtol=1e-14, atol=1e-300)


def test_average_of_many_workers_approaches_mean_gradient():
    """Alg. 1 with unbiased Q: the aggregate of K quantized copies of one vector tends
    to that vector, the error shrinking like 1/sqrt(K) (Sec. 2)."""
    rng = np.random.default_rng(2)
    d, bucket, s = 2048, 512, 3
    v = rng.standard_normal(d).astype(np.float32)
    nrm = oracle.bucket_norms(v, bucket).astype(np.float32)
    errs = []
    for K in (4, 64):
        parts = [oracle.encode(oracle.quantize(v, bucket, s, 1000 + k, nrm), bucket, s) for k in range(K)]
        out = oracle.decode_average([nrm] * K, [p[0] for p in parts], [p[1] for p in parts], d, bucket, s, 1.0 / K)
        errs.append(np.linalg.norm(out - v))
    assert errs[1] < errs[0] / 2.5
