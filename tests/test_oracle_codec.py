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


def erc_read(bits, pos):
    """Alg. 2's decoder on a '0'/'1' string, written out here so that the index is checked by a reader of its own:
    N = 1; while the next bit is 1, the next N + 1 bits are the new N; the 0 that follows ends the code."""
    n = 1
    while bits[pos] == "1":
        n, pos = int(bits[pos:pos + n + 1], 2), pos + n + 1
    return n, pos + 1


def test_sync_entries_worked_by_hand():
    """The decoder index of tests/golden/sync_examples.txt: offsets from Alg. 2's code lengths, pieces by hand."""
    for row in read_rows("sync_examples.txt"):
        bucket, s, stride, recs, bits, entries = [f.strip() for f in row.split("|")]
        bucket, s, stride = int(bucket), int(s), int(stride)
        q = np.zeros(bucket, np.uint8)
        if recs != "-":
            for r in recs.split():
                idx, lev = r.split(":")
                q[int(idx)] = abs(int(lev)) | (0x80 if int(lev) < 0 else 0)
        bit_off, words, sync = oracle.encode(q, bucket, s, stride)
        assert int(bit_off[1]) == int(bits)
        assert sync.tolist() == [int(e) for e in entries.split()], row
        assert oracle.num_sync(bucket, stride) == len(entries.split())


def test_num_sync_and_pieces():
    # blocks of 2048 coordinates, a power-of-two number of pieces of about `stride` coordinates each
    assert oracle.num_sync(8192, 256) == 4 * 8 and oracle.num_sync(8192, 512) == 4 * 4
    assert oracle.num_sync(16384, 256) == 8 * 8 and oracle.num_sync(32768, 64) == 16 * 32
    assert oracle.num_sync(512, 128) == 4 and oracle.num_sync(512, 512) == 1 and oracle.num_sync(100, 512) == 1
    assert oracle.num_sync(1000, 256) == 4 and oracle.num_sync(1300, 256) == 8      # 6 wanted -> 8
    assert oracle.num_sync(5000, 1024) == 3 * 2 and oracle.num_sync(8192, 0) == 0


@pytest.mark.parametrize("bucket,s,stride", [(8192, 3, 512), (8192, 3, 256), (16384, 7, 1024), (512, 3, 512),
                                             (512, 3, 128), (1000, 2, 256), (5000, 4, 64), (8192, 4, 0)])
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
    if not ns:
        return
    # What the index promises a decoder, checked without the rule that places the entries: the entries of a bucket
    # cut its bit string into pieces; decoding piece (t, g) from its entry's offset, with the first index taken from
    # the entry instead of the first gap code, up to the next entry's offset yields records that all lie in block t;
    # the pieces of a block together yield exactly the block's records, in order; and their record counts differ by
    # at most one (that is what the index is for: equal work per piece).
    P = oracle.sync_pieces(bucket, stride)
    assert ns % P == 0 and ns // P == (bucket + 2047) // 2048
    for b in range(oracle.num_buckets(d, bucket)):
        seg = q[b * bucket:(b + 1) * bucket]
        start = (int(bit_off[b]) + 31) // 32 * 32
        length = int(bit_off[b + 1]) - start
        ent = [int(e) for e in sync[b * ns:(b + 1) * ns]]
        offs = [e & 0x1FFFFF for e in ent] + [length]
        assert offs == sorted(offs)
        for t in range(ns // P):
            want = [i for i in np.flatnonzero(seg & 0x7F) if 2048 * t <= i < 2048 * (t + 1)]
            got, counts = [], []
            for g in range(P):
                e = t * P + g
                bits = oracle.words_to_bits(words, start + offs[e], start + offs[e + 1])
                pos, idx, cnt = 0, None, 0
                while pos < len(bits):
                    gap, pos = erc_read(bits, pos)
                    idx = 2048 * t + (ent[e] >> 21) if idx is None else idx + gap
                    neg = bits[pos] == "1"
                    lev, pos = erc_read(bits, pos + 1)
                    assert seg[idx] == (lev | (0x80 if neg else 0))
                    got.append(idx)
                    cnt += 1
                counts.append(cnt)
            assert got == want
            assert max(counts) - min(counts) <= 1


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
