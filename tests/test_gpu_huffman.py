"""GPU parity of the Huffman-coded levels through the C ABI against the CPU oracle: histogram exact, code lengths
equal (host arithmetic on both sides), messages (offsets, words, sync entries) bit-exact, decoded bytes equal, the
average of decoded bytes within 1e-6."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from test_gpu_parity import make_vector

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import gpu_util
    return gpu_util


CASES = [
    # (d, bucket, s, sync stride, K, kind)
    (100_000, 8192, 3, 256, 3, "mixed"),
    (100_003, 8192, 4, 1024, 2, "gauss"),
    (70_001, 16384, 7, 512, 2, "mixed"),
    (70_001, 16384, 7, 0, 1, "mixed"),
    (40_000, 512, 3, 128, 4, "mixed"),
    (40_000, 512, 3, 64, 2, "edges"),
    (33_333, 1000, 2, 256, 3, "mixed"),
    (9_999, 1001, 5, 128, 2, "mixed"),
    (3_000, 7, 1, 0, 3, "mixed"),
    (10_000, 2048, 14, 512, 2, "mixed"),
    (120_000, 32768, 3, 1024, 2, "mixed"),
    (66_000, 1536, 9, 64, 2, "edges"),         # six float4 rows per thread: sync boundaries inside a thread's chunk
    (1, 8192, 3, 512, 1, "gauss"),
    (20_000, 64, 3, 0, 8, "mixed"),            # many small buckets per workgroup: the average without value tables
    (30_000, 2000, 5, 256, 3, "mixed"),        # buckets that do not tile a workgroup's 4096 coordinates
]


@pytest.mark.parametrize("d,n,s,S,K,kind", CASES)
def test_histogram_code_message_decode_and_average(g, d, n, s, S, K, kind):
    nuq = g.nuq
    rng = np.random.default_rng(d + n + s + S)
    B = nuq.nuq_num_buckets(d, n)
    nsync = nuq.nuq_huffman_num_sync(n, S)
    cap = nuq.nuq_huffman_max_words(d, n)
    ws = torch.empty(nuq.nuq_encode_huffman_workspace_bytes(d, n), dtype=torch.uint8, device=g.DEV)
    lengths = None
    norms_list, q_list, q_np_list, msg_list, v_list = [], [], [], [], []
    for k in range(K):
        v_np = make_vector(kind, d, n, rng)
        v = torch.from_numpy(v_np).to(g.DEV)
        norms = torch.empty(B, dtype=torch.float32, device=g.DEV)
        nuq.nuq_bucket_norms(v, n, norms)
        q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
        nuq.nuq_quantize(v, n, s, 31 + k, norms, q)
        q_np = q.cpu().numpy()
        if lengths is None:                       # the code is built once, from the first worker's levels
            hist = torch.full((16,), -1, dtype=torch.int64, device=g.DEV)
            nuq.nuq_level_histogram(q, hist)
            hist_np = hist.cpu().numpy()
            np.testing.assert_array_equal(hist_np[: s + 2], oracle.level_histogram_of(q_np, s).astype(np.int64))
            assert not hist_np[s + 2:].any()
            lengths = nuq.nuq_huffman_lengths([int(x) for x in hist_np[: s + 2]], s)
            assert lengths == [int(x) for x in oracle.huffman_lengths(hist_np[: s + 2].astype(np.uint64), s)]
        bit_off = torch.full((B + 1,), -1, dtype=torch.int64, device=g.DEV)
        words = torch.zeros(cap, dtype=torch.int32, device=g.DEV)
        sync = torch.full((max(1, B * nsync),), 0x55555555, dtype=torch.int32, device=g.DEV)
        nuq.nuq_encode_huffman(q, n, s, S, lengths, bit_off, words, sync if nsync else None, ws)
        assert nuq.nuq_last_error_flags() == 0
        bo, w_ref, sync_ref = oracle.encode_huffman(q_np, n, s, lengths, S)
        np.testing.assert_array_equal(g.u64(bit_off), bo)
        np.testing.assert_array_equal(g.u32(words)[: w_ref.size], w_ref)
        assert not g.u32(words)[w_ref.size:].any()
        if sync_ref.size:
            np.testing.assert_array_equal(g.u32(sync)[: sync_ref.size], sync_ref)
        back = torch.full((d,), 0x7F, dtype=torch.uint8, device=g.DEV)
        nuq.nuq_decode_huffman(bit_off, words, sync if nsync else None, d, n, s, S, lengths, back)
        assert nuq.nuq_last_error_flags() == 0
        assert torch.equal(back, q)
        v_list.append(v)
        norms_list.append(norms)
        msg_list.append(nuq.Message(norms, bit_off, words, sync if nsync else None))
        q_list.append(back)
        q_np_list.append(q_np)
    # norms, quantizer and coding of all K workers in one launch (v read once) give the same norms and messages
    fused = [nuq.Message(torch.full((B,), -1.0, dtype=torch.float32, device=g.DEV),
                         torch.full((B + 1,), -1, dtype=torch.int64, device=g.DEV),
                         torch.zeros(cap, dtype=torch.int32, device=g.DEV),
                         torch.full((max(1, B * nsync),), 0x33333333, dtype=torch.int32, device=g.DEV)) for _ in range(K)]
    fws = torch.empty(nuq.nuq_encode_huffman_batch_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize_encode_huffman_batch(v_list, n, s, [31 + k for k in range(K)], S, lengths, fused, fws)
    assert nuq.nuq_last_error_flags() == 0
    for f, m in zip(fused, msg_list):
        assert torch.equal(f.norms, m.norms)
        assert torch.equal(f.bit_off, m.bit_off)
        nw = (int(m.bit_off[-1].item()) + 31) // 32
        assert torch.equal(f.words[:nw], m.words[:nw]) and not f.words[nw:].any()
        if nsync:
            assert torch.equal(f.sync[: B * nsync], m.sync[: B * nsync])
    # all K messages decoded in one launch give the same bytes
    again = [torch.full((d,), 0x7E, dtype=torch.uint8, device=g.DEV) for _ in range(K)]
    nuq.nuq_decode_huffman_batch(msg_list, d, n, s, S, lengths, again)
    assert nuq.nuq_last_error_flags() == 0
    for a_, b_ in zip(again, q_list):
        assert torch.equal(a_, b_)
    out = torch.full((d,), 2.0, dtype=torch.float32, device=g.DEV)
    nuq.nuq_average_levels(norms_list, q_list, d, n, s, 1.0 / K, False, out)
    scale32 = float(np.float32(1.0 / K))
    want = np.zeros(d)
    mag = np.zeros(d)
    for norms, q_np in zip(norms_list, q_np_list):
        deq = oracle.dequantize(q_np, n, s, norms.cpu().numpy())
        want += deq
        mag += np.abs(deq)
    diff = np.abs(out.cpu().numpy().astype(np.float64) - want * scale32)
    assert np.all(diff <= 1e-6 * mag * scale32 + 1e-45)
    # decode + average of the K messages in one launch (no bytes in between): the same average, written or added
    if fused_decode_fits(n, S, K):
        prior = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)
        for accumulate in (False, True):
            out2 = prior.clone()
            nuq.nuq_decode_accumulate_huffman(msg_list, d, n, s, S, lengths, 1.0 / K, accumulate, out2)
            assert nuq.nuq_last_error_flags() == 0
            ref = want * scale32
            got = out2.cpu().numpy().astype(np.float64)
            if accumulate:
                # the sum is rounded to fp32 first, then added to the old value in fp32
                ref32 = ref.astype(np.float32)
                p64 = prior.cpu().numpy().astype(np.float64)
                assert np.all(np.abs(got - (ref32.astype(np.float64) + p64))
                              <= 1e-6 * mag * scale32 + 6e-8 * (np.abs(ref) + np.abs(p64)) + 1e-45)
            else:
                assert np.all(np.abs(got - ref) <= 1e-6 * mag * scale32 + 1e-45)
    else:
        with pytest.raises(nuq.NuqError):
            nuq.nuq_decode_accumulate_huffman(msg_list, d, n, s, S, lengths, 1.0 / K, False, out)


def fused_decode_fits(n, S, K):
    """The geometry nuq_decode_accumulate_huffman takes (include/nuq.h): an index, and a lane per piece within the
    power-of-two group of lanes that a message has in a tile."""
    if S == 0 or n <= S:
        return False
    if n <= 2048:
        streams = min(2048 // n, 64 // K) * K
        pieces = -(-n // S)
    else:
        streams, pieces = K, 2048 // S
    lanes = 1
    while 2 * lanes * streams <= 64:
        lanes *= 2
    return pieces <= lanes


def _random_huffman_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        n = int(rng.integers(1, 300)) * 16 if rng.random() < 0.7 else int(rng.integers(1, 5000))
        d = int(rng.integers(1, 9 * n + 2)) if rng.random() < 0.5 else int(rng.integers(1, 120_000))
        s = int(rng.integers(1, 15))
        S = int(rng.choice([0, 64, 128, 256, 512, 1024]))
        K = int(rng.choice([1, 2, 3, 5, 8]))
        cases.append((d, n, s, S, K, str(rng.choice(["gauss", "mixed", "edges"]))))
    return cases


@pytest.mark.parametrize("d,n,s,S,K,kind", _random_huffman_cases(24, 78))
def test_random_shapes(g, d, n, s, S, K, kind):
    """Seeded draws over bucket size (mostly multiples of 16: the direct decoder and the wide average), vector
    length, levels, sync stride and workers."""
    test_histogram_code_message_decode_and_average(g, d, n, s, S, K, kind)


@pytest.mark.parametrize("s,n,S,hist", [
    (3, 8192, 256, [1, 10, 100, 1000, 10000]),                 # level 0 has the longest codeword: no four-at-a-time
    (3, 512, 128, [5, 4, 3, 2, 1]),                            # codeword of level 0 two bits long
    (14, 2048, 256, [2 ** j for j in range(16)]),              # codewords up to 15 bits, frequent levels short
    (14, 4096, 64, [2 ** (15 - j) for j in range(16)]),        # codewords up to 15 bits on levels that do occur
    (7, 1536, 512, [1] * 9),                                   # all codewords 3 or 4 bits
])
def test_codes_that_do_not_fit_the_data(g, s, n, S, hist):
    """Level bytes drawn uniformly over all levels and signs, coded with lengths built from an unrelated histogram:
    long codewords for frequent levels, codeword plus sign beyond eight bits, no short level-0 codeword."""
    nuq = g.nuq
    d = 5 * n + n // 2 + 16
    rng = np.random.default_rng(s * 1000 + n)
    level = rng.integers(0, s + 2, size=d).astype(np.uint8)
    level[rng.random(d) < 0.3] = 0
    q_np = (level | ((rng.random(d) < 0.5) & (level > 0)).astype(np.uint8) << 7).astype(np.uint8)
    lengths = nuq.nuq_huffman_lengths(hist, s)
    assert lengths == [int(x) for x in oracle.huffman_lengths(np.array(hist, dtype=np.uint64), s)]
    B, nsync = nuq.nuq_num_buckets(d, n), nuq.nuq_huffman_num_sync(n, S)
    q = torch.from_numpy(q_np).to(g.DEV)
    bit_off = torch.full((B + 1,), -1, dtype=torch.int64, device=g.DEV)
    words = torch.zeros(nuq.nuq_huffman_max_words(d, n), dtype=torch.int32, device=g.DEV)
    sync = torch.full((max(1, B * nsync),), 0x55555555, dtype=torch.int32, device=g.DEV)
    ws = torch.empty(nuq.nuq_encode_huffman_workspace_bytes(d, n), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_encode_huffman(q, n, s, S, lengths, bit_off, words, sync, ws)
    assert nuq.nuq_last_error_flags() == 0
    bo, w_ref, sync_ref = oracle.encode_huffman(q_np, n, s, lengths, S)
    np.testing.assert_array_equal(g.u64(bit_off), bo)
    np.testing.assert_array_equal(g.u32(words)[: w_ref.size], w_ref)
    np.testing.assert_array_equal(g.u32(sync)[: sync_ref.size], sync_ref)
    back = torch.full((d,), 0x7F, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_decode_huffman(bit_off, words, sync, d, n, s, S, lengths, back)
    assert nuq.nuq_last_error_flags() == 0
    np.testing.assert_array_equal(back.cpu().numpy(), q_np)
    np.testing.assert_array_equal(oracle.decode_huffman(bo, w_ref, d, n, s, lengths), q_np)
    # the same message through the fused decoder, with norms that differ per bucket
    norms_np = (10.0 ** rng.uniform(-2, 2, size=B)).astype(np.float32)
    msg = nuq.Message(torch.from_numpy(norms_np).to(g.DEV), bit_off, words, sync)
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate_huffman([msg], d, n, s, S, lengths, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == 0
    want = oracle.dequantize(oracle.decode_huffman(bo, w_ref, d, n, s, lengths), n, s, norms_np)
    np.testing.assert_allclose(out.cpu().numpy().astype(np.float64), want, rtol=1e-6, atol=1e-45)


def test_malformed_messages_raise_the_flag(g):
    nuq = g.nuq
    d, n, s, S = 4096, 1024, 3, 256
    rng = np.random.default_rng(0)
    q_np = np.where(rng.random(d) < 0.2, rng.integers(1, s + 2, d), 0).astype(np.uint8)
    lengths = [int(x) for x in oracle.huffman_lengths(oracle.level_histogram_of(q_np, s), s)]
    bo, words, sync = oracle.encode_huffman(q_np, n, s, lengths, S)
    dev = lambda a, dt: torch.from_numpy(a.view(dt)).to(g.DEV)
    q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_decode_huffman(dev(bo, np.int64), dev(words, np.int32), dev(sync, np.int32), d, n, s, S, lengths, q)
    assert nuq.nuq_last_error_flags() == 0 and np.array_equal(q.cpu().numpy(), q_np)
    bad_sync = sync.copy()
    bad_sync[1] += 1                                  # a segment that starts one bit late
    nuq.nuq_decode_huffman(dev(bo, np.int64), dev(words, np.int32), dev(bad_sync, np.int32), d, n, s, S, lengths, q)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_MALFORMED
    bad_bo = bo.copy()
    bad_bo[-1] -= 1                                   # the last bucket one bit short
    nuq.nuq_decode_huffman(dev(bad_bo, np.int64), dev(words, np.int32), dev(sync, np.int32), d, n, s, S, lengths, q)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_MALFORMED
    # the fused decoder sees the same damage
    norms = torch.ones(d // n, dtype=torch.float32, device=g.DEV)
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    mk = lambda b_, s_: nuq.Message(norms, dev(b_, np.int64), dev(words, np.int32), dev(s_, np.int32))
    nuq.nuq_decode_accumulate_huffman([mk(bo, sync)], d, n, s, S, lengths, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == 0
    np.testing.assert_allclose(out.cpu().numpy(), oracle.dequantize(q_np, n, s, np.ones(d // n, np.float32)), rtol=1e-6)
    nuq.nuq_decode_accumulate_huffman([mk(bo, bad_sync)], d, n, s, S, lengths, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_MALFORMED
    nuq.nuq_decode_accumulate_huffman([mk(bad_bo, sync)], d, n, s, S, lengths, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_MALFORMED
    short = nuq.Message(norms, dev(bo, np.int64), dev(words, np.int32)[: words.size // 2], dev(sync, np.int32))
    nuq.nuq_decode_accumulate_huffman([short], d, n, s, S, lengths, 1.0, False, out)      # words cut off
    assert nuq.nuq_last_error_flags() == nuq.FLAG_MALFORMED
    with pytest.raises(nuq.NuqError):                 # lengths that are no complete code are refused on the host
        nuq.nuq_decode_huffman(dev(bo, np.int64), dev(words, np.int32), dev(sync, np.int32), d, n, s, S,
                               [1, 1, 2, 3, 3], q)


def test_config3_worker_at_full_size(g):
    """One worker of config 3 at full size: code from its own histogram, message against the oracle on sampled
    buckets, decode gives the bytes back."""
    nuq = g.nuq
    w = workloads.workload(3)
    d, n, s, S = w.d, w.bucket, w.s, 256
    B, nsync = nuq.nuq_num_buckets(d, n), nuq.nuq_huffman_num_sync(n, S)
    v = workloads.generate(w, 0, g.DEV)
    norms = torch.empty(B, dtype=torch.float32, device=g.DEV)
    nuq.nuq_bucket_norms(v, n, norms)
    q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize(v, n, s, 0, norms, q)
    hist = torch.empty(16, dtype=torch.int64, device=g.DEV)
    nuq.nuq_level_histogram(q, hist)
    lengths = nuq.nuq_huffman_lengths([int(x) for x in hist.cpu().numpy()[: s + 2]], s)
    bit_off = torch.empty(B + 1, dtype=torch.int64, device=g.DEV)
    words = torch.zeros(nuq.nuq_huffman_max_words(d, n) // 4, dtype=torch.int32, device=g.DEV)   # ~1.1 bits/coord fit
    sync = torch.empty(B * nsync, dtype=torch.int32, device=g.DEV)
    ws = torch.empty(nuq.nuq_encode_huffman_workspace_bytes(d, n), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_encode_huffman(q, n, s, S, lengths, bit_off, words, sync, ws)
    assert nuq.nuq_last_error_flags() == 0
    bo = g.u64(bit_off)
    rng = np.random.default_rng(2)
    for b in [0, B - 1] + [int(x) for x in rng.integers(0, B, size=20)]:
        sl = slice(b * n, min(d, (b + 1) * n))
        rbo, rw, rs = oracle.encode_huffman(q[sl].cpu().numpy(), n, s, lengths, S)
        start = (int(bo[b]) + 31) // 32 * 32
        assert int(bo[b + 1]) - start == int(rbo[1])
        np.testing.assert_array_equal(g.u32(words[start // 32: start // 32 + rw.size]), rw)
        np.testing.assert_array_equal(g.u32(sync[b * nsync:(b + 1) * nsync]), rs)
    back = torch.empty_like(q)
    nuq.nuq_decode_huffman(bit_off, words, sync, d, n, s, S, lengths, back)
    assert nuq.nuq_last_error_flags() == 0
    assert torch.equal(back, q)
    assert 1.0 < float(bo[-1]) / d < 1.5              # one bit per zero, a few more for the 7 % that are not


def test_config3_fused_decode_at_full_size(g):
    """Config 3 at full size, all 8 workers coded in one launch and decoded + averaged in one launch, the way
    bench.py --huffman runs them: on sampled runs of buckets every worker's message piece is the oracle's and the
    average is the oracle's average of what those pieces decode to."""
    nuq = g.nuq
    w = workloads.workload(3)
    d, n, s, S, K = w.d, w.bucket, w.s, 256, w.K
    B, nsync = nuq.nuq_num_buckets(d, n), nuq.nuq_huffman_num_sync(n, S)
    vs = [workloads.generate(w, k, g.DEV) for k in range(K)]
    seeds = [w.quant_seed(k) for k in range(K)]
    # the code: from worker 0's levels
    norms0 = torch.empty(B, dtype=torch.float32, device=g.DEV)
    nuq.nuq_bucket_norms(vs[0], n, norms0)
    q0 = torch.empty(d, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize(vs[0], n, s, seeds[0], norms0, q0)
    hist = torch.empty(16, dtype=torch.int64, device=g.DEV)
    nuq.nuq_level_histogram(q0, hist)
    lengths = nuq.nuq_huffman_lengths([int(x) for x in hist.cpu().numpy()[: s + 2]], s)
    del q0
    cap = nuq.nuq_huffman_max_words(d, n) // 4
    msgs = [nuq.Message(torch.empty(B, dtype=torch.float32, device=g.DEV),
                        torch.empty(B + 1, dtype=torch.int64, device=g.DEV),
                        torch.full((cap,), 0x5A5A5A5A, dtype=torch.int32, device=g.DEV),
                        torch.empty(B * nsync, dtype=torch.int32, device=g.DEV)) for _ in range(K)]
    ws = torch.empty(nuq.nuq_encode_huffman_batch_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize_encode_huffman_batch(vs, n, s, seeds, S, lengths, msgs, ws)
    assert nuq.nuq_last_error_flags() == 0
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate_huffman(msgs, d, n, s, S, lengths, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() == 0
    rng = np.random.default_rng(4)
    run = 3
    scale32 = float(np.float32(1.0 / K))
    for b_lo in sorted({0, B - run} | {int(x) for x in rng.integers(0, B - run, size=16)}):
        c_lo, c_hi = b_lo * n, min(d, (b_lo + run) * n)
        want, mag = np.zeros(c_hi - c_lo), np.zeros(c_hi - c_lo)
        for v, m, seed in zip(vs, msgs, seeds):
            norms = m.norms[b_lo:b_lo + run].cpu().numpy()
            g.check_norms(v[c_lo:c_hi].cpu().numpy(), n, norms)
            q = oracle.quantize(v[c_lo:c_hi].cpu().numpy(), n, s, seed, norms, b_lo)
            bo, words, sync = oracle.encode_huffman(q, n, s, lengths, S)
            got_bo = g.u64(m.bit_off[b_lo:b_lo + run + 1])
            start = (int(got_bo[0]) + 31) // 32 * 32
            np.testing.assert_array_equal(got_bo[1:] - np.uint64(start), bo[1:])
            np.testing.assert_array_equal(g.u32(m.words[start // 32: start // 32 + words.size]), words)
            np.testing.assert_array_equal(g.u32(m.sync[b_lo * nsync:(b_lo + run) * nsync]), sync)
            deq = oracle.dequantize(oracle.decode_huffman(bo, words, c_hi - c_lo, n, s, lengths), n, s, norms)
            want += deq
            mag += np.abs(deq)
        diff = np.abs(out[c_lo:c_hi].cpu().numpy().astype(np.float64) - want * scale32)
        assert np.all(diff <= 1e-6 * mag * scale32 + 1e-45)
