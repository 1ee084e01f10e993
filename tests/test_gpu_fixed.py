"""GPU parity of the fixed-width coding (b bits per coordinate) through the C ABI against the CPU oracle: packed
words bit-exact (from bytes, and from the fused norms + quantizer + packing when the oracle is fed the GPU's norms),
unpacked averages within 1e-6 (the GPU sums in fp64 in worker order like the oracle)."""
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
    # (d, bucket, s, b, K, kind)
    (100_000, 8192, 3, 4, 3, "mixed"),
    (100_003, 8192, 6, 4, 8, "gauss"),
    (70_001, 16384, 7, 8, 2, "mixed"),
    (40_000, 512, 2, 3, 4, "mixed"),
    (40_000, 512, 3, 4, 4, "edges"),
    (33_333, 1000, 9, 5, 3, "mixed"),
    (9_999, 1001, 5, 4, 2, "mixed"),         # bucket not a multiple of 4: scalar unpack, unaligned loads
    (3_000, 7, 1, 3, 5, "mixed"),
    (120_000, 32768, 14, 8, 2, "mixed"),
    (66_000, 20000, 3, 7, 3, "edges"),
    (10_000, 2048, 14, 5, 1, "mixed"),
    (1, 8192, 3, 4, 1, "gauss"),
    (20_000, 64, 3, 4, 8, "mixed"),          # many small buckets per workgroup: value tables too large, arithmetic route
    (30_000, 96, 2, 3, 4, "mixed"),          # the same with buckets that do not tile a workgroup's 8192 coordinates
    (50_000, 2016, 3, 5, 3, "mixed"),        # tables, workgroups starting inside a bucket
    (90_000, 4096, 14, 8, 5, "mixed"),       # 32-entry tables indexed by (sign, level)
]


@pytest.mark.parametrize("d,n,s,b,K,kind", CASES)
def test_pack_fused_pack_and_unpack_average(g, d, n, s, b, K, kind):
    nuq = g.nuq
    rng = np.random.default_rng(d + n + s + b)
    B = nuq.nuq_num_buckets(d, n)
    W = nuq.nuq_fixed_words(d, n, b)
    assert W == oracle.fixed_words(d, n, b)
    vs_np = [make_vector(kind, d, n, rng) for _ in range(K)]
    vs = [torch.from_numpy(v).to(g.DEV) for v in vs_np]
    seeds = [int(x) for x in rng.integers(0, 2 ** 63, size=K)]
    norms = [torch.full((B,), -1.0, dtype=torch.float32, device=g.DEV) for _ in range(K)]
    packed = [torch.full((W,), 0x55555555, dtype=torch.int32, device=g.DEV) for _ in range(K)]
    nuq.nuq_quantize_pack_fixed_batch(vs, n, s, b, seeds, norms, packed)
    assert nuq.nuq_last_error_flags() == 0
    norms_np, packed_np = [], []
    for k in range(K):
        nk = norms[k].cpu().numpy()
        g.check_norms(vs_np[k], n, nk)
        q_ref = oracle.quantize(vs_np[k], n, s, seeds[k], nk)
        want = oracle.pack_fixed(q_ref, n, s, b)
        np.testing.assert_array_equal(g.u32(packed[k]), want)
        norms_np.append(nk)
        packed_np.append(want)
        if k == 0:       # the unfused chain gives the same words: norms -> bytes -> packing
            n2 = torch.empty(B, dtype=torch.float32, device=g.DEV)
            nuq.nuq_bucket_norms(vs[0], n, n2)
            assert torch.equal(n2, norms[0])
            q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
            nuq.nuq_quantize(vs[0], n, s, seeds[0], n2, q)
            p2 = torch.full((W,), 0x33333333, dtype=torch.int32, device=g.DEV)
            nuq.nuq_pack_fixed(q, n, s, b, p2)
            assert torch.equal(p2, packed[0])
    out = torch.full((d,), 9.0, dtype=torch.float32, device=g.DEV)
    nuq.nuq_unpack_accumulate_fixed(norms, packed, d, n, s, b, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() == 0
    check(norms_np, packed_np, d, n, s, b, 1.0 / K, out.cpu().numpy())
    prior = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)
    out2 = prior.clone()
    nuq.nuq_unpack_accumulate_fixed(norms, packed, d, n, s, b, 0.5, True, out2)
    check(norms_np, packed_np, d, n, s, b, 0.5, out2.cpu().numpy(), prior=prior.cpu().numpy().astype(np.float64))


def check(norms_np, packed_np, d, n, s, b, scale, got, prior=None):
    scale32 = float(np.float32(scale))
    want = oracle.unpack_average_fixed(norms_np, packed_np, d, n, s, b, scale32, prior=prior)
    mag = np.zeros(d)
    for norms, packed in zip(norms_np, packed_np):
        mag += np.abs(oracle.dequantize(oracle.unpack_fixed(packed, d, n, s, b), n, s, norms))
    mag = mag * abs(scale32) + (np.abs(prior) if prior is not None else 0.0)
    diff = np.abs(got.astype(np.float64) - want)
    assert np.all(diff <= 1e-6 * mag + 1e-45), float(np.max(diff / np.maximum(mag, 1e-300)))


TABLE_CASES = [
    # (d, bucket, table kind, s, p, norm, b, K, kind)
    (100_000, 8192, "uniform", 3, 0.0, "linf", 4, 3, "mixed"),      # QSGDinf, 4 bits
    (100_003, 8192, "uniform", 6, 0.0, "l2", 4, 8, "gauss"),        # QSGD, 4 bits (seven levels)
    (70_001, 16384, "uniform", 14, 0.0, "linf", 8, 2, "mixed"),
    (40_000, 512, "exp", 3, 0.3, "l2", 4, 4, "mixed"),
    (33_333, 1000, "exp", 6, 0.7, "linf", 5, 3, "edges"),
    (9_999, 1001, "uniform", 5, 0.0, "linf", 4, 2, "mixed"),        # scalar unpack
    (20_000, 64, "uniform", 3, 0.0, "linf", 4, 8, "mixed"),         # arithmetic route of the wide unpack
    (90_000, 4096, "exp", 14, 0.5, "l2", 8, 5, "mixed"),            # the main scheme's levels as a table
]


@pytest.mark.parametrize("d,n,tkind,s,p,norm,b,K,kind", TABLE_CASES)
def test_level_tables_and_maximum_norm(g, d, n, tkind, s, p, norm, b, K, kind):
    """The fused pack and the unpack + average for a level table and either norm (QSGD and QSGDinf at fixed width):
    norms to the bar (maximum norms exact), packed words bit-exact against pack_fixed(quantize_table) of the oracle
    fed the GPU's norms, averages of norm * sign * levels[j] within the bar."""
    nuq = g.nuq
    rng = np.random.default_rng(d + n + s + b + 1)
    lev = workloads.level_table(tkind, s, p if p else 0.5)
    B, W = nuq.nuq_num_buckets(d, n), nuq.nuq_fixed_words(d, n, b)
    vs_np = [make_vector(kind, d, n, rng) for _ in range(K)]
    vs = [torch.from_numpy(v).to(g.DEV) for v in vs_np]
    seeds = [int(x) for x in rng.integers(0, 2 ** 63, size=K)]
    norms = [torch.full((B,), -1.0, dtype=torch.float32, device=g.DEV) for _ in range(K)]
    packed = [torch.full((W,), 0x55555555, dtype=torch.int32, device=g.DEV) for _ in range(K)]
    nuq.nuq_quantize_pack_fixed_table_batch(vs, n, lev, nuq.NORM_LINF if norm == "linf" else nuq.NORM_L2, b, seeds,
                                            norms, packed)
    assert nuq.nuq_last_error_flags() == 0
    norms_np, packed_np = [], []
    for k in range(K):
        nk = norms[k].cpu().numpy()
        if norm == "linf":
            np.testing.assert_array_equal(nk.astype(np.float64), oracle.bucket_norms_linf(vs_np[k], n))
        else:
            g.check_norms(vs_np[k], n, nk)
        want = oracle.pack_fixed(oracle.quantize_table(vs_np[k], n, lev, seeds[k], nk), n, s, b)
        np.testing.assert_array_equal(g.u32(packed[k]), want)
        norms_np.append(nk)
        packed_np.append(want)
    for scale, prior in ((1.0 / K, None), (0.5, rng.standard_normal(d).astype(np.float32))):
        out = torch.full((d,), 9.0, dtype=torch.float32, device=g.DEV) if prior is None else torch.from_numpy(prior).to(g.DEV)
        nuq.nuq_unpack_accumulate_fixed_table(norms, packed, d, n, lev, b, scale, prior is not None, out)
        assert nuq.nuq_last_error_flags() == 0
        scale32 = float(np.float32(scale))
        want, mag = np.zeros(d), np.zeros(d)
        for nk, pk in zip(norms_np, packed_np):
            deq = oracle.dequantize_table(oracle.unpack_fixed(pk, d, n, s, b), n, lev, nk)
            want += deq
            mag += np.abs(deq)
        want, mag = want * scale32, mag * abs(scale32)
        got = out.cpu().numpy().astype(np.float64)
        if prior is not None:
            p64 = prior.astype(np.float64)
            assert np.all(np.abs(got - (want.astype(np.float32).astype(np.float64) + p64))
                          <= 1e-6 * mag + 6e-8 * (np.abs(want) + np.abs(p64)) + 1e-45)
        else:
            assert np.all(np.abs(got - want) <= 1e-6 * mag + 1e-45)


def _random_fixed_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        b = int(rng.integers(3, 9))
        s = int(rng.integers(1, min(14, 2 ** (b - 1) - 2) + 1))
        n = int(rng.integers(1, 400)) * 32 if rng.random() < 0.7 else int(rng.integers(1, 5000))
        d = int(rng.integers(1, 9 * n + 2)) if rng.random() < 0.5 else int(rng.integers(1, 120_000))
        K = int(rng.choice([1, 2, 3, 5, 8, 13]))
        cases.append((d, n, s, b, K, str(rng.choice(["gauss", "mixed", "edges"]))))
    return cases


@pytest.mark.parametrize("d,n,s,b,K,kind", _random_fixed_cases(24, 77))
def test_random_shapes(g, d, n, s, b, K, kind):
    """Seeded draws over the parameters: code width, levels, bucket size (mostly multiples of 32: the wide unpack
    kernel with and without value tables), vector length, workers."""
    test_pack_fused_pack_and_unpack_average(g, d, n, s, b, K, kind)


@pytest.mark.parametrize("b,s,nbuckets", [(4, 2, 1), (8, 2, 1), (8, 14, 1), (5, 2, 1), (3, 1, 1), (5, 2, 200), (4, 2, 300)])
def test_malformed_codes_raise_the_flag(g, b, s, nbuckets):
    # every route of the unpack kernel: value tables with the whole-word test (b = 4, 8) and the per-code test
    # (b = 3, 5), and the arithmetic route (many buckets per workgroup); the top valid level must not raise it
    nuq = g.nuq
    n = 64
    d = n * nbuckets
    wpb = n * b // 32
    norms = [torch.ones(nbuckets, dtype=torch.float32, device=g.DEV)]
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    top = 32 - b                                  # shift of a field's first code
    cases = [((s + 2) << top, True), (1 << 31, True), ((s + 1) << top, False), ((1 << 31) | ((s + 1) << top), False)]
    if s + 2 >= 1 << (b - 1):
        cases = cases[1:]                         # no level index above s + 1 fits the code
    for word, bad in cases:
        words = np.zeros(nbuckets * wpb, dtype=np.uint32)
        words[(nbuckets - 1) * wpb] = word        # first code of the last bucket
        packed = [torch.from_numpy(words.view(np.int32)).to(g.DEV)]
        nuq.nuq_unpack_accumulate_fixed(norms, packed, d, n, s, b, 1.0, False, out)
        assert nuq.nuq_last_error_flags() == (nuq.FLAG_MALFORMED if bad else 0), (hex(word), bad)
        if not bad:
            want = 1.0 * (-1.0 if word >> 31 else 1.0)          # norm * sign * 2^0
            assert out[(nbuckets - 1) * n].item() == want and out.abs().sum().item() == 1.0


def test_four_bit_at_benchmark_size(g):
    """Config 3 at full size, 4 bits: all 8 workers packed in one launch; sampled buckets against the oracle, the
    average on the same buckets."""
    nuq = g.nuq
    w = workloads.workload(3)
    d, n, s, K, b = w.d, w.bucket, w.s, w.K, 4
    B, W = nuq.nuq_num_buckets(d, n), nuq.nuq_fixed_words(d, n, b)
    wpb = W // B
    vs = [workloads.generate(w, k, g.DEV) for k in range(K)]
    seeds = [w.quant_seed(k) for k in range(K)]
    norms = [torch.empty(B, dtype=torch.float32, device=g.DEV) for _ in range(K)]
    packed = [torch.empty(W, dtype=torch.int32, device=g.DEV) for _ in range(K)]
    nuq.nuq_quantize_pack_fixed_batch(vs, n, s, b, seeds, norms, packed)
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_unpack_accumulate_fixed(norms, packed, d, n, s, b, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() == 0
    rng = np.random.default_rng(3)
    for bk in [0, B - 1] + [int(x) for x in rng.integers(0, B, size=10)]:
        sl = slice(bk * n, min(d, (bk + 1) * n))
        nn, pp = [], []
        for k in range(K):
            v_np = vs[k][sl].cpu().numpy()
            nk = norms[k][bk:bk + 1].cpu().numpy()
            want = oracle.pack_fixed(oracle.quantize(v_np, n, s, seeds[k], nk, first_bucket=bk), n, s, b)
            np.testing.assert_array_equal(g.u32(packed[k][bk * wpb:(bk + 1) * wpb]), want)
            nn.append(nk)
            pp.append(want)
        check(nn, pp, sl.stop - sl.start, n, s, b, 1.0 / K, out[sl].cpu().numpy())
