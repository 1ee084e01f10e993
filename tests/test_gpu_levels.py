"""GPU parity of the level-table variant (arbitrary level sequences, maximum norm) through the C ABI against the
CPU oracle on the same seeded inputs.  Bars as for the main path: maximum norms exact; level|sign bytes bit-exact
when the oracle is fed the GPU's norms (both sides decide u / 2^24 < p(r) over the real numbers: the oracle always by
an exact sum, the kernels by rounded fp64 operations that hand near-ties to an exact sum of their own); the message of
those bytes bit-exact; decoded averages within 1e-6."""
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


TABLES = {
    "nuq3": ("exp", 3, 0.5),          # the main scheme's own levels: must reproduce nuq_quantize
    "uniform3": ("uniform", 3, 0.0),  # QSGD
    "uniform7": ("uniform", 7, 0.0),
    "exp4_03": ("exp", 4, 0.3),
    "exp6_07": ("exp", 6, 0.7),
    "exp14": ("exp", 14, 0.5),
    "uniform14": ("uniform", 14, 0.0),
}

CASES = [
    # (d, bucket, table, norm, kind)
    (100_000, 8192, "uniform3", "l2", "mixed"),
    (100_003, 8192, "uniform3", "linf", "gauss"),
    (70_001, 16384, "uniform7", "linf", "mixed"),
    (40_000, 512, "exp4_03", "l2", "mixed"),
    (40_000, 512, "uniform3", "linf", "edges"),
    (33_333, 1000, "exp6_07", "l2", "mixed"),
    (9_999, 1001, "exp4_03", "linf", "mixed"),      # bucket not a multiple of 4
    (3_000, 7, "uniform3", "linf", "mixed"),
    (120_000, 32768, "exp14", "l2", "mixed"),
    (66_000, 20000, "uniform14", "l2", "edges"),
    (50_000, 2048, "nuq3", "l2", "mixed"),
    (1, 8192, "uniform3", "linf", "gauss"),
]


def table(name):
    kind, s, p = TABLES[name]
    return workloads.level_table(kind, s, p), s


@pytest.mark.parametrize("d,n,tname,norm,kind", CASES)
def test_norms_quantizer_message_and_average_match_oracle(g, d, n, tname, norm, kind):
    nuq = g.nuq
    lev, s = table(tname)
    S = 256 if n > 256 else 0
    rng = np.random.default_rng(d + n + s)
    K = 3
    msgs, msgs_np, vs = [], [], []
    for k in range(K):
        v_np = make_vector(kind, d, n, rng)
        v = torch.from_numpy(v_np).to(g.DEV)
        B = nuq.nuq_num_buckets(d, n)
        norms = torch.full((B,), -1.0, dtype=torch.float32, device=g.DEV)
        if norm == "linf":
            nuq.nuq_bucket_norms_linf(v, n, norms)
            np.testing.assert_array_equal(norms.cpu().numpy().astype(np.float64), oracle.bucket_norms_linf(v_np, n))
        else:
            nuq.nuq_bucket_norms(v, n, norms)
            g.check_norms(v_np, n, norms.cpu().numpy())
        norms_np = norms.cpu().numpy()
        q = torch.full((d,), 0x7F, dtype=torch.uint8, device=g.DEV)
        nuq.nuq_quantize_table(v, n, lev, 77 + k, norms, q)
        q_ref = oracle.quantize_table(v_np, n, lev, 77 + k, norms_np)
        np.testing.assert_array_equal(q.cpu().numpy(), q_ref)
        if tname == "nuq3":          # on its own levels the table rule is the main quantizer
            q_main = torch.empty_like(q)
            nuq.nuq_quantize(v, n, s, 77 + k, norms, q_main)
            assert torch.equal(q, q_main)
        m = g.alloc_message(d, n, s, S)
        m.norms.copy_(norms)
        nuq.nuq_encode(q, n, s, S, m.bit_off, m.words, m.sync if nuq.nuq_num_sync(n, S) else None, g.workspace(d, n, s))
        bo, words, sync = oracle.encode(q_ref, n, s, S)
        np.testing.assert_array_equal(g.u64(m.bit_off), bo)
        np.testing.assert_array_equal(g.u32(m.words)[: words.size], words)
        if sync.size:
            np.testing.assert_array_equal(g.u32(m.sync)[: sync.size], sync)
        msgs.append(m)
        msgs_np.append((norms_np, bo, words))
        vs.append(v)
    # the fused call (v read once, all workers in one launch) gives the same norms and messages, bit for bit
    fused = [g.alloc_message(d, n, s, S) for _ in range(K)]
    ws = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize_encode_table_batch(vs, n, lev, nuq.NORM_LINF if norm == "linf" else nuq.NORM_L2,
                                        [77 + k for k in range(K)], S, fused, ws)
    for f, (norms_np, bo, words) in zip(fused, msgs_np):
        np.testing.assert_array_equal(f.norms.cpu().numpy(), norms_np)
        np.testing.assert_array_equal(g.u64(f.bit_off), bo)
        np.testing.assert_array_equal(g.u32(f.words)[: words.size], words)
        assert not g.u32(f.words)[words.size:].any()
    assert nuq.nuq_last_error_flags() == 0
    out = torch.full((d,), 5.0, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate_table(msgs, d, n, lev, S, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() == 0
    check_average_table(msgs_np, d, n, lev, 1.0 / K, out.cpu().numpy())
    prior = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)
    out2 = prior.clone()
    nuq.nuq_decode_accumulate_table(msgs, d, n, lev, S, 0.25, True, out2)
    check_average_table(msgs_np, d, n, lev, 0.25, out2.cpu().numpy(), prior=prior.cpu().numpy().astype(np.float64))
    assert nuq.nuq_last_error_flags() == 0


def check_average_table(msgs_np, d, n, lev, scale, out_gpu, prior=None):
    """The bars of gpu_util.check_average with the table's level values."""
    s = len(lev) - 2
    scale32 = float(np.float32(scale))
    want = oracle.decode_average_table([m[0] for m in msgs_np], [m[1] for m in msgs_np], [m[2] for m in msgs_np],
                                       d, n, lev, scale32, prior=prior)
    mag = np.zeros(d)
    for norms, bo, words in msgs_np:
        q = oracle.decode_levels(bo, words, d, n, s)
        mag += np.abs(oracle.dequantize_table(q, n, lev, norms))
    mag = mag * abs(scale32) + (np.abs(prior) if prior is not None else 0.0)
    got = out_gpu.astype(np.float64)
    diff = np.abs(got - want)
    assert np.all(diff <= 1e-6 * mag + 1e-45), float(np.max(diff / np.maximum(mag, 1e-300)))
    for b in range((d + n - 1) // n):
        sl = slice(b * n, min(d, (b + 1) * n))
        assert np.linalg.norm(got[sl] - want[sl]) <= 1e-6 * np.linalg.norm(want[sl]) + 2.0 ** -149 * np.sqrt(n)


@pytest.mark.parametrize("d,n,S,K", [(100_000, 8192, 256, 1), (100_000, 8192, 256, 3), (40_000, 512, 128, 1),
                                     (70_001, 16384, 512, 4), (9_999, 1001, 0, 1), (66_000, 2048, 64, 1)])
def test_table_of_the_main_levels_decodes_like_the_main_path(g, d, n, S, K):
    """The level table 2^(j-1-s) through the table decoder (tile kernel, every K) against the main entry point
    (for K = 1 the kernel that stores values directly; 4096-coordinate tiles for large buckets of few workers):
    the same bits, written and added."""
    nuq = g.nuq
    s = 3
    rng = np.random.default_rng(d + n + K)
    vs = [torch.from_numpy(make_vector("mixed", d, n, rng)).to(g.DEV) for _ in range(K)]
    msgs = g.batched_encode(vs, n, s, list(range(K)), S)
    lev = [0.0] + [2.0 ** (j - 1 - s) for j in range(1, s + 2)]
    prior = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)
    for accumulate in (False, True):
        a, b = prior.clone(), prior.clone()
        nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, accumulate, a)
        nuq.nuq_decode_accumulate_table(msgs, d, n, lev, S, 1.0 / K, accumulate, b)
        assert torch.equal(a, b)
    assert nuq.nuq_last_error_flags() == 0


def test_uniform_levels_at_benchmark_size(g):
    """Config 3's shape (ResNet-50-sized gradient, bucket 8192) with QSGD's uniform levels and the maximum norm
    (QSGDinf), one worker at full size: bytes bit-exact on sampled buckets, the rest by count."""
    nuq = g.nuq
    w = workloads.workload(3)
    lev = workloads.level_table("uniform", 3)
    v = workloads.generate(w, 0, g.DEV)
    d, n = w.d, w.bucket
    B = nuq.nuq_num_buckets(d, n)
    norms = torch.empty(B, dtype=torch.float32, device=g.DEV)
    nuq.nuq_bucket_norms_linf(v, n, norms)
    q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize_table(v, n, lev, 5, norms, q)
    rng = np.random.default_rng(1)
    for b in [0, B - 1] + [int(x) for x in rng.integers(0, B, size=24)]:
        sl = slice(b * n, min(d, (b + 1) * n))
        v_np = v[sl].cpu().numpy()
        nb = norms[b:b + 1].cpu().numpy()
        assert float(nb[0]) == float(np.abs(v_np).max())
        want = oracle.quantize_table(v_np, n, lev, 5, nb, first_bucket=b)
        np.testing.assert_array_equal(q[sl].cpu().numpy(), want)
    assert nuq.nuq_last_error_flags() == 0


def test_near_ties_of_the_rounding_decision(g):
    """tests/golden/table_near_ties.txt: coordinates and draws at which both sides of the rounding test agree to
    within one rounding of fp64, so that a rounded evaluation decides them wrongly.  Positions at which the counter
    generator delivers each listed draw are looked up with the oracle's generator, the listed coordinate (with
    either sign) is planted there under the listed norm, and the bytes of nuq_quantize_table must equal the
    oracle's: up, as the exact rule says."""
    from test_oracle_levels import near_ties
    nuq = g.nuq
    n, B = 32768, 2048
    d = n * B
    ties = near_ties()
    assert len({tuple(t[0]) for t in ties}) == 1          # one level table for all listed examples
    lev = ties[0][0]
    s = len(lev) - 2
    planted = 0
    for seed in range(101, 109):
        u = oracle.rng_fill(seed, d, n)
        v = np.zeros(d, dtype=np.float32)
        norms = np.ones(B, dtype=np.float32)
        used = set()
        want_up = []
        for _, norm, a, draw, up in ties:
            for i in np.flatnonzero(u == draw):
                b = int(i) // n
                if b in used:
                    continue
                used.add(b)
                norms[b] = np.float32(norm)
                v[i] = np.float32(a) * (1 if (i & 1) else -1)
                want_up.append((int(i), up))
        if not want_up:
            continue
        planted += len(want_up)
        # ordinary coordinates around them
        rng = np.random.default_rng(seed)
        fill = rng.random(d) < 0.001
        fill[[i for i, _ in want_up]] = False
        v[fill] = (rng.standard_normal(int(fill.sum())) * 0.3).astype(np.float32)
        want = oracle.quantize_table(v, n, lev, seed, norms)
        for i, up in want_up:                              # the oracle puts them one level up from their bin
            j = max(t for t in range(s + 1) if np.float64(np.float32(lev[t])) * np.float64(norms[i // n]) <= abs(float(v[i])))
            assert int(want[i] & 0x7F) == j + up
        q = torch.empty(d, dtype=torch.uint8, device=g.DEV)
        nuq.nuq_quantize_table(torch.from_numpy(v).to(g.DEV), n, lev, seed, torch.from_numpy(norms).to(g.DEV), q)
        got = q.cpu().numpy()
        np.testing.assert_array_equal(got, want)
        if planted >= 4:
            break
    assert planted >= 2
