"""GPU parity: every step of the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bars (the benchmark spec the benchmark spec): level indices, signs, offsets, bit strings and sync
entries bit-exact when the oracle is fed the GPU's norms; norms within 1e-6 relative of the oracle's fp64
norms; decoded averages within 1e-6 relative."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import gpu_util
    return gpu_util


def make_vector(kind, d, n, rng):
    if kind == "gauss":
        return (rng.standard_normal(d) * 0.01).astype(np.float32)
    if kind == "mixed":          # per-chunk scales over many decades, some zero runs, some spikes
        v = rng.standard_normal(d)
        scale = 10.0 ** rng.uniform(-6, 1, size=(d + 99) // 100)
        v *= np.repeat(scale, 100)[:d]
        v[rng.random(d) < 0.05] = 0.0
        v[rng.integers(0, d, size=max(1, d // 500))] *= 300.0
        return v.astype(np.float32)
    if kind == "edges":          # zero bucket, single spike, on-level ratios, -0.0, constant bucket
        v = (rng.standard_normal(d) * 0.1).astype(np.float32)
        if d >= 4 * n:
            v[0:n] = 0.0
            v[n:2 * n] = 0.0
            v[n + n // 2] = -7.5
            v[2 * n:3 * n] = 0.25
            v[3 * n:3 * n + min(n, 16)] = -0.0
        return v
    raise ValueError(kind)


SHAPES = [
    # (d, bucket, s, sync_stride, kind)
    (8192, 8192, 3, 512, "gauss"),
    (100_000, 8192, 3, 512, "mixed"),        # several buckets + ragged tail
    (100_003, 8192, 4, 1024, "mixed"),
    (50_000, 8192, 3, 0, "edges"),
    (5000, 8192, 3, 512, "gauss"),           # d < bucket
    (70_001, 16384, 7, 1024, "mixed"),
    (70_001, 16384, 7, 0, "mixed"),          # large bucket without a sync index
    (40_000, 512, 3, 512, "mixed"),
    (40_000, 512, 3, 64, "edges"),
    (33_333, 1000, 2, 256, "mixed"),
    (9_999, 1001, 5, 128, "mixed"),          # bucket not a multiple of 4: unaligned path
    (3_000, 7, 1, 0, "mixed"),
    (1_000, 1, 3, 0, "gauss"),               # bucket of one coordinate: r = 1 always
    (10_000, 2048, 14, 512, "mixed"),
    (120_000, 32768, 3, 1024, "mixed"),
    (66_000, 20000, 9, 512, "edges"),
    (1, 8192, 3, 512, "gauss"),
]


@pytest.mark.parametrize("d,n,s,S,kind", SHAPES)
def test_each_step_and_fused_path_match_oracle(g, d, n, s, S, kind):
    nuq = g.nuq
    rng = np.random.default_rng(d * 31 + n + s)
    v_np = make_vector(kind, d, n, rng)
    v = torch.from_numpy(v_np).to(g.DEV)
    B = nuq.nuq_num_buckets(d, n)
    seed = 0x1234_5678_9ABC_DEF0 + d

    # step 1
    norms = torch.empty(B, dtype=torch.float32, device=g.DEV)
    nuq.nuq_bucket_norms(v, n, norms)
    norms_np = norms.cpu().numpy()
    g.check_norms(v_np, n, norms_np)

    # step 2: level|sign bytes, bit-exact
    q = torch.full((d,), 0x7F, dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize(v, n, s, seed, norms, q)
    q_ref = oracle.quantize(v_np, n, s, seed, norms_np)
    np.testing.assert_array_equal(q.cpu().numpy(), q_ref)

    # step 3: ENCODE of those bytes, bit-exact
    m = g.alloc_message(d, n, s, S)
    nuq.nuq_encode(q, n, s, S, m.bit_off, m.words, m.sync if nuq.nuq_num_sync(n, S) else None, g.workspace(d, n, s))
    bo, words, sync = oracle.encode(q_ref, n, s, S)
    np.testing.assert_array_equal(g.u64(m.bit_off), bo)
    np.testing.assert_array_equal(g.u32(m.words)[: words.size], words)
    assert not g.u32(m.words)[words.size:].any()
    if sync.size:
        np.testing.assert_array_equal(g.u32(m.sync)[: sync.size], sync)

    # fused steps 1-3: same norms as step 1 (bit for bit), same message
    mf = g.fused_encode(v, n, s, seed, S)
    np.testing.assert_array_equal(mf.norms.cpu().numpy(), norms_np)
    g.check_message_against_oracle(v_np, n, s, seed, S, mf)
    assert nuq.nuq_last_error_flags() == 0

    # step 4 with K = 1: DECODE(ENCODE(x)) reproduces Q_s(v)
    out = torch.full((d,), 7.0, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate([mf], d, n, s, S, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == 0
    g.check_average([(norms_np, bo, words)], d, n, s, 1.0, out.cpu().numpy())
    # ... and adds onto what is there (one message: values go straight to the output, no tile), also through a
    # pointer off the 16-byte grid
    prior_np = rng.standard_normal(d + 1).astype(np.float32)
    for shift in (0, 1):
        out2 = torch.from_numpy(prior_np).to(g.DEV)[shift:shift + d]
        nuq.nuq_decode_accumulate([mf], d, n, s, S, -0.25, True, out2)
        g.check_average([(norms_np, bo, words)], d, n, s, -0.25, out2.cpu().numpy(),
                        prior=prior_np[shift:shift + d].astype(np.float64))
        out3 = torch.full((d + 1,), 7.0, dtype=torch.float32, device=g.DEV)[shift:shift + d]
        nuq.nuq_decode_accumulate([mf], d, n, s, S, 1.0, False, out3)
        assert torch.equal(out3, out)
    assert nuq.nuq_last_error_flags() == 0


@pytest.mark.parametrize("d,n,s,S,K", [(60_000, 8192, 3, 512, 8), (30_000, 512, 3, 0, 4), (50_000, 16384, 7, 1024, 4),
                                       (20_000, 1000, 4, 256, 32), (9_000, 8192, 3, 512, 3)])
def test_decode_average_of_K_workers(g, d, n, s, S, K):
    nuq = g.nuq
    rng = np.random.default_rng(K * 1000 + n)
    msgs, msgs_np = [], []
    for k in range(K):
        v_np = make_vector("mixed", d, n, rng)
        m = g.fused_encode(torch.from_numpy(v_np).to(g.DEV), n, s, k, S)
        q, bo, words, _ = g.check_message_against_oracle(v_np, n, s, k, S, m)
        msgs.append(m)
        msgs_np.append((m.norms.cpu().numpy(), bo, words))
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, False, out)
    g.check_average(msgs_np, d, n, s, 1.0 / K, out.cpu().numpy())
    # accumulate = 1 adds to what is there
    prior = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)
    out2 = prior.clone()
    nuq.nuq_decode_accumulate(msgs, d, n, s, S, 0.5, True, out2)
    g.check_average(msgs_np, d, n, s, 0.5, out2.cpu().numpy(), prior=prior.cpu().numpy().astype(np.float64))
    assert nuq.nuq_last_error_flags() == 0


def random_cases(count, seed):
    """Seeded draws over the whole parameter space of the entry points: vector length, bucket size (log-uniform
    over 1..32768), s, sync stride, number of workers, value distribution."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        n = int(round(2.0 ** rng.uniform(0, 15)))
        if rng.random() < 0.3:
            n = int(2 ** rng.integers(6, 16))                  # powers of two: whole rows, aligned buckets
        d = int(rng.integers(1, 12 * n + 2)) if rng.random() < 0.5 else int(rng.integers(1, 150_000))
        s = int(rng.integers(1, 15))
        S = int(rng.choice([0, 64, 128, 256, 512, 1024]))
        K = int(rng.choice([1, 2, 3, 5, 8]))
        kind = str(rng.choice(["gauss", "mixed", "edges"]))
        cases.append((d, n, s, S, K, kind))
    return cases


@pytest.mark.parametrize("d,n,s,S,K,kind", random_cases(40, 20240607))
def test_random_shapes(g, d, n, s, S, K, kind):
    """Batched fused encode of K workers and decode + average on randomly drawn shapes: messages bit-exact,
    norms and averages to the bars."""
    nuq = g.nuq
    rng = np.random.default_rng([d, n, s, S, K])
    vs_np = [make_vector(kind, d, n, rng) for _ in range(K)]
    vs = [torch.from_numpy(v).to(g.DEV) for v in vs_np]
    seeds = [int(x) for x in rng.integers(0, 2 ** 63, size=K)]
    msgs = g.batched_encode(vs, n, s, seeds, S)
    msgs_np = []
    for v_np, m, seed in zip(vs_np, msgs, seeds):
        g.check_norms(v_np, n, m.norms.cpu().numpy())
        _, bo, words, _ = g.check_message_against_oracle(v_np, n, s, seed, S, m)
        msgs_np.append((m.norms.cpu().numpy(), bo, words))
    out = torch.full((d,), 3.0, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() == 0
    g.check_average(msgs_np, d, n, s, 1.0 / K, out.cpu().numpy())


@pytest.mark.parametrize("d,n,s,S,K", [(70_000, 8192, 3, 512, 8), (20_000, 512, 3, 0, 4), (40_000, 16384, 7, 256, 3)])
def test_batched_encode_equals_per_worker_encode(g, d, n, s, S, K):
    nuq = g.nuq
    rng = np.random.default_rng(5 * K + n)
    vs = [torch.from_numpy(make_vector("mixed", d, n, rng)).to(g.DEV) for _ in range(K)]
    seeds = [1000 + 7 * k for k in range(K)]
    msgs = [g.alloc_message(d, n, s, S) for _ in range(K)]
    ws = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=g.DEV)
    nuq.nuq_quantize_encode_batch(vs, n, s, seeds, S, msgs, ws)
    assert nuq.nuq_last_error_flags() == 0
    for k in range(K):
        g.check_message_against_oracle(vs[k].cpu().numpy(), n, s, seeds[k], S, msgs[k])
        one = g.fused_encode(vs[k], n, s, seeds[k], S)
        np.testing.assert_array_equal(one.norms.cpu().numpy(), msgs[k].norms.cpu().numpy())
        np.testing.assert_array_equal(g.u64(one.bit_off), g.u64(msgs[k].bit_off))


def test_extreme_magnitudes_and_subnormals(g):
    """Tiny norms (the bucket is rescaled inside the kernel), subnormal coordinates, huge values."""
    nuq = g.nuq
    n, s, S = 512, 3, 0
    rng = np.random.default_rng(77)
    parts = [rng.standard_normal(n) * sc for sc in (1e-30, 1e-38, 3e-41, 1e-44, 1e18, 1e-19, 1e-22, 1.0)]
    parts[7][:] = 0.0
    parts[7][5] = 1e-45          # a single subnormal coordinate: r = 1
    v_np = np.concatenate(parts).astype(np.float32)
    v = torch.from_numpy(v_np).to(g.DEV)
    m = g.fused_encode(v, n, s, 3, S)
    g.check_norms(v_np, n, m.norms.cpu().numpy())
    q, bo, words, _ = g.check_message_against_oracle(v_np, n, s, 3, S, m)
    assert (q[: 6 * n] & 0x7F).any()
    out = torch.empty(v_np.size, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate([m], v_np.size, n, s, S, 1.0, False, out)
    g.check_average([(m.norms.cpu().numpy(), bo, words)], v_np.size, n, s, 1.0, out.cpu().numpy())
    assert nuq.nuq_last_error_flags() == 0


def test_device_flags(g):
    nuq = g.nuq
    d, n, s = 20_000, 8192, 3
    v = torch.from_numpy(np.random.default_rng(20_000).standard_normal(d).astype(np.float32)).to(g.DEV)
    # capacity: offsets are complete, flag raised
    m = g.fused_encode(v, n, s, 1, 512, words_cap=10)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_CAPACITY
    full = g.fused_encode(v, n, s, 1, 512)
    assert nuq.nuq_last_error_flags() == 0
    np.testing.assert_array_equal(g.u64(m.bit_off), g.u64(full.bit_off))
    # non-finite input: flagged, that bucket encoded empty, others untouched
    v2 = v.clone()
    v2[100] = float("inf")
    m2 = g.fused_encode(v2, n, s, 1, 512)
    assert nuq.nuq_last_error_flags() == nuq.FLAG_NONFINITE
    bo2, bo = g.u64(m2.bit_off), g.u64(full.bit_off)
    assert bo2[1] == 0 and bo2[2] - bo2[1] == bo[2] - ((bo[1] + 31) // 32 * 32)
    # malformed stream: corrupt an offset so a record is cut; decode flags it and returns.  (Two bits: no record is
    # that short, so the cut cannot fall on a record boundary and leave a shorter, well-formed string.)
    bad = nuq.Message(full.norms, full.bit_off.clone(), full.words, full.sync)
    bad.bit_off[1] -= 2
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate([bad], d, n, s, 512, 1.0, False, out)
    assert nuq.nuq_last_error_flags() & nuq.FLAG_MALFORMED


def test_full_size_configs_1_to_3(g):
    """BASELINE configs 1-3 at full size, every bucket compared (the oracle needs a few seconds each)."""
    nuq = g.nuq
    for cfg in (1, 2, 3):
        w = workloads.workload(cfg)
        S = 512
        K = min(w.K, 2)                 # config 3: two of the eight workers element by element
        msgs, msgs_np = [], []
        for k in range(K):
            v = workloads.generate(w, k, g.DEV)
            m = g.fused_encode(v, w.bucket, w.s, w.quant_seed(k), S)
            v_np = v.cpu().numpy()
            g.check_norms(v_np, w.bucket, m.norms.cpu().numpy())
            q, bo, words, _ = g.check_message_against_oracle(v_np, w.bucket, w.s, w.quant_seed(k), S, m)
            msgs.append(m)
            msgs_np.append((m.norms.cpu().numpy(), bo, words))
            print("cfg %d worker %d: bits/coord %.4f" % (cfg, k, (32 * len(bo) - 32 + int(bo[-1])) / w.d), flush=True)
        out = torch.empty(w.d, dtype=torch.float32, device=g.DEV)
        nuq.nuq_decode_accumulate(msgs, w.d, w.bucket, w.s, S, 1.0 / K, False, out)
        g.check_average(msgs_np, w.d, w.bucket, w.s, 1.0 / K, out.cpu().numpy())
        assert nuq.nuq_last_error_flags() == 0


@pytest.mark.gpu
@pytest.mark.parametrize("n,s,S", [(8192, 3, 256), (16384, 7, 512), (32768, 3, 1024), (2048, 14, 128), (512, 3, 128)])
def test_encode_of_dense_buckets(g, n, s, S):
    """Buckets far denser than gradients produce: more nonzeros than the encoder's LDS index list holds, or a bit
    string longer than its LDS buffer (these buckets take the encoder's slower paths), next to ordinary ones.
    Level|sign bytes are crafted and go through nuq_encode; the message must equal the oracle's and decode back."""
    nuq = g.nuq
    rng = np.random.default_rng(n + s)
    nb = 7
    d = nb * n - 5
    q = np.zeros(d, dtype=np.uint8)

    def fill(b, density, top_heavy):
        lo, hi = b * n, min(d, (b + 1) * n)
        m = rng.random(hi - lo) < density
        lev = np.full(hi - lo, s + 1, dtype=np.uint8) if top_heavy else rng.integers(1, s + 2, size=hi - lo, dtype=np.uint8)
        sign = (rng.random(hi - lo) < 0.5).astype(np.uint8) << 7
        q[lo:hi] = np.where(m, lev | sign, 0)
    fill(0, 1.0, True)       # every coordinate at the top level: the worst case
    fill(1, 0.05, False)     # ordinary
    fill(2, 0.26, True)      # a few more nonzeros than the list holds (large buckets)
    fill(3, 0.24, True)      # the list holds them, the bit string is too long for the buffer
    fill(4, 0.0, False)      # empty
    fill(5, 0.6, False)
    fill(6, 1.0, False)      # short last bucket, full
    qd = torch.from_numpy(q).to(g.DEV)
    m = g.alloc_message(d, n, s, S)
    nuq.nuq_encode(qd, n, s, S, m.bit_off, m.words, m.sync if nuq.nuq_num_sync(n, S) else None, g.workspace(d, n, s))
    assert nuq.nuq_last_error_flags() == 0
    bo, words, sync = oracle.encode(q, n, s, S)
    np.testing.assert_array_equal(g.u64(m.bit_off), bo)
    np.testing.assert_array_equal(g.u32(m.words)[: words.size], words)
    assert not g.u32(m.words)[words.size:].any()
    if sync.size:
        np.testing.assert_array_equal(g.u32(m.sync)[: sync.size], sync)
    norms_np = (10.0 ** rng.uniform(-3, 3, size=nb)).astype(np.float32)
    m.norms.copy_(torch.from_numpy(norms_np))
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate([m], d, n, s, S, 1.0, False, out)
    assert nuq.nuq_last_error_flags() == 0
    g.check_average([(norms_np, bo, words)], d, n, s, 1.0, out.cpu().numpy())


@pytest.mark.gpu
def test_encode_and_decode_replayed_from_a_hip_graph(g):
    """The whole step (batched encode of K workers, decode + average) captured into a HIP graph and replayed
    several times with eager work in between: every replay must reproduce the eager messages and output."""
    nuq = g.nuq
    d, n, s, S, K = 200_000, 8192, 3, 256, 4
    rng = np.random.default_rng(7)
    vs = [torch.from_numpy((rng.standard_normal(d) * 0.01).astype(np.float32)).to(g.DEV) for _ in range(K)]
    seeds = [11 + k for k in range(K)]
    msgs = g.batched_encode(vs, n, s, seeds, S)                  # eager reference (also warms everything up)
    out_ref = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, False, out_ref)
    ref = [(m.bit_off.clone(), m.words.clone(), m.sync.clone(), m.norms.clone()) for m in msgs]

    B = nuq.nuq_num_buckets(d, n)
    ws = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=g.DEV)
    gm = [nuq.Message(torch.empty_like(m.norms), torch.empty_like(m.bit_off), torch.zeros_like(m.words),
                      torch.empty_like(m.sync)) for m in msgs]
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            nuq.nuq_quantize_encode_batch(vs, n, s, seeds, S, gm, ws)
            nuq.nuq_decode_accumulate(gm, d, n, s, S, 1.0 / K, False, out)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for m in gm:                      # eager work between replays: scrub the outputs
            m.bit_off.fill_(-1)
            m.words.zero_()
            m.sync.fill_(0x55)
            m.norms.fill_(-1.0)
        out.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for m, (bo, words, sync, norms) in zip(gm, ref):
            assert torch.equal(m.bit_off, bo) and torch.equal(m.words, words) and torch.equal(m.sync, sync)
            assert torch.equal(m.norms, norms)
        assert torch.equal(out, out_ref), rep
    assert nuq.nuq_last_error_flags() == 0


@pytest.mark.parametrize("d,n,s,S,K", [(300_000, 8192, 3, 256, 1), (300_000, 8192, 3, 256, 4), (90_000, 512, 3, 128, 4),
                                       (90_000, 512, 3, 0, 1), (200_000, 16384, 7, 0, 2), (400_000, 32768, 3, 1024, 2)])
def test_offsets_beyond_the_words_received(g, d, n, s, S, K):
    """A message cut short (fewer words than its offsets cover) and one whose offsets run backwards: the decoder
    raises the malformed flag, reads no word of the buckets concerned (they contribute nothing) and decodes every
    other bucket as usual.  The words tensors handed over are views of the full ones, so that even a decoder that
    ignored the length would stay inside allocated memory."""
    nuq = g.nuq
    rng = np.random.default_rng(d + K)
    vs = [torch.from_numpy((rng.standard_normal(d) * 0.01).astype(np.float32)).to(g.DEV) for _ in range(K)]
    seeds = [5 + k for k in range(K)]
    msgs = g.batched_encode(vs, n, s, seeds, S)
    B = nuq.nuq_num_buckets(d, n)
    parts = [(m.norms.cpu().numpy().copy(), g.u64(m.bit_off).copy(), g.u32(m.words).copy()) for m in msgs]
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)

    # worker 0's message loses its second half
    bo = parts[0][1]
    keep_words = int(bo[B // 2] + 31) // 32 + 1          # ends inside bucket B//2
    cut = nuq.Message(msgs[0].norms, msgs[0].bit_off, msgs[0].words[:keep_words], msgs[0].sync)
    nuq.nuq_decode_accumulate([cut] + msgs[1:], d, n, s, S, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() & nuq.FLAG_MALFORMED
    norms0 = parts[0][0].copy()
    norms0[bo[1:] > 32 * keep_words] = 0.0             # those buckets of worker 0 count for nothing
    assert (norms0 == 0).sum() >= B - B // 2 - 1 and (norms0 != 0).sum() >= B // 2 - 1
    g.check_average([(norms0, parts[0][1], parts[0][2])] + parts[1:], d, n, s, 1.0 / K, out.cpu().numpy())

    # the last worker's offsets run backwards at one bucket: that bucket and the next count for nothing
    b = B // 3
    bad_bo = msgs[-1].bit_off.clone()
    bad_bo[b + 1] = bad_bo[b] - 1 if int(bad_bo[b].item()) > 0 else bad_bo[b + 2] + 64
    back = nuq.Message(msgs[-1].norms, bad_bo, msgs[-1].words, msgs[-1].sync)
    nuq.nuq_decode_accumulate(msgs[:-1] + [back], d, n, s, S, 1.0 / K, False, out)
    assert nuq.nuq_last_error_flags() & nuq.FLAG_MALFORMED
    got = out.cpu().numpy()
    normsL = parts[-1][0].copy()
    normsL[b] = 0.0
    normsL[b + 1] = 0.0
    want_parts = parts[:-1] + [(normsL, parts[-1][1], parts[-1][2])]
    lo, hi = b * n, min(d, (b + 2) * n)
    ref = g.check_average([(p[0][: b], p[1][: b + 1], p[2]) for p in want_parts], lo, n, s, 1.0 / K, got[:lo]) if b else None
    # buckets b and b+1: the other workers' terms only, if the damaged ones were dropped whole (bucket b+1 may also
    # have been decoded from a start that is still inside the words: then its records were refused or kept)
    others = [(p[0], p[1], p[2]) for p in want_parts[:-1]]
    if others:
        w_all = oracle.decode_average([p[0] for p in others], [p[1] for p in others], [p[2] for p in others],
                                      d, n, s, float(np.float32(1.0 / K)))
        np.testing.assert_allclose(got[lo: b * n + n], w_all[lo: b * n + n], rtol=2e-6, atol=1e-30)
    else:
        assert not got[lo: b * n + n].any()


DIRTY = -0x5A5A5A5B           # 0xA5A5A5A5 as the int32 the word buffers are typed with


@pytest.mark.gpu
def test_full_size_in_the_benchmark_configuration(g):
    """BASELINE configs 3-5 at full size, launched the way bench.py launches them (all K workers in one encode
    call, bench's sync stride, one decode call over the K messages), into word buffers that hold a non-zero
    pattern before the encode.  Configs 3 and 4: every bucket of every worker's message bit-exact against the
    oracle, every element and bucket of the average within the bar.  Config 5: every bucket of every worker's
    message, and the average on sampled runs of buckets (the first, the last with the short bucket, seeded random
    ones).  Offsets non-decreasing with word-aligned starts accounted for, words
    beyond a message untouched, no error flags."""
    nuq = g.nuq
    for cfg in (3, 4, 5):
        w = workloads.workload(cfg)
        n, s, K, d = w.bucket, w.s, w.K, w.d
        S = workloads.sync_stride(w)
        B = nuq.nuq_num_buckets(d, n)
        print("cfg %d: generating %d x %d coordinates" % (cfg, K, d), flush=True)
        vs = [workloads.generate(w, k, g.DEV) for k in range(K)]
        seeds = [w.quant_seed(k) for k in range(K)]
        msgs = g.batched_encode(vs, n, s, seeds, S, fill=DIRTY)
        out = torch.empty(d, dtype=torch.float32, device=g.DEV)
        nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, False, out)
        assert nuq.nuq_last_error_flags() == 0
        for m in msgs:
            bo = m.bit_off
            assert int(bo[0].item()) == 0
            assert bool((bo[1:] >= (bo[:-1] + 31) // 32 * 32).all())      # a bucket ends at or after its aligned start
            W = (int(bo[-1].item()) + 31) // 32
            assert bool((m.words[W:] == DIRTY).all())                     # nothing written past the message
        if cfg != 5:
            g.check_every_bucket(vs, msgs, out, n, s, seeds, S, 1.0 / K)
            print("cfg %d: all %d buckets of %d workers bit-exact, averages within the bar" % (cfg, B, K), flush=True)
        else:
            g.check_every_bucket(vs, msgs, None, n, s, seeds, S, 1.0 / K)
            print("cfg 5: all %d buckets of %d workers bit-exact" % (B, K), flush=True)
            rng = np.random.default_rng(cfg)
            run_len = 64
            starts = {0, B - run_len} | {int(x) for x in rng.integers(0, B - run_len, size=96)}
            for b_lo in sorted(starts):
                g.check_bucket_run(vs, msgs, out, n, s, seeds, S, 1.0 / K, b_lo, b_lo + run_len)
            print("cfg 5: %d runs of %d buckets, all workers bit-exact, averages within the bar"
                  % (len(starts), run_len), flush=True)
        del vs, msgs, out
        torch.cuda.empty_cache()
