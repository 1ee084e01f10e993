"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the oracle on the
same inputs, compare to the bars the tests state."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_1908_06077_amd as nuq

DEV = torch.device("cuda:0")


def u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def u64(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def alloc_message(d, n, s, S, words_cap=None):
    B = nuq.nuq_num_buckets(d, n)
    cap = nuq.nuq_max_words(d, n, s) if words_cap is None else words_cap
    return nuq.Message(torch.full((B,), -1.0, dtype=torch.float32, device=DEV),
                       torch.full((B + 1,), -1, dtype=torch.int64, device=DEV),
                       torch.zeros(max(cap, 1), dtype=torch.int32, device=DEV),
                       torch.full((max(1, B * nuq.nuq_num_sync(n, S)),), 0x55555555, dtype=torch.int32, device=DEV))


def workspace(d, n, s):
    return torch.empty(nuq.nuq_encode_workspace_bytes(1, d, n, s), dtype=torch.uint8, device=DEV)


def fused_encode(v: torch.Tensor, n, s, seed, S, words_cap=None):
    m = alloc_message(v.numel(), n, s, S, words_cap)
    nuq.nuq_quantize_encode(v, n, s, seed, S, m.norms, m.bit_off, m.words, m.sync, workspace(v.numel(), n, s))
    return m


def check_norms(v_np, n, norms_gpu):
    want = oracle.bucket_norms(v_np, n)
    got = norms_gpu.astype(np.float64)
    # bar: 1e-6 relative to the fp64 norm (the benchmark spec); zero norms must be exactly zero.  A norm below the
    # smallest normal float cannot be held to 1e-6 by the fp32 output format itself: there the bar is half a
    # unit of the subnormal grid (2^-150), i.e. the correctly rounded value.
    tol = np.maximum(1e-6 * want, np.where(want > 0, 2.0 ** -150 * (1 + 1e-9), 0.0))
    assert np.all(np.abs(got - want) <= tol), float(np.max(np.abs(got - want) / np.maximum(want, 1e-300)))


def check_message_against_oracle(v_np, n, s, seed, S, m: "nuq.Message", first_bucket=0):
    """Bit-exact: levels/signs are implied by the bit strings; offsets, words and sync must be identical
    to the oracle's when it is fed the GPU's norms."""
    d = v_np.size
    norms = m.norms.cpu().numpy()
    q = oracle.quantize(v_np, n, s, seed, norms, first_bucket)
    bo, words, sync = oracle.encode(q, n, s, S)
    got_bo = u64(m.bit_off)
    np.testing.assert_array_equal(got_bo, bo)
    got_words = u32(m.words)
    np.testing.assert_array_equal(got_words[: words.size], words)
    assert not got_words[words.size:].any()          # nothing written past the end
    if sync.size:
        np.testing.assert_array_equal(u32(m.sync)[: sync.size], sync)
    return q, bo, words, sync


def check_average(msgs_np, d, n, s, scale, out_gpu: np.ndarray, prior=None):
    """bars: per bucket ||out - ref||_2 <= 1e-6 ||ref||_2 and per element |diff| <= 1e-6 * scale * sum_k |term_k|."""
    K = len(msgs_np)
    scale32 = float(np.float32(scale))
    want = oracle.decode_average([m[0] for m in msgs_np], [m[1] for m in msgs_np], [m[2] for m in msgs_np],
                                 d, n, s, scale32, prior=prior)
    mag = np.zeros(d)
    for norms, bo, words in msgs_np:
        q = oracle.decode_levels(bo, words, d, n, s)
        mag += np.abs(oracle.dequantize(q, n, s, norms))
    mag = mag * abs(scale32) + (np.abs(prior) if prior is not None else 0.0)
    got = out_gpu.astype(np.float64)
    diff = np.abs(got - want)
    assert np.all(diff <= 1e-6 * mag + 1e-45), float(np.max(diff / np.maximum(mag, 1e-300)))
    B = (d + n - 1) // n

    def bucket_l2(x):
        sq = np.zeros(B * n)
        sq[:d] = x * x
        return np.sqrt(sq.reshape(B, n).sum(axis=1))
    # (+ the fp32 subnormal grid, 2^-149 per element, for outputs below the smallest normal float)
    bad = bucket_l2(got - want) > 1e-6 * bucket_l2(want) + 2.0 ** -149 * np.sqrt(n)
    assert not bad.any(), np.flatnonzero(bad)[:8]
    return want


def batched_encode(vs, n, s, seeds, S, fill=0):
    """All workers in one launch, buffers sized like bench.py sizes them (a probe encode gives the lengths).
    `fill` is what every word of the message buffers holds before the encode."""
    d, K = vs[0].numel(), len(vs)
    B = nuq.nuq_num_buckets(d, n)
    nsync = nuq.nuq_num_sync(n, S)
    ws = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=DEV)

    def new_msg(nwords):
        return nuq.Message(torch.empty(B, dtype=torch.float32, device=DEV),
                           torch.empty(B + 1, dtype=torch.int64, device=DEV),
                           torch.full((nwords,), fill, dtype=torch.int32, device=DEV),
                           torch.empty(max(1, B * nsync), dtype=torch.int32, device=DEV))
    probes = [new_msg(16) for _ in range(K)]
    nuq.nuq_quantize_encode_batch(vs, n, s, seeds, S, probes, ws)
    assert nuq.nuq_last_error_flags() & ~nuq.FLAG_CAPACITY == 0
    msgs = [new_msg((int(p.bit_off[-1].item()) + 31) // 32 + 64) for p in probes]
    del probes
    nuq.nuq_quantize_encode_batch(vs, n, s, seeds, S, msgs, ws)
    assert nuq.nuq_last_error_flags() == 0
    return msgs


def check_bucket_run(vs, msgs, out, n, s, seeds, S, scale, b_lo, b_hi, prior=None):
    """Buckets [b_lo, b_hi) of a large problem: every worker's message pieces bit-exact against the oracle run
    on just those buckets (fed the GPU's norms), norms and the decoded average of the K workers to the bars."""
    d = vs[0].numel()
    c_lo, c_hi = b_lo * n, min(d, b_hi * n)
    nsync = nuq.nuq_num_sync(n, S)
    parts = []
    for v, m, seed in zip(vs, msgs, seeds):
        v_np = v[c_lo:c_hi].cpu().numpy()
        norms = m.norms[b_lo:b_hi].cpu().numpy()
        check_norms(v_np, n, norms)
        q = oracle.quantize(v_np, n, s, seed, norms, b_lo)
        bo, words, sync = oracle.encode(q, n, s, S)
        got_bo = u64(m.bit_off[b_lo:b_hi + 1])
        start = (int(got_bo[0]) + 31) // 32 * 32          # the run's first bucket starts on a word boundary
        np.testing.assert_array_equal(got_bo[1:] - np.uint64(start), bo[1:])
        got_words = u32(m.words[start // 32: start // 32 + words.size])
        np.testing.assert_array_equal(got_words, words)
        if sync.size:
            np.testing.assert_array_equal(u32(m.sync[b_lo * nsync: b_hi * nsync]), sync)
        parts.append((norms, bo, words))
    if out is not None:
        check_average(parts, c_hi - c_lo, n, s, scale, out[c_lo:c_hi].cpu().numpy(),
                      prior=None if prior is None else prior[c_lo:c_hi].cpu().numpy().astype(np.float64))
    return parts


def check_every_bucket(vs, msgs, out, n, s, seeds, S, scale, coords_per_run=1 << 20):
    """check_bucket_run over consecutive runs that cover every bucket, the runs dealt out to the host's cores (the
    oracle's calls release the interpreter lock).  Returns the number of buckets compared."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    d = vs[0].numel()
    B = nuq.nuq_num_buckets(d, n)
    run = max(1, coords_per_run // n)
    runs = [(lo, min(B, lo + run)) for lo in range(0, B, run)]
    with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1))) as pool:
        list(pool.map(lambda r: check_bucket_run(vs, msgs, out, n, s, seeds, S, scale, r[0], r[1]), runs))
    return B
