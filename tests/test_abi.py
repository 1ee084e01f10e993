"""The C-ABI library loads on a machine without a GPU and exports every symbol the header declares;
host-only size helpers and argument checks behave as include/nuq.h says.  No kernel is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nuq():
    lib = os.path.join(ROOT, "paper_1908_06077_amd", "libnuq.so")
    if not os.path.exists(lib):
        import __graft_entry__
        __graft_entry__.build()
    import paper_1908_06077_amd
    return paper_1908_06077_amd


def header_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(nuq_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(nuq):
    names = header_functions()
    assert names == nuq.exported_symbols()
    lib = ctypes.CDLL(nuq.library_path())
    for n in names:
        assert getattr(lib, n) is not None


def test_size_helpers(nuq):
    assert nuq.nuq_workspace_bytes(10 ** 6, 8192, 4) == nuq.nuq_encode_workspace_bytes(4, 10 ** 6, 8192, 14)
    assert nuq.nuq_workspace_bytes(10 ** 6, 8192, 4) >= nuq.nuq_encode_workspace_bytes(4, 10 ** 6, 8192, 3) > 0
    assert nuq.nuq_workspace_bytes(10 ** 6, 40000, 4) == 0 and nuq.nuq_workspace_bytes(0, 8192, 1) == 0
    assert nuq.nuq_num_buckets(25_557_032, 8192) == 3120
    assert nuq.nuq_num_buckets(8192, 8192) == 1 and nuq.nuq_num_buckets(8193, 8192) == 2
    # decoder index: blocks of 2048 coordinates x a power-of-two number of pieces of about sync_stride coordinates
    assert nuq.nuq_num_sync(8192, 512) == 4 * 4 and nuq.nuq_num_sync(512, 512) == 1
    assert nuq.nuq_num_sync(1000, 256) == 4 and nuq.nuq_num_sync(8192, 0) == 0 and nuq.nuq_num_sync(1300, 256) == 8
    assert nuq.nuq_num_sync(16384, 256) == 8 * 8 and nuq.nuq_num_sync(32768, 64) == 16 * 32
    assert nuq.nuq_num_sync(8192, 100) == 0                              # not a power of two in 64..1024
    assert nuq.nuq_huffman_num_sync(8192, 512) == 15 and nuq.nuq_huffman_num_sync(1000, 256) == 3
    # worst case: every coordinate nonzero at the top level: 1 (gap) + 1 (sign) + |ERC(s+1)| bits each
    assert nuq.nuq_max_words(8192, 8192, 3) == 8192 * 8 // 32 + 1        # |ERC(4)| = 6
    assert nuq.nuq_max_words(64, 64, 7) == (64 * 9 + 31) // 32 + 1       # |ERC(8)| = 7
    assert nuq.nuq_encode_workspace_bytes(1, 1 << 20, 8192, 3) >= 128 * 8192
    assert nuq.nuq_encode_workspace_bytes(1, 1 << 20, 0, 3) == 0


def test_argument_errors_are_reported_on_the_host(nuq):
    lib = ctypes.CDLL(nuq.library_path())
    lib.nuq_bucket_norms.restype = ctypes.c_int
    lib.nuq_bucket_norms.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    EINVAL = -1
    assert lib.nuq_bucket_norms(None, 10, 4, None, None) == EINVAL            # NULL pointers
    assert lib.nuq_bucket_norms(16, 0, 4, 16, None) == EINVAL                 # d = 0
    assert lib.nuq_bucket_norms(16, 10, 0, 16, None) == EINVAL                # bucket = 0
    assert lib.nuq_bucket_norms(16, 10, 40000, 16, None) == EINVAL            # bucket too large
    assert lib.nuq_bucket_norms(18, 10, 4, 16, None) == EINVAL                # misaligned v
    lib.nuq_quantize.restype = ctypes.c_int
    lib.nuq_quantize.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64,
                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.nuq_quantize(16, 10, 4, 0, 0, 16, 16, None) == EINVAL          # s = 0
    assert lib.nuq_quantize(16, 10, 4, 15, 0, 16, 16, None) == EINVAL         # s too large
    lib.nuq_last_error_flags.restype = ctypes.c_int
    lib.nuq_last_error_flags.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.nuq_last_error_flags(None, None) == EINVAL
    # level tables (host arrays) are validated before anything is launched
    lib.nuq_quantize_table.restype = ctypes.c_int
    lib.nuq_quantize_table.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    table = lambda *xs: (ctypes.c_float * len(xs))(*xs)
    assert lib.nuq_quantize_table(16, 10, 4, 3, None, 0, 16, 16, None) == EINVAL                            # no table
    assert lib.nuq_quantize_table(16, 10, 4, 3, table(0, .25, .5, .5, 1), 0, 16, 16, None) == EINVAL        # not increasing
    assert lib.nuq_quantize_table(16, 10, 4, 3, table(.1, .25, .5, .75, 1), 0, 16, 16, None) == EINVAL      # l_0 != 0
    assert lib.nuq_quantize_table(16, 10, 4, 3, table(0, .25, .5, .75, .9), 0, 16, 16, None) == EINVAL      # l_{s+1} != 1
    assert lib.nuq_quantize_table(16, 10, 4, 3, table(0, .25, float("nan"), .75, 1), 0, 16, 16, None) == EINVAL
    lib.nuq_bucket_norms_linf.restype = ctypes.c_int
    lib.nuq_bucket_norms_linf.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.nuq_bucket_norms_linf(None, 10, 4, None, None) == EINVAL


def test_argument_errors_of_the_update_entry_points(nuq):
    # rejected on the host before anything is launched
    lib = ctypes.CDLL(nuq.library_path())
    EINVAL, f32, vp, u64 = -1, ctypes.c_float, ctypes.c_void_p, ctypes.c_uint64
    lib.nuq_momentum_step.restype = ctypes.c_int
    lib.nuq_momentum_step.argtypes = [vp, vp, vp, u64, f32, f32, f32, vp]
    assert lib.nuq_momentum_step(16, 16, 16, 8, 0.1, 1.0, 0.0, None) == EINVAL              # mu = 1
    assert lib.nuq_momentum_step(16, 16, 16, 8, 0.1, -0.5, 0.0, None) == EINVAL             # mu < 0
    assert lib.nuq_momentum_step(16, 16, 16, 8, float("nan"), 0.5, 0.0, None) == EINVAL
    assert lib.nuq_momentum_step(16, 16, 16, 8, 0.1, 0.5, float("inf"), None) == EINVAL
    assert lib.nuq_momentum_step(None, 16, 16, 8, 0.1, 0.5, 0.0, None) == EINVAL            # NULL w
    assert lib.nuq_momentum_step(None, None, None, 0, 0.1, 0.5, 0.0, None) == 0             # d = 0: nothing to do
    lib.nuq_moments_accumulate.restype = ctypes.c_int
    lib.nuq_moments_accumulate.argtypes = [vp, vp, vp, u64, vp]
    assert lib.nuq_moments_accumulate(16, None, 16, 8, None) == EINVAL
    lib.nuq_normalized_variance.restype = ctypes.c_int
    lib.nuq_normalized_variance.argtypes = [vp, vp, u64, u64, vp, u64, vp, vp]
    assert lib.nuq_normalized_variance(16, 16, 8, 0, 16, 16384, 16, None) == EINVAL         # no draws
    assert lib.nuq_normalized_variance(16, 16, 8, 3, 16, 1024, 16, None) == EINVAL          # workspace too small
    assert lib.nuq_normalized_variance(16, 16, 8, 3, 20, 16384, 16, None) == EINVAL         # workspace misaligned
    assert lib.nuq_normalized_variance(16, 16, 8, 3, 16, 16384, None, None) == EINVAL       # no output
    lib.nuq_decode_momentum_step.restype = ctypes.c_int
    lib.nuq_decode_momentum_step.argtypes = [ctypes.c_uint32, vp, vp, vp, vp, vp, u64, ctypes.c_uint32, ctypes.c_uint32,
                                             ctypes.c_uint32, f32, f32, f32, f32, vp, vp, vp]
    one = (ctypes.c_void_p * 1)(16)
    n1 = (ctypes.c_uint64 * 1)(4)
    assert lib.nuq_decode_momentum_step(1, one, one, one, n1, one, 8, 4, 3, 0, 1.0, 0.1, 0.5, 0.0, 16, None, None) == EINVAL
    assert lib.nuq_decode_momentum_step(1, one, one, one, n1, one, 8, 4, 3, 0, 1.0, 0.1, 1.5, 0.0, 16, 16, None) == EINVAL
    assert lib.nuq_decode_momentum_step(0, one, one, one, n1, one, 8, 4, 3, 0, 1.0, 0.1, 0.5, 0.0, 16, 16, None) == EINVAL
    # the decoders want the length of every message's words
    lib.nuq_decode_accumulate.restype = ctypes.c_int
    lib.nuq_decode_accumulate.argtypes = [ctypes.c_uint32, vp, vp, vp, vp, vp, u64, ctypes.c_uint32, ctypes.c_uint32,
                                          ctypes.c_uint32, f32, ctypes.c_int, vp, vp]
    assert lib.nuq_decode_accumulate(1, one, one, one, None, one, 8, 4, 3, 0, 1.0, 0, 16, None) == EINVAL
    assert lib.nuq_decode_accumulate(1, one, one, one, n1, one, 8, 4, 3, 0, 1.0, 0, None, None) == EINVAL      # no out
    lib.nuq_fixed_words.restype = ctypes.c_uint64
    lib.nuq_fixed_words.argtypes = [u64, ctypes.c_uint32, ctypes.c_uint32]
    assert lib.nuq_fixed_words(100, 32, 4) == 4 * 4 and lib.nuq_fixed_words(100, 32, 2) == 0 and lib.nuq_fixed_words(100, 0, 4) == 0


def test_binding_checks_buffer_sizes(nuq, monkeypatch):
    """The wrappers refuse tensors shorter than d, bucket and sync_stride imply before anything reaches the
    library.  Host tensors stand in for device tensors (the placement check is switched off for all but the last
    case): every call here ends in the wrapper."""
    import torch
    from paper_1908_06077_amd import binding
    monkeypatch.setattr(binding, "_on_device", lambda t: True)
    d, n, s, S = 10_000, 1024, 3, 256
    B, per = nuq.nuq_num_buckets(d, n), nuq.nuq_num_sync(n, S)
    f = lambda k: torch.zeros(k, dtype=torch.float32)
    i32 = lambda k: torch.zeros(k, dtype=torch.int32)
    i64 = lambda k: torch.zeros(k, dtype=torch.int64)
    good = lambda: nuq.Message(f(B), i64(B + 1), i32(64), i32(B * per))
    ws = torch.zeros(64, dtype=torch.uint8)
    cases = [
        ("norms holds", lambda: nuq.nuq_bucket_norms(f(d), n, f(B - 1))),
        ("norms holds", lambda: nuq.nuq_bucket_norms_linf(f(d), n, f(B - 1))),
        ("norms holds", lambda: nuq.nuq_quantize(f(d), n, s, 1, f(B - 1), torch.zeros(d, dtype=torch.uint8))),
        ("q holds", lambda: nuq.nuq_quantize(f(d), n, s, 1, f(B), torch.zeros(d - 1, dtype=torch.uint8))),
        ("bit_off holds", lambda: nuq.nuq_encode(torch.zeros(d, dtype=torch.uint8), n, s, S, i64(B), i32(64), i32(B * per), ws)),
        ("sync holds", lambda: nuq.nuq_encode(torch.zeros(d, dtype=torch.uint8), n, s, S, i64(B + 1), i32(64), i32(B * per - 1), ws)),
        ("sync is needed", lambda: nuq.nuq_encode(torch.zeros(d, dtype=torch.uint8), n, s, S, i64(B + 1), i32(64), None, ws)),
        ("norms holds", lambda: nuq.nuq_quantize_encode(f(d), n, s, 1, S, f(B - 1), i64(B + 1), i32(64), i32(B * per), ws)),
        ("bit_off holds", lambda: nuq.nuq_quantize_encode_static(f(d), n, s, 1, S, f(B), i64(B), i32(64), i32(B * per))),
        ("sync holds", lambda: nuq.nuq_quantize_encode_batch([f(d)], n, s, [1], S, [nuq.Message(f(B), i64(B + 1), i32(64), i32(3))], ws)),
        ("bit_off holds", lambda: nuq.nuq_decode_accumulate([nuq.Message(f(B), i64(B), i32(64), i32(B * per))], d, n, s, S, 1.0, False, f(d))),
        ("norms holds", lambda: nuq.nuq_decode_accumulate([good(), nuq.Message(f(1), i64(B + 1), i32(64), i32(B * per))], d, n, s, S, 1.0, False, f(d))),
        ("out must hold", lambda: nuq.nuq_decode_accumulate([good()], d, n, s, S, 1.0, False, f(d - 1))),
        ("expected dtype", lambda: nuq.nuq_decode_accumulate([nuq.Message(f(B), i32(B + 1), i32(64), i32(B * per))], d, n, s, S, 1.0, False, f(d))),
        ("sync holds", lambda: nuq.nuq_decode_momentum_step([nuq.Message(f(B), i64(B + 1), i32(64), i32(1))], d, n, s, S, 1.0, 0.1, 0.5, 0.0, f(d), f(d))),
        ("sync holds", lambda: nuq.nuq_decode_accumulate_table([nuq.Message(f(B), i64(B + 1), i32(64), i32(1))], d, n, [0, .25, .5, .75, 1], S, 1.0, False, f(d))),
    ]
    for want, call in cases:
        with pytest.raises(ValueError, match=want):
            call()
    # tensors of the right sizes get as far as the placement check
    monkeypatch.undo()
    with pytest.raises(ValueError, match="device tensor"):
        nuq.nuq_decode_accumulate([good()], d, n, s, S, 1.0, False, f(d))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_huffman_lengths_on_the_host(nuq):
    """nuq_huffman_lengths is host arithmetic: the hand-built examples of tests/golden/huffman_examples.txt."""
    for line in open(os.path.join(ROOT, "tests", "golden", "huffman_examples.txt")):
        f = [x.strip() for x in line.split("|")]
        if f[0] != "L":
            continue
        s, hist, lengths = int(f[1]), [int(x) for x in f[2].split()], [int(x) for x in f[3].split()]
        assert nuq.nuq_huffman_lengths(hist, s) == lengths
    assert nuq.nuq_huffman_max_words(100, 10) == (100 * 16 + 31) // 32 + 10
    # the library's builder (a merge of two sorted queues) against the oracle's (repeated search for the two smallest
    # nodes): equal lengths, ties included, on random, tiny, huge and all-zero counts
    import numpy as np
    import oracle
    rng = np.random.default_rng(11)
    for t in range(3000):
        s = int(rng.integers(1, 15))
        hist = [rng.integers(0, 4, size=s + 2), rng.integers(0, 10 ** 7, size=s + 2),
                2 ** rng.integers(0, 45, size=s + 2), np.zeros(s + 2, dtype=np.int64)][t % 4]
        assert nuq.nuq_huffman_lengths([int(x) for x in hist], s) == \
            [int(x) for x in oracle.huffman_lengths(np.asarray(hist, dtype=np.uint64), s)]
