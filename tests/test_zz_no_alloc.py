"""The entry point that allocates nothing (nuq_quantize_encode_static: the encoder's workspace is a device array
inside the library) against nuq_quantize_encode with a caller-provided workspace: norms, offsets, bit strings
and decoder index bit for bit, on two calls in a row that share the array, the second on a smaller input."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_static_workspace_encoder_equals_the_workspace_one():
    import gpu_util as g
    nuq = g.nuq
    rng = np.random.default_rng(20261128)
    # a large first call (several hundred buckets, ragged tail), then a smaller one with another bucket size
    for d, n, s, S, seed in ((2_000_003, 8192, 3, 256, 5), (70_001, 512, 4, 128, 9)):
        v_np = (rng.standard_normal(d) * 10.0 ** rng.uniform(-4, 0, size=d)).astype(np.float32)
        v_np[rng.random(d) < 0.02] = 0.0
        v = torch.from_numpy(v_np).to(g.DEV)
        ref = g.fused_encode(v, n, s, seed, S)
        assert nuq.nuq_last_error_flags() == 0
        m = g.alloc_message(d, n, s, S)
        before = torch.cuda.memory_allocated()
        nuq.nuq_quantize_encode_static(v, n, s, seed, S, m.norms, m.bit_off, m.words, m.sync)
        assert torch.cuda.memory_allocated() == before            # (torch's own view: nothing was requested from it)
        assert nuq.nuq_last_error_flags() == 0
        assert torch.equal(m.norms, ref.norms)
        assert torch.equal(m.bit_off, ref.bit_off)
        assert torch.equal(m.words, ref.words)
        assert torch.equal(m.sync, ref.sync)
        # and the message is the oracle's (to the bar of the other parity tests: bit-exact)
        g.check_message_against_oracle(v_np, n, s, seed, S, m)


def test_static_workspace_encoder_rejects_what_does_not_fit():
    import gpu_util as g
    nuq = g.nuq
    d, n, s = 40_000_000, 8192, 3                                 # needs 40 MB of staging: above the 32 MiB array
    assert nuq.nuq_encode_workspace_bytes(1, d, n, s) > nuq.STATIC_WORKSPACE_BYTES
    v = torch.zeros(8, dtype=torch.float32, device=g.DEV)         # never read: the size check comes first
    m = g.alloc_message(8, n, s, 0)
    import ctypes                                                  # straight through the C ABI: d without a 160 MB tensor
    lib = ctypes.CDLL(nuq.library_path())
    lib.nuq_quantize_encode_static.restype = ctypes.c_int
    lib.nuq_quantize_encode_static.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                               ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
    rc = lib.nuq_quantize_encode_static(v.data_ptr(), d, n, s, 1, 0, m.norms.data_ptr(), m.bit_off.data_ptr(),
                                        m.words.data_ptr(), m.words.numel(), None, None)
    assert rc == -2                                                # NUQ_ECAPACITY, nothing enqueued
