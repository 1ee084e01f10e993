"""ctypes binding of the C ABI in include/nuq.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnuq.so")

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        "libnuq.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(or `python paper_1908_06077_amd/build.py`) first; there is no fallback path")

_lib = ctypes.CDLL(_LIB_PATH)

FLAG_CAPACITY, FLAG_NONFINITE, FLAG_MALFORMED = 1, 2, 4
SYNC_BLOCK = 2048
MAX_BUCKET, MAX_S, MAX_WORKERS = 32768, 14, 32

_u64, _u32, _i32, _vp, _f32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p, ctypes.c_float

_SIGNATURES = {
    "nuq_num_buckets": (_u64, [_u64, _u32]),
    "nuq_workspace_bytes": (_u64, [_u64, _u32, _u32]),
    "nuq_num_sync": (_u32, [_u32, _u32]),
    "nuq_huffman_num_sync": (_u32, [_u32, _u32]),
    "nuq_max_words": (_u64, [_u64, _u32, _u32]),
    "nuq_encode_workspace_bytes": (_u64, [_u32, _u64, _u32, _u32]),
    "nuq_quantize_encode_batch": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _u64, _vp]),
    "nuq_bucket_norms": (_i32, [_vp, _u64, _u32, _vp, _vp]),
    "nuq_quantize": (_i32, [_vp, _u64, _u32, _u32, _u64, _vp, _vp, _vp]),
    "nuq_encode": (_i32, [_vp, _u64, _u32, _u32, _u32, _vp, _vp, _u64, _vp, _vp, _u64, _vp]),
    "nuq_quantize_encode": (_i32, [_vp, _u64, _u32, _u32, _u64, _u32, _vp, _vp, _vp, _u64, _vp, _vp, _u64, _vp]),
    "nuq_quantize_encode_static": (_i32, [_vp, _u64, _u32, _u32, _u64, _u32, _vp, _vp, _vp, _u64, _vp, _vp]),
    "nuq_decode_accumulate": (_i32, [_u32, _vp, _vp, _vp, _vp, _vp, _u64, _u32, _u32, _u32, _f32, _i32, _vp, _vp]),
    "nuq_bucket_norms_linf": (_i32, [_vp, _u64, _u32, _vp, _vp]),
    "nuq_quantize_table": (_i32, [_vp, _u64, _u32, _u32, _vp, _u64, _vp, _vp, _vp]),
    "nuq_quantize_encode_table_batch": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _vp, _u32, _u32, _vp, _vp, _vp, _vp, _vp,
                                               _vp, _u64, _vp]),
    "nuq_decode_accumulate_huffman": (_i32, [_u32, _vp, _vp, _vp, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _f32, _i32, _vp,
                                             _vp]),
    "nuq_decode_accumulate_table": (_i32, [_u32, _vp, _vp, _vp, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _f32, _i32, _vp, _vp]),
    "nuq_fixed_words": (_u64, [_u64, _u32, _u32]),
    "nuq_pack_fixed": (_i32, [_vp, _u64, _u32, _u32, _u32, _vp, _vp]),
    "nuq_quantize_pack_fixed_batch": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp]),
    "nuq_unpack_accumulate_fixed": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _u32, _f32, _i32, _vp, _vp]),
    "nuq_quantize_pack_fixed_table_batch": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _vp, _u32, _u32, _vp, _vp, _vp]),
    "nuq_unpack_accumulate_fixed_table": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _vp, _u32, _f32, _i32, _vp, _vp]),
    "nuq_level_histogram": (_i32, [_vp, _u64, _vp, _vp]),
    "nuq_huffman_lengths": (_i32, [_vp, _u32, _vp]),
    "nuq_huffman_max_words": (_u64, [_u64, _u32]),
    "nuq_encode_huffman_workspace_bytes": (_u64, [_u64, _u32]),
    "nuq_encode_huffman": (_i32, [_vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp, _u64, _vp, _vp, _u64, _vp]),
    "nuq_decode_huffman": (_i32, [_vp, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp]),
    "nuq_encode_huffman_batch_workspace_bytes": (_u64, [_u32, _u64, _u32, _u32]),
    "nuq_quantize_encode_huffman_batch": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp, _vp, _vp, _vp,
                                                 _vp, _u64, _vp]),
    "nuq_decode_huffman_batch": (_i32, [_u32, _vp, _vp, _vp, _u64, _u32, _u32, _u32, _vp, _vp, _vp]),
    "nuq_average_levels": (_i32, [_u32, _vp, _vp, _u64, _u32, _u32, _f32, _i32, _vp, _vp]),
    "nuq_momentum_step": (_i32, [_vp, _vp, _vp, _u64, _f32, _f32, _f32, _vp]),
    "nuq_decode_momentum_step": (_i32, [_u32, _vp, _vp, _vp, _vp, _vp, _u64, _u32, _u32, _u32, _f32, _f32, _f32, _f32, _vp,
                                        _vp, _vp]),
    "nuq_moments_accumulate": (_i32, [_vp, _vp, _vp, _u64, _vp]),
    "nuq_normalized_variance": (_i32, [_vp, _vp, _u64, _u64, _vp, _u64, _vp, _vp]),
    "nuq_last_error_flags": (_i32, [_vp, _vp]),
    "nuq_timing_begin": (_i32, [_u32]),
    "nuq_timing_collect": (_i32, [_vp, _vp, _u32, _vp]),
}
for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def library_path() -> str:
    return _LIB_PATH


def exported_symbols() -> list[str]:
    return sorted(_SIGNATURES)


class NuqError(RuntimeError):
    def __init__(self, fn: str, code: int):
        names = {-1: "NUQ_EINVAL", -2: "NUQ_ECAPACITY", -3: "NUQ_ENONFINITE", -4: "NUQ_EHIP"}
        super().__init__("%s returned %s" % (fn, names.get(code, str(code))))
        self.code = code


def _check(fn: str, code: int) -> None:
    if code != 0:
        raise NuqError(fn, code)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _on_device(t: torch.Tensor) -> bool:
    return t.is_cuda


def _ptr(t: torch.Tensor | None, dtype: torch.dtype | None = None, need: int = 0, what: str = "tensor") -> int:
    """Device address of t after checking what the kernels take on trust: placement, contiguity, element type and
    that it holds at least `need` elements."""
    if t is None:
        if need:
            raise ValueError("%s is needed (%d elements)" % (what, need))
        return 0
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s: expected dtype %s, got %s" % (what, dtype, t.dtype))
    if t.numel() < need:
        raise ValueError("%s holds %d elements, %d are needed" % (what, t.numel(), need))
    if not _on_device(t) or not t.is_contiguous():
        raise ValueError("%s: expected a contiguous device tensor" % what)
    return t.data_ptr()


def _sizes(d: int, bucket: int, sync_stride: int, huffman: bool = False) -> tuple[int, int]:
    """(buckets, sync entries of a whole message) for the size checks; (0, 0) for arguments the library rejects."""
    B = _lib.nuq_num_buckets(d, bucket)
    per = (_lib.nuq_huffman_num_sync if huffman else _lib.nuq_num_sync)(bucket, sync_stride) if bucket else 0
    return B, B * per


def _message_arrays(messages, d: int, bucket: int, sync_stride: int, huffman: bool = False, norms: bool = True):
    """ctypes pointer arrays (norms, bit_off, words, words_len, sync) of K messages, every tensor checked against the
    size that d, bucket and sync_stride imply."""
    K = len(messages)
    B, nsync = _sizes(d, bucket, sync_stride, huffman)
    vp, u64 = ctypes.c_void_p * K, ctypes.c_uint64 * K
    return (vp(*[_ptr(m.norms, torch.float32, B, "norms") for m in messages]) if norms else None,
            vp(*[_ptr(m.bit_off, torch.int64, B + 1, "bit_off") for m in messages]),
            vp(*[_ptr(m.words, torch.int32, 0, "words") for m in messages]),
            u64(*[m.words.numel() for m in messages]),
            vp(*[_ptr(m.sync, torch.int32, nsync, "sync") for m in messages]))


# ------------------------------------------------------------------ sizes (host only)

def nuq_num_buckets(d: int, bucket: int) -> int:
    return _lib.nuq_num_buckets(d, bucket)


def nuq_num_sync(bucket: int, sync_stride: int) -> int:
    return _lib.nuq_num_sync(bucket, sync_stride)


def nuq_huffman_num_sync(bucket: int, sync_stride: int) -> int:
    return _lib.nuq_huffman_num_sync(bucket, sync_stride)


def nuq_max_words(d: int, bucket: int, s: int) -> int:
    return _lib.nuq_max_words(d, bucket, s)


def nuq_encode_workspace_bytes(K: int, d: int, bucket: int, s: int) -> int:
    return _lib.nuq_encode_workspace_bytes(K, d, bucket, s)


def nuq_workspace_bytes(d: int, bucket: int, K: int) -> int:
    return _lib.nuq_workspace_bytes(d, bucket, K)


# ------------------------------------------------------------------------- the path

def nuq_bucket_norms(v: torch.Tensor, bucket: int, norms: torch.Tensor) -> None:
    _check("nuq_bucket_norms",
           _lib.nuq_bucket_norms(_ptr(v, torch.float32), v.numel(), bucket,
                                 _ptr(norms, torch.float32, nuq_num_buckets(v.numel(), bucket), "norms"), _stream()))


def nuq_quantize(v: torch.Tensor, bucket: int, s: int, seed: int, norms: torch.Tensor, q: torch.Tensor) -> None:
    _check("nuq_quantize",
           _lib.nuq_quantize(_ptr(v, torch.float32), v.numel(), bucket, s, seed & (2 ** 64 - 1),
                             _ptr(norms, torch.float32, nuq_num_buckets(v.numel(), bucket), "norms"),
                             _ptr(q, torch.uint8, v.numel(), "q"), _stream()))


@dataclass
class Message:
    """One worker's encoded gradient: device tensors laid out as include/nuq.h describes."""
    norms: torch.Tensor       # float32 [B]
    bit_off: torch.Tensor     # int64 [B+1] (u64 bit pattern)
    words: torch.Tensor       # int32 [words_cap] (u32 bit pattern)
    sync: torch.Tensor | None  # int32 [B*nsync]


def nuq_encode(q: torch.Tensor, bucket: int, s: int, sync_stride: int, bit_off: torch.Tensor, words: torch.Tensor,
               sync: torch.Tensor | None, workspace: torch.Tensor) -> None:
    B, nsync = _sizes(q.numel(), bucket, sync_stride)
    _check("nuq_encode",
           _lib.nuq_encode(_ptr(q, torch.uint8), q.numel(), bucket, s, sync_stride,
                           _ptr(bit_off, torch.int64, B + 1, "bit_off"), _ptr(words, torch.int32), words.numel(),
                           _ptr(sync, torch.int32, nsync, "sync"), _ptr(workspace),
                           workspace.numel() * workspace.element_size(), _stream()))


def nuq_quantize_encode(v: torch.Tensor, bucket: int, s: int, seed: int, sync_stride: int, norms: torch.Tensor,
                        bit_off: torch.Tensor, words: torch.Tensor, sync: torch.Tensor | None,
                        workspace: torch.Tensor) -> None:
    B, nsync = _sizes(v.numel(), bucket, sync_stride)
    _check("nuq_quantize_encode",
           _lib.nuq_quantize_encode(_ptr(v, torch.float32), v.numel(), bucket, s, seed & (2 ** 64 - 1), sync_stride,
                                    _ptr(norms, torch.float32, B, "norms"), _ptr(bit_off, torch.int64, B + 1, "bit_off"),
                                    _ptr(words, torch.int32), words.numel(), _ptr(sync, torch.int32, nsync, "sync"),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


STATIC_WORKSPACE_BYTES = 32 << 20


def nuq_quantize_encode_static(v: torch.Tensor, bucket: int, s: int, seed: int, sync_stride: int, norms: torch.Tensor,
                               bit_off: torch.Tensor, words: torch.Tensor, sync: torch.Tensor | None) -> None:
    """nuq_quantize_encode with the library's own workspace: the call allocates nothing."""
    B, nsync = _sizes(v.numel(), bucket, sync_stride)
    _check("nuq_quantize_encode_static",
           _lib.nuq_quantize_encode_static(_ptr(v, torch.float32), v.numel(), bucket, s, seed & (2 ** 64 - 1),
                                           sync_stride, _ptr(norms, torch.float32, B, "norms"),
                                           _ptr(bit_off, torch.int64, B + 1, "bit_off"), _ptr(words, torch.int32),
                                           words.numel(), _ptr(sync, torch.int32, nsync, "sync"), _stream()))


def nuq_quantize_encode_batch(vs: list[torch.Tensor], bucket: int, s: int, seeds: list[int], sync_stride: int,
                              messages: list["Message"], workspace: torch.Tensor) -> None:
    K = len(vs)
    d = vs[0].numel()
    if any(v.numel() != d for v in vs) or len(seeds) != K or len(messages) != K:
        raise ValueError("K gradients of equal length, K seeds and K messages are needed")
    arr = lambda ts, dt=None: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    u64s = lambda xs: (ctypes.c_uint64 * K)(*[x & (2 ** 64 - 1) for x in xs])
    norms, offs, words, caps, sync = _message_arrays(messages, d, bucket, sync_stride)
    _check("nuq_quantize_encode_batch",
           _lib.nuq_quantize_encode_batch(K, arr(vs, torch.float32), u64s(seeds), d, bucket, s, sync_stride,
                                          norms, offs, words, caps, sync, _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()))


def nuq_decode_accumulate(messages: list[Message], d: int, bucket: int, s: int, sync_stride: int, scale: float,
                          accumulate: bool, out: torch.Tensor) -> None:
    K = len(messages)
    norms, offs, words, lens, sync = _message_arrays(messages, d, bucket, sync_stride)
    if out.numel() != d:
        raise ValueError("out must hold d floats")
    _check("nuq_decode_accumulate",
           _lib.nuq_decode_accumulate(K, norms, offs, words, lens, sync, d, bucket, s, sync_stride, float(scale),
                                      1 if accumulate else 0, _ptr(out, torch.float32), _stream()))


# ------------------------------------------- other level sequences, maximum norm

def _levels(levels, s: int):
    if len(levels) != s + 2:
        raise ValueError("a level table holds s + 2 values")
    return (ctypes.c_float * (s + 2))(*[float(x) for x in levels])


def nuq_bucket_norms_linf(v: torch.Tensor, bucket: int, norms: torch.Tensor) -> None:
    _check("nuq_bucket_norms_linf",
           _lib.nuq_bucket_norms_linf(_ptr(v, torch.float32), v.numel(), bucket,
                                      _ptr(norms, torch.float32, nuq_num_buckets(v.numel(), bucket), "norms"),
                                      _stream()))


def nuq_quantize_table(v: torch.Tensor, bucket: int, levels, seed: int, norms: torch.Tensor, q: torch.Tensor) -> None:
    s = len(levels) - 2
    _check("nuq_quantize_table",
           _lib.nuq_quantize_table(_ptr(v, torch.float32), v.numel(), bucket, s, _levels(levels, s),
                                   seed & (2 ** 64 - 1),
                                   _ptr(norms, torch.float32, nuq_num_buckets(v.numel(), bucket), "norms"),
                                   _ptr(q, torch.uint8, v.numel(), "q"), _stream()))


NORM_L2, NORM_LINF = 0, 1


def nuq_quantize_encode_table_batch(vs: list[torch.Tensor], bucket: int, levels, norm_kind: int, seeds: list[int],
                                    sync_stride: int, messages: list["Message"], workspace: torch.Tensor) -> None:
    K = len(vs)
    d = vs[0].numel()
    s = len(levels) - 2
    if any(v.numel() != d for v in vs) or len(seeds) != K or len(messages) != K:
        raise ValueError("K gradients of equal length, K seeds and K messages are needed")
    arr = lambda ts, dt=None: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    u64s = lambda xs: (ctypes.c_uint64 * K)(*[x & (2 ** 64 - 1) for x in xs])
    norms, offs, words, caps, sync = _message_arrays(messages, d, bucket, sync_stride)
    _check("nuq_quantize_encode_table_batch",
           _lib.nuq_quantize_encode_table_batch(K, arr(vs, torch.float32), u64s(seeds), d, bucket, s,
                                                _levels(levels, s), norm_kind, sync_stride, norms, offs, words, caps,
                                                sync, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                _stream()))


def nuq_decode_accumulate_table(messages: list[Message], d: int, bucket: int, levels, sync_stride: int, scale: float,
                                accumulate: bool, out: torch.Tensor) -> None:
    K = len(messages)
    s = len(levels) - 2
    norms, offs, words, lens, sync = _message_arrays(messages, d, bucket, sync_stride)
    if out.numel() != d:
        raise ValueError("out must hold d floats")
    _check("nuq_decode_accumulate_table",
           _lib.nuq_decode_accumulate_table(K, norms, offs, words, lens, sync, d, bucket, s, sync_stride,
                                            _levels(levels, s), float(scale), 1 if accumulate else 0,
                                            _ptr(out, torch.float32), _stream()))


# --------------------------------------------------------- fixed-width coding

def nuq_fixed_words(d: int, bucket: int, b: int) -> int:
    return _lib.nuq_fixed_words(d, bucket, b)


def nuq_pack_fixed(q: torch.Tensor, bucket: int, s: int, b: int, packed: torch.Tensor) -> None:
    _check("nuq_pack_fixed",
           _lib.nuq_pack_fixed(_ptr(q, torch.uint8), q.numel(), bucket, s, b, _ptr(packed, torch.int32), _stream()))


def nuq_quantize_pack_fixed_batch(vs: list[torch.Tensor], bucket: int, s: int, b: int, seeds: list[int],
                                  norms: list[torch.Tensor], packed: list[torch.Tensor]) -> None:
    K = len(vs)
    d = vs[0].numel()
    if any(v.numel() != d for v in vs) or len(seeds) != K or len(norms) != K or len(packed) != K:
        raise ValueError("K gradients of equal length, K seeds, K norm arrays and K packed arrays are needed")
    arr = lambda ts, dt: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    _check("nuq_quantize_pack_fixed_batch",
           _lib.nuq_quantize_pack_fixed_batch(K, arr(vs, torch.float32),
                                              (ctypes.c_uint64 * K)(*[x & (2 ** 64 - 1) for x in seeds]), d, bucket,
                                              s, b, arr(norms, torch.float32), arr(packed, torch.int32), _stream()))


def nuq_unpack_accumulate_fixed(norms: list[torch.Tensor], packed: list[torch.Tensor], d: int, bucket: int, s: int,
                                b: int, scale: float, accumulate: bool, out: torch.Tensor) -> None:
    K = len(norms)
    arr = lambda ts, dt: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    if out.numel() != d:
        raise ValueError("out must hold d floats")
    _check("nuq_unpack_accumulate_fixed",
           _lib.nuq_unpack_accumulate_fixed(K, arr(norms, torch.float32), arr(packed, torch.int32), d, bucket, s, b,
                                            float(scale), 1 if accumulate else 0, _ptr(out, torch.float32), _stream()))


def nuq_quantize_pack_fixed_table_batch(vs: list[torch.Tensor], bucket: int, levels, norm_kind: int, b: int,
                                        seeds: list[int], norms: list[torch.Tensor], packed: list[torch.Tensor]) -> None:
    K = len(vs)
    d = vs[0].numel()
    s = len(levels) - 2
    if any(v.numel() != d for v in vs) or len(seeds) != K or len(norms) != K or len(packed) != K:
        raise ValueError("K gradients of equal length, K seeds, K norm arrays and K packed arrays are needed")
    B, words = nuq_num_buckets(d, bucket), nuq_fixed_words(d, bucket, b)
    _check("nuq_quantize_pack_fixed_table_batch",
           _lib.nuq_quantize_pack_fixed_table_batch(
               K, (ctypes.c_void_p * K)(*[_ptr(v, torch.float32) for v in vs]),
               (ctypes.c_uint64 * K)(*[x & (2 ** 64 - 1) for x in seeds]), d, bucket, s, _levels(levels, s), norm_kind, b,
               (ctypes.c_void_p * K)(*[_ptr(t, torch.float32, B, "norms") for t in norms]),
               (ctypes.c_void_p * K)(*[_ptr(t, torch.int32, words, "packed") for t in packed]), _stream()))


def nuq_unpack_accumulate_fixed_table(norms: list[torch.Tensor], packed: list[torch.Tensor], d: int, bucket: int,
                                      levels, b: int, scale: float, accumulate: bool, out: torch.Tensor) -> None:
    K = len(norms)
    s = len(levels) - 2
    if out.numel() != d or len(packed) != K:
        raise ValueError("K norm arrays, K packed arrays and d floats of output are needed")
    B, words = nuq_num_buckets(d, bucket), nuq_fixed_words(d, bucket, b)
    _check("nuq_unpack_accumulate_fixed_table",
           _lib.nuq_unpack_accumulate_fixed_table(
               K, (ctypes.c_void_p * K)(*[_ptr(t, torch.float32, B, "norms") for t in norms]),
               (ctypes.c_void_p * K)(*[_ptr(t, torch.int32, words, "packed") for t in packed]), d, bucket, s,
               _levels(levels, s), b, float(scale), 1 if accumulate else 0, _ptr(out, torch.float32), _stream()))


# -------------------------------------------------------- Huffman-coded levels

def nuq_level_histogram(q: torch.Tensor, hist: torch.Tensor) -> None:
    """hist: int64[16] on the device, overwritten."""
    if hist.numel() < 16:
        raise ValueError("hist holds 16 counters")
    _check("nuq_level_histogram",
           _lib.nuq_level_histogram(_ptr(q, torch.uint8), q.numel(), _ptr(hist, torch.int64), _stream()))


def nuq_huffman_lengths(hist: list[int], s: int) -> list[int]:
    """Host arithmetic: code lengths of the level indices 0..s+1 from their counts."""
    if len(hist) != s + 2:
        raise ValueError("one count per level index 0..s+1")
    h = (ctypes.c_uint64 * (s + 2))(*[int(x) for x in hist])
    out = (ctypes.c_uint8 * (s + 2))()
    _check("nuq_huffman_lengths", _lib.nuq_huffman_lengths(h, s, out))
    return list(out)


def nuq_huffman_max_words(d: int, bucket: int) -> int:
    return _lib.nuq_huffman_max_words(d, bucket)


def nuq_encode_huffman_workspace_bytes(d: int, bucket: int) -> int:
    return _lib.nuq_encode_huffman_workspace_bytes(d, bucket)


def _lengths(lengths, s: int):
    if len(lengths) != s + 2:
        raise ValueError("one code length per level index 0..s+1")
    return (ctypes.c_uint8 * (s + 2))(*[int(x) for x in lengths])


def nuq_encode_huffman(q: torch.Tensor, bucket: int, s: int, sync_stride: int, lengths, bit_off: torch.Tensor,
                       words: torch.Tensor, sync: torch.Tensor | None, workspace: torch.Tensor) -> None:
    _check("nuq_encode_huffman",
           _lib.nuq_encode_huffman(_ptr(q, torch.uint8), q.numel(), bucket, s, sync_stride, _lengths(lengths, s),
                                   _ptr(bit_off, torch.int64), _ptr(words, torch.int32), words.numel(), _ptr(sync),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def nuq_decode_huffman(bit_off: torch.Tensor, words: torch.Tensor, sync: torch.Tensor | None, d: int, bucket: int,
                       s: int, sync_stride: int, lengths, q: torch.Tensor) -> None:
    if q.numel() != d:
        raise ValueError("q must hold d bytes")
    _check("nuq_decode_huffman",
           _lib.nuq_decode_huffman(_ptr(bit_off, torch.int64), _ptr(words, torch.int32), _ptr(sync), d, bucket, s,
                                   sync_stride, _lengths(lengths, s), _ptr(q, torch.uint8), _stream()))


def nuq_encode_huffman_batch_workspace_bytes(K: int, d: int, bucket: int, s: int) -> int:
    return _lib.nuq_encode_huffman_batch_workspace_bytes(K, d, bucket, s)


def nuq_quantize_encode_huffman_batch(vs: list[torch.Tensor], bucket: int, s: int, seeds: list[int], sync_stride: int,
                                      lengths, messages: list["Message"], workspace: torch.Tensor) -> None:
    K = len(vs)
    d = vs[0].numel()
    if any(v.numel() != d for v in vs) or len(seeds) != K or len(messages) != K:
        raise ValueError("K gradients of equal length, K seeds and K messages are needed")
    arr = lambda ts, dt=None: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    u64s = lambda xs: (ctypes.c_uint64 * K)(*[x & (2 ** 64 - 1) for x in xs])
    _check("nuq_quantize_encode_huffman_batch",
           _lib.nuq_quantize_encode_huffman_batch(K, arr(vs, torch.float32), u64s(seeds), d, bucket, s, sync_stride,
                                                  _lengths(lengths, s),
                                                  arr([m.norms for m in messages], torch.float32),
                                                  arr([m.bit_off for m in messages], torch.int64),
                                                  arr([m.words for m in messages], torch.int32),
                                                  u64s([m.words.numel() for m in messages]),
                                                  arr([m.sync for m in messages]), _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream()))


def nuq_decode_huffman_batch(messages: list[Message], d: int, bucket: int, s: int, sync_stride: int, lengths,
                             qs: list[torch.Tensor]) -> None:
    K = len(messages)
    if len(qs) != K or any(q.numel() != d for q in qs):
        raise ValueError("K messages and K byte arrays of d entries are needed")
    arr = lambda ts, dt=None: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    _check("nuq_decode_huffman_batch",
           _lib.nuq_decode_huffman_batch(K, arr([m.bit_off for m in messages], torch.int64),
                                         arr([m.words for m in messages], torch.int32),
                                         arr([m.sync for m in messages]), d, bucket, s, sync_stride,
                                         _lengths(lengths, s), arr(qs, torch.uint8), _stream()))


def nuq_decode_accumulate_huffman(messages: list[Message], d: int, bucket: int, s: int, sync_stride: int, lengths,
                                  scale: float, accumulate: bool, out: torch.Tensor) -> None:
    K = len(messages)
    norms, offs, words, lens, sync = _message_arrays(messages, d, bucket, sync_stride, huffman=True)
    if out.numel() != d:
        raise ValueError("out must hold d floats")
    _check("nuq_decode_accumulate_huffman",
           _lib.nuq_decode_accumulate_huffman(K, norms, offs, words, lens, sync, d, bucket, s, sync_stride,
                                              _lengths(lengths, s), float(scale), 1 if accumulate else 0,
                                              _ptr(out, torch.float32), _stream()))


def nuq_average_levels(norms: list[torch.Tensor], qs: list[torch.Tensor], d: int, bucket: int, s: int, scale: float,
                       accumulate: bool, out: torch.Tensor) -> None:
    K = len(norms)
    arr = lambda ts, dt: (ctypes.c_void_p * K)(*[_ptr(t, dt) for t in ts])
    if out.numel() != d or len(qs) != K:
        raise ValueError("K norm arrays, K byte arrays and d floats of output are needed")
    _check("nuq_average_levels",
           _lib.nuq_average_levels(K, arr(norms, torch.float32), arr(qs, torch.uint8), d, bucket, s, float(scale),
                                   1 if accumulate else 0, _ptr(out, torch.float32), _stream()))


# --------------------------------- parameter update and variance diagnostic

VARIANCE_WORKSPACE_BYTES = 16384


def nuq_momentum_step(w: torch.Tensor, yl: torch.Tensor, g: torch.Tensor, alpha: float, mu: float, l: float) -> None:
    d = w.numel()
    if yl.numel() != d or g.numel() != d:
        raise ValueError("w, yl and g hold d floats each")
    _check("nuq_momentum_step",
           _lib.nuq_momentum_step(_ptr(w, torch.float32), _ptr(yl, torch.float32), _ptr(g, torch.float32), d,
                                  float(alpha), float(mu), float(l), _stream()))


def nuq_decode_momentum_step(messages: list[Message], d: int, bucket: int, s: int, sync_stride: int, scale: float,
                             alpha: float, mu: float, l: float, w: torch.Tensor, yl: torch.Tensor) -> None:
    K = len(messages)
    norms, offs, words, lens, sync = _message_arrays(messages, d, bucket, sync_stride)
    if w.numel() != d or yl.numel() != d:
        raise ValueError("w and yl hold d floats each")
    _check("nuq_decode_momentum_step",
           _lib.nuq_decode_momentum_step(K, norms, offs, words, lens, sync, d, bucket,
                                         s, sync_stride, float(scale), float(alpha), float(mu), float(l),
                                         _ptr(w, torch.float32), _ptr(yl, torch.float32), _stream()))


def nuq_moments_accumulate(g: torch.Tensor, total: torch.Tensor, total_sq: torch.Tensor) -> None:
    d = g.numel()
    if total.numel() != d or total_sq.numel() != d:
        raise ValueError("the moment sums hold d doubles each")
    _check("nuq_moments_accumulate",
           _lib.nuq_moments_accumulate(_ptr(g, torch.float32), _ptr(total, torch.float64),
                                       _ptr(total_sq, torch.float64), d, _stream()))


def nuq_normalized_variance(total: torch.Tensor, total_sq: torch.Tensor, M: int, workspace: torch.Tensor,
                            out2: torch.Tensor) -> None:
    d = total.numel()
    if total_sq.numel() != d or out2.numel() != 2:
        raise ValueError("two moment sums of d doubles and two doubles of output are needed")
    _check("nuq_normalized_variance",
           _lib.nuq_normalized_variance(_ptr(total, torch.float64), _ptr(total_sq, torch.float64), d, M,
                                        _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _ptr(out2, torch.float64), _stream()))


def nuq_last_error_flags() -> int:
    flags = ctypes.c_uint32(0)
    _check("nuq_last_error_flags", _lib.nuq_last_error_flags(ctypes.byref(flags), _stream()))
    return flags.value


# ------------------------------------------------------------ measurement aid

T_NORMS, T_QUANTIZE, T_ENCODE, T_QUANTIZE_ENCODE, T_DECODE = 1, 2, 3, 4, 5


def nuq_timing_begin(max_launches: int) -> None:
    _check("nuq_timing_begin", _lib.nuq_timing_begin(max_launches))


def nuq_timing_collect(cap: int = 4096) -> list[tuple[int, float]]:
    """[(entry point id, milliseconds)] for the launches bracketed since nuq_timing_begin."""
    ms = (ctypes.c_float * cap)()
    entry = (ctypes.c_int32 * cap)()
    count = ctypes.c_uint32(0)
    _check("nuq_timing_collect", _lib.nuq_timing_collect(ms, entry, cap, ctypes.byref(count)))
    return [(entry[i], ms[i]) for i in range(count.value)]
