"""CPU oracle for the NUQSGD compression path.  TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``nuq_oracle.c`` (plain C, fp64, sequential).
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It imports nothing from the HIP package and the HIP
package imports nothing from here.

Each function names the passage of the paper its C counterpart follows; see
the header of ``nuq_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nuq_oracle.c")
_LIB = os.path.join(_HERE, "libnuq_oracle.so")

OK, EINVAL, ECAPACITY, EMALFORMED = 0, -1, -2, -5


def build(force: bool = False) -> str:
    """Compile nuq_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
             "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, u32, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        vp = ctypes.c_void_p
        L.nuqo_bucket_norms.argtypes = [vp, u64, u32, vp]
        L.nuqo_bucket_norms.restype = None
        L.nuqo_rng_key.argtypes = [u64, u64, vp, vp]
        L.nuqo_rng_key.restype = None
        L.nuqo_rng_u24.argtypes = [u32, u32, u32]
        L.nuqo_rng_u24.restype = u32
        L.nuqo_rng_fill.argtypes = [u64, u64, u32, vp]
        L.nuqo_rng_fill.restype = None
        L.nuqo_quantize_coord.argtypes = [ctypes.c_float, ctypes.c_float, i32, u32]
        L.nuqo_quantize_coord.restype = i32
        L.nuqo_quantize_coord_many.argtypes = [ctypes.c_float, ctypes.c_float, i32, vp, u64, vp]
        L.nuqo_quantize_coord_many.restype = None
        L.nuqo_level_histogram.argtypes = [ctypes.c_float, ctypes.c_float, i32, u32, u32, vp]
        L.nuqo_level_histogram.restype = None
        L.nuqo_quantize_given_u.argtypes = [vp, u64, u32, i32, vp, vp, vp]
        L.nuqo_quantize_given_u.restype = None
        L.nuqo_quantize.argtypes = [vp, u64, u32, i32, u64, vp, u64, vp]
        L.nuqo_quantize.restype = None
        L.nuqo_erc_encode.argtypes = [u64, ctypes.c_char_p]
        L.nuqo_erc_encode.restype = i32
        L.nuqo_erc_length.argtypes = [u64]
        L.nuqo_erc_length.restype = i32
        L.nuqo_erc_decode.argtypes = [vp, vp, u64, vp]
        L.nuqo_erc_decode.restype = i32
        L.nuqo_encode.argtypes = [vp, u64, u32, i32, u32, vp, vp, u64, vp]
        L.nuqo_encode.restype = i32
        L.nuqo_num_sync.argtypes = [u32, u32]
        L.nuqo_num_sync.restype = u64
        L.nuqo_decode_levels.argtypes = [vp, vp, u64, u32, i32, vp]
        L.nuqo_decode_levels.restype = i32
        L.nuqo_decode_average.argtypes = [u32, vp, vp, vp, u64, u32, i32, ctypes.c_double, i32, vp]
        L.nuqo_decode_average.restype = i32
        L.nuqo_fixed_words.argtypes = [u64, u32, u32]
        L.nuqo_fixed_words.restype = u64
        L.nuqo_pack_fixed.argtypes = [vp, u64, u32, i32, u32, vp]
        L.nuqo_pack_fixed.restype = i32
        L.nuqo_unpack_fixed.argtypes = [vp, u64, u32, i32, u32, vp]
        L.nuqo_unpack_fixed.restype = i32
        L.nuqo_huffman_lengths.argtypes = [vp, i32, vp]
        L.nuqo_huffman_lengths.restype = i32
        L.nuqo_huffman_codes.argtypes = [vp, i32, vp]
        L.nuqo_huffman_codes.restype = i32
        L.nuqo_encode_huffman.argtypes = [vp, u64, u32, i32, u32, vp, vp, vp, u64, vp]
        L.nuqo_encode_huffman.restype = i32
        L.nuqo_decode_huffman.argtypes = [vp, vp, u64, u32, i32, vp, vp]
        L.nuqo_decode_huffman.restype = i32
        L.nuqo_bucket_norms_linf.argtypes = [vp, u64, u32, vp]
        L.nuqo_bucket_norms_linf.restype = None
        L.nuqo_quantize_coord_table.argtypes = [ctypes.c_float, ctypes.c_float, i32, vp, u32]
        L.nuqo_quantize_coord_table.restype = i32
        L.nuqo_level_histogram_table.argtypes = [ctypes.c_float, ctypes.c_float, i32, vp, u32, u32, vp]
        L.nuqo_level_histogram_table.restype = None
        L.nuqo_quantize_table.argtypes = [vp, u64, u32, i32, vp, u64, vp, u64, vp]
        L.nuqo_quantize_table.restype = None
        L.nuqo_decode_average_table.argtypes = [u32, vp, vp, vp, u64, u32, i32, vp, ctypes.c_double, i32, vp]
        L.nuqo_decode_average_table.restype = i32
        _lib = L
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def num_buckets(d: int, bucket: int) -> int:
    return (d + bucket - 1) // bucket


SYNC_BLOCK = 2048


def sync_pieces(bucket: int, sync_stride: int) -> int:
    """Pieces per block of the decoder index: the smallest power of two >= min(bucket, 2048) / sync_stride."""
    need = (min(bucket, SYNC_BLOCK) + sync_stride - 1) // sync_stride
    P = 1
    while P < need:
        P *= 2
    return P


def num_sync(bucket: int, sync_stride: int) -> int:
    """Decoder index entries per bucket of an ERC message: blocks of 2048 coordinates times pieces per block."""
    return int(lib().nuqo_num_sync(bucket, sync_stride))


def num_sync_huffman(bucket: int, sync_stride: int) -> int:
    """Index entries per bucket of a Huffman-coded message: one per multiple of the stride inside the bucket."""
    return 0 if sync_stride == 0 else (bucket + sync_stride - 1) // sync_stride - 1


# ----------------------------------------------------------------- level set

def levels(s: int) -> list[Fraction]:
    """Sec. 3.1: (0, 2^-s, ..., 2^(s-1)/2^s, 1) as exact fractions, index j = 0..s+1."""
    return [Fraction(0)] + [Fraction(1, 2 ** (s + 1 - j)) for j in range(1, s + 2)]


# --------------------------------------------------------------------- norms

def bucket_norms(v: np.ndarray, bucket: int) -> np.ndarray:
    """Def. 1: Euclidean norm of each bucket, fp64."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    out = np.empty(num_buckets(v.size, bucket), dtype=np.float64)
    lib().nuqo_bucket_norms(_p(v), v.size, bucket, _p(out))
    return out


# ----------------------------------------------------------------------- rng

def rng_key(seed: int, bucket_index: int) -> tuple[int, int]:
    k0, k1 = ctypes.c_uint32(), ctypes.c_uint32()
    lib().nuqo_rng_key(seed & (2 ** 64 - 1), bucket_index, ctypes.addressof(k0), ctypes.addressof(k1))
    return k0.value, k1.value


def rng_fill(seed: int, d: int, bucket: int) -> np.ndarray:
    """The 24-bit draw of every coordinate of a d-vector cut into buckets."""
    u = np.empty(d, dtype=np.uint32)
    lib().nuqo_rng_fill(seed & (2 ** 64 - 1), d, bucket, _p(u))
    return u


# ----------------------------------------------------------------- quantizer

def quantize_coord(vi: float, norm: float, s: int, u24: int) -> int:
    """Def. 1 / App. B (h_case1), (h_case2): level index of one coordinate for draw u24."""
    return lib().nuqo_quantize_coord(float(np.float32(vi)), float(np.float32(norm)), s, u24)


def quantize_coord_many(vi: float, norm: float, s: int, u24: np.ndarray) -> np.ndarray:
    u24 = np.ascontiguousarray(u24, dtype=np.uint32)
    out = np.empty(u24.size, dtype=np.uint8)
    lib().nuqo_quantize_coord_many(float(np.float32(vi)), float(np.float32(norm)), s, _p(u24), u24.size, _p(out))
    return out


def level_histogram(vi: float, norm: float, s: int, u_begin: int = 0, u_end: int = 1 << 24) -> np.ndarray:
    """How many of the draws u in [u_begin, u_end) give each level index."""
    hist = np.zeros(16, dtype=np.uint64)
    lib().nuqo_level_histogram(float(np.float32(vi)), float(np.float32(norm)), s, u_begin, u_end, _p(hist))
    return hist


def quantize_given_u(v: np.ndarray, bucket: int, s: int, norms: np.ndarray, u24: np.ndarray) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float32)
    norms = np.ascontiguousarray(norms, dtype=np.float32)
    u24 = np.ascontiguousarray(u24, dtype=np.uint32)
    assert norms.size == num_buckets(v.size, bucket) and u24.size == v.size
    q = np.empty(v.size, dtype=np.uint8)
    lib().nuqo_quantize_given_u(_p(v), v.size, bucket, s, _p(norms), _p(u24), _p(q))
    return q


def quantize(v: np.ndarray, bucket: int, s: int, seed: int, norms: np.ndarray, first_bucket: int = 0) -> np.ndarray:
    """q[i] = level index | sign << 7, with the counter generator of the format text.
    `first_bucket` > 0 when v holds buckets first_bucket.. of a longer vector."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    norms = np.ascontiguousarray(norms, dtype=np.float32)
    assert norms.size == num_buckets(v.size, bucket)
    q = np.empty(v.size, dtype=np.uint8)
    lib().nuqo_quantize(_p(v), v.size, bucket, s, seed & (2 ** 64 - 1), _p(norms), first_bucket, _p(q))
    return q


def dequantize(q: np.ndarray, bucket: int, s: int, norms: np.ndarray) -> np.ndarray:
    """Def. 1: Q_s(v_i) = ||v|| * sign * l_j, fp64."""
    j = (q & 0x7F).astype(np.int64)
    h = np.where(j > 0, np.ldexp(1.0, j - 1 - s), 0.0)
    sign = np.where(q & 0x80, -1.0, 1.0)
    nrm = np.repeat(np.asarray(norms, dtype=np.float64), bucket)[: q.size]
    return nrm * sign * h


# ----------------------------------------------------------------------- ERC

def erc_encode(N: int) -> str:
    """App. A, Alg. 2 (encoder): the code of N as a '0'/'1' string."""
    buf = ctypes.create_string_buffer(96)
    n = lib().nuqo_erc_encode(N, buf)
    if n < 0:
        raise ValueError("ERC is defined for positive integers")
    return buf.raw[:n].decode()


def erc_length(N: int) -> int:
    return lib().nuqo_erc_length(N)


def bits_to_words(bits: str) -> np.ndarray:
    """Pack a '0'/'1' string MSB-first into uint32 words, zero padded."""
    nw = max(1, (len(bits) + 31) // 32)
    w = np.zeros(nw, dtype=np.uint32)
    for t, c in enumerate(bits):
        if c == "1":
            w[t >> 5] |= np.uint32(1 << (31 - (t & 31)))
    return w


def words_to_bits(words: np.ndarray, begin: int, end: int) -> str:
    return "".join("1" if (int(words[t >> 5]) >> (31 - (t & 31))) & 1 else "0" for t in range(begin, end))


def erc_decode(bits: str, pos: int = 0) -> tuple[int, int]:
    """App. A, Alg. 2 (decoder): returns (N, position after the code)."""
    w = bits_to_words(bits)
    p = ctypes.c_uint64(pos)
    n = ctypes.c_uint64(0)
    rc = lib().nuqo_erc_decode(_p(w), ctypes.addressof(p), len(bits), ctypes.addressof(n))
    if rc:
        raise ValueError("malformed ERC code")
    return n.value, p.value


# -------------------------------------------------------------------- ENCODE

def max_words(d: int, bucket: int, s: int) -> int:
    """Worst case: every coordinate nonzero at the top level, plus padding per bucket."""
    per = 2 + erc_length(s + 1)
    nb = num_buckets(d, bucket)
    return (d * per + 31) // 32 + nb


def encode(q: np.ndarray, bucket: int, s: int, sync_stride: int = 0, words_cap: int | None = None):
    """App. A ENCODE of every bucket. Returns (bit_off[B+1] u64, words u32 (trimmed), sync u32)."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    d = q.size
    nb = num_buckets(d, bucket)
    cap = max_words(d, bucket, s) if words_cap is None else words_cap
    bit_off = np.zeros(nb + 1, dtype=np.uint64)
    words = np.zeros(max(cap, 1), dtype=np.uint32)
    ns = num_sync(bucket, sync_stride)
    sync = np.zeros(max(nb * ns, 1), dtype=np.uint32)
    rc = lib().nuqo_encode(_p(q), d, bucket, s, sync_stride, _p(bit_off), _p(words), cap, _p(sync))
    if rc:
        raise RuntimeError("nuqo_encode failed: %d" % rc)
    nw = (int(bit_off[-1]) + 31) // 32
    return bit_off, words[:nw].copy(), sync[: nb * ns].copy()


# -------------------------------------------------------------------- DECODE

def decode_levels(bit_off: np.ndarray, words: np.ndarray, d: int, bucket: int, s: int) -> np.ndarray:
    """App. A DECODE back to q (level | sign << 7)."""
    bit_off = np.ascontiguousarray(bit_off, dtype=np.uint64)
    words = np.ascontiguousarray(words, dtype=np.uint32)
    if words.size == 0:
        words = np.zeros(1, dtype=np.uint32)
    q = np.empty(d, dtype=np.uint8)
    rc = lib().nuqo_decode_levels(_p(bit_off), _p(words), d, bucket, s, _p(q))
    if rc:
        raise ValueError("malformed stream: %d" % rc)
    return q


def decode_average(norms_list, bit_off_list, words_list, d: int, bucket: int, s: int,
                   scale: float, prior: np.ndarray | None = None) -> np.ndarray:
    """DECODE each worker and aggregate as in Alg. 1: [prior +] scale * sum_k Q_k, fp64."""
    K = len(norms_list)
    norms_list = [np.ascontiguousarray(a, dtype=np.float32) for a in norms_list]
    bit_off_list = [np.ascontiguousarray(a, dtype=np.uint64) for a in bit_off_list]
    words_list = [np.ascontiguousarray(a if a.size else np.zeros(1, np.uint32), dtype=np.uint32) for a in words_list]
    arr = lambda xs: (ctypes.c_void_p * K)(*[_p(x) for x in xs])
    out = np.zeros(d, dtype=np.float64) if prior is None else np.array(prior, dtype=np.float64)
    rc = lib().nuqo_decode_average(K, arr(norms_list), arr(bit_off_list), arr(words_list), d, bucket, s,
                                   float(scale), 0 if prior is None else 1, _p(out))
    if rc:
        raise ValueError("malformed stream: %d" % rc)
    return out


# ------------------------------------------------------- general level sets

def _table(lev, s: int) -> np.ndarray:
    lev = np.ascontiguousarray(lev, dtype=np.float32)
    assert lev.size == s + 2 and lev[0] == 0.0 and lev[-1] == 1.0 and np.all(np.diff(lev) > 0)
    return lev


def bucket_norms_linf(v: np.ndarray, bucket: int) -> np.ndarray:
    """Maximum norm of each bucket (QSGDinf's normalization)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    out = np.empty(num_buckets(v.size, bucket), dtype=np.float64)
    lib().nuqo_bucket_norms_linf(_p(v), v.size, bucket, _p(out))
    return out


def quantize_coord_table(vi: float, norm: float, lev, u24: int) -> int:
    """Def. 1 with an arbitrary level sequence (Sec. 4.1, generally spaced levels)."""
    s = len(lev) - 2
    lev = _table(lev, s)
    return lib().nuqo_quantize_coord_table(float(np.float32(vi)), float(np.float32(norm)), s, _p(lev), u24)


def level_histogram_table(vi: float, norm: float, lev, u_begin: int = 0, u_end: int = 1 << 24) -> np.ndarray:
    s = len(lev) - 2
    lev = _table(lev, s)
    hist = np.zeros(16, dtype=np.uint64)
    lib().nuqo_level_histogram_table(float(np.float32(vi)), float(np.float32(norm)), s, _p(lev), u_begin, u_end,
                                     _p(hist))
    return hist


def quantize_table(v: np.ndarray, bucket: int, lev, seed: int, norms: np.ndarray, first_bucket: int = 0) -> np.ndarray:
    """q[i] = level index | sign << 7 for the level sequence lev[0..s+1], counter generator as in quantize()."""
    s = len(lev) - 2
    lev = _table(lev, s)
    v = np.ascontiguousarray(v, dtype=np.float32)
    norms = np.ascontiguousarray(norms, dtype=np.float32)
    assert norms.size == num_buckets(v.size, bucket)
    q = np.empty(v.size, dtype=np.uint8)
    lib().nuqo_quantize_table(_p(v), v.size, bucket, s, _p(lev), seed & (2 ** 64 - 1), _p(norms), first_bucket, _p(q))
    return q


def dequantize_table(q: np.ndarray, bucket: int, lev, norms: np.ndarray) -> np.ndarray:
    """Def. 1: Q(v_i) = ||v|| * sign * l_j with l_j from the table, fp64."""
    lev = np.asarray(lev, dtype=np.float32).astype(np.float64)
    j = (q & 0x7F).astype(np.int64)
    sign = np.where(q & 0x80, -1.0, 1.0)
    nrm = np.repeat(np.asarray(norms, dtype=np.float64), bucket)[: q.size]
    return nrm * sign * lev[j]


def decode_average_table(norms_list, bit_off_list, words_list, d: int, bucket: int, lev,
                         scale: float, prior: np.ndarray | None = None) -> np.ndarray:
    """decode_average() with the table's level values."""
    s = len(lev) - 2
    lev = _table(lev, s)
    K = len(norms_list)
    norms_list = [np.ascontiguousarray(a, dtype=np.float32) for a in norms_list]
    bit_off_list = [np.ascontiguousarray(a, dtype=np.uint64) for a in bit_off_list]
    words_list = [np.ascontiguousarray(a if a.size else np.zeros(1, np.uint32), dtype=np.uint32) for a in words_list]
    arr = lambda xs: (ctypes.c_void_p * K)(*[_p(x) for x in xs])
    out = np.zeros(d, dtype=np.float64) if prior is None else np.array(prior, dtype=np.float64)
    rc = lib().nuqo_decode_average_table(K, arr(norms_list), arr(bit_off_list), arr(words_list), d, bucket, s,
                                         _p(lev), float(scale), 0 if prior is None else 1, _p(out))
    if rc:
        raise ValueError("malformed stream: %d" % rc)
    return out


# -------------------------------------------------------- fixed-width coding

def fixed_words(d: int, bucket: int, b: int) -> int:
    return lib().nuqo_fixed_words(d, bucket, b)


def pack_fixed(q: np.ndarray, bucket: int, s: int, b: int) -> np.ndarray:
    """Sec. 5's fixed-width variants: every coordinate's sign and level index in b bits (layout: design notes)."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    out = np.zeros(max(1, fixed_words(q.size, bucket, b)), dtype=np.uint32)
    rc = lib().nuqo_pack_fixed(_p(q), q.size, bucket, s, b, _p(out))
    if rc:
        raise ValueError("pack_fixed: %d" % rc)
    return out[: fixed_words(q.size, bucket, b)]


def unpack_fixed(packed: np.ndarray, d: int, bucket: int, s: int, b: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    assert packed.size >= fixed_words(d, bucket, b)
    q = np.empty(d, dtype=np.uint8)
    rc = lib().nuqo_unpack_fixed(_p(packed), d, bucket, s, b, _p(q))
    if rc:
        raise ValueError("unpack_fixed: %d" % rc)
    return q


def unpack_average_fixed(norms_list, packed_list, d: int, bucket: int, s: int, b: int, scale: float,
                         prior: np.ndarray | None = None) -> np.ndarray:
    """Unpack each worker, rebuild ||v|| * sign * l_j (Def. 1) and aggregate as in Alg. 1, fp64, workers in order."""
    out = np.zeros(d, dtype=np.float64)
    for norms, packed in zip(norms_list, packed_list):
        out += dequantize(unpack_fixed(packed, d, bucket, s, b), bucket, s, norms)
    out *= float(scale)
    return out if prior is None else np.asarray(prior, dtype=np.float64) + out


# ------------------------------------------------------ Huffman-coded levels

def level_histogram_of(q: np.ndarray, s: int) -> np.ndarray:
    """Counts of the level indices 0..s+1 in level|sign bytes."""
    return np.bincount(np.asarray(q, dtype=np.uint8) & 0x7F, minlength=s + 2)[: s + 2].astype(np.uint64)


def huffman_lengths(hist, s: int) -> np.ndarray:
    """Sec. 5 ("Efficient Encoding"): code lengths of the level indices from a sample's histogram."""
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    assert hist.size == s + 2
    out = np.zeros(s + 2, dtype=np.uint8)
    rc = lib().nuqo_huffman_lengths(_p(hist), s, _p(out))
    if rc:
        raise ValueError("huffman_lengths: %d" % rc)
    return out


def huffman_codes(lengths, s: int) -> list[str]:
    """Canonical codewords as '0'/'1' strings."""
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    codes = np.zeros(16, dtype=np.uint32)
    rc = lib().nuqo_huffman_codes(_p(lengths), s, _p(codes))
    if rc:
        raise ValueError("lengths do not describe a complete code")
    return [format(int(codes[j]), "0%db" % int(lengths[j])) for j in range(s + 2)]


def encode_huffman(q: np.ndarray, bucket: int, s: int, lengths, sync_stride: int = 0):
    """Codeword of every coordinate's level index, then its sign bit when nonzero.  Returns (bit_off, words, sync)."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    d = q.size
    nb = num_buckets(d, bucket)
    cap = (d * 16 + 31) // 32 + nb
    bit_off = np.zeros(nb + 1, dtype=np.uint64)
    words = np.zeros(max(cap, 1), dtype=np.uint32)
    ns = num_sync_huffman(bucket, sync_stride)
    sync = np.zeros(max(nb * ns, 1), dtype=np.uint32)
    rc = lib().nuqo_encode_huffman(_p(q), d, bucket, s, sync_stride, _p(lengths), _p(bit_off), _p(words), cap, _p(sync))
    if rc:
        raise RuntimeError("nuqo_encode_huffman failed: %d" % rc)
    return bit_off, words[: (int(bit_off[-1]) + 31) // 32].copy(), sync[: nb * ns].copy()


def decode_huffman(bit_off, words, d: int, bucket: int, s: int, lengths) -> np.ndarray:
    bit_off = np.ascontiguousarray(bit_off, dtype=np.uint64)
    words = np.ascontiguousarray(words if len(words) else np.zeros(1, np.uint32), dtype=np.uint32)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    q = np.empty(d, dtype=np.uint8)
    rc = lib().nuqo_decode_huffman(_p(bit_off), _p(words), d, bucket, s, _p(lengths), _p(q))
    if rc:
        raise ValueError("malformed stream: %d" % rc)
    return q


# ------------------------------------------------------- Alg. 1, the momentum rule, normalized variance
# Plain numpy in fp64; the quantizer, ENCODE and DECODE steps are the C functions above.

def momentum_step(w, yl_prev, g, alpha: float, mu: float, l: float):
    """Update rule of Sec. 4.2 ("NUQSGD with Momentum"): y = w - alpha g, y^l = w - l alpha g,
    w_next = y + mu (y^l - y^l_prev).  alpha, mu, l are taken at fp32 precision (what the caller can
    pass through the library).  Returns (w_next, y^l) in fp64; l = 0 is heavy ball, l = 1 Nesterov."""
    w = np.asarray(w, dtype=np.float64)
    yl_prev = np.asarray(yl_prev, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    alpha, mu, l = (float(np.float32(x)) for x in (alpha, mu, l))
    y = w - alpha * g
    yl = w - (l * alpha) * g
    return y + mu * (yl - yl_prev), yl


def normalized_variance(samples) -> float:
    """Mean normalized variance (App. J, "Additional Experiments"): over M draws of a gradient estimate (rows), the mean over
    coordinates of the variance across draws divided by the mean over coordinates of the second moment
    across draws.  Variance = mean squared deviation from the mean of the M draws."""
    x = np.asarray(samples, dtype=np.float64)
    mean = x.mean(axis=0)
    var = ((x - mean) ** 2).mean(axis=0)
    second = (x * x).mean(axis=0)
    return float(var.mean() / second.mean())


def step_seed(seed0: int, t: int, K: int, k: int) -> int:
    """Seed of worker k's quantizer at step t: every (t, k) draws from its own stream."""
    return (seed0 + t * K + k) & (2 ** 64 - 1)


def aggregate_quantized(grads, bucket: int, s: int, sync_stride: int, seeds) -> np.ndarray:
    """Inner loops of Alg. 1 for one step: every worker quantizes and ENCODEs its gradient, every
    receiver DECODEs the K messages; returns (1/K) sum_k Q(g_k) in fp64."""
    K = len(grads)
    d = grads[0].size
    norms_l, off_l, words_l = [], [], []
    for k in range(K):
        g = np.ascontiguousarray(grads[k], dtype=np.float32)
        norms = bucket_norms(g, bucket)
        q = quantize(g, bucket, s, seeds[k], norms)
        bit_off, words, _ = encode(q, bucket, s, sync_stride)
        norms_l.append(norms); off_l.append(bit_off); words_l.append(words)
    return decode_average(norms_l, off_l, words_l, d, bucket, s, 1.0 / K)


def data_parallel_sgd(w0, grad_fn, K: int, T: int, alpha: float, bucket: int, s: int, sync_stride: int = 0,
                      seed0: int = 0, mu: float = 0.0, l: float = 0.0) -> np.ndarray:
    """Alg. 1 with Omega = R^d (no projection): for t < T, worker k computes g = grad_fn(w_t, t, k)
    (fp32, length d), the K gradients are quantized, coded, decoded and averaged, and the parameters
    move by the plain rule w - alpha * average (mu == 0) or by the momentum rule.  Parameters and y^l are
    held in fp32 between steps, as the library's caller holds them.  Returns w_T (fp32)."""
    w = np.array(w0, dtype=np.float32)
    yl = w.copy()
    a32 = float(np.float32(alpha))
    for t in range(T):
        grads = [np.asarray(grad_fn(w, t, k), dtype=np.float32) for k in range(K)]
        avg = aggregate_quantized(grads, bucket, s, sync_stride, [step_seed(seed0, t, K, k) for k in range(K)])
        if mu == 0.0:
            w = (w.astype(np.float64) - a32 * avg).astype(np.float32)
        else:
            w_next, yl_next = momentum_step(w, yl, avg.astype(np.float32), alpha, mu, l)
            w, yl = w_next.astype(np.float32), yl_next.astype(np.float32)
    return w
