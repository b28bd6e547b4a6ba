"""CPU oracle for natural compression / natural dithering (test infrastructure only).

A ctypes view of oracle/natcomp_oracle.c with numpy arrays in and out.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the GPU library never does, and this package never imports the GPU one.
"""
import ctypes
import math
import os

import numpy as np

from . import build as _build

_lib = None

_u8p = ctypes.POINTER(ctypes.c_uint8)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_u32, _u64, _f64 = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_double

DOMAIN_NAT = 0
DOMAIN_DITHER = 1


def lib():
    """Load liboracle.so, compiling it first when it is missing or stale."""
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.orc_clip_encode.argtypes = [_f32p, _u64, _u64, _u32, _u64, _u8p]
        L.orc_clip_encode.restype = None
        L.orc_clip_decode.argtypes = [_u8p, _u64, _f32p]
        L.orc_clip_decode.restype = None
        L.orc_clip_aggregate.argtypes = [_u8p, _u64, _u32, _u64, _u64, _u32, _u64, _i64p, _u8p, _u8p]
        L.orc_clip_aggregate.restype = None
        L.orc_clip_round.argtypes = [ctypes.c_int64, _u32]
        L.orc_clip_round.restype = _u32
        L.orc_clip_count_up.argtypes = [ctypes.c_int64]
        L.orc_clip_count_up.restype = _u64
        L.orc_find_word_below.argtypes = [_u64, _u32, _u32, _u64, _u64, _u32]
        L.orc_find_word_below.restype = ctypes.c_int64
        L.orc_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_random_word.argtypes = [_u64, _u32, _u32, _u64]
        L.orc_random_word.restype = _u32
        L.orc_dither_word.argtypes = [_u64, _u32, _u64]
        L.orc_dither_word.restype = _u32
        L.orc_dither_word_of_call.argtypes = [_u32p, _u32]
        L.orc_dither_word_of_call.restype = _u32
        L.orc_nat_round.argtypes = [_u32, _u32]
        L.orc_nat_round.restype = _u32
        L.orc_nat_count_up.argtypes = [_u32]
        L.orc_nat_count_up.restype = _u64
        L.orc_nat_encode.argtypes = [_f32p, _u64, _u64, _u32, _u64, _u8p, _u8p]
        L.orc_nat_encode.restype = None
        L.orc_nat_decode.argtypes = [_u8p, _u8p, _u64, _f32p]
        L.orc_nat_decode.restype = None
        L.orc_pnorm.argtypes = [_f32p, _u64, _f64]
        L.orc_pnorm.restype = _f64
        L.orc_segment_count.argtypes = [_u64, _u64p, _u32, _u32]
        L.orc_segment_count.restype = _u64
        L.orc_pnorm_segments.argtypes = [_f32p, _u64, _u64p, _u32, _u32, _f64, _f64p]
        L.orc_pnorm_segments.restype = None
        L.orc_dither_level.argtypes = [_u32, _u32, _u32]
        L.orc_dither_level.restype = _u32
        L.orc_dither_count.argtypes = [_u32, _u32, _u32]
        L.orc_dither_count.restype = _u64
        L.orc_dither_inv_norm.argtypes = [ctypes.c_float]
        L.orc_dither_inv_norm.restype = ctypes.c_float
        L.orc_dither_y_bits.argtypes = [ctypes.c_float, ctypes.c_float]
        L.orc_dither_y_bits.restype = _u32
        L.orc_dither_code_bytes.argtypes = [_u64, _u32]
        L.orc_dither_code_bytes.restype = _u64
        L.orc_dither_sign_bytes.argtypes = [_u64, _u32]
        L.orc_dither_sign_bytes.restype = _u64
        L.orc_dither_encode.argtypes = [_f32p, _u64, _u64p, _u32, _u32, _u32, _f32p, _u64, _u32, _u64, _u8p, _u8p]
        L.orc_dither_encode.restype = None
        L.orc_dither_decode.argtypes = [_f32p, _u8p, _u8p, _u64, _u64p, _u32, _u32, _u32, _f32p]
        L.orc_dither_decode.restype = None
        L.orc_aggregate_nat.argtypes = [_u8p, _u64, _u8p, _u64, _u32, _u64, _f64p, _f32p, _f64p]
        L.orc_aggregate_nat.restype = None
        L.orc_aggregate_dither.argtypes = [_f32p, _u64, _u8p, _u64, _u8p, _u64, _u32, _u64, _u64p, _u32, _u32, _u32,
                                           _f64p, _f32p, _f64p]
        L.orc_aggregate_dither.restype = None
        L.orc_sparse_index.argtypes = [_u64, _u64, _u32, _u64]
        L.orc_sparse_index.restype = _u64
        L.orc_sparse_nat_encode.argtypes = [_f32p, _u64, _u64, ctypes.c_float, _u64, _u32, _u32p, _u8p, _u8p]
        L.orc_sparse_nat_encode.restype = None
        L.orc_sparse_nat_aggregate.argtypes = [_u32p, _u64, _u8p, _u64, _u8p, _u64, _u32, _u64, _u64, _f32p, _f64p, _f64p]
        L.orc_sparse_nat_aggregate.restype = None
        L.orc_master_nat.argtypes = [_u8p, _u64, _u8p, _u64, _u32, _u64, _u64, _u32, _u64, _f32p, _u8p, _u8p]
        L.orc_master_nat.restype = None
        L.orc_norm_compress.argtypes = [_f32p, _u64, _u64, _u32, _u8p, _f32p]
        L.orc_norm_compress.restype = None
        L.orc_sta_level.argtypes = [ctypes.c_float, _u32, _u32]
        L.orc_sta_level.restype = _u32
        L.orc_sta_count.argtypes = [ctypes.c_float, _u32, _u32]
        L.orc_sta_count.restype = _u64
        L.orc_sta_encode.argtypes = L.orc_dither_encode.argtypes
        L.orc_sta_encode.restype = None
        L.orc_sta_decode.argtypes = L.orc_dither_decode.argtypes
        L.orc_sta_decode.restype = None
        L.orc_threads.argtypes = []
        L.orc_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def threads():
    """OpenMP threads the element-parallel loops use."""
    return int(lib().orc_threads())


def set_threads(n):
    """Sets the number of OpenMP threads of the element-parallel loops (timing only: results do not depend on it)."""
    lib().orc_set_threads(int(n))


def _ptr(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _segs(d, offsets, bucket):
    """(offsets array or None, num_segments, bucket, count) after validation."""
    if offsets is not None:
        offsets = _c(offsets, np.uint64)
        assert offsets.ndim == 1 and offsets.size >= 2
        assert int(offsets[0]) == 0 and int(offsets[-1]) == d
        assert np.all(offsets[1:] >= offsets[:-1])
        return offsets, offsets.size - 1, 0, offsets.size - 1
    bucket = int(bucket or 0)
    return None, 0, bucket, (-(-d // bucket) if bucket else 1)


# ---------------------------------------------------------------- random words
def philox4x32_10(ctr, key):
    c = _c(ctr, np.uint32)
    k = _c(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_ptr(c, _u32p), _ptr(k, _u32p), _ptr(out, _u32p))
    return out


def random_word(seed, worker, domain, g):
    return int(lib().orc_random_word(seed, worker, domain, g))


# ------------------------------------------------------------ natural compression
def dither_word(seed, worker, g):
    """The 32-bit word the dithering operators draw for global element g (one call per 8 elements)."""
    return int(lib().orc_dither_word(seed, worker, g))


def dither_word_of_call(words, j):
    """Word of element j (0..7) of a group, given the four output words of the group's call."""
    w = np.asarray(words, np.uint32)
    return int(lib().orc_dither_word_of_call(_ptr(w, _u32p), j))


def nat_round(u_bits, r):
    """New exponent field of the binary32 value with bits u_bits, given the uniform word r."""
    return int(lib().orc_nat_round(u_bits, r))


def nat_count_up(u_bits):
    """Number of words r in [0, 2^32) for which the exponent is incremented."""
    return int(lib().orc_nat_count_up(u_bits))


def nat_encode(x, seed, worker=0, index_offset=0):
    x = _c(x, np.float32)
    d = x.size
    exp = np.zeros(d, np.uint8)
    sign = np.zeros((d + 7) // 8, np.uint8)
    lib().orc_nat_encode(_ptr(x, _f32p), d, seed, worker, index_offset, _ptr(exp, _u8p), _ptr(sign, _u8p))
    return exp, sign


def nat_decode(exp, sign, d):
    exp = _c(exp, np.uint8)
    sign = _c(sign, np.uint8)
    assert exp.size >= d and sign.size >= (d + 7) // 8
    out = np.zeros(d, np.float32)
    lib().orc_nat_decode(_ptr(exp, _u8p), _ptr(sign, _u8p), d, _ptr(out, _f32p))
    return out


# --------------------------------------------------------------------- norms
def pnorm(x, p):
    x = _c(x, np.float32)
    assert p in (1, 2, math.inf)
    return float(lib().orc_pnorm(_ptr(x, _f32p), x.size, float(p)))


def pnorm_segments(x, p, offsets=None, bucket=0):
    """float64 norm of every segment."""
    x = _c(x, np.float32)
    assert p in (1, 2, math.inf)
    off, nseg, bucket, count = _segs(x.size, offsets, bucket)
    out = np.zeros(count, np.float64)
    lib().orc_pnorm_segments(_ptr(x, _f32p), x.size, _ptr(off, _u64p), nseg, bucket, float(p), _ptr(out, _f64p))
    return out


# ------------------------------------------------------------ natural dithering
def dither_level(y_bits, s, r):
    assert 1 <= s <= 127
    return int(lib().orc_dither_level(y_bits, s, r))


def dither_count(y_bits, s, code):
    assert 1 <= s <= 127
    return int(lib().orc_dither_count(y_bits, s, code))


def dither_inv_norm(norm):
    return float(lib().orc_dither_inv_norm(np.float32(norm)))


def dither_y_bits(x, inv):
    return int(lib().orc_dither_y_bits(np.float32(x), np.float32(inv)))


def dither_code_bytes(d, s):
    return int(lib().orc_dither_code_bytes(d, s))


def dither_sign_bytes(d, s):
    return int(lib().orc_dither_sign_bytes(d, s))


def dither_encode(x, s, norms, seed, worker=0, index_offset=0, offsets=None, bucket=0):
    """Encode with the given binary32 segment norms; returns (code plane, sign plane)."""
    assert 1 <= s <= 127
    x = _c(x, np.float32)
    d = x.size
    off, nseg, bucket, count = _segs(d, offsets, bucket)
    norms = _c(norms, np.float32)
    assert norms.size == count
    code = np.zeros(dither_code_bytes(d, s), np.uint8)
    sign = np.zeros(max(dither_sign_bytes(d, s), 1), np.uint8)
    lib().orc_dither_encode(_ptr(x, _f32p), d, _ptr(off, _u64p), nseg, bucket, s, _ptr(norms, _f32p), seed, worker,
                            index_offset, _ptr(code, _u8p), _ptr(sign, _u8p))
    return code, sign[:dither_sign_bytes(d, s)]


def dither_decode(norms, code, sign, d, s, offsets=None, bucket=0):
    assert 1 <= s <= 127
    off, nseg, bucket, count = _segs(d, offsets, bucket)
    norms = _c(norms, np.float32)
    assert norms.size == count
    code = _c(code, np.uint8)
    assert code.size >= dither_code_bytes(d, s)
    sign = _c(sign, np.uint8) if dither_sign_bytes(d, s) else None
    out = np.zeros(d, np.float32)
    lib().orc_dither_decode(_ptr(norms, _f32p), _ptr(code, _u8p), _ptr(sign, _u8p), d, _ptr(off, _u64p), nseg, bucket,
                            s, _ptr(out, _f32p))
    return out


# ------------------------------------------------------------ sum over workers
def aggregate_nat(exp, sign, d):
    """exp: (n, >=d) uint8, sign: (n, >=ceil(d/8)) uint8 -> (sum in double, left-to-right binary32 sum, sum of |.|)."""
    exp = _c(exp, np.uint8)
    sign = _c(sign, np.uint8)
    n = exp.shape[0]
    assert exp.ndim == 2 and sign.ndim == 2 and sign.shape[0] == n
    assert exp.shape[1] >= d and sign.shape[1] >= (d + 7) // 8
    o64 = np.zeros(d, np.float64)
    o32 = np.zeros(d, np.float32)
    oa = np.zeros(d, np.float64)
    lib().orc_aggregate_nat(_ptr(exp, _u8p), exp.shape[1], _ptr(sign, _u8p), sign.shape[1], n, d, _ptr(o64, _f64p),
                            _ptr(o32, _f32p), _ptr(oa, _f64p))
    return o64, o32, oa


def aggregate_dither(norms, code, sign, d, s, offsets=None, bucket=0):
    """norms: (n, segments) float32, code: (n, bytes) uint8, sign: (n, bytes) uint8 or None."""
    assert 1 <= s <= 127
    off, nseg, bucket, count = _segs(d, offsets, bucket)
    norms = _c(norms, np.float32)
    code = _c(code, np.uint8)
    n = code.shape[0]
    assert norms.shape == (n, count)
    assert code.shape[1] >= dither_code_bytes(d, s)
    if dither_sign_bytes(d, s):
        sign = _c(sign, np.uint8)
        assert sign.shape[0] == n and sign.shape[1] >= dither_sign_bytes(d, s)
        sstride = sign.shape[1]
    else:
        sign, sstride = None, 0
    o64 = np.zeros(d, np.float64)
    o32 = np.zeros(d, np.float32)
    oa = np.zeros(d, np.float64)
    lib().orc_aggregate_dither(_ptr(norms, _f32p), norms.shape[1], _ptr(code, _u8p), code.shape[1], _ptr(sign, _u8p),
                               sstride, n, d, _ptr(off, _u64p), nseg, bucket, s, _ptr(o64, _f64p), _ptr(o32, _f32p),
                               _ptr(oa, _f64p))
    return o64, o32, oa


# ------------------------------------------------ random sparsification composed with C_nat
DOMAIN_SPARSE = 2


def sparse_index(d, seed, worker, j):
    """pi(j): the j-th kept coordinate of the keyed permutation of [0, d)."""
    assert 0 <= j < d <= 1 << 32
    return int(lib().orc_sparse_index(d, seed, worker, j))


def sparse_nat_encode(x, k, scale, seed, worker=0):
    """(indices uint32[k], exponent plane uint8[k], sign plane uint8[ceil(k/8)])."""
    x = _c(x, np.float32)
    d = x.size
    assert 0 < k <= d <= 1 << 32
    idx = np.zeros(k, np.uint32)
    exp = np.zeros(k, np.uint8)
    sign = np.zeros((k + 7) // 8, np.uint8)
    lib().orc_sparse_nat_encode(_ptr(x, _f32p), d, k, np.float32(scale), seed, worker, _ptr(idx, _u32p),
                                _ptr(exp, _u8p), _ptr(sign, _u8p))
    return idx, exp, sign


def sparse_nat_aggregate(idx, exp, sign, k, d, only32=False):
    """idx (n, >=k) uint32, exp (n, >=k) uint8, sign (n, >=ceil(k/8)) uint8 -> (binary32 sum in worker
    order, double sum, sum of magnitudes), dense vectors of length d (only32: the last two are None)."""
    idx = _c(idx, np.uint32)
    exp = _c(exp, np.uint8)
    sign = _c(sign, np.uint8)
    n = idx.shape[0]
    assert idx.ndim == 2 and exp.shape[0] == n and sign.shape[0] == n
    assert idx.shape[1] >= k and exp.shape[1] >= k and sign.shape[1] >= (k + 7) // 8
    assert int(idx[:, :k].max()) < d
    o32 = np.zeros(d, np.float32)
    o64 = None if only32 else np.zeros(d, np.float64)
    oa = None if only32 else np.zeros(d, np.float64)
    lib().orc_sparse_nat_aggregate(_ptr(idx, _u32p), idx.shape[1], _ptr(exp, _u8p), exp.shape[1], _ptr(sign, _u8p),
                                   sign.shape[1], n, k, d, _ptr(o32, _f32p), _ptr(o64, _f64p), _ptr(oa, _f64p))
    return o32, o64, oa


# ------------------------------------------------------------------ master-side compression
DOMAIN_MASTER = 3


def master_nat(exp, sign, d, seed, master=0, index_offset=0):
    """Sum of the n decoded C_nat streams (binary32, worker order), then C_nat of the sum with the
    master's stream: returns (sum, exponent plane, sign plane)."""
    exp = _c(exp, np.uint8)
    sign = _c(sign, np.uint8)
    n = exp.shape[0]
    assert exp.ndim == 2 and sign.ndim == 2 and sign.shape[0] == n
    assert exp.shape[1] >= d and sign.shape[1] >= (d + 7) // 8
    total = np.zeros(d, np.float32)
    e = np.zeros(d, np.uint8)
    s = np.zeros((d + 7) // 8, np.uint8)
    lib().orc_master_nat(_ptr(exp, _u8p), exp.shape[1], _ptr(sign, _u8p), sign.shape[1], n, d, seed, master,
                         index_offset, _ptr(total, _f32p), _ptr(e, _u8p), _ptr(s, _u8p))
    return total, e, s


# ------------------------------------------------------------------ compressed norm
DOMAIN_NORM = 4


def norm_compress(norms, seed, worker=0):
    """C_nat of every (non-negative) norm: (exponent bytes, the powers of two they stand for)."""
    norms = _c(norms, np.float32)
    e = np.zeros(norms.size, np.uint8)
    q = np.zeros(norms.size, np.float32)
    lib().orc_norm_compress(_ptr(norms, _f32p), norms.size, seed, worker, _ptr(e, _u8p), _ptr(q, _f32p))
    return e, q


# ------------------------------------------------------------------ standard dithering
def sta_level(y, s, r):
    assert 1 <= s <= 255
    return int(lib().orc_sta_level(np.float32(y), s, r))


def sta_count(y, s, code):
    assert 1 <= s <= 255
    return int(lib().orc_sta_count(np.float32(y), s, code))


def sta_encode(x, s, norms, seed, worker=0, index_offset=0, offsets=None, bucket=0):
    assert 1 <= s <= 255
    x = _c(x, np.float32)
    d = x.size
    off, nseg, bucket, count = _segs(d, offsets, bucket)
    norms = _c(norms, np.float32)
    assert norms.size == count
    code = np.zeros(dither_code_bytes(d, s), np.uint8)
    sign = np.zeros(max(dither_sign_bytes(d, s), 1), np.uint8)
    lib().orc_sta_encode(_ptr(x, _f32p), d, _ptr(off, _u64p), nseg, bucket, s, _ptr(norms, _f32p), seed, worker,
                         index_offset, _ptr(code, _u8p), _ptr(sign, _u8p))
    return code, sign[:dither_sign_bytes(d, s)]


def sta_decode(norms, code, sign, d, s, offsets=None, bucket=0):
    assert 1 <= s <= 255
    off, nseg, bucket, count = _segs(d, offsets, bucket)
    norms = _c(norms, np.float32)
    code = _c(code, np.uint8)
    sign = _c(sign, np.uint8) if dither_sign_bytes(d, s) else None
    out = np.zeros(d, np.float32)
    lib().orc_sta_decode(_ptr(norms, _f32p), _ptr(code, _u8p), _ptr(sign, _u8p), d, _ptr(off, _u64p), nseg, bucket,
                         s, _ptr(out, _f32p))
    return out


# ------------------------------------------------------------------ clipped 8-bit format, integer aggregation
def clip_encode(x, seed, worker=0, index_offset=0):
    """One byte per element: sign << 7 | zero flag << 6 | clip(exponent of C_nat(x), -50, 10) + 50."""
    x = _c(x, np.float32)
    out = np.zeros(x.size, np.uint8)
    lib().orc_clip_encode(_ptr(x, _f32p), x.size, seed, worker, index_offset, _ptr(out, _u8p))
    return out


def clip_decode(code):
    code = _c(code, np.uint8)
    out = np.zeros(code.size, np.float32)
    lib().orc_clip_decode(_ptr(code, _u8p), code.size, _ptr(out, _f32p))
    return out


def clip_aggregate(code, d, seed, master=0, index_offset=0):
    """Integer sum (units of 2^-50) of the n byte streams and C_nat of it: (sums int64, exponent plane,
    sign plane)."""
    code = _c(code, np.uint8)
    assert code.ndim == 2 and code.shape[1] >= d
    total = np.zeros(d, np.int64)
    e = np.zeros(d, np.uint8)
    s = np.zeros((d + 7) // 8, np.uint8)
    lib().orc_clip_aggregate(_ptr(code, _u8p), code.shape[1], code.shape[0], d, seed, master, index_offset,
                             _ptr(total, _i64p), _ptr(e, _u8p), _ptr(s, _u8p))
    return total, e, s


def clip_round(total, r):
    """Exponent field of C_nat(total * 2^-50) for the word r (0 for total = 0)."""
    return lib().orc_clip_round(total, r)


def clip_count_up(total):
    """Number of words r, out of 2^32, that round |total| up to the next power of two."""
    return lib().orc_clip_count_up(total)


def find_word_below(seed, worker, domain, start, count, bound):
    """First global index in [start, start + count) whose random word is below `bound`, or -1."""
    return lib().orc_find_word_below(seed, worker, domain, start, count, bound)
