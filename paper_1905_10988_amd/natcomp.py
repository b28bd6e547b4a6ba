"""ctypes binding of libnatcomp's C ABI (include/natcomp.h).

Argument marshalling only: every function checks tensor device/dtype/contiguity, passes
raw device pointers, sizes and the current HIP stream to the entry point of the same
name, and raises on a non-zero status.  PyTorch is used for device memory and streams
and for nothing else.  There is no fallback: if libnatcomp.so has not been built the
first call raises.
"""
import ctypes
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnatcomp.so")

NC_KIND_NAT = 0
NC_KIND_DITHER = 1
NC_KIND_DITHER_STA = 2
NC_KIND_DITHER_NORM8 = 3

_vp, _u32, _u64, _sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t


class AggDesc(ctypes.Structure):
    """Mirror of nc_agg_desc."""
    _fields_ = [
        ("kind", ctypes.c_int32), ("n", _u32), ("d", _u64), ("s", _u32), ("bucket", _u32),
        ("code", _vp), ("code_stride", _sz),
        ("sign", _vp), ("sign_stride", _sz),
        ("norms", _vp), ("norm_stride", _sz),
        ("seg_offsets", _vp), ("num_segments", _u32), ("reserved", _u32),
    ]


class NatcompError(RuntimeError):
    pass


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise NatcompError(f"{LIB_PATH} is missing: run `python -m paper_1905_10988_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        L.nc_status_string.argtypes = [ctypes.c_int]
        L.nc_status_string.restype = ctypes.c_char_p
        for name, args in {
            "nc_nat_exp_bytes": [_u64], "nc_sign_bytes": [_u64],
            "nc_dither_code_bytes": [_u64, _u32], "nc_dither_sign_bytes": [_u64, _u32],
            "nc_plane_stride": [_sz],
            "nc_dither_workspace_bytes": [_u64, _u32, _u32, ctypes.c_int],
        }.items():
            getattr(L, name).argtypes = args
            getattr(L, name).restype = _sz
        L.nc_segment_count.argtypes = [_u64, _u32, _u32, ctypes.c_int]
        L.nc_segment_count.restype = _u64
        L.nc_nat_encode.argtypes = [_vp, _u64, _u64, _u32, _u64, _vp, _vp, _vp]
        L.nc_nat_encode_batch.argtypes = [_vp, _sz, _u32, _u64, _u64, _u32, _u64, _vp, _sz, _vp, _sz, _vp]
        L.nc_nat_decode.argtypes = [_vp, _vp, _u64, _vp, _vp]
        L.nc_dither_encode.argtypes = [_vp, _u64, _vp, _u32, _u32, ctypes.c_float, _u32, _u64, _u32, _u64,
                                       _vp, _vp, _vp, _vp, _sz, _vp]
        L.nc_dither_encode_static.argtypes = [_vp, _u64, _vp, _u32, _u32, ctypes.c_float, _u32, _u64, _u32, _u64,
                                              _vp, _vp, _vp, _vp]
        L.nc_dither_encode_static.restype = ctypes.c_int
        L.nc_static_scratch_init.argtypes = []
        L.nc_static_scratch_init.restype = ctypes.c_int
        L.nc_static_scratch_bytes.argtypes = []
        L.nc_static_scratch_bytes.restype = _sz
        L.nc_dither_decode.argtypes = [_vp, _vp, _vp, _u64, _vp, _u32, _u32, _u32, _vp, _vp]
        L.nc_dither_sta_encode.argtypes = L.nc_dither_encode.argtypes
        L.nc_dither_sta_decode.argtypes = L.nc_dither_decode.argtypes
        L.nc_dither_decode_norm8.argtypes = L.nc_dither_decode.argtypes
        L.nc_dither_decode_norm8.restype = ctypes.c_int
        L.nc_dither_sta_encode.restype = ctypes.c_int
        L.nc_dither_sta_decode.restype = ctypes.c_int
        L.nc_aggregate_sum.argtypes = [ctypes.POINTER(AggDesc), _vp, _vp]
        L.nc_sparse_nat_encode.argtypes = [_vp, _u64, _u64, ctypes.c_float, _u64, _u32, _vp, _vp, _vp, _vp]
        L.nc_sparse_nat_encode_batch.argtypes = [_vp, _sz, _u32, _u64, _u64, ctypes.c_float, _u64, _u32, _vp, _sz,
                                                 _vp, _sz, _vp, _sz, _vp]
        L.nc_sparse_nat_aggregate.argtypes = [_vp, _sz, _vp, _sz, _vp, _sz, _u32, _u64, _u64, _vp, _vp]
        L.nc_sparse_nat_aggregate_ws.argtypes = [_vp, _sz, _vp, _sz, _vp, _sz, _u32, _u64, _u64, _vp, _vp, _sz, _vp]
        L.nc_sparse_nat_aggregate_ws.restype = ctypes.c_int
        L.nc_sparse_aggregate_workspace_bytes.argtypes = [_u32, _u64, _u64]
        L.nc_sparse_aggregate_workspace_bytes.restype = _sz
        L.nc_norm_compress.argtypes = [_vp, _u64, _u64, _u32, _vp, _vp, _vp]
        L.nc_norm_compress.restype = ctypes.c_int
        L.nc_master_nat.argtypes = [ctypes.POINTER(AggDesc), _u64, _u32, _u64, _vp, _vp, _vp]
        L.nc_nat_clip_encode.argtypes = [_vp, ctypes.c_size_t, _u32, _u64, _u64, _u32, _u64, _vp, ctypes.c_size_t, _vp]
        L.nc_nat_clip_encode.restype = ctypes.c_int
        L.nc_nat_clip_decode.argtypes = [_vp, _u64, _vp, _vp]
        L.nc_nat_clip_decode.restype = ctypes.c_int
        L.nc_clip_aggregate_int.argtypes = [_vp, ctypes.c_size_t, _u32, _u64, _u64, _u32, _u64, _vp, _vp, _vp, _vp]
        L.nc_clip_aggregate_int.restype = ctypes.c_int
        L.nc_master_nat.restype = ctypes.c_int
        for name in ("nc_sparse_nat_encode", "nc_sparse_nat_encode_batch", "nc_sparse_nat_aggregate"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("nc_nat_encode", "nc_nat_encode_batch", "nc_nat_decode", "nc_dither_encode",
                     "nc_dither_decode", "nc_aggregate_sum"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise NatcompError(lib().nc_status_string(status).decode())


def _stream():
    return _vp(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t


def _ptr(t):
    return _vp(0 if t is None else t.data_ptr())


# ------------------------------------------------------------------ sizes
def nat_exp_bytes(d):
    return lib().nc_nat_exp_bytes(d)


def sign_bytes(d):
    return lib().nc_sign_bytes(d)


def dither_code_bytes(d, s):
    return lib().nc_dither_code_bytes(d, s)


def dither_sign_bytes(d, s):
    return lib().nc_dither_sign_bytes(d, s)


def plane_stride(nbytes):
    return lib().nc_plane_stride(nbytes)


def segment_count(d, num_segments=0, bucket=0, have_offsets=False):
    return lib().nc_segment_count(d, num_segments, bucket, int(have_offsets))


def dither_workspace_bytes(d, num_segments=0, bucket=0, have_offsets=False):
    return lib().nc_dither_workspace_bytes(d, num_segments, bucket, int(have_offsets))


# ------------------------------------------------------------------ natural compression
def nat_encode(x, seed, worker=0, index_offset=0, exp_out=None, sign_out=None):
    """nc_nat_encode: returns (exponent plane, sign plane) as uint8 tensors."""
    x = _dev(x, torch.float32, "x")
    d = x.numel()
    if exp_out is None:
        exp_out = torch.empty(nat_exp_bytes(d), dtype=torch.uint8, device=x.device)
    if sign_out is None:
        sign_out = torch.empty(sign_bytes(d), dtype=torch.uint8, device=x.device)
    _dev(exp_out, torch.uint8, "exp_out")
    _dev(sign_out, torch.uint8, "sign_out")
    assert exp_out.numel() >= nat_exp_bytes(d) and sign_out.numel() >= sign_bytes(d)
    _check(lib().nc_nat_encode(_ptr(x), d, seed, worker, index_offset, _ptr(exp_out), _ptr(sign_out), _stream()))
    return exp_out, sign_out


def nat_encode_batch(x, seed, first_worker=0, index_offset=0, exp_out=None, sign_out=None, d=None):
    """nc_nat_encode_batch: x is (n, row) float32 with the first d entries of each row used;
    outputs are (n, exp_stride) and (n, sign_stride) uint8 with 256-byte-multiple strides."""
    x = _dev(x, torch.float32, "x")
    assert x.dim() == 2
    n, row = x.shape
    d = row if d is None else d
    assert d <= row
    if exp_out is None:
        exp_out = torch.empty((n, plane_stride(nat_exp_bytes(d))), dtype=torch.uint8, device=x.device)
    if sign_out is None:
        sign_out = torch.empty((n, plane_stride(sign_bytes(d))), dtype=torch.uint8, device=x.device)
    _dev(exp_out, torch.uint8, "exp_out")
    _dev(sign_out, torch.uint8, "sign_out")
    assert exp_out.shape[0] == n and sign_out.shape[0] == n
    assert exp_out.shape[1] >= nat_exp_bytes(d) and sign_out.shape[1] >= sign_bytes(d)
    _check(lib().nc_nat_encode_batch(_ptr(x), row, n, d, seed, first_worker, index_offset, _ptr(exp_out),
                                     exp_out.shape[1], _ptr(sign_out), sign_out.shape[1], _stream()))
    return exp_out, sign_out


def nat_decode(exp, sign, d, out=None):
    """nc_nat_decode."""
    exp = _dev(exp, torch.uint8, "exp")
    sign = _dev(sign, torch.uint8, "sign")
    assert exp.numel() >= nat_exp_bytes(d) and sign.numel() >= sign_bytes(d)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=exp.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    _check(lib().nc_nat_decode(_ptr(exp), _ptr(sign), d, _ptr(out), _stream()))
    return out


# ------------------------------------------------------------------ natural dithering
def _segments(d, seg_offsets, bucket):
    if seg_offsets is not None:
        seg_offsets = _dev(seg_offsets, torch.int64, "seg_offsets")   # uint64 values held in an int64 tensor
        return seg_offsets, seg_offsets.numel() - 1, 0, seg_offsets.numel() - 1
    bucket = int(bucket or 0)
    return None, 0, bucket, segment_count(d, 0, bucket, False)


def dither_encode(x, p, s, seed, worker=0, index_offset=0, seg_offsets=None, bucket=0,
                  norms_out=None, code_out=None, sign_out=None, workspace=None, standard=False):
    """nc_dither_encode (standard=True: nc_dither_sta_encode): returns (norms, code plane, sign plane or None)."""
    x = _dev(x, torch.float32, "x")
    d = x.numel()
    off, nseg, bucket, count = _segments(d, seg_offsets, bucket)
    if norms_out is None:
        norms_out = torch.empty(count, dtype=torch.float32, device=x.device)
    if code_out is None:
        code_out = torch.empty(dither_code_bytes(d, s), dtype=torch.uint8, device=x.device)
    nsign = dither_sign_bytes(d, s)
    if sign_out is None and nsign:
        sign_out = torch.empty(nsign, dtype=torch.uint8, device=x.device)
    need = dither_workspace_bytes(d, nseg, bucket, off is not None)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _dev(norms_out, torch.float32, "norms_out")
    _dev(code_out, torch.uint8, "code_out")
    _dev(sign_out, torch.uint8, "sign_out")
    _dev(workspace, torch.uint8, "workspace")
    assert norms_out.numel() >= count and code_out.numel() >= dither_code_bytes(d, s)
    assert nsign == 0 or sign_out.numel() >= nsign
    fn = lib().nc_dither_sta_encode if standard else lib().nc_dither_encode
    _check(fn(_ptr(x), d, _ptr(off), nseg, bucket, float(p), s, seed, worker, index_offset,
              _ptr(norms_out), _ptr(code_out), _ptr(sign_out), _ptr(workspace),
              0 if workspace is None else workspace.numel(), _stream()))
    return norms_out, code_out, sign_out


def static_scratch_bytes():
    return lib().nc_static_scratch_bytes()


def static_scratch_init():
    """nc_static_scratch_init on torch's current device."""
    _check(lib().nc_static_scratch_init())


def dither_encode_static(x, p, s, seed, norms_out, code_out, sign_out=None, worker=0, index_offset=0,
                         seg_offsets=None, bucket=0):
    """nc_dither_encode_static: every output is the caller's; nothing is allocated here or in the library."""
    x = _dev(x, torch.float32, "x")
    d = x.numel()
    off, nseg, bucket, count = _segments(d, seg_offsets, bucket)
    _dev(norms_out, torch.float32, "norms_out")
    _dev(code_out, torch.uint8, "code_out")
    _dev(sign_out, torch.uint8, "sign_out")
    assert norms_out.numel() >= count and code_out.numel() >= dither_code_bytes(d, s)
    assert dither_sign_bytes(d, s) == 0 or (sign_out is not None and sign_out.numel() >= dither_sign_bytes(d, s))
    _check(lib().nc_dither_encode_static(_ptr(x), d, _ptr(off), nseg, bucket, float(p), s, seed, worker, index_offset,
                                         _ptr(norms_out), _ptr(code_out), _ptr(sign_out), _stream()))
    return norms_out, code_out, sign_out


def dither_decode(norms, code, sign, d, s, seg_offsets=None, bucket=0, out=None, standard=False):
    """nc_dither_decode (standard=True: nc_dither_sta_decode; uint8 norms: nc_dither_decode_norm8)."""
    norm8 = norms.dtype == torch.uint8
    norms = _dev(norms, torch.uint8 if norm8 else torch.float32, "norms")
    code = _dev(code, torch.uint8, "code")
    sign = _dev(sign, torch.uint8, "sign")
    off, nseg, bucket, count = _segments(d, seg_offsets, bucket)
    assert norms.numel() >= count and code.numel() >= dither_code_bytes(d, s)
    assert dither_sign_bytes(d, s) == 0 or (sign is not None and sign.numel() >= dither_sign_bytes(d, s))
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=code.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    assert not (norm8 and standard)
    fn = lib().nc_dither_decode_norm8 if norm8 else lib().nc_dither_sta_decode if standard else lib().nc_dither_decode
    _check(fn(_ptr(norms), _ptr(code), _ptr(sign), d, _ptr(off), nseg, bucket, s, _ptr(out), _stream()))
    return out


# ------------------------------------------------------------------ sum over workers
def aggregate_sum(kind, d, code, sign=None, norms=None, s=0, seg_offsets=None, bucket=0, out=None):
    """nc_aggregate_sum over the rows of 2-D plane tensors (row w = worker w)."""
    code = _dev(code, torch.uint8, "code")
    sign = _dev(sign, torch.uint8, "sign")
    norms = _dev(norms, torch.uint8 if kind == NC_KIND_DITHER_NORM8 else torch.float32, "norms")
    assert code.dim() == 2
    n = code.shape[0]
    desc = AggDesc()
    desc.kind, desc.n, desc.d, desc.s = kind, n, d, s
    desc.code, desc.code_stride = code.data_ptr(), code.shape[1]
    if sign is not None:
        assert sign.dim() == 2 and sign.shape[0] == n
        desc.sign, desc.sign_stride = sign.data_ptr(), sign.shape[1]
    if kind == NC_KIND_NAT:
        assert code.shape[1] >= nat_exp_bytes(d) and sign is not None and sign.shape[1] >= sign_bytes(d)
    if kind in (NC_KIND_DITHER, NC_KIND_DITHER_STA, NC_KIND_DITHER_NORM8):
        assert code.shape[1] >= dither_code_bytes(d, s)
        assert dither_sign_bytes(d, s) == 0 or (sign is not None and sign.shape[1] >= dither_sign_bytes(d, s))
        off, nseg, bucket, count = _segments(d, seg_offsets, bucket)
        assert norms is not None and norms.dim() == 2 and norms.shape[0] == n and norms.shape[1] >= count
        desc.norms, desc.norm_stride = norms.data_ptr(), norms.shape[1]
        desc.seg_offsets = 0 if off is None else off.data_ptr()
        desc.num_segments, desc.bucket = nseg, bucket
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=code.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    _check(lib().nc_aggregate_sum(ctypes.byref(desc), _ptr(out), _stream()))
    return out


# ------------------------------------------------------------------ sparsification + C_nat
def sparse_nat_encode_batch(x, k, scale, seed, first_worker=0, d=None, idx_out=None, exp_out=None, sign_out=None):
    """nc_sparse_nat_encode_batch: x is (n, row) float32; returns (idx int32-typed uint32 values (n, ks),
    exp (n, es), sign (n, ss)) with strides rounded up so every row is 256-byte aligned."""
    x = _dev(x, torch.float32, "x")
    assert x.dim() == 2
    n, row = x.shape
    d = row if d is None else d
    assert 0 < k <= d <= row
    if idx_out is None:
        idx_out = torch.empty((n, plane_stride(4 * k) // 4), dtype=torch.int32, device=x.device)
    if exp_out is None:
        exp_out = torch.empty((n, plane_stride(k)), dtype=torch.uint8, device=x.device)
    if sign_out is None:
        sign_out = torch.empty((n, plane_stride(sign_bytes(k))), dtype=torch.uint8, device=x.device)
    _dev(idx_out, torch.int32, "idx_out")
    _dev(exp_out, torch.uint8, "exp_out")
    _dev(sign_out, torch.uint8, "sign_out")
    assert idx_out.shape[0] == n and exp_out.shape[0] == n and sign_out.shape[0] == n
    assert idx_out.shape[1] >= k and exp_out.shape[1] >= k and sign_out.shape[1] >= sign_bytes(k)
    _check(lib().nc_sparse_nat_encode_batch(_ptr(x), row, n, d, k, float(scale), seed, first_worker, _ptr(idx_out),
                                            idx_out.shape[1], _ptr(exp_out), exp_out.shape[1], _ptr(sign_out),
                                            sign_out.shape[1], _stream()))
    return idx_out, exp_out, sign_out


def sparse_nat_encode(x, k, scale, seed, worker=0):
    """nc_sparse_nat_encode on a 1-D tensor: (idx (k,), exp (k,), sign (ceil(k/8),))."""
    x = _dev(x, torch.float32, "x")
    d = x.numel()
    if not 0 < k <= d:
        raise NatcompError("NC_ERR_INVALID")
    idx = torch.empty(k, dtype=torch.int32, device=x.device)
    exp = torch.empty(k, dtype=torch.uint8, device=x.device)
    sign = torch.empty(sign_bytes(k), dtype=torch.uint8, device=x.device)
    _check(lib().nc_sparse_nat_encode(_ptr(x), d, k, float(scale), seed, worker, _ptr(idx), _ptr(exp), _ptr(sign),
                                      _stream()))
    return idx, exp, sign


def sparse_nat_aggregate(idx, exp, sign, k, d, out=None):
    """nc_sparse_nat_aggregate over the rows of 2-D tensors (row w = worker w)."""
    idx = _dev(idx, torch.int32, "idx")
    exp = _dev(exp, torch.uint8, "exp")
    sign = _dev(sign, torch.uint8, "sign")
    assert idx.dim() == 2 and exp.dim() == 2 and sign.dim() == 2
    n = idx.shape[0]
    assert exp.shape[0] == n and sign.shape[0] == n
    assert idx.shape[1] >= k and exp.shape[1] >= k and sign.shape[1] >= sign_bytes(k)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=idx.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    _check(lib().nc_sparse_nat_aggregate(_ptr(idx), idx.shape[1], _ptr(exp), exp.shape[1], _ptr(sign), sign.shape[1],
                                         n, k, d, _ptr(out), _stream()))
    return out


def sparse_aggregate_workspace_bytes(n, k, d):
    return int(lib().nc_sparse_aggregate_workspace_bytes(n, k, d))


def sparse_nat_aggregate_ws(idx, exp, sign, k, d, out=None, workspace=None):
    """nc_sparse_nat_aggregate_ws over the rows of 2-D tensors (row w = worker w); the workspace is a
    uint8 tensor of at least sparse_aggregate_workspace_bytes(n, k, d) bytes (allocated here if None)."""
    idx = _dev(idx, torch.int32, "idx")
    exp = _dev(exp, torch.uint8, "exp")
    sign = _dev(sign, torch.uint8, "sign")
    assert idx.dim() == 2 and exp.dim() == 2 and sign.dim() == 2
    n = idx.shape[0]
    assert exp.shape[0] == n and sign.shape[0] == n
    assert idx.shape[1] >= k and exp.shape[1] >= k and sign.shape[1] >= sign_bytes(k)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=idx.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    if workspace is None:
        workspace = torch.empty(max(1, sparse_aggregate_workspace_bytes(n, k, d)), dtype=torch.uint8, device=idx.device)
    _dev(workspace, torch.uint8, "workspace")
    _check(lib().nc_sparse_nat_aggregate_ws(_ptr(idx), idx.shape[1], _ptr(exp), exp.shape[1], _ptr(sign),
                                            sign.shape[1], n, k, d, _ptr(out), _ptr(workspace), workspace.numel(),
                                            _stream()))
    return out


def norm_compress(norms, seed, worker=0):
    """nc_norm_compress: (exponent bytes, power-of-two norms)."""
    norms = _dev(norms, torch.float32, "norms")
    e = torch.empty(norms.numel(), dtype=torch.uint8, device=norms.device)
    q = torch.empty(norms.numel(), dtype=torch.float32, device=norms.device)
    _check(lib().nc_norm_compress(_ptr(norms), norms.numel(), seed, worker, _ptr(e), _ptr(q), _stream()))
    return e, q


def master_nat(d, exp, sign, seed, master=0, index_offset=0, exp_out=None, sign_out=None):
    """nc_master_nat over the rows of 2-D plane tensors: returns (exponent plane, sign plane) of C_nat(sum)."""
    exp = _dev(exp, torch.uint8, "exp")
    sign = _dev(sign, torch.uint8, "sign")
    assert exp.dim() == 2 and sign.dim() == 2 and sign.shape[0] == exp.shape[0]
    desc = AggDesc()
    desc.kind, desc.n, desc.d = NC_KIND_NAT, exp.shape[0], d
    desc.code, desc.code_stride = exp.data_ptr(), exp.shape[1]
    desc.sign, desc.sign_stride = sign.data_ptr(), sign.shape[1]
    if exp_out is None:
        exp_out = torch.empty(nat_exp_bytes(d), dtype=torch.uint8, device=exp.device)
    if sign_out is None:
        sign_out = torch.empty(sign_bytes(d), dtype=torch.uint8, device=exp.device)
    _dev(exp_out, torch.uint8, "exp_out")
    _dev(sign_out, torch.uint8, "sign_out")
    assert exp_out.numel() >= nat_exp_bytes(d) and sign_out.numel() >= sign_bytes(d)
    _check(lib().nc_master_nat(ctypes.byref(desc), seed, master, index_offset, _ptr(exp_out), _ptr(sign_out), _stream()))
    return exp_out, sign_out


def nat_clip_encode(x, seed, first_worker=0, index_offset=0, code_out=None, d=None):
    """nc_nat_clip_encode: x is (d,) or (n, row) float32; returns uint8 codes of shape (d,) or (n, stride)."""
    x = _dev(x, torch.float32, "x")
    single = x.dim() == 1
    x2 = x.unsqueeze(0) if single else x
    assert x2.dim() == 2
    n, row = x2.shape
    d = row if d is None else d
    assert d <= row
    if code_out is None:
        code_out = torch.empty((n, plane_stride(d)), dtype=torch.uint8, device=x.device)
        if single:
            code_out = code_out[0, :d]
    _dev(code_out, torch.uint8, "code_out")
    c2 = code_out.unsqueeze(0) if code_out.dim() == 1 else code_out
    assert c2.shape[0] == n and c2.shape[1] >= d
    _check(lib().nc_nat_clip_encode(_ptr(x2), row, n, d, seed, first_worker, index_offset, _ptr(c2), c2.shape[1],
                                    _stream()))
    return code_out


def nat_clip_decode(code, d, out=None):
    """nc_nat_clip_decode."""
    code = _dev(code, torch.uint8, "code")
    assert code.numel() >= d
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=code.device)
    _dev(out, torch.float32, "out")
    assert out.numel() >= d
    _check(lib().nc_nat_clip_decode(_ptr(code), d, _ptr(out), _stream()))
    return out


def clip_aggregate_int(code, d, seed, master=0, index_offset=0, want_sum=False, want_planes=True, sum_out=None,
                       exp_out=None, sign_out=None):
    """nc_clip_aggregate_int over the rows of a 2-D code tensor: returns (sums int64 or None, exponent plane or
    None, sign plane or None)."""
    code = _dev(code, torch.uint8, "code")
    assert code.dim() == 2 and code.shape[1] >= d
    if want_sum and sum_out is None:
        sum_out = torch.empty(d, dtype=torch.int64, device=code.device)
    if want_planes and exp_out is None:
        exp_out = torch.empty(nat_exp_bytes(d), dtype=torch.uint8, device=code.device)
    if want_planes and sign_out is None:
        sign_out = torch.empty(sign_bytes(d), dtype=torch.uint8, device=code.device)
    if sum_out is not None:
        _dev(sum_out, torch.int64, "sum_out")
        assert sum_out.numel() >= d
    if exp_out is not None:
        _dev(exp_out, torch.uint8, "exp_out")
        assert exp_out.numel() >= nat_exp_bytes(d)
    if sign_out is not None:
        _dev(sign_out, torch.uint8, "sign_out")
        assert sign_out.numel() >= sign_bytes(d)
    _check(lib().nc_clip_aggregate_int(_ptr(code), code.shape[1], code.shape[0], d, seed, master, index_offset,
                                       _ptr(sum_out), _ptr(exp_out), _ptr(sign_out), _stream()))
    return sum_out, exp_out, sign_out


def p_value(p):
    """The float the ABI expects for p (math.inf for the max-norm)."""
    return math.inf if p in ("inf", math.inf) else float(p)
