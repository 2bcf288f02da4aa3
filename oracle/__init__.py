"""ctypes front end of the CPU oracle (oracle/diloco_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests, by the smoke check and by the benchmark's CPU-baseline
leg; never by the product package.  It takes and returns numpy arrays in host memory and does no
arithmetic of its own: every number comes out of the C file.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")

STATUS_DEGENERATE = 1
STATUS_NONFINITE = 2
STATUS_EMPTY = 4


class QParams(ctypes.Structure):
    _fields_ = [("mean", ctypes.c_double), ("std", ctypes.c_double), ("lo", ctypes.c_float),
                ("inv_w", ctypes.c_float), ("n", ctypes.c_uint64), ("status", ctypes.c_uint32),
                ("pad", ctypes.c_uint32)]


QPARAMS_DTYPE = np.dtype([("mean", "<f8"), ("std", "<f8"), ("lo", "<f4"), ("inv_w", "<f4"),
                          ("n", "<u8"), ("status", "<u4"), ("pad", "<u4")])
assert QPARAMS_DTYPE.itemsize == ctypes.sizeof(QParams) == 40

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(t: int) -> None:
    lib().oracle_set_num_threads(int(t))


PAPER_RANGE_SIGMAS = 6.0          # Section 2.2: the range is mean +- 6 standard deviations


def _variant(range_sigmas, codebook):
    """The quantiser's two knobs as C arguments; the defaults are the paper's."""
    if codebook not in ("mean", "midpoint"):
        raise ValueError(codebook)
    return ctypes.c_double(float(range_sigmas)), ctypes.c_int(int(codebook == "midpoint"))


def _p(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _chk(a, dtype, name):
    if a.dtype != np.dtype(dtype) or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(dtype)}, got {a.dtype}")
    return a


def _segs(seg_offsets, n):
    so = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.uint64))
    if so.ndim != 1 or so.size < 2 or so[0] != 0 or so[-1] != n or np.any(np.diff(so.astype(np.int64)) < 0):
        raise ValueError("seg_offsets must ascend from 0 to n")
    return so


def pseudograd(theta_outer, theta_local, local_is_bf16=False):
    """d = theta_outer - theta_local (fp32).  bf16 theta_local is passed as uint16 bit patterns."""
    to = _chk(theta_outer, np.float32, "theta_outer")
    tl = _chk(theta_local, np.uint16 if local_is_bf16 else np.float32, "theta_local")
    assert to.size == tl.size
    d = np.empty(to.size, dtype=np.float32)
    lib().oracle_pseudograd(_p(to), _p(tl), ctypes.c_int(int(local_is_bf16)),
                            ctypes.c_uint64(to.size), _p(d))
    return d


def quantize(x, range_sigmas=PAPER_RANGE_SIGMAS, codebook="mean"):
    """Q on one tensor -> (codes u8[n], lut f32[256], qparams record)."""
    x = _chk(x, np.float32, "x")
    codes = np.empty(x.size, dtype=np.uint8)
    lut = np.empty(256, dtype=np.float32)
    qp = np.zeros(1, dtype=QPARAMS_DTYPE)
    lib().oracle_quantize(_p(x), ctypes.c_uint64(x.size), *_variant(range_sigmas, codebook), _p(codes), _p(lut),
                          _p(qp))
    return codes, lut, qp[0]


def dequantize(codes, lut):
    codes = _chk(codes, np.uint8, "codes")
    lut = _chk(lut, np.float32, "lut")
    out = np.empty(codes.size, dtype=np.float32)
    lib().oracle_dequantize(_p(codes), _p(lut), ctypes.c_uint64(codes.size), _p(out))
    return out


def quantize_segments(x, seg_offsets, range_sigmas=PAPER_RANGE_SIGMAS, codebook="mean"):
    x = _chk(x, np.float32, "x")
    so = _segs(seg_offsets, x.size)
    T = so.size - 1
    codes = np.empty(x.size, dtype=np.uint8)
    luts = np.empty((T, 256), dtype=np.float32)
    qps = np.zeros(T, dtype=QPARAMS_DTYPE)
    lib().oracle_quantize_segments(_p(x), _p(so), ctypes.c_uint32(T), *_variant(range_sigmas, codebook),
                                   _p(codes), _p(luts), _p(qps))
    return codes, luts, qps


def pseudograd_quantize(theta_outer, theta_local, seg_offsets, local_is_bf16=False,
                        range_sigmas=PAPER_RANGE_SIGMAS, codebook="mean"):
    """Stage 1 -> (codes, luts[T][256], qparams[T], d) where d is the fp32 pseudo-gradient."""
    to = _chk(theta_outer, np.float32, "theta_outer")
    tl = _chk(theta_local, np.uint16 if local_is_bf16 else np.float32, "theta_local")
    assert to.size == tl.size
    so = _segs(seg_offsets, to.size)
    T = so.size - 1
    d = np.empty(to.size, dtype=np.float32)
    codes = np.empty(to.size, dtype=np.uint8)
    luts = np.empty((T, 256), dtype=np.float32)
    qps = np.zeros(T, dtype=QPARAMS_DTYPE)
    lib().oracle_pseudograd_quantize(_p(to), _p(tl), ctypes.c_int(int(local_is_bf16)),
                                     ctypes.c_uint64(to.size), _p(so), ctypes.c_uint32(T),
                                     *_variant(range_sigmas, codebook), _p(d), _p(codes), _p(luts), _p(qps))
    return codes, luts, qps, d


def reduce(peer_codes, peer_luts, seg_offsets, divisor, local_fp32=None,
           range_sigmas=PAPER_RANGE_SIGMAS, codebook="mean"):
    """Stage 2 -> (acc f32[n], codes_out, luts_out, qparams_out).

    peer_codes: list of W uint8[n]; peer_luts: list of W float32[T][256]."""
    W = len(peer_codes)
    assert len(peer_luts) == W
    if W:
        n = peer_codes[0].size
    else:
        n = local_fp32.size
    so = _segs(seg_offsets, n)
    T = so.size - 1
    pcs = [_chk(c, np.uint8, "peer_codes") for c in peer_codes]
    pls = [_chk(np.ascontiguousarray(l).reshape(T, 256), np.float32, "peer_luts") for l in peer_luts]
    for c in pcs:
        assert c.size == n
    code_ptrs = (ctypes.c_void_p * max(W, 1))(*[c.ctypes.data for c in pcs])
    lut_ptrs = (ctypes.c_void_p * max(W, 1))(*[l.ctypes.data for l in pls])
    loc = _chk(local_fp32, np.float32, "local_fp32") if local_fp32 is not None else None
    if loc is not None:
        assert loc.size == n
    acc = np.empty(n, dtype=np.float32)
    codes = np.empty(n, dtype=np.uint8)
    luts = np.empty((T, 256), dtype=np.float32)
    qps = np.zeros(T, dtype=QPARAMS_DTYPE)
    lib().oracle_reduce(code_ptrs, lut_ptrs, ctypes.c_uint32(W), _p(loc), ctypes.c_uint32(divisor),
                        ctypes.c_uint64(n), _p(so), ctypes.c_uint32(T), *_variant(range_sigmas, codebook),
                        _p(acc), _p(codes), _p(luts), _p(qps))
    return acc, codes, luts, qps


def outer_step(theta, momentum, lr, beta, delta_fp32=None, delta_codes=None, delta_luts=None,
               seg_offsets=None, local_out_dtype=None):
    """Stage 3, IN PLACE on theta and momentum (float32 arrays).

    Returns theta_local_out (float32, or uint16 bf16 bit patterns) when local_out_dtype is
    "fp32" / "bf16", else None."""
    th = _chk(theta, np.float32, "theta")
    mo = _chk(momentum, np.float32, "momentum")
    N = th.size
    assert mo.size == N
    assert (delta_fp32 is None) != (delta_codes is None)
    so = None
    T = 0
    if delta_fp32 is not None:
        df = _chk(delta_fp32, np.float32, "delta_fp32")
        assert df.size == N
        dc = dl = None
    else:
        df = None
        dc = _chk(delta_codes, np.uint8, "delta_codes")
        assert dc.size == N
        so = _segs(seg_offsets, N)
        T = so.size - 1
        dl = _chk(np.ascontiguousarray(delta_luts).reshape(T, 256), np.float32, "delta_luts")
    out = None
    is_bf16 = 0
    if local_out_dtype == "fp32":
        out = np.empty(N, dtype=np.float32)
    elif local_out_dtype == "bf16":
        out = np.empty(N, dtype=np.uint16)
        is_bf16 = 1
    elif local_out_dtype is not None:
        raise ValueError(local_out_dtype)
    lib().oracle_outer_step(_p(th), _p(mo), _p(df), _p(dc), _p(dl), _p(so), ctypes.c_uint32(T),
                            ctypes.c_uint64(N), ctypes.c_float(lr), ctypes.c_float(beta), _p(out),
                            ctypes.c_int(is_bf16))
    return out
