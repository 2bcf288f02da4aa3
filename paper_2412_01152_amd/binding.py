"""ctypes binding of libdiloco_mi355.so (C ABI: include/diloco_mi355.h).

Argument marshalling only: torch tensors supply device memory and the current HIP stream; every
step of the computation runs in the library's kernels.  There is no fallback: if the library has
not been built (python -m paper_2412_01152_amd.build) loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdiloco_mi355.so")

DTYPE_FP32 = 0
DTYPE_BF16 = 1
MAX_PEERS = 16
STATIC_MAX_SEGMENTS = 512
STATUS_DEGENERATE = 1
STATUS_NONFINITE = 2
STATUS_EMPTY = 4

QPARAMS_DTYPE = np.dtype([("mean", "<f8"), ("std", "<f8"), ("lo", "<f4"), ("inv_w", "<f4"),
                          ("n", "<u8"), ("status", "<u4"), ("pad", "<u4")])
QPARAMS_BYTES = 40
assert QPARAMS_DTYPE.itemsize == QPARAMS_BYTES

EXPORTS = ("diloco_workspace_bytes", "diloco_strerror", "diloco_pseudograd_quantize",
           "int8_reduce_chunk", "outer_nesterov_step", "diloco_profile_passes",
           "diloco_pseudograd_quantize_variant", "int8_reduce_chunk_variant", "diloco_ring_order",
           "diloco_tune_write_phase", "int8_reduce_chunk_static", "diloco_placement")

CODEBOOK_MEAN, CODEBOOK_MIDPOINT = 0, 1

_lib = None


class DilocoError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load().diloco_strerror(ctypes.c_int32(code)).decode()
        super().__init__(f"{where}: {msg} (code {code})")


def load() -> ctypes.CDLL:
    """Load the built library; raises if it is missing (no CPU path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2412_01152_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u64, u32, i32, f32, sz = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32,
                                  ctypes.c_float, ctypes.c_size_t)
    lib.diloco_workspace_bytes.restype = sz
    lib.diloco_workspace_bytes.argtypes = [u32]
    lib.diloco_strerror.restype = ctypes.c_char_p
    lib.diloco_strerror.argtypes = [i32]
    lib.diloco_pseudograd_quantize.restype = i32
    lib.diloco_pseudograd_quantize.argtypes = [vp, vp, i32, u64, vp, u32, vp, vp, vp, vp, sz, vp]
    lib.int8_reduce_chunk.restype = i32
    lib.int8_reduce_chunk.argtypes = [vp, vp, u32, vp, u32, u64, vp, u32, vp, vp, vp, vp, vp, sz, vp]
    lib.int8_reduce_chunk_static.restype = i32
    lib.int8_reduce_chunk_static.argtypes = [vp, vp, u32, vp, u32, u64, vp, u32, vp, vp, vp, vp, vp]
    f64 = ctypes.c_double
    lib.diloco_pseudograd_quantize_variant.restype = i32
    lib.diloco_pseudograd_quantize_variant.argtypes = lib.diloco_pseudograd_quantize.argtypes + [f64, u32]
    lib.int8_reduce_chunk_variant.restype = i32
    lib.int8_reduce_chunk_variant.argtypes = lib.int8_reduce_chunk.argtypes + [f64, u32]
    lib.diloco_ring_order.restype = i32
    lib.diloco_ring_order.argtypes = [vp, u32, vp, vp]
    lib.outer_nesterov_step.restype = i32
    lib.outer_nesterov_step.argtypes = [vp, vp, vp, vp, vp, vp, u32, u64, f32, f32, vp, i32, vp, sz, vp]
    lib.diloco_profile_passes.restype = i32
    lib.diloco_profile_passes.argtypes = [vp]
    lib.diloco_placement.restype = i32
    lib.diloco_placement.argtypes = [u64, vp]
    lib.diloco_tune_write_phase.restype = i32
    lib.diloco_tune_write_phase.argtypes = [i32, i32]
    _lib = lib
    return lib


def profile_passes(events: Optional[Sequence[int]]) -> None:
    """diloco_profile_passes: 4 raw hipEvent_t handles (ints), or None to stop recording."""
    lib = load()
    if events is None:
        lib.diloco_profile_passes(ctypes.c_void_p(0))
        return
    assert len(events) == 4
    arr = (ctypes.c_void_p * 4)(*events)
    lib.diloco_profile_passes(ctypes.cast(arr, ctypes.c_void_p))


def tune_write_phase(period_us: int, window_us: int = 0) -> None:
    """diloco_tune_write_phase: < 0 the built-in choice, 0 write at once, else (period, window) in us."""
    rc = load().diloco_tune_write_phase(ctypes.c_int32(period_us), ctypes.c_int32(window_us))
    if rc != 0:
        raise DilocoError(rc, "diloco_tune_write_phase")


def placement(arena_bytes: int) -> Tuple[int, int, int]:
    """diloco_placement: byte offsets of the "read", "state" and "out" groups in an arena of arena_bytes."""
    out = (ctypes.c_uint64 * 3)()
    rc = load().diloco_placement(ctypes.c_uint64(arena_bytes), ctypes.cast(out, ctypes.c_void_p))
    if rc != 0:
        raise DilocoError(rc, "diloco_placement")
    return int(out[0]), int(out[1]), int(out[2])


def workspace_bytes(T: int) -> int:
    return int(load().diloco_workspace_bytes(ctypes.c_uint32(T)))


def new_workspace(T: int, device) -> torch.Tensor:
    return torch.empty(workspace_bytes(T), dtype=torch.uint8, device=device)


def new_qparams(T: int, device) -> torch.Tensor:
    return torch.empty(T * QPARAMS_BYTES, dtype=torch.uint8, device=device)


def qparams_to_numpy(qp: torch.Tensor) -> np.ndarray:
    return qp.cpu().numpy().view(QPARAMS_DTYPE).copy()


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _seg_array(seg_offsets: Sequence[int]):
    so = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.uint64))
    return so, so.size - 1


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _variant_args(variant):
    range_sigmas, codebook = variant
    return ctypes.c_double(float(range_sigmas)), ctypes.c_uint32(int(codebook))


def _local_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DTYPE_FP32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"theta_local must be float32 or bfloat16, got {t.dtype}")


def pseudograd_quantize(theta_outer: torch.Tensor, theta_local: torch.Tensor, seg_offsets,
                        codes_out: Optional[torch.Tensor] = None, lut_out: Optional[torch.Tensor] = None,
                        qparams_out: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, stream=None, variant=None):
    """diloco_pseudograd_quantize -> (codes u8[N], lut f32[T,256], qparams bytes[T*40]).

    variant = (range_sigmas, codebook) calls diloco_pseudograd_quantize_variant instead."""
    lib = load()
    assert theta_outer.dtype == torch.float32
    N = theta_outer.numel()
    assert theta_local.numel() == N
    so, T = _seg_array(seg_offsets)
    dev = theta_outer.device
    codes_out = torch.empty(N, dtype=torch.uint8, device=dev) if codes_out is None else codes_out
    lut_out = torch.empty((max(T, 0), 256), dtype=torch.float32, device=dev) if lut_out is None else lut_out
    qparams_out = new_qparams(max(T, 0), dev) if qparams_out is None else qparams_out
    workspace = new_workspace(T, dev) if workspace is None else workspace
    fn, name, extra = lib.diloco_pseudograd_quantize, "diloco_pseudograd_quantize", ()
    if variant is not None:
        fn, name, extra = lib.diloco_pseudograd_quantize_variant, name + "_variant", _variant_args(variant)
    rc = fn(_ptr(theta_outer), _ptr(theta_local), _local_dtype(theta_local), ctypes.c_uint64(N),
            ctypes.c_void_p(so.ctypes.data), ctypes.c_uint32(T), _ptr(codes_out), _ptr(lut_out), _ptr(qparams_out),
            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(stream), *extra)
    if rc != 0:
        raise DilocoError(rc, name)
    return codes_out, lut_out, qparams_out


def reduce_chunk(peer_codes: List[torch.Tensor], peer_luts: List[torch.Tensor], seg_offsets, divisor: int,
                 local_fp32: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                 codes_out: Optional[torch.Tensor] = None, lut_out: Optional[torch.Tensor] = None,
                 qparams_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 stream=None, variant=None):
    """int8_reduce_chunk -> (codes u8[n], lut f32[T,256], qparams bytes[T*40]); acc_out filled if given.

    variant = (range_sigmas, codebook) calls int8_reduce_chunk_variant instead."""
    lib = load()
    W = len(peer_codes)
    assert len(peer_luts) == W
    so, T = _seg_array(seg_offsets)
    n = int(so[-1]) if so.size else 0
    ref = peer_codes[0] if W else local_fp32
    dev = ref.device
    for c in peer_codes:
        assert c.dtype == torch.uint8 and c.numel() == n
    for l in peer_luts:
        assert l.dtype == torch.float32 and l.numel() == T * 256
    code_ptrs = (ctypes.c_void_p * max(W, 1))(*[c.data_ptr() for c in peer_codes])
    lut_ptrs = (ctypes.c_void_p * max(W, 1))(*[l.data_ptr() for l in peer_luts])
    codes_out = torch.empty(n, dtype=torch.uint8, device=dev) if codes_out is None else codes_out
    lut_out = torch.empty((T, 256), dtype=torch.float32, device=dev) if lut_out is None else lut_out
    qparams_out = new_qparams(T, dev) if qparams_out is None else qparams_out
    workspace = new_workspace(T, dev) if workspace is None else workspace
    fn, name, extra = lib.int8_reduce_chunk, "int8_reduce_chunk", ()
    if variant is not None:
        fn, name, extra = lib.int8_reduce_chunk_variant, name + "_variant", _variant_args(variant)
    rc = fn(ctypes.cast(code_ptrs, ctypes.c_void_p), ctypes.cast(lut_ptrs, ctypes.c_void_p), ctypes.c_uint32(W),
            _ptr(local_fp32), ctypes.c_uint32(divisor), ctypes.c_uint64(n), ctypes.c_void_p(so.ctypes.data),
            ctypes.c_uint32(T), _ptr(acc_out), _ptr(codes_out), _ptr(lut_out), _ptr(qparams_out), _ptr(workspace),
            ctypes.c_size_t(workspace.numel()), _stream(stream), *extra)
    if rc != 0:
        raise DilocoError(rc, name)
    return codes_out, lut_out, qparams_out


def reduce_chunk_static(peer_codes: List[torch.Tensor], peer_luts: List[torch.Tensor], seg_offsets, divisor: int,
                        codes_out: torch.Tensor, lut_out: torch.Tensor, qparams_out: torch.Tensor,
                        local_fp32: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """int8_reduce_chunk_static: every output buffer comes from the caller, the scratch from the library's
    static device array; nothing is allocated here or in the library."""
    lib = load()
    W = len(peer_codes)
    assert len(peer_luts) == W
    so, T = _seg_array(seg_offsets)
    n = int(so[-1]) if so.size else 0
    code_ptrs = (ctypes.c_void_p * max(W, 1))(*[c.data_ptr() for c in peer_codes])
    lut_ptrs = (ctypes.c_void_p * max(W, 1))(*[l.data_ptr() for l in peer_luts])
    rc = lib.int8_reduce_chunk_static(ctypes.cast(code_ptrs, ctypes.c_void_p), ctypes.cast(lut_ptrs, ctypes.c_void_p),
                                      ctypes.c_uint32(W), _ptr(local_fp32), ctypes.c_uint32(divisor),
                                      ctypes.c_uint64(n), ctypes.c_void_p(so.ctypes.data), ctypes.c_uint32(T),
                                      _ptr(acc_out), _ptr(codes_out), _ptr(lut_out), _ptr(qparams_out),
                                      _stream(stream))
    if rc != 0:
        raise DilocoError(rc, "int8_reduce_chunk_static")


def outer_step(theta_outer: torch.Tensor, momentum: torch.Tensor, lr: float, beta: float,
               delta_fp32: Optional[torch.Tensor] = None, delta_codes: Optional[torch.Tensor] = None,
               delta_lut: Optional[torch.Tensor] = None, seg_offsets=None,
               theta_local_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
               stream=None) -> None:
    """outer_nesterov_step, in place on theta_outer and momentum."""
    lib = load()
    N = theta_outer.numel()
    assert theta_outer.dtype == torch.float32 and momentum.dtype == torch.float32
    assert momentum.numel() == N
    T = 0
    so_ptr = ctypes.c_void_p(0)
    so = None
    if seg_offsets is not None:
        so, T = _seg_array(seg_offsets)
        so_ptr = ctypes.c_void_p(so.ctypes.data)
    if delta_codes is not None and workspace is None:
        workspace = new_workspace(T, theta_outer.device)
    ws_bytes = workspace.numel() if workspace is not None else 0
    out_dtype = _local_dtype(theta_local_out) if theta_local_out is not None else DTYPE_FP32
    rc = lib.outer_nesterov_step(_ptr(theta_outer), _ptr(momentum), _ptr(delta_fp32), _ptr(delta_codes),
                                 _ptr(delta_lut), so_ptr, ctypes.c_uint32(T), ctypes.c_uint64(N),
                                 ctypes.c_float(lr), ctypes.c_float(beta), _ptr(theta_local_out),
                                 ctypes.c_int32(out_dtype), _ptr(workspace), ctypes.c_size_t(ws_bytes),
                                 _stream(stream))
    if rc != 0:
        raise DilocoError(rc, "outer_nesterov_step")


def ring_order(bandwidth) -> Tuple[List[int], float]:
    """diloco_ring_order: (order, bottleneck) for an [n][n] matrix of link bandwidths (host data)."""
    lib = load()
    w = np.ascontiguousarray(np.asarray(bandwidth, dtype=np.float64))
    if w.ndim != 2 or w.shape[0] != w.shape[1]:
        raise ValueError("bandwidth must be a square matrix")
    n = w.shape[0]
    order = np.zeros(max(n, 1), dtype=np.uint32)
    bottleneck = ctypes.c_double(0.0)
    rc = lib.diloco_ring_order(ctypes.c_void_p(w.ctypes.data), ctypes.c_uint32(n), ctypes.c_void_p(order.ctypes.data),
                               ctypes.cast(ctypes.byref(bottleneck), ctypes.c_void_p))
    if rc != 0:
        raise DilocoError(rc, "diloco_ring_order")
    return [int(v) for v in order[:n]], float(bottleneck.value)
