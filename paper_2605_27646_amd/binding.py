"""ctypes binding of libhqmq.so.  Argument marshalling only: every step of encode and decode
runs in the library's kernels.  There is no fallback: if the library is not built, loading
raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhqmq.so")

HQMQ_OK = 0
HQMQ_FLAG_NO_OUTLIERS = 1
HQMQ_FLAG_CHECK_FINITE = 2
HQMQ_FLAG_ATTEND_TABLES = 4
HQMQ_STATUS_OUTLIER_OVERFLOW = 1
HQMQ_STATUS_NONFINITE = 2
HQMQ_MAX_S = 2730
HQMQ_STATIC_SCRATCH_BYTES = 16 << 20
_ERRORS = {-1: "HQMQ_ERR_INVALID_ARG", -2: "HQMQ_ERR_UNSUPPORTED", -3: "HQMQ_ERR_BUFFER_TOO_SMALL",
           -4: "HQMQ_ERR_HIP"}


class HqmqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed: {_ERRORS.get(code, code)}")


class HqmqParams(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("T", C.c_int32), ("D", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64),
                ("S", C.c_int32), ("b_r", C.c_int32), ("C", C.c_float), ("flags", C.c_uint32)]


class HqmqSizeInfo(C.Structure):
    _fields_ = [("n_rows", C.c_uint64), ("index_bits", C.c_uint32), ("code_bits", C.c_uint32),
                ("code_bytes", C.c_uint64), ("sigma_bytes", C.c_uint64), ("flag_bytes", C.c_uint64),
                ("row_off_bytes", C.c_uint64), ("n_outliers_bytes", C.c_uint64),
                ("status_bytes", C.c_uint64), ("outlier_capacity_max", C.c_uint64),
                ("outlier_bytes_max", C.c_uint64), ("workspace_bytes", C.c_uint64),
                ("chunks_per_row", C.c_uint32), ("code_words_per_row", C.c_uint32)]


class _Encoded(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("sigma", C.c_void_p), ("flags", C.c_void_p),
                ("row_off", C.c_void_p), ("outliers", C.c_void_p), ("n_outliers", C.c_void_p),
                ("status", C.c_void_p)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_27646_amd.build` "
                "(there is no fallback path)")
        lib = C.CDLL(_LIB_PATH)
        lib.hqmq_build_codebooks.restype = C.c_int32
        lib.hqmq_build_codebooks.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        lib.hqmq_sizes.restype = C.c_int32
        lib.hqmq_sizes.argtypes = [C.POINTER(HqmqParams), C.POINTER(HqmqSizeInfo)]
        lib.hqmq_encode.restype = C.c_int32
        lib.hqmq_encode.argtypes = [C.POINTER(HqmqParams), C.c_void_p, C.c_void_p, C.POINTER(_Encoded),
                                    C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
        lib.hqmq_encode_static.restype = C.c_int32
        lib.hqmq_encode_static.argtypes = [C.POINTER(HqmqParams), C.c_void_p, C.c_void_p, C.POINTER(_Encoded),
                                           C.c_uint64, C.c_void_p]
        lib.hqmq_encode_timed.restype = C.c_int32
        lib.hqmq_encode_timed.argtypes = lib.hqmq_encode.argtypes + [C.POINTER(C.c_void_p)]
        lib.hqmq_encode_given_thresholds.restype = C.c_int32
        lib.hqmq_encode_given_thresholds.argtypes = [C.POINTER(HqmqParams), C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.POINTER(_Encoded), C.c_uint64, C.c_void_p, C.c_uint64,
                                                     C.c_void_p]
        lib.hqmq_encode_batch_given_thresholds.restype = C.c_int32
        lib.hqmq_encode_batch_given_thresholds.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.POINTER(C.c_void_p),
                                                           C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                                           C.POINTER(_Encoded), C.POINTER(C.c_uint64), C.c_void_p,
                                                           C.c_uint64, C.c_void_p]
        lib.hqmq_thresholds.restype = C.c_int32
        lib.hqmq_thresholds.argtypes = [C.POINTER(HqmqParams), C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p,
                                        C.c_void_p]
        lib.hqmq_init.restype = C.c_int32
        lib.hqmq_init.argtypes = []
        lib.hqmq_shard_median_pass.restype = C.c_int32
        lib.hqmq_shard_median_pass.argtypes = [C.POINTER(HqmqParams), C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p,
                                               C.c_uint64, C.c_void_p]
        lib.hqmq_shard_median_region.restype = C.c_int32
        lib.hqmq_shard_median_region.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.POINTER(C.c_uint64),
                                                 C.POINTER(C.c_uint64)]
        lib.hqmq_encode_batch.restype = C.c_int32
        lib.hqmq_encode_batch.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.POINTER(C.c_void_p),
                                          C.POINTER(C.c_void_p), C.POINTER(_Encoded), C.POINTER(C.c_uint64),
                                          C.c_void_p, C.c_uint64, C.c_void_p, C.POINTER(C.c_void_p)]
        lib.hqmq_decode.restype = C.c_int32
        lib.hqmq_decode.argtypes = [C.POINTER(HqmqParams), C.POINTER(_Encoded), C.c_uint64, C.c_void_p,
                                    C.c_void_p, C.c_void_p]
        lib.hqmq_decode_batch.restype = C.c_int32
        lib.hqmq_decode_batch.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.POINTER(_Encoded),
                                          C.POINTER(C.c_uint64), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                          C.c_void_p]
        lib.hqmq_attend.restype = C.c_int32
        lib.hqmq_attend.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.c_void_p, C.c_float,
                                    C.POINTER(_Encoded), C.c_uint64, C.c_void_p,
                                    C.POINTER(_Encoded), C.c_uint64, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        lib.hqmq_attend_lse.restype = C.c_int32
        lib.hqmq_attend_lse.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.c_void_p, C.c_float, C.POINTER(_Encoded),
                                        C.c_uint64, C.c_void_p, C.POINTER(_Encoded), C.c_uint64, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        lib.hqmq_attend_masked.restype = C.c_int32
        lib.hqmq_attend_masked.argtypes = [C.POINTER(HqmqParams), C.c_int32, C.c_void_p, C.c_float,
                                           C.POINTER(_Encoded), C.c_uint64, C.c_void_p, C.POINTER(_Encoded),
                                           C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_uint64, C.c_void_p]
        lib.hqmq_attend_workspace_bytes.restype = C.c_uint64
        lib.hqmq_attend_workspace_bytes.argtypes = [C.POINTER(HqmqParams), C.c_int32]
        lib.hqmq_last_hip_error.restype = C.c_int32
        lib.hqmq_last_hip_error.argtypes = []
        _lib = lib
    return _lib


def _check(rc: int, where: str) -> None:
    if rc != HQMQ_OK:
        raise HqmqError(rc, where)


def params_for(x: torch.Tensor, S: int, b_r: int = 6, Cmul: float = 3.0, flags: int = 0) -> HqmqParams:
    """hqmq_params describing tensor x [B, H, T, D] (any strides with D contiguous)."""
    if x.dim() != 4 or x.stride(3) != 1:
        raise ValueError("x must be [B, H, T, D] with D contiguous")
    B, H, T, D = x.shape
    return HqmqParams(B, H, T, D, x.stride(0), x.stride(1), x.stride(2), S, b_r, Cmul, flags)


@dataclass
class EncodedBuffers:
    """Caller-owned device buffers of one encoded tensor (see hqmq_encoded in hqmq.h)."""
    codes: torch.Tensor        # int32 [n_rows, w]   (bit patterns of uint32)
    sigma: torch.Tensor        # float16 [n_rows]
    flags: torch.Tensor        # int32 [n_rows]
    row_off: torch.Tensor      # int32 [n_rows + 1]
    outliers: torch.Tensor     # float16 [capacity, 4]
    n_outliers: torch.Tensor   # int32 [H + 1]
    status: torch.Tensor       # int32 [1]

    @property
    def outlier_capacity(self) -> int:
        return self.outliers.shape[0]

    def as_struct(self) -> _Encoded:
        return _Encoded(self.codes.data_ptr(), self.sigma.data_ptr(), self.flags.data_ptr(),
                        self.row_off.data_ptr(), self.outliers.data_ptr(), self.n_outliers.data_ptr(),
                        self.status.data_ptr())

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in
                   (self.codes, self.sigma, self.flags, self.row_off, self.outliers, self.n_outliers, self.status))


def hqmq_last_hip_error() -> int:
    return int(_load().hqmq_last_hip_error())


def hqmq_init() -> None:
    """Per-device set-up of the library for torch's current device (optional except before a stream capture)."""
    _check(_load().hqmq_init(), "hqmq_init")


def hqmq_build_codebooks(seed: int, n_layers: int, n_kv_heads: int, S: int) -> torch.Tensor:
    """fp32 [n_layers, 2, n_kv_heads, S, 4] on the host (role 0 = K, 1 = V)."""
    if n_layers <= 0 or n_kv_heads <= 0 or S <= 0:
        _check(-1, "hqmq_build_codebooks")
    out = torch.empty(n_layers, 2, n_kv_heads, S, 4, dtype=torch.float32)
    _check(_load().hqmq_build_codebooks(seed, n_layers, n_kv_heads, S, out.data_ptr()), "hqmq_build_codebooks")
    return out


def hqmq_sizes(params: HqmqParams) -> HqmqSizeInfo:
    info = HqmqSizeInfo()
    _check(_load().hqmq_sizes(C.byref(params), C.byref(info)), "hqmq_sizes")
    return info


def alloc_encoded(params: HqmqParams, device, outlier_capacity: int | None = None) -> EncodedBuffers:
    """Allocate the encoded buffers with torch (memory plumbing only)."""
    info = hqmq_sizes(params)
    cap = int(info.outlier_capacity_max if outlier_capacity is None else outlier_capacity)
    n = int(info.n_rows)
    return EncodedBuffers(
        codes=torch.empty(n, info.code_words_per_row, dtype=torch.int32, device=device),
        sigma=torch.empty(n, dtype=torch.float16, device=device),
        flags=torch.empty(n, dtype=torch.int32, device=device),
        row_off=torch.empty(n + 1, dtype=torch.int32, device=device),
        outliers=torch.empty(max(cap, 1), 4, dtype=torch.float16, device=device)[:cap],
        n_outliers=torch.empty(params.H + 1, dtype=torch.int32, device=device),
        status=torch.empty(1, dtype=torch.int32, device=device),
    )


def alloc_workspace(params: HqmqParams, device) -> torch.Tensor:
    info = hqmq_sizes(params)
    return torch.empty(int(info.workspace_bytes), dtype=torch.uint8, device=device)


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def hqmq_encode(params: HqmqParams, x: torch.Tensor, sec: torch.Tensor, enc: EncodedBuffers,
                workspace: torch.Tensor, stream=None) -> None:
    """Enqueue the encode of x (fp16 device tensor described by params) against sec
    (fp32 [H, S, 4] on the device) on `stream` (default: torch's current stream)."""
    if x.dtype != torch.float16 or not x.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
        raise ValueError("x must be a device fp16 tensor and sec a device fp32 tensor")
    if not sec.is_contiguous() or tuple(sec.shape) != (params.H, params.S, 4):
        raise ValueError("sec must be contiguous [H, S, 4]")
    rc = _load().hqmq_encode(C.byref(params), x.data_ptr(), sec.data_ptr(), C.byref(enc.as_struct()),
                             enc.outlier_capacity, workspace.data_ptr(), workspace.numel(),
                             _stream_ptr(stream))
    _check(rc, "hqmq_encode")


def hqmq_encode_static(params: HqmqParams, x: torch.Tensor, sec: torch.Tensor, enc: EncodedBuffers,
                       stream=None) -> None:
    """hqmq_encode on the library's own static workspace: nothing is allocated by the call.  Shapes whose
    workspace exceeds HQMQ_STATIC_SCRATCH_BYTES are refused; calls that overlap on one GPU race."""
    if x.dtype != torch.float16 or not x.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
        raise ValueError("x must be a device fp16 tensor and sec a device fp32 tensor")
    if not sec.is_contiguous() or tuple(sec.shape) != (params.H, params.S, 4):
        raise ValueError("sec must be contiguous [H, S, 4]")
    rc = _load().hqmq_encode_static(C.byref(params), x.data_ptr(), sec.data_ptr(), C.byref(enc.as_struct()),
                                    enc.outlier_capacity, _stream_ptr(stream))
    _check(rc, "hqmq_encode_static")


def hqmq_encode_timed(params: HqmqParams, x: torch.Tensor, sec: torch.Tensor, enc: EncodedBuffers,
                      workspace: torch.Tensor, phase_events, stream=None) -> None:
    """hqmq_encode that also records up to four torch.cuda.Event (already created, i.e.
    recorded once) around its phases; entries may be None."""
    handles = (C.c_void_p * 4)(*[None if e is None else e.cuda_event for e in phase_events])
    rc = _load().hqmq_encode_timed(C.byref(params), x.data_ptr(), sec.data_ptr(), C.byref(enc.as_struct()),
                                   enc.outlier_capacity, workspace.data_ptr(), workspace.numel(),
                                   _stream_ptr(stream), handles)
    _check(rc, "hqmq_encode_timed")


def hqmq_decode(params: HqmqParams, enc: EncodedBuffers, sec: torch.Tensor, out: torch.Tensor,
                stream=None) -> None:
    """Enqueue the decode into `out` (fp16 device tensor with the strides params holds)."""
    if out.dtype != torch.float16 or not out.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
        raise ValueError("out must be a device fp16 tensor and sec a device fp32 tensor")
    if not sec.is_contiguous() or tuple(sec.shape) != (params.H, params.S, 4):
        raise ValueError("sec must be contiguous [H, S, 4]")
    rc = _load().hqmq_decode(C.byref(params), C.byref(enc.as_struct()), enc.outlier_capacity,
                             sec.data_ptr(), out.data_ptr(), _stream_ptr(stream))
    _check(rc, "hqmq_decode")


def hqmq_encode_given_thresholds(params: HqmqParams, x: torch.Tensor, sec: torch.Tensor, thr: torch.Tensor,
                                 enc: EncodedBuffers, workspace: torch.Tensor, stream=None) -> None:
    """hqmq_encode with the caller's thresholds on squared chunk norms (device fp64 [H])."""
    if x.dtype != torch.float16 or not x.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
        raise ValueError("x must be a device fp16 tensor and sec a device fp32 tensor")
    if not thr.is_cuda or thr.dtype != torch.float64 or not thr.is_contiguous() or thr.numel() != params.H:
        raise ValueError("thr must be a contiguous device fp64 tensor of H entries")
    rc = _load().hqmq_encode_given_thresholds(C.byref(params), x.data_ptr(), sec.data_ptr(), thr.data_ptr(),
                                              C.byref(enc.as_struct()), enc.outlier_capacity,
                                              workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                              _stream_ptr(stream))
    _check(rc, "hqmq_encode_given_thresholds")


def hqmq_thresholds(params: HqmqParams, workspace: torch.Tensor, slice_index: int = 0, stream=None) -> torch.Tensor:
    """Device fp64 [H]: the thresholds the last encode on this workspace (slice) applied."""
    out = torch.empty(params.H, dtype=torch.float64, device=workspace.device)
    rc = _load().hqmq_thresholds(C.byref(params), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                 int(slice_index), out.data_ptr(), _stream_ptr(stream))
    _check(rc, "hqmq_thresholds")
    return out


def hqmq_shard_median_pass(params: HqmqParams, total_chunks_per_head: int, pass_index: int, x: torch.Tensor,
                           workspace: torch.Tensor, stream=None) -> None:
    """One pass (0..5 counting, 6 finish) of the sequence-sharded median on this shard's slice x."""
    rc = _load().hqmq_shard_median_pass(C.byref(params), int(total_chunks_per_head), int(pass_index), x.data_ptr(),
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                        _stream_ptr(stream))
    _check(rc, "hqmq_shard_median_pass")


def hqmq_shard_median_region(params: HqmqParams, pass_index: int, workspace: torch.Tensor) -> torch.Tensor:
    """The histogram pass 0..5 left in the workspace, as an int32 view of it: what the shards sum."""
    off, n = C.c_uint64(), C.c_uint64()
    _check(_load().hqmq_shard_median_region(C.byref(params), int(pass_index), C.byref(off), C.byref(n)),
           "hqmq_shard_median_region")
    return workspace.view(torch.uint8)[off.value: off.value + 4 * n.value].view(torch.int32)


class EncodeBatch:
    """Marshalled argument arrays of hqmq_encode_batch, built once and reusable across calls (the
    tensors' buffers must stay alive and in place).  `workspace` holds min(n, 32) slices of
    hqmq_sizes().workspace_bytes."""

    def __init__(self, params: HqmqParams, xs, secs, encs, workspace: torch.Tensor):
        n = len(xs)
        if not (n == len(secs) == len(encs)) or n == 0:
            raise ValueError("xs, secs and encs must be non-empty lists of equal length")
        for x, sec in zip(xs, secs):
            if x.dtype != torch.float16 or not x.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
                raise ValueError("xs must be device fp16 tensors and secs device fp32 tensors")
            if not sec.is_contiguous() or tuple(sec.shape) != (params.H, params.S, 4):
                raise ValueError("every sec must be contiguous [H, S, 4]")
            if (x.stride(0), x.stride(1), x.stride(2)) != (params.stride_b, params.stride_h, params.stride_t) or \
                    x.stride(3) != 1:
                raise ValueError("every x must have the strides params holds")
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous device tensor")
        self.params = params
        self.n = n
        self.keep = (list(xs), list(secs), list(encs), workspace)
        self.x = (C.c_void_p * n)(*[t.data_ptr() for t in xs])
        self.sec = (C.c_void_p * n)(*[t.data_ptr() for t in secs])
        self.enc = (_Encoded * n)(*[e.as_struct() for e in encs])
        self.cap = (C.c_uint64 * n)(*[e.outlier_capacity for e in encs])
        self.workspace = workspace


class ThresholdBatch:
    """Marshalled threshold pointers of hqmq_encode_batch_given_thresholds for one EncodeBatch, built once and
    reusable across calls (a generation loop appends with the same buffers every step)."""

    def __init__(self, batch: "EncodeBatch", thrs):
        if len(thrs) != batch.n:
            raise ValueError("one threshold tensor per batch entry")
        for t in thrs:
            if not t.is_cuda or t.dtype != torch.float64 or not t.is_contiguous() or t.numel() != batch.params.H:
                raise ValueError("thresholds must be contiguous device fp64 tensors of H entries")
        self.keep = list(thrs)
        self.n = batch.n
        self.ptrs = (C.c_void_p * batch.n)(*[t.data_ptr() for t in thrs])


def hqmq_encode_batch_given_thresholds(batch: "EncodeBatch", thrs, stream=None) -> None:
    """hqmq_encode_batch with one caller-supplied threshold vector (device fp64 [H]) per tensor: a list of
    tensors, or a ThresholdBatch built from one."""
    if not isinstance(thrs, ThresholdBatch):
        thrs = ThresholdBatch(batch, thrs)
    if thrs.n != batch.n:
        raise ValueError("one threshold tensor per batch entry")
    ptrs = thrs.ptrs
    ws = batch.workspace
    rc = _load().hqmq_encode_batch_given_thresholds(C.byref(batch.params), batch.n, batch.x, batch.sec, ptrs,
                                                    batch.enc, batch.cap, ws.data_ptr(),
                                                    ws.numel() * ws.element_size(), _stream_ptr(stream))
    _check(rc, "hqmq_encode_batch_given_thresholds")


def alloc_batch_workspace(params: HqmqParams, n_tensors: int, device) -> torch.Tensor:
    per = int(hqmq_sizes(params).workspace_bytes)
    return torch.empty(per * min(int(n_tensors), 32), dtype=torch.uint8, device=device)


def hqmq_encode_batch(batch: EncodeBatch, phase_events=None, stream=None) -> None:
    """Enqueue the encode of every tensor of the batch (up to 32 per kernel launch).  phase_events:
    None or four torch.cuda.Event (already recorded once), see hqmq_encode_timed."""
    handles = None
    if phase_events is not None:
        handles = (C.c_void_p * 4)(*[None if e is None else e.cuda_event for e in phase_events])
    ws = batch.workspace
    rc = _load().hqmq_encode_batch(C.byref(batch.params), batch.n, batch.x, batch.sec, batch.enc, batch.cap,
                                   ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream), handles)
    _check(rc, "hqmq_encode_batch")


class DecodeBatch:
    """Marshalled argument arrays of hqmq_decode_batch, built once and reusable across calls
    (the tensors' buffers must stay alive and in place)."""

    def __init__(self, params: HqmqParams, encs, secs, outs):
        n = len(encs)
        if not (n == len(secs) == len(outs)) or n == 0:
            raise ValueError("encs, secs and outs must be non-empty lists of equal length")
        for sec, out in zip(secs, outs):
            if out.dtype != torch.float16 or not out.is_cuda or not sec.is_cuda or sec.dtype != torch.float32:
                raise ValueError("outs must be device fp16 tensors and secs device fp32 tensors")
            if not sec.is_contiguous() or tuple(sec.shape) != (params.H, params.S, 4):
                raise ValueError("every sec must be contiguous [H, S, 4]")
            if (out.stride(0), out.stride(1), out.stride(2)) != (params.stride_b, params.stride_h, params.stride_t):
                raise ValueError("every out must have the strides params holds")
        self.params = params
        self.n = n
        self.keep = (list(encs), list(secs), list(outs))
        self.enc = (_Encoded * n)(*[e.as_struct() for e in encs])
        self.cap = (C.c_uint64 * n)(*[e.outlier_capacity for e in encs])
        self.sec = (C.c_void_p * n)(*[t.data_ptr() for t in secs])
        self.out = (C.c_void_p * n)(*[t.data_ptr() for t in outs])


def hqmq_decode_batch(batch: DecodeBatch, stream=None) -> None:
    """Enqueue the decode of every tensor of the batch (one shape) on `stream`."""
    rc = _load().hqmq_decode_batch(C.byref(batch.params), batch.n, batch.enc, batch.cap, batch.sec, batch.out,
                                   _stream_ptr(stream))
    _check(rc, "hqmq_decode_batch")


def hqmq_attend_workspace_bytes(params: HqmqParams, n_q_heads: int) -> int:
    return int(_load().hqmq_attend_workspace_bytes(C.byref(params), int(n_q_heads)))


def _check_attend_args(params, q, out, sec_k, sec_v, workspace):
    for t in (q, out):
        if t.dtype != torch.float16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 3:
            raise ValueError("q and out must be contiguous device fp16 [B, n_q_heads, D]")
    if q.shape != out.shape or q.shape[0] != params.B or q.shape[2] != params.D:
        raise ValueError("q / out shape does not match params")
    for sec in (sec_k, sec_v):
        if not sec.is_cuda or sec.dtype != torch.float32 or not sec.is_contiguous() or \
                tuple(sec.shape) != (params.H, params.S, 4):
            raise ValueError("sec must be contiguous device fp32 [H, S, 4]")
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")


def hqmq_attend(params: HqmqParams, q: torch.Tensor, scale: float, enc_k: EncodedBuffers,
                sec_k: torch.Tensor, enc_v: EncodedBuffers, sec_v: torch.Tensor, out: torch.Tensor,
                workspace: torch.Tensor, stream=None) -> None:
    """Enqueue single-query attention over the packed K and V caches: q and out are contiguous
    device fp16 [B, n_q_heads, D], D = 64, 96 or 128."""
    _check_attend_args(params, q, out, sec_k, sec_v, workspace)
    rc = _load().hqmq_attend(C.byref(params), int(q.shape[1]), q.data_ptr(), float(scale),
                             C.byref(enc_k.as_struct()), enc_k.outlier_capacity, sec_k.data_ptr(),
                             C.byref(enc_v.as_struct()), enc_v.outlier_capacity, sec_v.data_ptr(),
                             out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                             _stream_ptr(stream))
    _check(rc, "hqmq_attend")


def hqmq_attend_lse(params: HqmqParams, q: torch.Tensor, scale: float, enc_k: EncodedBuffers,
                    sec_k: torch.Tensor, enc_v: EncodedBuffers, sec_v: torch.Tensor, out: torch.Tensor,
                    lse: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """hqmq_attend that also writes lse (contiguous device fp32 [B, n_q_heads]): the natural log of each
    query head's softmax denominator, for combining results over several token ranges."""
    _check_attend_args(params, q, out, sec_k, sec_v, workspace)
    if lse.dtype != torch.float32 or not lse.is_cuda or not lse.is_contiguous() or tuple(lse.shape) != tuple(q.shape[:2]):
        raise ValueError("lse must be contiguous device fp32 [B, n_q_heads]")
    rc = _load().hqmq_attend_lse(C.byref(params), int(q.shape[1]), q.data_ptr(), float(scale),
                                 C.byref(enc_k.as_struct()), enc_k.outlier_capacity, sec_k.data_ptr(),
                                 C.byref(enc_v.as_struct()), enc_v.outlier_capacity, sec_v.data_ptr(),
                                 out.data_ptr(), lse.data_ptr(), workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(rc, "hqmq_attend_lse")


def hqmq_attend_masked(params: HqmqParams, q: torch.Tensor, scale: float, enc_k: EncodedBuffers,
                       sec_k: torch.Tensor, enc_v: EncodedBuffers, sec_v: torch.Tensor, visible: torch.Tensor,
                       out: torch.Tensor, workspace: torch.Tensor, lse: torch.Tensor | None = None, stream=None) -> None:
    """hqmq_attend with a causal limit per query head: visible is contiguous device int32 [B, n_q_heads],
    head hq sees the cached tokens t < visible[b, hq].  lse as in hqmq_attend_lse, optional."""
    _check_attend_args(params, q, out, sec_k, sec_v, workspace)
    if visible.dtype != torch.int32 or not visible.is_cuda or not visible.is_contiguous() or \
            tuple(visible.shape) != tuple(q.shape[:2]):
        raise ValueError("visible must be contiguous device int32 [B, n_q_heads]")
    if lse is not None and (lse.dtype != torch.float32 or not lse.is_cuda or not lse.is_contiguous() or
                            tuple(lse.shape) != tuple(q.shape[:2])):
        raise ValueError("lse must be contiguous device fp32 [B, n_q_heads]")
    rc = _load().hqmq_attend_masked(C.byref(params), int(q.shape[1]), q.data_ptr(), float(scale),
                                    C.byref(enc_k.as_struct()), enc_k.outlier_capacity, sec_k.data_ptr(),
                                    C.byref(enc_v.as_struct()), enc_v.outlier_capacity, sec_v.data_ptr(),
                                    visible.data_ptr(), out.data_ptr(), None if lse is None else lse.data_ptr(),
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                    _stream_ptr(stream))
    _check(rc, "hqmq_attend_masked")
