"""Thin Python binding over the C ABI of libknn.so (see include/knn.h).

Argument marshalling only: every step of the computation runs in the HIP
kernels of the library.  torch is used for device memory and streams.  There is
no CPU fallback: if the library is missing or the device call fails, the call
raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libknn.so")

KNN_SQEUCLIDEAN = 0
KNN_COSINE = 1
KNN_HELLINGER = 2
KNN_L1 = 3
KNN_LINF = 4
KNN_KL = 5
KNN_OK, KNN_EINVAL, KNN_EUNSUPPORTED, KNN_ENOMEM, KNN_EDEVICE = range(5)
KNN_MAX_K = 128
METRICS = {"sqeuclidean": KNN_SQEUCLIDEAN, "cosine": KNN_COSINE, "hellinger": KNN_HELLINGER,
           "l1": KNN_L1, "linf": KNN_LINF, "kl": KNN_KL}

PLAN_AUTO, PLAN_FUSED_STREAMING, PLAN_FUSED, PLAN_TWO_PHASE, PLAN_SPLIT_BF16 = 0, 1, 3, 4, 6
NO_LIMIT = ctypes.c_size_t(-1).value      # knn_plan: "whatever workspace the preferred plan wants"

STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ["knn_build", "knn_build_ex", "knn_search", "knn_search_ex", "knn_search_static", "knn_workspace_bytes",
           "knn_workspace_bytes_ex", "knn_workspace_bytes_min", "knn_plan", "knn_select",
           "knn_select_workspace_bytes",
           "knn_mfma_calibration", "knn_mfma_bf16_calibration", "knn_contraction_calibration", "knn_valu_calibration", "knn_read_calibration", "knn_status_string",
           "knn_last_device_error"]


class KnnProfile(ctypes.Structure):
    _fields_ = [("ms_prepare", ctypes.c_float), ("ms_main", ctypes.c_float),
                ("ms_finalize", ctypes.c_float), ("ms_total", ctypes.c_float),
                ("main_launches", ctypes.c_int32), ("symmetric", ctypes.c_int32),
                ("pairs_computed", ctypes.c_int64), ("ms_select", ctypes.c_float),
                ("two_phase", ctypes.c_int32)]


class KnnOptions(ctypes.Structure):
    _fields_ = [("symmetric", ctypes.c_int32), ("rescore", ctypes.c_int32),
                ("r_splits", ctypes.c_int32), ("variant", ctypes.c_int32),
                ("block_rows", ctypes.c_int32), ("center", ctypes.c_int32),
                ("profile", ctypes.POINTER(KnnProfile)), ("uncertified", ctypes.c_void_p)]


class KnnPlanInfo(ctypes.Structure):
    _fields_ = [("plan", ctypes.c_int32), ("symmetric", ctypes.c_int32), ("two_phase", ctypes.c_int32),
                ("main_launches", ctypes.c_int32), ("workspace_bytes", ctypes.c_uint64),
                ("kernel", ctypes.c_char * 32)]

    def __repr__(self) -> str:
        return (f"KnnPlanInfo(plan={self.plan}, symmetric={self.symmetric}, two_phase={self.two_phase}, "
                f"main_launches={self.main_launches}, workspace_bytes={self.workspace_bytes}, "
                f"kernel={self.kernel.decode()!r})")


class KnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(text)
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen libknn.so and declare its entry points; raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_0906_0231_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    optp = ctypes.POINTER(KnnOptions)
    lib.knn_build.restype = i32
    lib.knn_build.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.knn_build_ex.restype = i32
    lib.knn_build_ex.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, sz, vp, optp]
    lib.knn_search.restype = i32
    lib.knn_search.argtypes = [vp, i64, vp, i64, i32, i32, i32, i64, vp, vp, vp, sz, vp]
    lib.knn_search_ex.restype = i32
    lib.knn_search_ex.argtypes = [vp, i64, vp, i64, i32, i32, i32, i64, vp, vp, vp, sz, vp, optp]
    lib.knn_search_static.restype = i32
    lib.knn_search_static.argtypes = [vp, i64, vp, i64, i32, i32, i32, i64, vp, vp, vp]
    lib.knn_workspace_bytes.restype = sz
    lib.knn_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32]
    lib.knn_workspace_bytes_ex.restype = sz
    lib.knn_workspace_bytes_ex.argtypes = [i64, i64, i32, i32, i32, i32, optp]
    lib.knn_workspace_bytes_min.restype = sz
    lib.knn_workspace_bytes_min.argtypes = [i64, i64, i32, i32, i32, i32]
    lib.knn_plan.restype = i32
    lib.knn_plan.argtypes = [i64, i64, i32, i32, i32, i32, optp, sz, ctypes.POINTER(KnnPlanInfo)]
    lib.knn_select.restype = i32
    lib.knn_select.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]
    lib.knn_select_workspace_bytes.restype = sz
    lib.knn_select_workspace_bytes.argtypes = [i64, i64, i32]
    lib.knn_mfma_calibration.restype = i32
    lib.knn_mfma_calibration.argtypes = [i64, i32, vp, sz, ctypes.POINTER(i64), vp]
    lib.knn_mfma_bf16_calibration.restype = i32
    lib.knn_mfma_bf16_calibration.argtypes = [i64, i32, i32, vp, sz, ctypes.POINTER(i64), vp]
    lib.knn_contraction_calibration.restype = i32
    lib.knn_contraction_calibration.argtypes = [i32, i32, i64, vp, vp, sz, ctypes.POINTER(i64), vp]
    lib.knn_read_calibration.restype = i32
    lib.knn_read_calibration.argtypes = [vp, i64, i64, vp, sz, vp]
    lib.knn_valu_calibration.restype = i32
    lib.knn_valu_calibration.argtypes = [i64, i32, vp, sz, ctypes.POINTER(i64), vp]
    lib.knn_status_string.restype = ctypes.c_char_p
    lib.knn_status_string.argtypes = [i32]
    lib.knn_last_device_error.restype = ctypes.c_char_p
    lib.knn_last_device_error.argtypes = []
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != KNN_OK:
        lib = load_library()
        text = lib.knn_status_string(status).decode()
        if status == KNN_EDEVICE:
            text += " (" + lib.knn_last_device_error().decode() + ")"
        raise KnnError(status, text)


def _metric(metric) -> int:
    return METRICS[metric] if isinstance(metric, str) else int(metric)


def _options(symmetric: int, rescore: int, r_splits: int, profile: bool, variant: int = 0,
             block_rows: int = 0, uncertified: Optional[torch.Tensor] = None, center: bool = False):
    opt = KnnOptions()
    opt.symmetric, opt.rescore, opt.r_splits, opt.variant = symmetric, rescore, r_splits, variant
    opt.block_rows = block_rows
    opt.center = int(center)
    if uncertified is not None:
        if not uncertified.is_cuda or uncertified.dtype != torch.int32 or uncertified.numel() < 1:
            raise ValueError("uncertified must be an int32 tensor on the GPU")
        opt.uncertified = uncertified.data_ptr()
    prof = KnnProfile() if profile else None
    if prof is not None:
        opt.profile = ctypes.pointer(prof)
    return opt, prof


def _dev_matrix(x: torch.Tensor, name: str) -> torch.Tensor:
    if not isinstance(x, torch.Tensor) or x.dim() != 2:
        raise TypeError(f"{name} must be a 2-D torch tensor")
    if not x.is_cuda:
        raise ValueError(f"{name} must live on the GPU (no CPU path exists)")
    if x.dtype != torch.float32 or not x.is_contiguous():
        raise ValueError(f"{name} must be contiguous fp32")
    return x


def knn_workspace_bytes(nq: int, nr: int, d: int, k: int, metric="sqeuclidean",
                        symmetric: bool = False, r_splits: int = 0, variant: int = 0,
                        schedule: int = 0, block_rows: int = 0, center: bool = False) -> int:
    """Workspace of knn_build (symmetric=True) or knn_search for the same options; `schedule`
    is the value of their `symmetric` option (0 auto, 1 triangle, 2 full square)."""
    lib = load_library()
    opt, _ = _options(schedule, 0, r_splits, False, variant, block_rows, None, center)
    return int(lib.knn_workspace_bytes_ex(nq, nr, d, k, _metric(metric), int(symmetric),
                                          ctypes.byref(opt)))


def knn_workspace_bytes_min(nq: int, nr: int, d: int, k: int, metric="sqeuclidean",
                            symmetric: bool = False) -> int:
    """Smallest workspace with which a call with default options succeeds (the fused plan's)."""
    return int(load_library().knn_workspace_bytes_min(nq, nr, d, k, _metric(metric), int(symmetric)))


def knn_plan(nq: int, nr: int, d: int, k: int, metric="sqeuclidean", symmetric: bool = False, *,
             workspace_bytes: int = NO_LIMIT, r_splits: int = 0, variant: int = 0, schedule: int = 0,
             block_rows: int = 0, center: bool = False) -> KnnPlanInfo:
    """What knn_build (symmetric=True) or knn_search with these sizes and options would do if
    given a workspace of `workspace_bytes`; see knn_plan in knn.h."""
    lib = load_library()
    opt, _ = _options(schedule, 0, r_splits, False, variant, block_rows, None, center)
    info = KnnPlanInfo()
    _check(lib.knn_plan(nq, nr, d, k, _metric(metric), int(symmetric), ctypes.byref(opt), workspace_bytes,
                        ctypes.byref(info)))
    return info


def _own_workspace(lib, opt, nq, nr, d, k, metric, self_flag, device) -> torch.Tensor:
    """Workspace for a call that brought none: what the preferred plan wants (it may hold
    distances, up to 72 GiB) or, if the device cannot spare that, what the fused plan needs.
    The library takes its plan from the size it is handed; KnnResult.plan says which ran."""
    nbytes = int(lib.knn_workspace_bytes_ex(nq, nr, d, k, _metric(metric), self_flag, ctypes.byref(opt)))
    try:
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    except torch.cuda.OutOfMemoryError:
        if opt.variant != 0:
            raise
        nbytes = int(lib.knn_workspace_bytes_min(nq, nr, d, k, _metric(metric), self_flag))
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _plan_of(lib, opt, nq, nr, d, k, metric, self_flag, workspace) -> KnnPlanInfo:
    info = KnnPlanInfo()
    _check(lib.knn_plan(nq, nr, d, k, _metric(metric), self_flag, ctypes.byref(opt), workspace.numel(),
                        ctypes.byref(info)))
    return info


@dataclass
class KnnResult:
    idx: torch.Tensor                 # [nq, k] int32
    dist: torch.Tensor                # [nq, k] fp32, ascending
    profile: Optional[KnnProfile] = None
    plan: Optional[KnnPlanInfo] = None  # the plan the library took for this call


def knn_build(X: torch.Tensor, k: int, metric="sqeuclidean", *, symmetric: int = 0,
              rescore: int = 0, r_splits: int = 0, variant: int = 0, block_rows: int = 0,
              profile: bool = False, workspace: Optional[torch.Tensor] = None,
              out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
              uncertified: Optional[torch.Tensor] = None, center: bool = False) -> KnnResult:
    """All-pairs self kNN of the rows of X (device tensor); see knn_build in knn.h.
    `uncertified`: int32 device tensor that receives knn_options_t.uncertified (plan 6 only);
    `center`: knn_options_t.center (squared Euclidean: column means subtracted first)."""
    lib = load_library()
    X = _dev_matrix(X, "X")
    n, d = X.shape
    with torch.cuda.device(X.device):
        idx, dist = out if out is not None else (
            torch.empty((n, k), dtype=torch.int32, device=X.device),
            torch.empty((n, k), dtype=torch.float32, device=X.device))
        opt, prof = _options(symmetric, rescore, r_splits, profile, variant, block_rows, uncertified, center)
        if workspace is None:
            workspace = _own_workspace(lib, opt, n, n, d, k, metric, 1, X.device)
        stream = torch.cuda.current_stream(X.device).cuda_stream
        _check(lib.knn_build_ex(X.data_ptr(), n, d, k, _metric(metric), idx.data_ptr(),
                                dist.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                stream, ctypes.byref(opt)))
        plan = _plan_of(lib, opt, n, n, d, k, metric, 1, workspace)
    return KnnResult(idx, dist, prof, plan)


def knn_search(Q: torch.Tensor, R: torch.Tensor, k: int, metric="sqeuclidean",
               self_offset: int = -1, *, rescore: int = 0, r_splits: int = 0, variant: int = 0,
               profile: bool = False, workspace: Optional[torch.Tensor] = None,
               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
               uncertified: Optional[torch.Tensor] = None, center: bool = False) -> KnnResult:
    """Neighbours of every row of Q among the rows of R; see knn_search in knn.h."""
    lib = load_library()
    Q = _dev_matrix(Q, "Q")
    R = _dev_matrix(R, "R")
    if Q.shape[1] != R.shape[1] or Q.device != R.device:
        raise ValueError("Q and R must share dimension and device")
    nq, d = Q.shape
    nr = R.shape[0]
    with torch.cuda.device(Q.device):
        idx, dist = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int32, device=Q.device),
            torch.empty((nq, k), dtype=torch.float32, device=Q.device))
        opt, prof = _options(0, rescore, r_splits, profile, variant, 0, uncertified, center)
        if workspace is None:
            workspace = _own_workspace(lib, opt, nq, nr, d, k, metric, 0, Q.device)
        stream = torch.cuda.current_stream(Q.device).cuda_stream
        _check(lib.knn_search_ex(Q.data_ptr(), nq, R.data_ptr(), nr, d, k, _metric(metric),
                                 self_offset, idx.data_ptr(), dist.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), stream,
                                 ctypes.byref(opt)))
        plan = _plan_of(lib, opt, nq, nr, d, k, metric, 0, workspace)
    return KnnResult(idx, dist, prof, plan)


def knn_search_static(Q: torch.Tensor, R: torch.Tensor, k: int, metric="sqeuclidean", self_offset: int = -1, *,
                      out: Tuple[torch.Tensor, torch.Tensor]) -> KnnResult:
    """knn_search on the library's static scratch array: no workspace, and this binding allocates
    nothing either -- the caller brings the outputs (`out` = (idx int32 [nq,k], dist fp32 [nq,k])).
    See knn_search_static in knn.h; sizes beyond the array raise KnnError(KNN_ENOMEM)."""
    lib = load_library()
    Q = _dev_matrix(Q, "Q")
    R = _dev_matrix(R, "R")
    if Q.shape[1] != R.shape[1] or Q.device != R.device:
        raise ValueError("Q and R must share dimension and device")
    nq, d = Q.shape
    nr = R.shape[0]
    idx, dist = out
    if idx.shape != (nq, k) or dist.shape != (nq, k) or idx.dtype != torch.int32 or dist.dtype != torch.float32 \
            or not idx.is_contiguous() or not dist.is_contiguous() or idx.device != Q.device or dist.device != Q.device:
        raise ValueError("out must be contiguous device tensors (int32 [nq,k], fp32 [nq,k])")
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream(Q.device).cuda_stream
        _check(lib.knn_search_static(Q.data_ptr(), nq, R.data_ptr(), nr, d, k, _metric(metric), self_offset,
                                     idx.data_ptr(), dist.data_ptr(), stream))
    return KnnResult(idx, dist)


def knn_select(A: torch.Tensor, k: int, *, workspace: Optional[torch.Tensor] = None,
               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """k smallest entries of every row of the device matrix A; see knn_select in knn.h.
    A may be a row-strided view (stride(1) == 1).  Returns (idx int32 [m,k], val fp32 [m,k])."""
    lib = load_library()
    if not isinstance(A, torch.Tensor) or A.dim() != 2 or not A.is_cuda or A.dtype != torch.float32:
        raise ValueError("A must be a 2-D fp32 tensor on the GPU")
    if A.stride(1) != 1 or A.stride(0) < A.shape[1]:
        raise ValueError("rows of A must be contiguous")
    m, n = A.shape
    with torch.cuda.device(A.device):
        idx, val = out if out is not None else (
            torch.empty((m, k), dtype=torch.int32, device=A.device),
            torch.empty((m, k), dtype=torch.float32, device=A.device))
        if workspace is None:
            nbytes = int(lib.knn_select_workspace_bytes(m, n, k))
            workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=A.device)
        stream = torch.cuda.current_stream(A.device).cuda_stream
        _check(lib.knn_select(A.data_ptr(), m, n, A.stride(0), k, idx.data_ptr(), val.data_ptr(),
                              workspace.data_ptr(), workspace.numel(), stream))
    return idx, val


def knn_mfma_calibration(mfma_per_wave: int = 1 << 20, waves_per_simd: int = 2, device=None) -> Tuple[float, float]:
    """Time the library's matrix-instruction-only kernel; returns (TFLOP/s, ms).  See
    knn_mfma_calibration in knn.h: a calibration of the device, not part of the method."""
    lib = load_library()
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    with torch.cuda.device(dev):
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        sink = torch.empty(cus * waves_per_simd * 256, dtype=torch.float32, device=dev)
        stream = torch.cuda.current_stream(dev)
        waves = ctypes.c_int64(0)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record(stream)
        _check(lib.knn_mfma_calibration(mfma_per_wave, waves_per_simd, sink.data_ptr(), sink.numel() * 4,
                                        ctypes.byref(waves), stream.cuda_stream))
        stop.record(stream)
        stop.synchronize()
        ms = start.elapsed_time(stop)
    return waves.value * mfma_per_wave * 4096.0 / (ms * 1e-3) / 1e12, ms


def knn_mfma_bf16_calibration(mfma_per_wave: int = 1 << 21, waves_per_simd: int = 2, chains: int = 4,
                              device=None) -> Tuple[float, float]:
    """Time the library's bf16 matrix-instruction-only kernel; returns (TFLOP/s, ms).  See
    knn_mfma_bf16_calibration in knn.h."""
    lib = load_library()
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    with torch.cuda.device(dev):
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        sink = torch.empty(cus * waves_per_simd * 256, dtype=torch.float32, device=dev)
        stream = torch.cuda.current_stream(dev)
        waves = ctypes.c_int64(0)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record(stream)
        _check(lib.knn_mfma_bf16_calibration(mfma_per_wave, waves_per_simd, chains, sink.data_ptr(), sink.numel() * 4,
                                             ctypes.byref(waves), stream.cuda_stream))
        stop.record(stream)
        stop.synchronize()
        ms = start.elapsed_time(stop)
    return waves.value * mfma_per_wave * 32768.0 / (ms * 1e-3) / 1e12, ms


def knn_contraction_calibration(shape: int = 0, dc: int = 32, tiles_per_workgroup: int = 2048,
                                device=None) -> Tuple[float, float]:
    """Time the library's contraction-only kernel (see knn_contraction_calibration in knn.h):
    `shape` 0 = 32x32x2, 1 = 16x16x4 fp32 matrix instruction, `dc` coordinates per LDS step.
    Returns (TFLOP/s, ms)."""
    lib = load_library()
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    with torch.cuda.device(dev):
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        g = torch.Generator(device="cpu").manual_seed(7)
        rows = torch.randn(64, 256, generator=g, dtype=torch.float32).to(dev)
        sink = torch.empty(2 * cus * 256, dtype=torch.float32, device=dev)
        stream = torch.cuda.current_stream(dev)
        wgs = ctypes.c_int64(0)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record(stream)
        _check(lib.knn_contraction_calibration(shape, dc, tiles_per_workgroup, rows.data_ptr(), sink.data_ptr(),
                                               sink.numel() * 4, ctypes.byref(wgs), stream.cuda_stream))
        stop.record(stream)
        stop.synchronize()
        ms = start.elapsed_time(stop)
    return wgs.value * tiles_per_workgroup * 4194304.0 / (ms * 1e-3) / 1e12, ms


def knn_valu_calibration(pairs_per_wave: int = 1 << 22, waves_per_simd: int = 4, device=None) -> Tuple[float, float]:
    """Time the library's vector-instruction-only kernel; returns (1e12 lane operations per second,
    ms).  See knn_valu_calibration in knn.h."""
    lib = load_library()
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    with torch.cuda.device(dev):
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        sink = torch.empty(cus * waves_per_simd * 256 + 16, dtype=torch.float32, device=dev)
        stream = torch.cuda.current_stream(dev)
        waves = ctypes.c_int64(0)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record(stream)
        _check(lib.knn_valu_calibration(pairs_per_wave, waves_per_simd, sink.data_ptr(), sink.numel() * 4,
                                        ctypes.byref(waves), stream.cuda_stream))
        stop.record(stream)
        stop.synchronize()
        ms = start.elapsed_time(stop)
    return waves.value * pairs_per_wave * 128.0 / (ms * 1e-3) / 1e12, ms


def knn_read_calibration(buf: torch.Tensor, floats_per_wave: int = 1 << 18) -> Tuple[float, float]:
    """Time the library's read-only kernel over `buf` (fp32, contiguous, a multiple of 2048
    elements); returns (GB/s, ms).  See knn_read_calibration in knn.h."""
    lib = load_library()
    if buf.dtype != torch.float32 or not buf.is_contiguous() or not buf.is_cuda:
        raise ValueError("buf must be a contiguous fp32 CUDA tensor")
    dev = buf.device
    with torch.cuda.device(dev):
        sink = torch.empty(1024, dtype=torch.float32, device=dev)
        stream = torch.cuda.current_stream(dev)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record(stream)
        _check(lib.knn_read_calibration(buf.data_ptr(), buf.numel(), floats_per_wave, sink.data_ptr(),
                                        sink.numel() * 4, stream.cuda_stream))
        stop.record(stream)
        stop.synchronize()
        ms = start.elapsed_time(stop)
    return buf.numel() * 4.0 / (ms * 1e-3) / 1e9, ms
