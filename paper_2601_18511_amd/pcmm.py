"""ctypes binding of libpcmm.so: same names as the C ABI, argument marshalling only.

There is no CPU fallback: if the HIP library cannot be loaded the import of a function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch  # imported before the library so that both share one HIP runtime

from . import build as _build

PCMM_OK, PCMM_EINVAL, PCMM_EUNSUPPORTED, PCMM_ENOMEM, PCMM_EDEVICE = range(5)

EXPORTED = (
    "pcmm_plan_create",
    "pcmm_plan_workspace_bytes",
    "pcmm_plan_digits",
    "pcmm_run",
    "pcmm_run_profiled",
    "pcmm_run_noalloc",
    "pcmm_plan_destroy",
    "pcmm_status_str",
    "pcmm_mfma_probe",
    "pcmm_ring_decompose",
    "pcmm_ring_compose",
    "pcmm_slot_rearrange",
    "pcmv_plan_create",
    "pcmv_plan_workspace_bytes",
    "pcmv_run",
    "pcmv_plan_destroy",
)

_lib: Optional[ctypes.CDLL] = None


class PcmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s" % (where, pcmm_status_str(status)))


def load_library() -> ctypes.CDLL:
    """Load libpcmm.so; it is built first if there is none or if it was built from other sources than the
    present ones (a stale binary must not pass for the code under test)."""
    global _lib
    if _lib is not None:
        return _lib
    _build.build_library(force=False)
    lib = ctypes.CDLL(_build.LIB)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.pcmm_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, i32, vp, i32, i32, vp, i32, vp]
    lib.pcmm_plan_create.restype = ctypes.c_int
    lib.pcmm_plan_workspace_bytes.argtypes = [vp]
    lib.pcmm_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.pcmm_plan_digits.argtypes = [vp]
    lib.pcmm_plan_digits.restype = i32
    lib.pcmm_run.argtypes = [vp, vp, vp, vp]
    lib.pcmm_run.restype = ctypes.c_int
    lib.pcmm_run_noalloc.argtypes = [vp, vp, vp, vp]
    lib.pcmm_run_noalloc.restype = ctypes.c_int
    lib.pcmm_run_profiled.argtypes = [vp, vp, vp, vp, ctypes.POINTER(ctypes.c_float)]
    lib.pcmm_run_profiled.restype = ctypes.c_int
    lib.pcmm_mfma_probe.argtypes = [i32, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.pcmm_mfma_probe.restype = ctypes.c_int
    for fn in (lib.pcmm_ring_decompose, lib.pcmm_ring_compose):
        fn.argtypes = [vp, vp, i64, i64, i64, i32, vp]
        fn.restype = ctypes.c_int
    lib.pcmm_slot_rearrange.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, i32, vp]
    lib.pcmm_slot_rearrange.restype = ctypes.c_int
    lib.pcmv_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, i32, vp, i32, vp, i32, vp]
    lib.pcmv_plan_create.restype = ctypes.c_int
    lib.pcmv_plan_workspace_bytes.argtypes = [vp]
    lib.pcmv_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.pcmv_run.argtypes = [vp, vp, vp, vp]
    lib.pcmv_run.restype = ctypes.c_int
    lib.pcmv_plan_destroy.argtypes = [vp]
    lib.pcmv_plan_destroy.restype = None
    lib.pcmm_plan_destroy.argtypes = [vp]
    lib.pcmm_plan_destroy.restype = None
    lib.pcmm_status_str.argtypes = [ctypes.c_int]
    lib.pcmm_status_str.restype = ctypes.c_char_p
    _lib = lib
    return lib


def pcmm_status_str(status: int) -> str:
    return load_library().pcmm_status_str(int(status)).decode()


class PcmmPlan:
    """Owner of one pcmm_plan handle."""

    def __init__(self, handle: int, M: int, K: int, Ncols: int, L: int, device: int):
        self.handle = handle
        self.M, self.K, self.Ncols, self.L, self.device = M, K, Ncols, L, device

    def destroy(self) -> None:
        if self.handle:
            load_library().pcmm_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def pcmm_plan_create(W: torch.Tensor, primes: Sequence[int], prime_bits: int, Ncols: int, stream=None) -> PcmmPlan:
    """Plan for the device tensor W ([M][K], int8 or int16) and the host list of primes."""
    if not W.is_cuda or W.dim() != 2 or W.dtype not in (torch.int8, torch.int16) or not W.is_contiguous():
        raise ValueError("W must be a contiguous 2-D int8 or int16 tensor on the GPU")
    M, K = W.shape
    L = len(primes)
    arr = (ctypes.c_uint64 * max(L, 1))(*[int(q) for q in primes])
    out = ctypes.c_void_p()
    w_bits = 8 if W.dtype == torch.int8 else 16
    with torch.cuda.device(W.device):
        rc = load_library().pcmm_plan_create(
            ctypes.byref(out), M, K, int(Ncols), L, ctypes.cast(arr, ctypes.c_void_p), int(prime_bits), w_bits,
            W.data_ptr(), W.device.index, _stream_handle(stream),
        )
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_plan_create")
    return PcmmPlan(out.value, M, K, int(Ncols), L, W.device.index)


def pcmm_plan_workspace_bytes(plan: PcmmPlan) -> int:
    return int(load_library().pcmm_plan_workspace_bytes(plan.handle))


def pcmm_plan_digits(plan: PcmmPlan) -> int:
    return int(load_library().pcmm_plan_digits(plan.handle))


def _check_io(plan: PcmmPlan, A: torch.Tensor, C: torch.Tensor) -> None:
    if plan.handle is None:
        raise ValueError("plan was destroyed")
    for name, t, rows in (("A", A, plan.K), ("C", C, plan.M)):
        if not t.is_cuda or t.device.index != plan.device or not t.is_contiguous():
            raise ValueError("%s must be a contiguous tensor on the plan's device" % name)
        if t.dtype not in (torch.int64, torch.uint64) or tuple(t.shape) != (plan.L, rows, plan.Ncols):
            raise ValueError("%s must be 64-bit integers of shape [L][%d][Ncols]" % (name, rows))


def pcmm_run(plan: PcmmPlan, A: torch.Tensor, C: torch.Tensor, stream=None) -> None:
    """Enqueue C[j] = W . A[j] mod q_j on `stream` (default: torch's current stream). Asynchronous."""
    _check_io(plan, A, C)
    with torch.cuda.device(plan.device):
        rc = load_library().pcmm_run(plan.handle, A.data_ptr(), C.data_ptr(), _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_run")


NOALLOC_SCRATCH_BYTES = 64 << 20     # PCMM_NOALLOC_SCRATCH_BYTES of include/pcmm.h


def pcmm_run_noalloc(plan: PcmmPlan, A: torch.Tensor, C: torch.Tensor, stream=None) -> None:
    """pcmm_run through the library's static digit scratch: the call allocates nothing. Asynchronous."""
    _check_io(plan, A, C)
    with torch.cuda.device(plan.device):
        rc = load_library().pcmm_run_noalloc(plan.handle, A.data_ptr(), C.data_ptr(), _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_run_noalloc")


def pcmm_run_profiled(plan: PcmmPlan, A: torch.Tensor, C: torch.Tensor, stream=None):
    """pcmm_run with per-kernel HIP-event timing; returns (ms_split, ms_gemm) after synchronising."""
    _check_io(plan, A, C)
    ms = (ctypes.c_float * 2)()
    with torch.cuda.device(plan.device):
        rc = load_library().pcmm_run_profiled(plan.handle, A.data_ptr(), C.data_ptr(), _stream_handle(stream), ms)
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_run_profiled")
    return float(ms[0]), float(ms[1])


def pcmm_mfma_probe(device: int = 0, iters: int = 200000, random_operands: bool = True):
    """MFMA-only sustained rate on `device`: returns (TOP/s, shader clock in MHz). Synchronous."""
    tops, mhz = ctypes.c_double(), ctypes.c_double()
    rc = load_library().pcmm_mfma_probe(int(device), int(iters), 1 if random_operands else 0,
                                        ctypes.byref(tops), ctypes.byref(mhz))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_mfma_probe")
    return float(tops.value), float(mhz.value)


def _ring_call(name: str, src: torch.Tensor, dst: torch.Tensor, N: int, k: int, stream) -> None:
    for t in (src, dst):
        if not t.is_cuda or not t.is_contiguous() or t.dtype not in (torch.int64, torch.uint64):
            raise ValueError("ring switching moves contiguous 64-bit integer tensors on the GPU")
    if src.device != dst.device or src.numel() != dst.numel() or src.numel() % int(N):
        raise ValueError("source and destination must hold the same whole number of polynomials of degree N")
    with torch.cuda.device(src.device):
        rc = getattr(load_library(), name)(src.data_ptr(), dst.data_ptr(), src.numel() // int(N), int(N), int(k),
                                           src.device.index, _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, name)


def pcmm_ring_decompose(p: torch.Tensor, parts: torch.Tensor, N: int, k: int, stream=None) -> None:
    """parts[..., j, i] = p[..., i*k + j]: p is [..][N], parts is [..][k][N/k]. Asynchronous."""
    _ring_call("pcmm_ring_decompose", p, parts, N, k, stream)


def pcmm_ring_compose(parts: torch.Tensor, p: torch.Tensor, N: int, k: int, stream=None) -> None:
    """p[..., i*k + j] = parts[..., j, i]: the inverse of pcmm_ring_decompose. Asynchronous."""
    _ring_call("pcmm_ring_compose", parts, p, N, k, stream)


def pcmm_slot_rearrange(S: torch.Tensor, out: torch.Tensor, d: int, ell: int, b: int, k_first: int = 0,
                        k_count: Optional[int] = None, stream=None) -> None:
    """out[e][k - k_first][r][c] = S[e][(r - ell k - (k // b) b) mod d][(c + k) mod d]: the rearranged plaintexts
    number k_first .. k_first + k_count - 1 of the slot-encoded PCMM, from the stored S = tau^ell o sigma(pt_A).
    S is [..][d][d], out is [..][k_count][d][d]. Asynchronous."""
    if k_count is None:
        k_count = int(d) - int(k_first)
    for t in (S, out):
        if not t.is_cuda or not t.is_contiguous() or t.dtype not in (torch.int64, torch.uint64):
            raise ValueError("the rearrangement moves contiguous 64-bit integer tensors on the GPU")
    d = int(d)
    if d <= 0 or S.numel() % (d * d) or S.device != out.device or out.numel() != S.numel() * int(k_count):
        raise ValueError("S must hold whole d x d matrices and out k_count times as many words")
    with torch.cuda.device(S.device):
        rc = load_library().pcmm_slot_rearrange(S.data_ptr(), out.data_ptr(), S.numel() // (d * d), d, int(ell), int(b),
                                                int(k_first), int(k_count), S.device.index, _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmm_slot_rearrange")


class PcmvPlan:
    """Owner of one pcmv_plan handle."""

    def __init__(self, handle: int, Mp: int, Kp: int, N: int, L: int, device: int):
        self.handle = handle
        self.Mp, self.Kp, self.N, self.L, self.device = Mp, Kp, N, L, device

    def destroy(self) -> None:
        if self.handle:
            load_library().pcmv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def pcmv_plan_create(pt: torch.Tensor, primes: Sequence[int], prime_bits: int, stream=None) -> PcmvPlan:
    """PCMv plan for the device tensor pt ([Mp][Kp][N] int32 plaintext coefficients) and the host list of primes."""
    if not pt.is_cuda or pt.dim() != 3 or pt.dtype != torch.int32 or not pt.is_contiguous():
        raise ValueError("pt must be a contiguous [Mp][Kp][N] int32 tensor on the GPU")
    Mp, Kp, N = pt.shape
    L = len(primes)
    arr = (ctypes.c_uint64 * max(L, 1))(*[int(q) for q in primes])
    out = ctypes.c_void_p()
    with torch.cuda.device(pt.device):
        rc = load_library().pcmv_plan_create(ctypes.byref(out), Mp, Kp, N, L, ctypes.cast(arr, ctypes.c_void_p),
                                             int(prime_bits), pt.data_ptr(), pt.device.index, _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmv_plan_create")
    return PcmvPlan(out.value, Mp, Kp, N, L, pt.device.index)


def pcmv_plan_workspace_bytes(plan: PcmvPlan) -> int:
    return int(load_library().pcmv_plan_workspace_bytes(plan.handle))


def pcmv_run(plan: PcmvPlan, ct: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """Enqueue out[j][m][c] = sum_k pt[m][k] * ct[j][k][c] in Z_{q_j}[X]/(X^N+1). ct is [L][Kp][2][N], out [L][Mp][2][N]."""
    if plan.handle is None:
        raise ValueError("plan was destroyed")
    for name, t, rows in (("ct", ct, plan.Kp), ("out", out, plan.Mp)):
        if not t.is_cuda or t.device.index != plan.device or not t.is_contiguous():
            raise ValueError("%s must be a contiguous tensor on the plan's device" % name)
        if t.dtype not in (torch.int64, torch.uint64) or tuple(t.shape) != (plan.L, rows, 2, plan.N):
            raise ValueError("%s must be 64-bit integers of shape [L][%d][2][N]" % (name, rows))
    with torch.cuda.device(plan.device):
        rc = load_library().pcmv_run(plan.handle, ct.data_ptr(), out.data_ptr(), _stream_handle(stream))
    if rc != PCMM_OK:
        raise PcmmError(rc, "pcmv_run")


def pcmv_plan_destroy(plan: PcmvPlan) -> None:
    plan.destroy()


def pcmm_plan_destroy(plan: PcmmPlan) -> None:
    plan.destroy()
