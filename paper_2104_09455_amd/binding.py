"""ctypes binding of libabft.so: the same entry points as include/abft.h.

Argument marshalling only -- every step of the path runs in the library's HIP
kernels.  Tensors are PyTorch device tensors (PyTorch is used for device memory
and streams, nothing else); their ``data_ptr()`` goes straight through the C ABI.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libabft.so")

# enums of abft.h
NONE, GLOBAL, THREAD, AUTO, REPLICA, THREAD_HALF, TWOSIDED, GLOBAL_WEIGHTED = 0, 1, 2, 3, 4, 5, 6, 7
ACT_NONE, ACT_RELU = 0, 1
F16, BF16, I8 = 0, 1, 2
B_NK, B_KN = 0, 1
OK = 0

MODE_NAMES = {NONE: "none", GLOBAL: "global", THREAD: "thread", AUTO: "auto", REPLICA: "replica",
              THREAD_HALF: "thread_half", TWOSIDED: "twosided", GLOBAL_WEIGHTED: "global_weighted"}
DTYPE_NAMES = {F16: "f16", BF16: "bf16", I8: "i8"}


class Fault(ctypes.Structure):
    _fields_ = [("row", ctypes.c_int64), ("col", ctypes.c_int64), ("bit", ctypes.c_int32),
                ("k_after", ctypes.c_int32)]


class Conv(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("Cin", ctypes.c_int32), ("KH", ctypes.c_int32), ("KW", ctypes.c_int32),
                ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


class Report(ctypes.Structure):
    _fields_ = [("lhs", ctypes.c_double), ("rhs", ctypes.c_double), ("tau", ctypes.c_double),
                ("worst_ratio", ctypes.c_double), ("tiles", ctypes.c_uint64),
                ("frob", ctypes.c_double), ("l1", ctypes.c_double), ("lock", ctypes.c_uint32),
                ("region", ctypes.c_uint32), ("fault_row", ctypes.c_int32), ("fault_col", ctypes.c_int32),
                ("fault_delta", ctypes.c_double), ("ratio_rows", ctypes.c_double), ("ratio_cols", ctypes.c_double)]


class Layer(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("N", ctypes.c_int32), ("K", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("b_layout", ctypes.c_int32), ("has_conv", ctypes.c_int32),
                ("conv", Conv), ("B", ctypes.c_void_p), ("ldb", ctypes.c_int64)]


EXPORTS = [
    "abft_gemm", "abft_conv", "abft_workspace_bytes", "abft_weight_checksum",
    "abft_activation_checksum", "abft_arithmetic_intensity", "abft_cmr", "abft_set_cmr",
    "abft_select", "abft_tile_shape", "abft_tolerance_coeff", "abft_plan_create", "abft_plan_run",
    "abft_plan_mode", "abft_plan_times", "abft_plan_destroy", "abft_strerror", "abft_version",
    "abft_set_kernel_events", "abft_region_shape", "abft_tolerance_bias_coeff",
    "abft_plan_run_all", "abft_plan_set_mode", "abft_k_ways", "abft_beta_bytes", "abft_conv_workspace_bytes",
    "abft_plan_set_activation", "abft_plan_activation", "abft_gemm_static", "abft_static_scratch_bytes",
    "abft_tolerance_half_coeff", "abft_plan_run_chain", "abft_plan_chain_status", "abft_plan_chain_reset",
    "abft_plan_set_diagnostics", "abft_handover_launches", "abft_mfma_probe", "abft_mfma_probe_bytes",
]

_lib = None


def lib() -> ctypes.CDLL:
    """Load libabft.so (once).  Raises if it was not built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2104_09455_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, i64, sz, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_double
    ip = ctypes.POINTER(ctypes.c_int)
    L.abft_gemm.restype = ci
    L.abft_gemm.argtypes = [ci, ci, ci, vp, i64, vp, i64, ci, vp, i64, ci, ci, vp, vp, sz, vp, vp,
                            ctypes.POINTER(Fault), vp]
    L.abft_gemm_static.restype = ci
    L.abft_gemm_static.argtypes = [ci, ci, ci, vp, i64, vp, i64, ci, vp, i64, ci, ci, vp, vp, vp,
                                   ctypes.POINTER(Fault), vp]
    L.abft_static_scratch_bytes.restype = sz
    L.abft_static_scratch_bytes.argtypes = []
    L.abft_conv.restype = ci
    L.abft_conv.argtypes = [ctypes.POINTER(Conv), ci, vp, vp, i64, ci, vp, i64, ci, ci, vp, vp, sz, vp, vp,
                            ctypes.POINTER(Fault), vp]
    L.abft_workspace_bytes.restype = sz
    L.abft_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    L.abft_conv_workspace_bytes.restype = sz
    L.abft_conv_workspace_bytes.argtypes = [ctypes.POINTER(Conv), ci, ci, ci]
    L.abft_beta_bytes.restype = sz
    L.abft_beta_bytes.argtypes = [ci, ci, ci]
    L.abft_weight_checksum.restype = ci
    L.abft_weight_checksum.argtypes = [ci, ci, vp, i64, ci, ci, ci, vp, vp]
    L.abft_activation_checksum.restype = ci
    L.abft_activation_checksum.argtypes = [ci, ci, vp, i64, ctypes.POINTER(Conv), ci, vp, vp]
    L.abft_arithmetic_intensity.restype = dbl
    L.abft_arithmetic_intensity.argtypes = [ci, ci, ci, ci]
    L.abft_cmr.restype = dbl
    L.abft_cmr.argtypes = [ci]
    L.abft_set_cmr.restype = None
    L.abft_set_cmr.argtypes = [ci, dbl]
    L.abft_select.restype = ci
    L.abft_select.argtypes = [ci, ci, ci, ci]
    L.abft_tile_shape.restype = ci
    L.abft_tile_shape.argtypes = [ci, ci, ci, ci, ci, ip, ip, ip]
    L.abft_region_shape.restype = ci
    L.abft_region_shape.argtypes = [ci, ci, ci, ci, ci, ip, ip]
    L.abft_tolerance_bias_coeff.restype = dbl
    L.abft_tolerance_bias_coeff.argtypes = [ci, ci, ci]
    L.abft_tolerance_half_coeff.restype = dbl
    L.abft_tolerance_half_coeff.argtypes = [ci, ci, ci, ci]
    L.abft_tolerance_coeff.restype = dbl
    L.abft_tolerance_coeff.argtypes = [ci, ci, ci]
    L.abft_plan_create.restype = ci
    L.abft_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Layer), ci, ci, vp]
    L.abft_plan_run.restype = ci
    L.abft_plan_run.argtypes = [vp, ci, vp, i64, vp, i64, vp, vp]
    L.abft_plan_run_all.restype = ci
    L.abft_plan_run_all.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.POINTER(vp),
                                    ctypes.POINTER(i64), vp, ci, vp]
    L.abft_plan_run_chain.restype = ci
    L.abft_plan_run_chain.argtypes = [vp, ci, ci, vp, i64, ctypes.POINTER(vp), ctypes.POINTER(i64), vp, vp]
    L.abft_plan_chain_status.restype = ci
    L.abft_plan_chain_status.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), vp]
    L.abft_plan_chain_reset.restype = ci
    L.abft_plan_chain_reset.argtypes = [vp, ci, vp]
    L.abft_handover_launches.restype = ctypes.c_longlong
    L.abft_handover_launches.argtypes = []
    L.abft_mfma_probe_bytes.restype = ctypes.c_size_t
    L.abft_mfma_probe_bytes.argtypes = []
    L.abft_mfma_probe.restype = ctypes.c_int
    L.abft_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    L.abft_plan_set_diagnostics.restype = ci
    L.abft_plan_set_diagnostics.argtypes = [vp, ci, vp, ctypes.POINTER(Fault)]
    L.abft_plan_set_mode.restype = ci
    L.abft_plan_set_mode.argtypes = [vp, ci, ci]
    L.abft_plan_set_activation.restype = ci
    L.abft_plan_set_activation.argtypes = [vp, ci, ci]
    L.abft_plan_activation.restype = ci
    L.abft_plan_activation.argtypes = [vp, ci]
    L.abft_k_ways.restype = ci
    L.abft_k_ways.argtypes = [ci, ci, ci, ci, ci, ci, ip, ip]
    L.abft_plan_mode.restype = ci
    L.abft_plan_mode.argtypes = [vp, ci]
    L.abft_plan_times.restype = ci
    L.abft_plan_times.argtypes = [vp, ci, ctypes.POINTER(dbl)]
    L.abft_plan_destroy.restype = None
    L.abft_plan_destroy.argtypes = [vp]
    L.abft_strerror.restype = ctypes.c_char_p
    L.abft_strerror.argtypes = [ci]
    L.abft_version.restype = ci
    L.abft_version.argtypes = []
    L.abft_set_kernel_events.restype = None
    L.abft_set_kernel_events.argtypes = [vp, vp]
    _lib = L
    return L


class AbftError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"abft error {code}: {abft_strerror(code)}")


def _check(rc: int) -> None:
    if rc != OK:
        raise AbftError(rc)


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---- thin wrappers, one per entry point ------------------------------------
def abft_strerror(code: int) -> str:
    return lib().abft_strerror(code).decode()


def abft_version() -> int:
    return lib().abft_version()


def abft_arithmetic_intensity(M, N, K, dtype) -> float:
    return lib().abft_arithmetic_intensity(M, N, K, dtype)


def abft_cmr(dtype) -> float:
    return lib().abft_cmr(dtype)


def abft_set_cmr(dtype, value) -> None:
    lib().abft_set_cmr(dtype, value)


def abft_select(M, N, K, dtype) -> int:
    rc = lib().abft_select(M, N, K, dtype)
    if rc < 0:
        raise AbftError(rc)
    return rc


def abft_tile_shape(M, N, K, dtype, aligned=True):
    tm, tn, ks = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().abft_tile_shape(M, N, K, dtype, 1 if aligned else 0, ctypes.byref(tm), ctypes.byref(tn),
                                 ctypes.byref(ks)))
    return tm.value, tn.value, ks.value


def abft_k_ways(M, N, K, dtype, mode, aligned=True):
    """(ways, step): wavefront w of `ways` multiplies the k with (k // step) % ways == w."""
    w, st = ctypes.c_int(), ctypes.c_int()
    _check(lib().abft_k_ways(M, N, K, dtype, 1 if aligned else 0, mode, ctypes.byref(w), ctypes.byref(st)))
    return w.value, st.value


def abft_k_parts(M, N, K, dtype, mode, aligned=True):
    """The parts the accumulators of the product are split into along k, as lists of k indices,
    as abft_k_ways says (only tells which accumulator an injected fault lands in).  One part =
    range(K): not split."""
    ways, step = abft_k_ways(M, N, K, dtype, mode, aligned)
    return [[k for k in range(K) if (k // step) % ways == w] for w in range(ways)]


def abft_tolerance_coeff(K, dtype, mode) -> float:
    return lib().abft_tolerance_coeff(K, dtype, mode)


def abft_workspace_bytes(M, N, K, dtype, mode) -> int:
    return lib().abft_workspace_bytes(M, N, K, dtype, mode)


def abft_conv_workspace_bytes(conv, N, dtype, mode) -> int:
    return lib().abft_conv_workspace_bytes(ctypes.byref(conv), N, dtype, mode)


def abft_beta_bytes(K, N, block_n=0) -> int:
    return lib().abft_beta_bytes(K, N, block_n)


def abft_weight_checksum(K, N, B, ldb, b_layout, dtype, beta, block_n=0, stream=None) -> None:
    _check(lib().abft_weight_checksum(K, N, _ptr(B), ldb, b_layout, dtype, block_n, _ptr(beta), _stream(stream)))


def abft_region_shape(M, N, K, dtype, aligned=True):
    rm, rn = ctypes.c_int(), ctypes.c_int()
    _check(lib().abft_region_shape(M, N, K, dtype, 1 if aligned else 0, ctypes.byref(rm), ctypes.byref(rn)))
    return rm.value, rn.value


def abft_tolerance_bias_coeff(K, dtype, mode) -> float:
    return lib().abft_tolerance_bias_coeff(K, dtype, mode)


def abft_tolerance_half_coeff(dtype, mode, tile_m, tile_n) -> float:
    return lib().abft_tolerance_half_coeff(dtype, mode, tile_m, tile_n)


def abft_activation_checksum(M, K, A, lda, dtype, alpha, conv: Optional[Conv] = None, stream=None) -> None:
    cp = ctypes.byref(conv) if conv is not None else None
    _check(lib().abft_activation_checksum(M, K, _ptr(A), lda, cp, dtype, _ptr(alpha), _stream(stream)))


def abft_gemm(M, N, K, A, lda, B, ldb, b_layout, C, ldc, dtype, mode, beta=None, workspace=None,
              workspace_bytes=0, fault_flag=None, report=None, inject: Optional[Fault] = None,
              stream=None) -> None:
    ip = ctypes.byref(inject) if inject is not None else None
    _check(lib().abft_gemm(M, N, K, _ptr(A), lda, _ptr(B), ldb, b_layout, _ptr(C), ldc, dtype, mode,
                           _ptr(beta), _ptr(workspace), workspace_bytes, _ptr(fault_flag), _ptr(report),
                           ip, _stream(stream)))


def abft_gemm_static(M, N, K, A, lda, B, ldb, b_layout, C, ldc, dtype, mode, beta=None, fault_flag=None,
                     report=None, inject: Optional[Fault] = None, stream=None) -> None:
    ip = ctypes.byref(inject) if inject is not None else None
    _check(lib().abft_gemm_static(M, N, K, _ptr(A), lda, _ptr(B), ldb, b_layout, _ptr(C), ldc, dtype, mode,
                                  _ptr(beta), _ptr(fault_flag), _ptr(report), ip, _stream(stream)))


def abft_static_scratch_bytes() -> int:
    return lib().abft_static_scratch_bytes()


def abft_conv(conv: Conv, N, x, B, ldb, b_layout, C, ldc, dtype, mode, beta=None, workspace=None,
              workspace_bytes=0, fault_flag=None, report=None, inject: Optional[Fault] = None,
              stream=None) -> None:
    ip = ctypes.byref(inject) if inject is not None else None
    _check(lib().abft_conv(ctypes.byref(conv), N, _ptr(x), _ptr(B), ldb, b_layout, _ptr(C), ldc, dtype, mode,
                           _ptr(beta), _ptr(workspace), workspace_bytes, _ptr(fault_flag), _ptr(report), ip,
                           _stream(stream)))


def abft_plan_create(layers, profile=False, stream=None) -> int:
    arr = (Layer * len(layers))(*layers)
    handle = ctypes.c_void_p()
    _check(lib().abft_plan_create(ctypes.byref(handle), arr, len(layers), 1 if profile else 0, _stream(stream)))
    return handle.value


def abft_plan_run(plan, layer, A, lda, C, ldc, fault_flag, stream=None) -> None:
    _check(lib().abft_plan_run(plan, layer, _ptr(A), lda, _ptr(C), ldc, _ptr(fault_flag), _stream(stream)))


class PlanIO:
    """Marshalled per-layer input / output pointers for abft_plan_run_all (built once, reused)."""

    def __init__(self, A, lda, C, ldc):
        n = len(A)
        self.A = (ctypes.c_void_p * n)(*[_ptr(a) for a in A])
        self.C = (ctypes.c_void_p * n)(*[_ptr(c) for c in C])
        self.lda = (ctypes.c_int64 * n)(*lda)
        self.ldc = (ctypes.c_int64 * n)(*ldc)


def abft_plan_run_all(plan, io: PlanIO, fault_flag, event_layer=-1, stream=None) -> None:
    _check(lib().abft_plan_run_all(plan, io.A, io.lda, io.C, io.ldc, _ptr(fault_flag), event_layer,
                                   _stream(stream)))


def abft_plan_run_chain(plan, first, count, A, lda, C, ldc, fault_flag, stream=None) -> None:
    """C: list of `count` output tensors (or pointers), ldc: their leading dimensions."""
    cp = (ctypes.c_void_p * count)(*[_ptr(c) for c in C])
    lp = (ctypes.c_int64 * count)(*ldc)
    _check(lib().abft_plan_run_chain(plan, first, count, _ptr(A), lda, cp, lp, _ptr(fault_flag), _stream(stream)))


def abft_plan_chain_status(plan, stream=None) -> int:
    st = ctypes.c_uint32()
    _check(lib().abft_plan_chain_status(plan, ctypes.byref(st), _stream(stream)))
    return st.value


def abft_plan_chain_reset(plan, spin_limit=-1, stream=None) -> None:
    _check(lib().abft_plan_chain_reset(plan, spin_limit, _stream(stream)))


def abft_handover_launches() -> int:
    return int(lib().abft_handover_launches())


def abft_mfma_probe_bytes() -> int:
    return int(lib().abft_mfma_probe_bytes())


def abft_mfma_probe(shape: int, dtype: int, iters: int, operands, sink, stream=None) -> float:
    """One launch of the registers-only MFMA kernel; returns the operations (2 x multiply-adds) it did."""
    ops = ctypes.c_double(0.0)
    _check(lib().abft_mfma_probe(shape, dtype, iters, _ptr(operands), _ptr(sink), ctypes.byref(ops), stream))
    return ops.value


def abft_plan_set_diagnostics(plan, layer, report=None, inject: Optional[Fault] = None) -> None:
    ip = ctypes.byref(inject) if inject is not None else None
    _check(lib().abft_plan_set_diagnostics(plan, layer, _ptr(report), ip))


def abft_plan_set_mode(plan, layer, mode) -> None:
    _check(lib().abft_plan_set_mode(plan, layer, mode))


def abft_plan_set_activation(plan, layer, act) -> None:
    _check(lib().abft_plan_set_activation(plan, layer, act))


def abft_plan_activation(plan, layer) -> int:
    rc = lib().abft_plan_activation(plan, layer)
    if rc < 0:
        raise AbftError(rc)
    return rc


def abft_plan_mode(plan, layer) -> int:
    rc = lib().abft_plan_mode(plan, layer)
    if rc < 0:
        raise AbftError(rc)
    return rc


def abft_plan_times(plan, layer):
    out = (ctypes.c_double * 3)()
    _check(lib().abft_plan_times(plan, layer, out))
    return list(out)


def abft_plan_destroy(plan) -> None:
    lib().abft_plan_destroy(plan)


def abft_set_kernel_events(start_event, stop_event) -> None:
    """hipEvent_t handles (ints) recorded around the matrix-product kernel; None, None = off."""
    lib().abft_set_kernel_events(start_event, stop_event)
