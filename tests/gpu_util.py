"""Helpers for the GPU parity tests: move seeded numpy operands to the device, call the
library through its C ABI (via the ctypes binding) and bring results back."""
import ctypes

import numpy as np
import torch

from paper_2104_09455_amd import binding as B

DT = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}
DEV = "cuda:0"


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    x = np.ascontiguousarray(x)
    if dtype == "f16":
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.float16)
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(x).to(DEV)


def c_to_host(C: torch.Tensor, dtype: str) -> np.ndarray:
    """Device C -> float64 (fp16/bf16, exact widening) or int64 (int8 path)."""
    if dtype == "i8":
        return C.cpu().numpy().astype(np.int64)
    return C.cpu().to(torch.float64).numpy()


class Result:
    def __init__(self, C, flag, report):
        self.C, self.flag, self.report = C, flag, report


def read_report(rep_t):
    raw = rep_t.cpu().numpy().tobytes()
    return B.Report.from_buffer_copy(raw)


def run_gemm(A, Bm, dtype, mode, layout=B.B_NK, inject=None, use_beta=False, want_report=True,
             lda_pad=0, ldb_pad=0, ldc_pad=0, misalign=0) -> Result:
    """A: M x K storage array, Bm: K x N storage array (paper orientation)."""
    dt = DT[dtype]
    M, K = A.shape
    N = Bm.shape[1]
    es = 1 if dtype == "i8" else 2

    def padded(x, pad, mis):
        r, c = x.shape
        buf = np.zeros(r * (c + pad) + mis, dtype=x.dtype)
        view = buf[mis:].reshape(r, c + pad)
        view[:, :c] = x
        return buf, c + pad

    a_buf, lda = padded(A, lda_pad, misalign)
    b_src = Bm.T if layout == B.B_NK else Bm
    b_buf, ldb = padded(np.ascontiguousarray(b_src), ldb_pad, misalign)
    dA, dB = to_dev(a_buf, dtype), to_dev(b_buf, dtype)
    ldc = N + ldc_pad
    c_t = torch.int32 if dtype == "i8" else (torch.float16 if dtype == "f16" else torch.bfloat16)
    dC = torch.zeros(M * ldc, dtype=c_t, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV) if want_report else None
    resolved = mode if mode != B.AUTO else B.abft_select(M, N, K, dt)
    wsb = B.abft_workspace_bytes(M, N, K, dt, resolved)
    ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=DEV)
    beta = None
    if use_beta:
        aligned = misalign == 0 and (K * es) % 16 == 0 and (lda * es) % 16 == 0 and (ldb * es) % 16 == 0 \
            and layout == B.B_NK
        _, rn = B.abft_region_shape(M, N, K, dt, aligned)
        beta = torch.zeros(B.abft_beta_bytes(K, N, rn) // 8, dtype=torch.float64, device=DEV)
        B.abft_weight_checksum(K, N, dB.data_ptr() + misalign * es, ldb, layout, dt, beta, block_n=rn)
    B.abft_gemm(M, N, K, dA.data_ptr() + misalign * es, lda, dB.data_ptr() + misalign * es, ldb, layout,
                dC, ldc, dt, mode, beta=beta, workspace=ws, workspace_bytes=wsb, fault_flag=flag,
                report=rep, inject=inject)
    torch.cuda.synchronize()
    C = c_to_host(dC.view(M, ldc)[:, :N], dtype)
    return Result(C, int(flag.item()), read_report(rep) if want_report else None)


def c_close(C_gpu, C_ref, dtype):
    """The parity bar: bit-exact for int8->int32; |dC| <= 1e-2 |C_ref| + 1e-2 rms(C_ref) for
    fp16/bf16 outputs of fp32 accumulators."""
    if dtype == "i8":
        return np.array_equal(C_gpu, C_ref)
    rms = float(np.sqrt(np.mean(C_ref * C_ref))) if C_ref.size else 0.0
    return bool(np.all(np.abs(C_gpu - C_ref) <= 1e-2 * np.abs(C_ref) + 1e-2 * rms))


def normwise_error(C_gpu, C_ref):
    d = np.linalg.norm(C_ref)
    return float(np.linalg.norm(C_gpu - C_ref) / d) if d > 0 else 0.0
