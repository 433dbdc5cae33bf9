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


def sample_rows(M, n, band=256, seed=0):
    """About n row indices of 0..M-1 that hit every band of `band` rows (its first and last row
    among them), the rest drawn from a seeded generator; all rows when M <= n."""
    if M <= n:
        return np.arange(M)
    rng = np.random.default_rng(seed)
    rows = set()
    bands = range(0, M, band)
    per = max(2, n // max(1, len(bands)))
    for b0 in bands:
        b1 = min(b0 + band, M)
        rows.update((b0, b1 - 1))
        rows.update(int(r) for r in rng.integers(b0, b1, size=max(0, per - 2)))
    while len(rows) < n:   # (draws that coincided)
        rows.add(int(rng.integers(M)))
    return np.array(sorted(rows))


class DeviceGemm:
    """Device-resident operands of one product (weights stored N x K), reused over many calls."""

    def __init__(self, M, N, K, dtype, seed, dist_a="normal", dist_b=None, operands=None):
        from paper_2104_09455_amd import workloads as wl
        self.M, self.N, self.K, self.dtype, self.dt = M, N, K, dtype, DT[dtype]
        if operands is None:
            operands = wl.gemm_operands(M, N, K, dtype, seed, dist_a=dist_a, dist_b=dist_b or dist_a)
        self.A, self.Bm = operands
        self.dA = to_dev(self.A, dtype)
        self.dB = to_dev(np.ascontiguousarray(self.Bm.T), dtype)
        c_t = torch.int32 if dtype == "i8" else (torch.float16 if dtype == "f16" else torch.bfloat16)
        self.dC = torch.zeros((M, N), dtype=c_t, device=DEV)
        self.flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        self.rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV)
        self.wsb = max(B.abft_workspace_bytes(M, N, K, self.dt, m) for m in (B.NONE, B.GLOBAL, B.THREAD))
        self.ws = torch.zeros(max(self.wsb, 256), dtype=torch.uint8, device=DEV)
        es = 1 if dtype == "i8" else 2
        self.aligned = (K * es) % 16 == 0
        self.rm, self.rn = B.abft_region_shape(M, N, K, self.dt, self.aligned)
        self.tm, self.tn, self.k_step = B.abft_tile_shape(M, N, K, self.dt, self.aligned)
        self.beta = torch.zeros(B.abft_beta_bytes(K, N, self.rn) // 8, dtype=torch.float64, device=DEV)
        B.abft_weight_checksum(K, N, self.dB, K, B.B_NK, self.dt, self.beta, block_n=self.rn)  # offline (Sec. 2.5)

    def run(self, mode, inject=None, want_report=True):
        self.flag.zero_()
        self.rep.zero_()
        B.abft_gemm(self.M, self.N, self.K, self.dA, self.K, self.dB, self.K, B.B_NK, self.dC, self.N, self.dt,
                    mode, beta=self.beta, workspace=self.ws, workspace_bytes=self.wsb, fault_flag=self.flag,
                    report=self.rep if want_report else None, inject=inject)
        torch.cuda.synchronize()
        return int(self.flag.item()), (read_report(self.rep) if want_report else None)

    def C(self, rows=None, cols=None):
        c = self.dC
        if rows is not None:
            c = c[torch.as_tensor(np.asarray(rows), device=DEV)]
        if cols is not None:
            c = c[:, torch.as_tensor(np.asarray(cols), device=DEV)]
        return c_to_host(c, self.dtype)

    def region_of(self, i, j, mode):
        """(r0, r1, c0, c1) of the comparison region of `mode` that holds element (i, j)."""
        bm, bn = (self.rm, self.rn) if mode == B.GLOBAL else (self.tm, self.tn)
        r0, c0 = i // bm * bm, j // bn * bn
        return r0, min(r0 + bm, self.M), c0, min(c0 + bn, self.N)


class DeviceConv:
    """Device-resident operands of one convolution layer (NHWC input, weights N x K)."""

    def __init__(self, c, dtype, seed, lowered=True):
        from paper_2104_09455_amd import workloads as wl
        self.c, self.dtype, self.dt = c, dtype, DT[dtype]
        self.x, self.Wm = wl.conv_operands(c, dtype, seed)
        self.M, self.K, self.N = c.batch * c.OH * c.OW, c.KH * c.KW * c.Cin, c.Cout
        self.dx = to_dev(self.x, dtype)
        self.dB = to_dev(np.ascontiguousarray(self.Wm.T), dtype)
        c_t = torch.int32 if dtype == "i8" else (torch.float16 if dtype == "f16" else torch.bfloat16)
        self.dC = torch.zeros((self.M, self.N), dtype=c_t, device=DEV)
        self.flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        self.rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV)
        self.conv = B.Conv(c.batch, c.H, c.W, c.Cin, c.KH, c.KW, c.stride, c.pad)
        modes = (B.NONE, B.GLOBAL, B.THREAD)
        self.wsb = max(B.abft_workspace_bytes(self.M, self.N, self.K, self.dt, m) for m in modes)
        if lowered:   # room for the padded input copy and the re-ordered weights of a few-channel layer
            self.wsb = max(self.wsb, max(B.abft_conv_workspace_bytes(self.conv, self.N, self.dt, m) for m in modes))
        self.ws = torch.zeros(max(self.wsb, 256), dtype=torch.uint8, device=DEV)

    def run(self, mode, inject=None, want_report=True):
        self.flag.zero_()
        self.rep.zero_()
        B.abft_conv(self.conv, self.N, self.dx, self.dB, self.K, B.B_NK, self.dC, self.N, self.dt, mode,
                    workspace=self.ws, workspace_bytes=self.wsb, fault_flag=self.flag,
                    report=self.rep if want_report else None, inject=inject)
        torch.cuda.synchronize()
        return int(self.flag.item()), (read_report(self.rep) if want_report else None)

    def C(self, rows=None):
        c = self.dC if rows is None else self.dC[torch.as_tensor(np.asarray(rows), device=DEV)]
        return c_to_host(c, self.dtype)


WAVE_LEVEL = (B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED)   # one comparison per wavefront tile


def wave_check(mode, A, Bm, C, dtype, region, tile):
    """The oracle's check of one wavefront register tile (region = r0, r1, c0, c1; tile = the
    nominal tile shape) under the wavefront-level scheme `mode`."""
    import oracle
    if mode == B.REPLICA:
        return oracle.replica_check(A, Bm, C, dtype, *region)
    return oracle.tile_check(A, Bm, C, dtype, *region, two_sided=mode == B.TWOSIDED,
                             operand_sums=tuple(tile) if mode in (B.THREAD_HALF, B.TWOSIDED) else None)
