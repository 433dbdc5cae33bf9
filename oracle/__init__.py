"""CPU oracle for ABFT-protected matrix multiplication -- TEST INFRASTRUCTURE ONLY.

Plain fp64 / int64 definitions of what the protected GEMM path computes, written
from the paper ("Arithmetic-Intensity-Guided Fault Tolerance for Neural Network
Inference on GPUs", SC '21).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product never does, and this
package imports nothing from the product.

The heavy loops live in ``abft_oracle.c`` (built by ``oracle/build.py`` into
``libabft_oracle.so``); this module marshals numpy arrays into them and adds the
few scalar formulas (tolerance, comparison, selector) on top.

Conventions (Sec. 2.1): A is M x K activations, B is K x N weights, C = A.B.
Floating-point operands arrive as *storage* arrays -- ``numpy.float16`` for fp16,
``numpy.uint16`` bit patterns for bf16 -- and are widened exactly to fp64 before
any arithmetic; int8 operands are widened to int64.

Parity pins (tests/test_oracle_*.py): the GEMM against brute force and
``numpy.matmul``; the checksum identity exactly over integers and within a
rigorous rounding bound in fp64; the tile checks against the global identity
they telescope to; detection exhaustively over every bit of every element on
small integer cases; arithmetic intensity / CMR / selector against every value
the paper prints (Fig. 5, Fig. 11 axis labels, Fig. 10 labels, Sec. 3.3); the
layer chain (activation function, storage rounding) against closed forms, every
representable fp16 / bf16 value and its midpoints, and an exact integer chain.
Parity unpinned by the paper: the floating-point tolerance itself -- the paper never states one
(it says "equality check").  Its constants are this build's reading; the tests pin them from
both sides against things derived apart from them: ``C_TOL`` against a binary32 accumulation
simulated with plain IEEE arithmetic (residuals stay under a quarter of the tolerance) and
against the first-order worst-case bound of recursive summation (the tolerance stays far below
it), ``U_CHI`` against the representation error of a sum handed on in fp16 / bf16 pieces,
``C_BIAS`` as a fixed fraction of that worst-case bound; the size of ``C_BIAS`` additionally
rests on measurements of the accelerator's accumulation.
"""
from __future__ import annotations

import ctypes
import math
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libabft_oracle.so")
_lib = None

F16, BF16, I8 = "f16", "bf16", "i8"

# Floating-point tolerance of the checksum comparison (this build's reading; the
# paper is silent).  Accumulators are binary32, so one rounding is at most
# U32 = 2^-24 relative.  An accumulator that receives K products one after the
# other carries a random-walk error of about U32 * sqrt(K) * |C_ij| / 2.4, and
# the errors of the entries of C add in quadrature when C is summed, giving
# about 0.4 * U32 * sqrt(K) * ||C||_F; the checksum side of the thread-level
# scheme is accumulated the same way and contributes as much again.  C_TOL = 8
# therefore sits more than ten standard deviations above the noise.
U32 = 2.0 ** -24
C_TOL = 8.0


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} not built: run `python oracle/build.py` (or __graft_entry__.build())")
    lib = ctypes.CDLL(_LIB_PATH)
    dp = ctypes.POINTER(ctypes.c_double)
    i8p = ctypes.POINTER(ctypes.c_int8)
    i64p = ctypes.POINTER(ctypes.c_int64)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    ip = ctypes.POINTER(ctypes.c_int)
    ci, cd = ctypes.c_int, ctypes.c_double
    sig = {
        "orc_threads": (ci, []),
        "orc_f16_bits_to_f64": (cd, [ctypes.c_uint16]),
        "orc_bf16_bits_to_f64": (cd, [ctypes.c_uint16]),
        "orc_widen_f16": (None, [u16p, ctypes.c_size_t, dp]),
        "orc_widen_bf16": (None, [u16p, ctypes.c_size_t, dp]),
        "orc_gemm_f64": (None, [ci, ci, ci, dp, dp, dp]),
        "orc_gemm_i8": (None, [ci, ci, ci, i8p, i8p, i64p]),
        "orc_gemm_rows_f64": (None, [ci, ip, ci, ci, dp, dp, dp]),
        "orc_gemm_rows_i8": (None, [ci, ip, ci, ci, i8p, i8p, i64p]),
        "orc_partial_dot_f64": (cd, [ci, ci, dp, dp, ci, ci, ci, ci]),
        "orc_partial_dot_i8": (ctypes.c_int64, [ci, ci, i8p, i8p, ci, ci, ci, ci]),
        "orc_col_checksum_f64": (None, [ci, ci, dp, dp]),
        "orc_row_checksum_f64": (None, [ci, ci, dp, dp]),
        "orc_col_checksum_i8": (None, [ci, ci, i8p, i64p]),
        "orc_row_checksum_i8": (None, [ci, ci, i8p, i64p]),
        "orc_dot_f64": (cd, [ci, dp, dp]),
        "orc_dot_i64": (ctypes.c_int64, [ci, i64p, i64p]),
        "orc_block_sum_f64": (cd, [ci, dp, ci, ci, ci, ci]),
        "orc_block_sum_i64": (ctypes.c_int64, [ci, i64p, ci, ci, ci, ci]),
        "orc_phi_f64": (cd, [ci, ci, ci, dp, dp]),
        "orc_sabs_f64": (cd, [ci, ci, ci, dp, dp]),
        "orc_tile_one_sided_f64": (None, [ci, ci, dp, dp, dp, ci, ci, ci, ci, dp, dp]),
        "orc_tile_one_sided_i8": (None, [ci, ci, i8p, i8p, i64p, ci, ci, ci, ci, i64p, i64p]),
        "orc_tile_two_sided_f64": (None, [ci, ci, dp, dp, dp, ci, ci, ci, ci, dp, dp]),
        "orc_tile_two_sided_i8": (None, [ci, ci, i8p, i8p, i64p, ci, ci, ci, ci, i64p, i64p]),
        "orc_flip_bit_f32": (cd, [cd, ci]),
        "orc_flip_bit_i32": (ctypes.c_int64, [ctypes.c_int64, ci]),
        "orc_flops": (cd, [cd, cd, cd, ci]),
        "orc_bytes": (cd, [cd, cd, cd, cd, cd, cd, ci]),
        "orc_arithmetic_intensity": (cd, [cd, cd, cd, cd, cd, cd, ci]),
        "orc_cmr": (cd, [cd, cd]),
        "orc_compute_bound": (ci, [cd, cd]),
        "orc_select": (ci, [cd, cd]),
        "orc_im2col_f64": (None, [ci, ci, ci, ci, ci, ci, ci, ci, dp, dp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _d(a):
    return _p(a, ctypes.c_double)


def threads() -> int:
    """Host threads the OpenMP loops of the oracle use."""
    return _load().orc_threads()


# --------------------------------------------------------------------------- #
# widening
# --------------------------------------------------------------------------- #
def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> exact fp64 (fp16/bf16) or the int8 array itself, C-contiguous."""
    lib = _load()
    x = np.ascontiguousarray(x)
    if x.dtype == np.float64 and dtype in (F16, BF16):
        return x  # already widened (e.g. the output of im2col)
    if dtype == F16:
        bits = x.view(np.uint16) if x.dtype == np.float16 else x
        assert bits.dtype == np.uint16
        out = np.empty(bits.shape, dtype=np.float64)
        lib.orc_widen_f16(_p(bits, ctypes.c_uint16), bits.size, _d(out))
        return out
    if dtype == BF16:
        assert x.dtype == np.uint16, "bf16 operands are passed as uint16 bit patterns"
        out = np.empty(x.shape, dtype=np.float64)
        lib.orc_widen_bf16(_p(x, ctypes.c_uint16), x.size, _d(out))
        return out
    if dtype == I8:
        assert x.dtype == np.int8
        return x
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# GEMM
# --------------------------------------------------------------------------- #
def gemm(A: np.ndarray, B: np.ndarray, dtype: str) -> np.ndarray:
    """C = A.B from storage operands: fp64 for fp16/bf16 inputs, int64 for int8 (Sec. 2.1)."""
    lib = _load()
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    M, K = Aw.shape
    K2, N = Bw.shape
    assert K == K2
    if dtype == I8:
        C = np.empty((M, N), dtype=np.int64)
        lib.orc_gemm_i8(M, N, K, _p(Aw, ctypes.c_int8), _p(Bw, ctypes.c_int8), _p(C, ctypes.c_int64))
    else:
        C = np.empty((M, N), dtype=np.float64)
        lib.orc_gemm_f64(M, N, K, _d(Aw), _d(Bw), _d(C))
    return C


def gemm_rows(A: np.ndarray, B: np.ndarray, dtype: str, rows) -> np.ndarray:
    """Rows ``rows`` of C = A.B only (spot checks at sizes where all of C is too slow)."""
    lib = _load()
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    M, K = Aw.shape
    N = Bw.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert rows.min() >= 0 and rows.max() < M
    if dtype == I8:
        out = np.empty((len(rows), N), dtype=np.int64)
        lib.orc_gemm_rows_i8(len(rows), _p(rows, ctypes.c_int), N, K, _p(Aw, ctypes.c_int8),
                             _p(Bw, ctypes.c_int8), _p(out, ctypes.c_int64))
    else:
        out = np.empty((len(rows), N), dtype=np.float64)
        lib.orc_gemm_rows_f64(len(rows), _p(rows, ctypes.c_int), N, K, _d(Aw), _d(Bw), _d(out))
    return out


def partial_dot(A, B, dtype, i, j, k_begin, k_end):
    """sum_{k_begin <= k < k_end} A[i,k] B[k,j]: the running accumulator of element (i, j)."""
    lib = _load()
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    K, N = Bw.shape
    if dtype == I8:
        return int(lib.orc_partial_dot_i8(N, K, _p(Aw, ctypes.c_int8), _p(Bw, ctypes.c_int8), i, j,
                                          k_begin, k_end))
    return float(lib.orc_partial_dot_f64(N, K, _d(Aw), _d(Bw), i, j, k_begin, k_end))


# --------------------------------------------------------------------------- #
# the ABFT checksums (Sec. 2.4 steps 1-3)
# --------------------------------------------------------------------------- #
def col_checksum(A, dtype):
    """alpha[k] = sum_i A[i,k]: the 1 x K activation checksum."""
    lib = _load()
    Aw = widen(A, dtype)
    M, K = Aw.shape
    if dtype == I8:
        out = np.empty(K, dtype=np.int64)
        lib.orc_col_checksum_i8(M, K, _p(Aw, ctypes.c_int8), _p(out, ctypes.c_int64))
    else:
        out = np.empty(K, dtype=np.float64)
        lib.orc_col_checksum_f64(M, K, _d(Aw), _d(out))
    return out


def row_checksum(B, dtype):
    """beta[k] = sum_j B[k,j]: the K x 1 weight checksum."""
    lib = _load()
    Bw = widen(B, dtype)
    K, N = Bw.shape
    if dtype == I8:
        out = np.empty(K, dtype=np.int64)
        lib.orc_row_checksum_i8(K, N, _p(Bw, ctypes.c_int8), _p(out, ctypes.c_int64))
    else:
        out = np.empty(K, dtype=np.float64)
        lib.orc_row_checksum_f64(K, N, _d(Bw), _d(out))
    return out


def checksum_dot(alpha, beta):
    lib = _load()
    if alpha.dtype == np.int64:
        return int(lib.orc_dot_i64(len(alpha), _p(alpha, ctypes.c_int64), _p(beta, ctypes.c_int64)))
    return float(lib.orc_dot_f64(len(alpha), _d(alpha), _d(beta)))


def block_sum(C, r0=0, r1=None, c0=0, c1=None):
    """Sum of C[r0:r1, c0:c1] (the output summation; whole matrix by default)."""
    lib = _load()
    C = np.ascontiguousarray(C)
    M, N = C.shape
    r1 = M if r1 is None else r1
    c1 = N if c1 is None else c1
    if C.dtype == np.int64:
        return int(lib.orc_block_sum_i64(N, _p(C, ctypes.c_int64), r0, r1, c0, c1))
    return float(lib.orc_block_sum_f64(N, _d(C), r0, r1, c0, c1))


def phi(A, B, dtype):
    lib = _load()
    Aw, Bw = widen(A, dtype).astype(np.float64), widen(B, dtype).astype(np.float64)
    M, K = Aw.shape
    N = Bw.shape[1]
    return float(lib.orc_phi_f64(M, N, K, _d(np.ascontiguousarray(Aw)), _d(np.ascontiguousarray(Bw))))


def s_abs(A, B, dtype):
    lib = _load()
    Aw, Bw = widen(A, dtype).astype(np.float64), widen(B, dtype).astype(np.float64)
    M, K = Aw.shape
    N = Bw.shape[1]
    return float(lib.orc_sabs_f64(M, N, K, _d(np.ascontiguousarray(Aw)), _d(np.ascontiguousarray(Bw))))


# --------------------------------------------------------------------------- #
# tolerance and comparison (Sec. 2.4 step 4)
# --------------------------------------------------------------------------- #
def frob(C, r0=0, r1=None, c0=0, c1=None) -> float:
    blk = np.asarray(C, dtype=np.float64)[r0:r1, c0:c1]
    with np.errstate(over="ignore", invalid="ignore"):
        return float(np.sqrt(np.sum(blk * blk)))


# Precision of the tile checksum operand in the thread-level scheme: the checksum of
# B_t is formed in binary32 and handed to the matrix unit as two fp16 pieces (22 bits)
# or three bf16 pieces (24 bits), so it adds a relative 2^-22 / 2^-23 on top of the
# accumulation noise.  The global scheme keeps its checksums in fp64 and adds nothing.
U_CHI = {F16: 2.0 ** -22, BF16: 2.0 ** -23}

# Global scheme only: the accelerator's binary32 accumulation is not perfectly unbiased;
# measured on MI355X, every entry of C carries a same-sign error of up to about
# 2e-4 * 2^-24 * K * |C_ij| when the operands have the same sign, which adds coherently
# under the output summation.  C_BIAS = 1e-3 covers it five times over.  (In the
# thread-level scheme both sides of the comparison are accumulated the same way and
# the bias cancels.)
C_BIAS = 1.0e-3


def l1norm(C, r0=0, r1=None, c0=0, c1=None) -> float:
    blk = np.asarray(C, dtype=np.float64)[r0:r1, c0:c1]
    with np.errstate(over="ignore", invalid="ignore"):
        return float(np.sum(np.abs(blk)))


# Thread-level schemes that add their checksums in the operand type (the paper's packed
# half-precision adds, Sec. 5.2.2): every such add rounds to U_HALF.  The rounding errors of
# the B-side checksum enter the comparison weighted with the column sums of the A tile, each at
# most sqrt(tile rows) times the norm of that column (Cauchy-Schwarz), and the other way round
# for the A-side checksum of the two-sided scheme.  C_HALF = 4 sits on top of that bound.
U_HALF = {F16: 2.0 ** -11, BF16: 2.0 ** -8}
C_HALF = 4.0


def half_sum_term(dtype, frob_norm, tile_m, tile_n, two_sided, block=32):
    """What the roundings of checksums added in the operand type add to the tolerance of a
    tile_m x tile_n register tile made of block x block outputs of the matrix instruction: the
    B-side checksum takes tile_n / block - 1 adds per element, the A-side one (two-sided scheme
    only) tile_m / block - 1."""
    if dtype == I8:
        return 0.0
    n_b = max(tile_n // block - 1, 0)
    n_a = max(tile_m // block - 1, 0) if two_sided else 0
    return C_HALF * U_HALF[dtype] * math.sqrt(n_b * tile_m + n_a * tile_n) * frob_norm


def tolerance(K: int, frob_norm: float, dtype: str, scheme: int = 1, l1_norm: float = 0.0) -> float:
    """Tolerance of one comparison over a region S of C (fp32 accumulators):
         global (scheme=1):  tau = C_TOL * 2^-24 * sqrt(K) * ||C_S||_F + C_BIAS * 2^-24 * K * ||C_S||_1
         thread (scheme=2):  tau = C_TOL * (2^-24 * sqrt(K) + U_CHI[dtype]) * ||C_S||_F
       (the schemes that add checksums in the operand type add half_sum_term to the latter)
       0 for int8 (exact comparison)."""
    if dtype == I8:
        return 0.0
    if scheme == 2:
        return C_TOL * (U32 * math.sqrt(K) + U_CHI[dtype]) * frob_norm
    return C_TOL * U32 * math.sqrt(K) * frob_norm + C_BIAS * U32 * K * l1_norm


def rigorous_bound(M, N, K, sabs):
    """|s_C - s_AB| <= gamma * S_abs can never be violated by rounding alone in binary32
    accumulation (K adds per entry, ceil(log2(MN)) levels of summation, slack 4)."""
    return (K + math.ceil(math.log2(max(M * N, 2))) + 4) * U32 * sabs


def mismatch(lhs, rhs, tau) -> bool:
    """True when the two checksums disagree.  Written so that NaN and infinities flag."""
    if isinstance(lhs, (int, np.integer)) and isinstance(rhs, (int, np.integer)):
        return int(lhs) != int(rhs)
    if not (math.isfinite(lhs) and math.isfinite(rhs)):
        return True
    return not (abs(lhs - rhs) <= tau)


@dataclass
class Check:
    lhs: float  # output summation (of C or of the tile)
    rhs: float  # checksum product
    tau: float
    flag: bool

    @property
    def residual(self):
        return self.lhs - self.rhs


def global_check(A, B, C, dtype) -> Check:
    """Global ABFT (Sec. 2.4): (1^T A)(B 1) against sum(C) for the C that is passed in."""
    K = A.shape[1]
    s_ab = checksum_dot(col_checksum(A, dtype), row_checksum(B, dtype))
    s_c = block_sum(C)
    tau = tolerance(K, frob(C), dtype, scheme=1, l1_norm=l1norm(C))
    return Check(s_c, s_ab, tau, mismatch(s_c, s_ab, tau))


def region_check(A, B, C, dtype, r0, r1, c0, c1) -> Check:
    """Global ABFT restricted to the block rows r0..r1 x columns c0..c1 of C: the checksum
    of those rows of A times the checksum of those columns of B against the block's sum."""
    lib = _load()
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    K, N = Bw.shape
    C = np.ascontiguousarray(C)
    if dtype == I8:
        lhs, rhs = ctypes.c_int64(), ctypes.c_int64()
        lib.orc_tile_two_sided_i8(N, K, _p(Aw, ctypes.c_int8), _p(Bw, ctypes.c_int8), _p(C, ctypes.c_int64),
                                  r0, r1, c0, c1, ctypes.byref(lhs), ctypes.byref(rhs))
        return Check(lhs.value, rhs.value, 0.0, lhs.value != rhs.value)
    lhs, rhs = ctypes.c_double(), ctypes.c_double()
    lib.orc_tile_two_sided_f64(N, K, _d(Aw), _d(Bw), _d(C), r0, r1, c0, c1, ctypes.byref(lhs),
                               ctypes.byref(rhs))
    tau = tolerance(K, frob(C, r0, r1, c0, c1), dtype, scheme=1, l1_norm=l1norm(C, r0, r1, c0, c1))
    return Check(lhs.value, rhs.value, tau, mismatch(lhs.value, rhs.value, tau))


def global_check_blocks(A, B, C, dtype, block_m, block_n):
    """Global ABFT with one comparison per block_m x block_n block of C (the identity of
    Sec. 2.4 applied to each row block of A and column block of B; summed over the blocks
    it is the whole-matrix identity).  The layer is flagged when any block is."""
    M, N = C.shape
    checks = [region_check(A, B, C, dtype, *t) for t in tiles(M, N, block_m, block_n)]
    return any(c.flag for c in checks), checks


@dataclass
class WeightedCheck:
    """Three comparisons of one region (Sec. 2.4, last paragraph: several checksums from
    independent linear combinations): plain, rows weighted, columns weighted."""
    plain: Check
    rows: Check
    cols: Check

    @property
    def flag(self):
        return self.plain.flag or self.rows.flag or self.cols.flag


def weighted_region_check(A, B, C, dtype, r0, r1, c0, c1, block_m=None, block_n=None) -> WeightedCheck:
    """Global ABFT of the block rows r0..r1 x columns c0..c1 of C with three independent checksum
    pairs: with 1 the all-ones vector, w the row weights and v the column weights of the block,
         plain:  (1^T A_S)(B_S 1)  against  sum_ij C_ij
         rows:   (w^T A_S)(B_S 1)  against  sum_ij w_i C_ij
         cols:   (1^T A_S)(B_S v)  against  sum_ij v_j C_ij
    Integer operands: w_i = i + 1, v_j = j + 1 (local indices), exact comparisons.  Floating
    point: w_i = (i + 1) / block_m, v_j = (j + 1) / block_n (block_m, block_n: the nominal block
    shape, default the block itself), tolerance as for the global scheme on the weighted block.
    One wrong element (i, j) of the block off by delta leaves the residuals delta, w_i delta and
    v_j delta (locate); two wrong elements whose errors cancel in the plain sum still show in the
    weighted ones unless they share the row and the column weights."""
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    K = Aw.shape[1]
    bm, bn = block_m or (r1 - r0), block_n or (c1 - c0)
    acc_t = np.int64 if dtype == I8 else np.float64
    As = np.asarray(Aw[r0:r1], dtype=acc_t)
    Bs = np.asarray(Bw[:, c0:c1], dtype=acc_t)
    Cs = np.asarray(C, dtype=acc_t)[r0:r1, c0:c1]
    w = np.arange(1, r1 - r0 + 1, dtype=acc_t)
    v = np.arange(1, c1 - c0 + 1, dtype=acc_t)
    if dtype != I8:
        w, v = w / bm, v / bn
    alpha, alpha_w = As.sum(axis=0), (w[:, None] * As).sum(axis=0)     # 1^T A_S, w^T A_S
    beta, beta_v = Bs.sum(axis=1), (Bs * v[None, :]).sum(axis=1)       # B_S 1,   B_S v
    out = []
    for a_vec, b_vec, Cw in ((alpha, beta, Cs), (alpha_w, beta, w[:, None] * Cs), (alpha, beta_v, Cs * v[None, :])):
        if dtype == I8:
            lhs, rhs = int(Cw.sum()), int(np.dot(a_vec, b_vec))
            out.append(Check(lhs, rhs, 0.0, lhs != rhs))
        else:
            with np.errstate(over="ignore", invalid="ignore"):
                lhs, rhs = float(Cw.sum()), float(np.dot(a_vec, b_vec))
                tau = tolerance(K, float(np.sqrt(np.sum(Cw * Cw))), dtype, scheme=1, l1_norm=float(np.sum(np.abs(Cw))))
            out.append(Check(lhs, rhs, tau, mismatch(lhs, rhs, tau)))
    return WeightedCheck(*out)


def locate(wc: WeightedCheck, dtype, block_m, block_n):
    """(row, col, delta) of a single wrong element of the block, local indices, from the three
    residuals: w_i = rows residual / plain residual, v_j likewise.  None when the plain
    comparison holds (nothing to locate, or errors that cancel in the plain sum)."""
    d0 = wc.plain.residual
    if not wc.plain.flag or d0 == 0:
        return None
    if dtype == I8:
        i, j = wc.rows.residual // d0 - 1, wc.cols.residual // d0 - 1
    else:
        i, j = round(block_m * wc.rows.residual / d0) - 1, round(block_n * wc.cols.residual / d0) - 1
    return int(i), int(j), d0


def tiles(M, N, tile_m, tile_n):
    """The partition of C into register tiles (edge tiles clipped), row-major order."""
    for r0 in range(0, M, tile_m):
        for c0 in range(0, N, tile_n):
            yield r0, min(r0 + tile_m, M), c0, min(c0 + tile_n, N)


def tile_check(A, B, C, dtype, r0, r1, c0, c1, two_sided=False, operand_sums=None) -> Check:
    """Thread-level ABFT for one tile (Sec. 5.2.2): one-sided by default, two-sided (Sec. 5.2.1)
    on request.  operand_sums = (tile_m, tile_n): the checksums are added up in the operand type
    on register tiles of that nominal shape, which widens the tolerance (half_sum_term); the two
    sides of the comparison are the exact ones either way."""
    lib = _load()
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    K, N = Bw.shape
    C = np.ascontiguousarray(C)
    if dtype == I8:
        lhs, rhs = ctypes.c_int64(), ctypes.c_int64()
        fn = lib.orc_tile_two_sided_i8 if two_sided else lib.orc_tile_one_sided_i8
        fn(N, K, _p(Aw, ctypes.c_int8), _p(Bw, ctypes.c_int8), _p(C, ctypes.c_int64), r0, r1, c0, c1,
           ctypes.byref(lhs), ctypes.byref(rhs))
        return Check(lhs.value, rhs.value, 0.0, lhs.value != rhs.value)
    lhs, rhs = ctypes.c_double(), ctypes.c_double()
    fn = lib.orc_tile_two_sided_f64 if two_sided else lib.orc_tile_one_sided_f64
    fn(N, K, _d(Aw), _d(Bw), _d(C), r0, r1, c0, c1, ctypes.byref(lhs), ctypes.byref(rhs))
    f = frob(C, r0, r1, c0, c1)
    tau = tolerance(K, f, dtype, scheme=2)
    if operand_sums is not None:
        tau += half_sum_term(dtype, f, operand_sums[0], operand_sums[1], two_sided)
    return Check(lhs.value, rhs.value, tau, mismatch(lhs.value, rhs.value, tau))


def thread_check(A, B, C, dtype, tile_m, tile_n, two_sided=False):
    """All tile checks of a partition; the layer is flagged when any tile is."""
    M, N = C.shape
    checks = [tile_check(A, B, C, dtype, *t, two_sided=two_sided) for t in tiles(M, N, tile_m, tile_n)]
    return any(c.flag for c in checks), checks


def replica_check(A, B, C, dtype, r0, r1, c0, c1, block_n=32) -> Check:
    """Thread-level replication with single accumulation for one tile (Sec. 5.1): every product
    of the tile is formed a second time, the tile's column blocks of width ``block_n`` (the
    matrix instruction's output width) all added into one block; the sum of that block against
    the output summation of the tile of the C that is passed in."""
    Aw, Bw = widen(A, dtype), widen(B, dtype)
    K = Aw.shape[1]
    At = np.ascontiguousarray(Aw[r0:r1])
    acc_t = np.int64 if dtype == I8 else np.float64
    rep = np.zeros((r1 - r0, block_n), dtype=acc_t)
    for b0 in range(c0, c1, block_n):
        blk = gemm(At, np.ascontiguousarray(Bw[:, b0:min(b0 + block_n, c1)]), dtype)
        rep[:, :blk.shape[1]] += blk
    lhs = block_sum(C, r0, r1, c0, c1)
    if dtype == I8:
        rhs = int(rep.sum())
        return Check(int(lhs), rhs, 0.0, int(lhs) != rhs)
    rhs = math.fsum(rep.ravel().tolist())
    tau = tolerance(K, frob(C, r0, r1, c0, c1), dtype, scheme=2)
    return Check(lhs, rhs, tau, mismatch(lhs, rhs, tau))


# --------------------------------------------------------------------------- #
# fault injection (fault model of Sec. 2.3)
# --------------------------------------------------------------------------- #
def flip_bit(value, bit: int, dtype: str):
    """One flipped bit in the accumulator that holds ``value``: binary32 for the
    floating-point paths, int32 for int8."""
    lib = _load()
    assert 0 <= bit < 32
    if dtype == I8:
        return int(lib.orc_flip_bit_i32(int(value), bit))
    return float(lib.orc_flip_bit_f32(float(value), bit))


def inject(A, B, C, dtype, row, col, bit, k_after=-1, k_begin=0, k_set=None):
    """Copy of C with one fault in element (row, col).

    The accumulator that is hit holds the products k_begin <= k < k_after (k_after < 0 or
    >= K: up to K) -- with ``k_set`` (a collection of k indices) only those of them whose k is
    in the set, for an accumulator that takes a subset of the k range.  Its value is flipped and
    everything else is added to the corrupted value (the fault persists to the end).
    k_begin = 0, k_after < 0, no k_set: a flip of the final value of C[row, col].
    """
    Cf = np.array(C, copy=True)
    K = A.shape[1]
    if k_after < 0 or k_after > K:
        k_after = K
    if k_set is None and k_begin == 0 and k_after == K:
        Cf[row, col] = flip_bit(C[row, col], bit, dtype)
        return Cf
    # only row `row` of A and column `col` of B take part
    a = np.ascontiguousarray(np.asarray(A)[row:row + 1])
    b = np.ascontiguousarray(np.asarray(B)[:, col:col + 1])
    hit = range(k_begin, k_after) if k_set is None else sorted(k for k in k_set if k_begin <= k < k_after)
    inside = np.zeros(K + 1, dtype=bool)
    inside[list(hit)] = True
    # maximal runs of consecutive k inside / outside the hit accumulator, each summed in ascending k
    head = rest = 0 if dtype == I8 else 0.0
    k = 0
    while k < K:
        e = k
        while e < K and inside[e] == inside[k]:
            e += 1
        term = partial_dot(a, b, dtype, 0, 0, k, e)
        if inside[k]:
            head += term
        else:
            rest += term
        k = e
    Cf[row, col] = flip_bit(head, bit, dtype) + rest
    return Cf


def part_of(k_parts, k):
    """Index of the part (a collection of k indices) that holds k."""
    for s, part in enumerate(k_parts):
        if k in part:
            return s
    raise ValueError(k)


# --------------------------------------------------------------------------- #
# arithmetic intensity, CMR, selector (Sec. 3.1 Eq. 1, Sec. 5.3)
# --------------------------------------------------------------------------- #
STORAGE_BYTES = {F16: (2, 2, 2), BF16: (2, 2, 2), I8: (1, 1, 4)}  # (A, B, C) bytes per element

GLOBAL, THREAD = 1, 2


def flops(M, N, K, pad_to=1):
    return _load().orc_flops(M, N, K, pad_to)


def bytes_moved(M, N, K, dtype=F16, pad_to=1):
    sa, sb, sc = STORAGE_BYTES[dtype]
    return _load().orc_bytes(M, N, K, sa, sb, sc, pad_to)


def arithmetic_intensity(M, N, K, dtype=F16, pad_to=1):
    sa, sb, sc = STORAGE_BYTES[dtype]
    return _load().orc_arithmetic_intensity(M, N, K, sa, sb, sc, pad_to)


def aggregate_intensity(layers, dtype=F16, pad_to=1):
    """Sum of FLOPs over sum of bytes across the linear layers of a network (Sec. 3.2)."""
    f = sum(flops(M, N, K, pad_to) for (M, N, K) in layers)
    b = sum(bytes_moved(M, N, K, dtype, pad_to) for (M, N, K) in layers)
    return f / b


def cmr(peak_ops_per_s, bytes_per_s):
    return _load().orc_cmr(peak_ops_per_s, bytes_per_s)


def select(M, N, K, dtype, cmr_value, pad_to=1):
    """GLOBAL when the layer is compute bound by Eq. 1, THREAD otherwise (Sec. 5.3)."""
    return _load().orc_select(arithmetic_intensity(M, N, K, dtype, pad_to), cmr_value)


# --------------------------------------------------------------------------- #
# convolution as a matrix product (Sec. 2.1)
# --------------------------------------------------------------------------- #
def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def im2col(x, dtype, KH, KW, stride, pad):
    """NHWC activations -> the (batch*OH*OW) x (KH*KW*Cin) matrix A, in fp64 (int8: int8)."""
    lib = _load()
    xw = widen(x, dtype)
    n, H, W, Cin = xw.shape
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    xd = np.ascontiguousarray(xw, dtype=np.float64)
    out = np.empty((n * OH * OW, KH * KW * Cin), dtype=np.float64)
    lib.orc_im2col_f64(n, H, W, Cin, KH, KW, stride, pad, _d(xd), _d(out))
    if dtype == I8:
        return out.astype(np.int8)
    return out


# --------------------------------------------------------------------------- #
# a chain of layers: activation function and storage rounding (Sec. 2.4 step 4)
# --------------------------------------------------------------------------- #
def activation(C, act="relu"):
    """The activation function a layer applies to its output: "relu" is max(x, 0), None passes."""
    if act is None or act == "none":
        return C
    if act == "relu":
        return np.maximum(C, 0)
    raise ValueError(act)


def round_out(C, dtype):
    """fp64 values -> the storage array of the output type, rounded once to nearest, ties to
    even (numpy.float16, or uint16 bf16 bit patterns); int8 products stay int64."""
    if dtype == I8:
        return C
    C = np.asarray(C, dtype=np.float64)
    if dtype == F16:
        with np.errstate(over="ignore"):
            return C.astype(np.float16)
    if dtype == BF16:
        # 8 significant bits; exponent range of binary32 (least normal 2^-126)
        m, e = np.frexp(C)                              # C = m 2^e, 0.5 <= |m| < 1
        ulp = np.ldexp(1.0, np.maximum(e, -125) - 8)
        q = np.rint(C / ulp) * ulp                      # rint: ties to even
        q = np.where(np.isfinite(C), q, C)
        big = np.ldexp(255.0, 120)                      # largest finite bf16
        q = np.where(np.abs(q) > big, np.copysign(np.inf, q), q)
        return (q.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def mlp_forward(x, weights, dtype, acts):
    """A chain of fully-connected layers: layer l computes act_l(a_l . W_l) and hands it, stored
    in the operand type, to layer l + 1 (a_0 = x).  Returns every layer's stored output."""
    outs, a = [], x
    for W, act in zip(weights, acts):
        a = round_out(activation(gemm(a, W, dtype), act), dtype)
        outs.append(a)
    return outs
