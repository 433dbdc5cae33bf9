"""Pins for the oracle's widening and matrix product (CPU only).

Independent references used here: exact rational arithmetic (fractions.Fraction) with
hand-written index loops, numpy's own float16 -> float64 conversion and numpy.matmul.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import workloads as wl


def test_f16_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, "f16")
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, "bf16")
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])


def test_known_values():
    # 0x3C00 = 1, 0xC000 = -2, 0x3555 ~ 1/3, 0x0001 = 2^-24, 0x7BFF = 65504
    bits = np.array([0x3C00, 0xC000, 0x0001, 0x7BFF], dtype=np.uint16)
    assert oracle.widen(bits, "f16").tolist() == [1.0, -2.0, 2.0 ** -24, 65504.0]
    b = np.array([0x3F80, 0xC040, 0x0080], dtype=np.uint16)  # 1, -3, 2^-126
    assert oracle.widen(b, "bf16").tolist() == [1.0, -3.0, 2.0 ** -126]


def _brute(A, B):
    """C[i][j] = sum_k A[i][k] B[k][j] in exact rational arithmetic, j-i-k loop order."""
    M, K = A.shape
    N = B.shape[1]
    C = [[Fraction(0)] * N for _ in range(M)]
    for j in range(N):
        for i in range(M):
            s = Fraction(0)
            for k in reversed(range(K)):
                s += Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            C[i][j] = s
    return C


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (8, 8, 8), (5, 2, 7), (3, 8, 1)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_gemm_against_exact_brute_force(M, N, K, dtype):
    A, B = wl.gemm_operands(M, N, K, dtype, seed=11 + M + 10 * N + 100 * K)
    C = oracle.gemm(A, B, dtype)
    Aw = oracle.widen(A, dtype).astype(np.float64)
    Bw = oracle.widen(B, dtype).astype(np.float64)
    exact = _brute(Aw, Bw)
    for i in range(M):
        for j in range(N):
            if dtype == "i8":
                assert int(C[i, j]) == exact[i][j]
            else:
                # fp64 accumulation of <= 8 products of 11-bit (8-bit) significands
                err = abs(Fraction(float(C[i, j])) - exact[i][j])
                assert err <= Fraction(2) ** -50 * max(abs(exact[i][j]), Fraction(1, 1 << 20))


def test_gemm_detects_transposition_shapes():
    # a wrong index or transposed operand cannot survive a non-square one-hot product
    A = np.zeros((3, 5), dtype=np.float16)
    B = np.zeros((5, 4), dtype=np.float16)
    A[2, 1] = 2.0
    B[1, 3] = 3.0
    C = oracle.gemm(A, B, "f16")
    want = np.zeros((3, 4))
    want[2, 3] = 6.0
    assert np.array_equal(C, want)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (37, 129, 200), (130, 70, 333)])
def test_gemm_against_numpy_matmul(M, N, K, dtype):
    A, B = wl.gemm_operands(M, N, K, dtype, seed=5)
    C = oracle.gemm(A, B, dtype)
    Aw, Bw = oracle.widen(A, dtype), oracle.widen(B, dtype)
    ref = np.matmul(Aw, Bw)
    scale = np.abs(Aw) @ np.abs(Bw)
    assert np.all(np.abs(C - ref) <= 4 * K * 2.0 ** -53 * scale)


@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (33, 65, 257)])
def test_gemm_int8_against_numpy(M, N, K):
    A, B = wl.gemm_operands(M, N, K, "i8", seed=6)
    C = oracle.gemm(A, B, "i8")
    assert C.dtype == np.int64
    assert np.array_equal(C, A.astype(np.int64) @ B.astype(np.int64))
    # extremes: -128 * -128 * K must not wrap
    A[:] = -128
    B[:] = -128
    assert np.all(oracle.gemm(A, B, "i8") == 16384 * K)


def test_gemm_rows_and_partial_dot_agree_with_full():
    A, B = wl.gemm_operands(20, 17, 50, "f16", seed=3)
    C = oracle.gemm(A, B, "f16")
    rows = [0, 7, 19]
    assert np.array_equal(oracle.gemm_rows(A, B, "f16", rows), C[rows])
    assert oracle.partial_dot(A, B, "f16", 7, 5, 0, 50) == C[7, 5]
    head = oracle.partial_dot(A, B, "f16", 7, 5, 0, 20)
    want = float(np.sum(A[7, :20].astype(np.float64) * B[:20, 5].astype(np.float64)))
    assert abs(head - want) < 1e-12
    Ai, Bi = wl.gemm_operands(9, 6, 40, "i8", seed=4)
    Ci = oracle.gemm(Ai, Bi, "i8")
    assert np.array_equal(oracle.gemm_rows(Ai, Bi, "i8", [8, 1]), Ci[[8, 1]])
    assert oracle.partial_dot(Ai, Bi, "i8", 2, 3, 0, 17) + oracle.partial_dot(Ai, Bi, "i8", 2, 3, 17, 40) == Ci[2, 3]


def test_im2col_against_direct_convolution():
    """Lowered conv == direct sliding-window convolution written with explicit loops."""
    c = wl.Conv(batch=2, H=6, W=5, Cin=3, Cout=4, KH=3, KW=3, stride=2, pad=1)
    x, Wm = wl.conv_operands(c, "f16", seed=8)
    A = oracle.im2col(x, "f16", c.KH, c.KW, c.stride, c.pad)
    assert A.shape == (c.batch * c.OH * c.OW, c.KH * c.KW * c.Cin)
    C = oracle.gemm(A, Wm, "f16").reshape(c.batch, c.OH, c.OW, c.Cout)
    xf = x.astype(np.float64)
    Wf = Wm.astype(np.float64).reshape(c.KH, c.KW, c.Cin, c.Cout)
    xp = np.zeros((c.batch, c.H + 2, c.W + 2, c.Cin))
    xp[:, 1:-1, 1:-1, :] = xf
    for n in range(c.batch):
        for oh in range(c.OH):
            for ow in range(c.OW):
                patch = xp[n, oh * 2:oh * 2 + 3, ow * 2:ow * 2 + 3, :]
                want = np.einsum("hwc,hwco->o", patch, Wf)
                assert np.allclose(C[n, oh, ow], want, rtol=1e-12, atol=1e-12)


def test_im2col_1x1_is_a_reshape():
    c = wl.Conv(batch=2, H=4, W=3, Cin=8, Cout=2, KH=1, KW=1, stride=1, pad=0)
    x, _ = wl.conv_operands(c, "f16", seed=9)
    A = oracle.im2col(x, "f16", 1, 1, 1, 0)
    assert np.array_equal(A, x.astype(np.float64).reshape(-1, 8))
