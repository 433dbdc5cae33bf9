"""Pins for the oracle's checksum schemes, fault injection and tolerance (CPU only)."""
import math

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import workloads as wl

SHAPES = [(8, 8, 8), (64, 64, 64), (33, 70, 129), (1, 5, 13), (16, 1, 256)]


# ------------------------------------------------------------------ invariant
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_integer_invariant_is_exact(M, N, K):
    """sum(C) == (1^T A)(B 1) exactly over the integers (Sec. 2.4)."""
    A, B = wl.gemm_operands(M, N, K, "i8", seed=M + N + K)
    C = oracle.gemm(A, B, "i8")
    alpha, beta = oracle.col_checksum(A, "i8"), oracle.row_checksum(B, "i8")
    # checksums against numpy's own reductions
    assert np.array_equal(alpha, A.astype(np.int64).sum(axis=0))
    assert np.array_equal(beta, B.astype(np.int64).sum(axis=1))
    assert alpha.shape == (K,) and beta.shape == (K,)
    assert oracle.checksum_dot(alpha, beta) == oracle.block_sum(C) == int(C.sum())
    chk = oracle.global_check(A, B, C, "i8")
    assert chk.tau == 0.0 and not chk.flag and chk.residual == 0


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_fp_invariant_within_rigorous_bound(M, N, K, dtype):
    A, B = wl.gemm_operands(M, N, K, dtype, seed=1)
    C = oracle.gemm(A, B, dtype)
    chk = oracle.global_check(A, B, C, dtype)
    # everything is fp64 here: the residual is far below even the fp32 bound
    sabs = oracle.s_abs(A, B, dtype)
    assert abs(chk.residual) <= (K + M * N) * 2.0 ** -52 * sabs
    assert abs(chk.residual) <= oracle.rigorous_bound(M, N, K, sabs)
    assert not chk.flag


def test_a_dropped_row_or_column_breaks_the_invariant():
    """The pins above would catch a checksum that skips a row/column or mixes up axes."""
    A, B = wl.gemm_operands(7, 9, 11, "i8", seed=2)
    C = oracle.gemm(A, B, "i8")
    alpha, beta = oracle.col_checksum(A, "i8"), oracle.row_checksum(B, "i8")
    assert oracle.checksum_dot(alpha, beta) == int(C.sum())
    assert oracle.checksum_dot(oracle.col_checksum(A[:-1], "i8"), beta) != int(C.sum())
    assert oracle.checksum_dot(alpha, oracle.row_checksum(B[:, :-1], "i8")) != int(C.sum())


def test_phi_and_sabs_closed_forms():
    # all-ones operands: Phi = sqrt(K * M * N), S_abs = K * M * N, sum(C) = K * M * N
    M, N, K = 6, 10, 12
    A = np.ones((M, K), dtype=np.float16)
    B = np.ones((K, N), dtype=np.float16)
    assert oracle.phi(A, B, "f16") == pytest.approx(math.sqrt(K * M * N))
    assert oracle.s_abs(A, B, "f16") == K * M * N
    C = oracle.gemm(A, B, "f16")
    assert oracle.block_sum(C) == K * M * N
    assert oracle.frob(C) == pytest.approx(K * math.sqrt(M * N))
    assert oracle.tolerance(K, oracle.frob(C), "f16") == pytest.approx(
        8 * 2.0 ** -24 * math.sqrt(K) * K * math.sqrt(M * N))
    assert oracle.tolerance(K, 123.0, "i8") == 0.0


# ----------------------------------------------------------------- tile scheme
@pytest.mark.parametrize("tile", [(4, 4), (8, 16), (32, 32), (5, 3), (64, 64), (128, 16)])
def test_tile_checks_telescope_to_the_global_identity(tile):
    M, N, K = 40, 50, 24
    A, B = wl.gemm_operands(M, N, K, "i8", seed=3)
    C = oracle.gemm(A, B, "i8")
    flag, checks = oracle.thread_check(A, B, C, "i8", *tile)
    assert not flag
    assert len(checks) == math.ceil(M / tile[0]) * math.ceil(N / tile[1])
    assert all(c.lhs == c.rhs for c in checks)
    assert sum(c.lhs for c in checks) == int(C.sum())
    g = oracle.global_check(A, B, C, "i8")
    assert sum(c.rhs for c in checks) == g.rhs


def test_tile_one_sided_matches_definition_by_numpy():
    """rho_i = sum_k A[i,k] * (sum_{j in T} B[k,j]) written with numpy slices."""
    M, N, K = 24, 40, 16
    A, B = wl.gemm_operands(M, N, K, "f16", seed=4)
    C = oracle.gemm(A, B, "f16")
    Aw, Bw = A.astype(np.float64), B.astype(np.float64)
    r0, r1, c0, c1 = 8, 24, 16, 33
    chk = oracle.tile_check(A, B, C, "f16", r0, r1, c0, c1)
    chi = Bw[:, c0:c1].sum(axis=1)
    rho = Aw[r0:r1] @ chi
    assert chk.rhs == pytest.approx(rho.sum(), rel=1e-13)
    assert chk.lhs == pytest.approx(C[r0:r1, c0:c1].sum(), rel=1e-13)
    two = oracle.tile_check(A, B, C, "f16", r0, r1, c0, c1, two_sided=True)
    assert two.rhs == pytest.approx(chk.rhs, rel=1e-12)
    assert two.rhs == pytest.approx(float(Aw[r0:r1].sum(axis=0) @ chi), rel=1e-13)
    # a tile check must not see elements outside its tile
    C2 = C.copy()
    C2[0, 0] += 100.0
    assert oracle.tile_check(A, B, C2, "f16", r0, r1, c0, c1).lhs == chk.lhs


# ------------------------------------------------------------------- injection
def test_flip_bit_semantics():
    assert oracle.flip_bit(1.0, 31, "f16") == -1.0            # sign
    assert oracle.flip_bit(1.0, 23, "f16") == 0.5             # lowest exponent bit of 1.0 (127 -> 126)
    assert oracle.flip_bit(1.0, 22, "f16") == 1.5             # top mantissa bit
    assert oracle.flip_bit(1.0, 0, "f16") == 1.0 + 2.0 ** -23
    assert oracle.flip_bit(1.0, 30, "f16") == math.inf        # exponent 0x7f -> 0xff
    assert math.isnan(oracle.flip_bit(1.5, 30, "f16"))
    assert oracle.flip_bit(0, 0, "i8") == 1
    assert oracle.flip_bit(0, 31, "i8") == -2 ** 31
    assert oracle.flip_bit(-1, 31, "i8") == 2 ** 31 - 1
    assert oracle.flip_bit(5, 2, "i8") == 1


@pytest.mark.parametrize("M,N,K,tile", [(8, 8, 8, (4, 4)), (64, 64, 64, (32, 32))])
def test_int8_every_single_bit_flip_is_detected(M, N, K, tile):
    """Exhaustive: all 32 bits of every element of C (Sec. 2.3: one faulty value)."""
    A, B = wl.gemm_operands(M, N, K, "i8", seed=5)
    C = oracle.gemm(A, B, "i8")
    s_ab = oracle.global_check(A, B, C, "i8").rhs
    s_c = int(C.sum())
    tile_rhs = {t: oracle.tile_check(A, B, C, "i8", *t).rhs for t in oracle.tiles(M, N, *tile)}
    step = 1 if M <= 8 else 7  # 64^3: every 7th element keeps the loop short
    n = 0
    for i in range(0, M, step):
        for j in range(0, N, step):
            for bit in range(32):
                bad = oracle.flip_bit(C[i, j], bit, "i8")
                delta = bad - int(C[i, j])
                assert delta != 0
                assert oracle.mismatch(s_c + delta, s_ab, 0.0)
                t = (i // tile[0] * tile[0], min(i // tile[0] * tile[0] + tile[0], M),
                     j // tile[1] * tile[1], min(j // tile[1] * tile[1] + tile[1], N))
                assert oracle.mismatch(tile_rhs[t] + delta, tile_rhs[t], 0.0)
                n += 1
    assert n >= 32 * 64


def test_incremental_evaluation_matches_full_recomputation():
    """s_C' = s_C + delta (used by large campaigns) == recomputing the check on corrupted C."""
    M, N, K = 48, 40, 96
    for dtype in ("i8", "f16"):
        A, B = wl.gemm_operands(M, N, K, dtype, seed=6)
        C = oracle.gemm(A, B, dtype)
        rng = np.random.default_rng(7)
        for _ in range(40):
            i, j, bit = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(32))
            k_after = int(rng.choice([-1, 32, 64]))
            Cf = oracle.inject(A, B, C, dtype, i, j, bit, k_after)
            full = oracle.global_check(A, B, Cf, dtype)
            clean = oracle.global_check(A, B, C, dtype)
            if dtype == "i8":
                assert full.lhs == clean.lhs + (int(Cf[i, j]) - int(C[i, j]))
                assert full.flag
            elif math.isfinite(Cf[i, j]):
                assert full.lhs == pytest.approx(clean.lhs + (Cf[i, j] - C[i, j]), rel=1e-12, abs=1e-9)
            assert np.array_equal(np.delete(Cf.ravel(), i * N + j), np.delete(C.ravel(), i * N + j))


def test_mid_loop_injection_persists_additively():
    A, B = wl.gemm_operands(4, 4, 64, "i8", seed=8)
    C = oracle.gemm(A, B, "i8")
    head = oracle.partial_dot(A, B, "i8", 1, 2, 0, 16)
    Cf = oracle.inject(A, B, C, "i8", 1, 2, 3, k_after=16)
    assert Cf[1, 2] - C[1, 2] == oracle.flip_bit(head, 3, "i8") - head
    assert abs(Cf[1, 2] - C[1, 2]) == 8


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_fp_flips_outside_the_dont_care_band(dtype):
    """|delta| >= 2 tau must flag, |delta| <= tau/2 must not; NaN/Inf must flag."""
    M, N, K = 64, 64, 64
    A, B = wl.gemm_operands(M, N, K, dtype, seed=9)
    C = oracle.gemm(A, B, dtype)
    rng = np.random.default_rng(10)
    seen = {"flag": 0, "quiet": 0, "nonfinite": 0}
    for _ in range(300):
        i, j, bit = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(32))
        Cf = oracle.inject(A, B, C, dtype, i, j, bit)
        g = oracle.global_check(A, B, Cf, dtype)
        t_flag, _ = oracle.thread_check(A, B, Cf, dtype, 32, 32)
        if not math.isfinite(Cf[i, j]):
            assert g.flag and t_flag
            seen["nonfinite"] += 1
            continue
        delta = abs(Cf[i, j] - float(np.float32(C[i, j])))
        if delta >= 2 * g.tau:
            assert g.flag
            seen["flag"] += 1
        elif delta <= g.tau / 2:
            assert not g.flag
            seen["quiet"] += 1
    assert min(seen.values()) > 0


# --------------------------------------------------------------- clean campaigns
@pytest.mark.parametrize("dist_a,dist_b", [("uniform_pm1", "uniform_pm1"), ("uniform_01", "weights"),
                                           ("normal", "normal"), ("uniform_01", "uniform_01")])
def test_no_false_alarm_on_fp32_accumulated_products(dist_a, dist_b):
    """The tolerance must clear real binary32 accumulation noise.  numpy's float32 matmul
    (a library SGEMM, binary32 accumulators) stands in for the accelerator here; 1000 seeds."""
    M, N, K = 64, 64, 64
    worst = 0.0
    for seed in range(1000):
        A, B = wl.gemm_operands(M, N, K, "f16", seed=seed, dist_a=dist_a, dist_b=dist_b)
        C32 = np.matmul(A.astype(np.float32), B.astype(np.float32)).astype(np.float64)
        g = oracle.global_check(A, B, C32, "f16")
        assert not g.flag, (seed, g)
        worst = max(worst, abs(g.residual) / g.tau)
    assert worst < 0.5  # comfortable margin, not a near miss


def test_no_false_alarm_tiles_fp32_accumulated_larger():
    M, N, K = 256, 256, 1024
    for seed in range(3):
        A, B = wl.gemm_operands(M, N, K, "f16", seed=seed, dist_a="uniform_01", dist_b="weights")
        C32 = np.matmul(A.astype(np.float32), B.astype(np.float32)).astype(np.float64)
        flag, checks = oracle.thread_check(A, B, C32, "f16", 128, 128)
        assert not flag
        assert not oracle.global_check(A, B, C32, "f16").flag


# -------------------------------------------------------- per-block global check
@pytest.mark.parametrize("block", [(16, 16), (64, 64), (7, 20), (256, 256)])
def test_block_checks_telescope_to_the_whole_matrix_identity(block):
    """One comparison per block of C: every block passes on clean data, and the block
    checksum products add up to (1^T A)(B 1) exactly over the integers."""
    M, N, K = 40, 50, 24
    A, B = wl.gemm_operands(M, N, K, "i8", seed=13)
    C = oracle.gemm(A, B, "i8")
    flag, checks = oracle.global_check_blocks(A, B, C, "i8", *block)
    assert not flag and all(c.lhs == c.rhs for c in checks)
    whole = oracle.global_check(A, B, C, "i8")
    assert sum(c.rhs for c in checks) == whole.rhs and sum(c.lhs for c in checks) == whole.lhs
    # block checksum product written out with numpy for one block
    r0, r1, c0, c1 = 0, min(block[0], M), 0, min(block[1], N)
    want = int(A[r0:r1].astype(np.int64).sum(axis=0) @ B[:, c0:c1].astype(np.int64).sum(axis=1))
    assert checks[0].rhs == want
    # a fault is seen by exactly the block that holds it
    Cf = oracle.inject(A, B, C, "i8", 17, 33, 5)
    flag, checks = oracle.global_check_blocks(A, B, Cf, "i8", *block)
    assert flag and sum(c.flag for c in checks) == 1


def test_global_tolerance_has_the_bias_term():
    K = 100
    C = np.full((4, 5), 2.0)
    f, l1 = oracle.frob(C), oracle.l1norm(C)
    assert l1 == 40.0 and f == pytest.approx(2.0 * math.sqrt(20))
    tau = oracle.tolerance(K, f, "f16", scheme=1, l1_norm=l1)
    assert tau == pytest.approx(8 * 2.0 ** -24 * 10 * f + 1e-3 * 2.0 ** -24 * 100 * 40)
    assert oracle.tolerance(K, f, "f16", scheme=2) == pytest.approx(8 * (2.0 ** -24 * 10 + 2.0 ** -22) * f)
    A, B = wl.gemm_operands(8, 8, 8, "f16", seed=14)
    Cc = oracle.gemm(A, B, "f16")
    one = oracle.region_check(A, B, Cc, "f16", 0, 8, 0, 8)
    whole = oracle.global_check(A, B, Cc, "f16")
    assert one.tau == pytest.approx(whole.tau) and one.rhs == pytest.approx(whole.rhs, rel=1e-13)


def _accumulate_binary32(A, B):
    """C = A.B with one binary32 accumulator per entry that takes the K products in ascending k,
    one round-to-nearest add each (a product of two fp16 / bf16 values is exact in binary32)."""
    A32, B32 = A.astype(np.float32), B.astype(np.float32)
    acc = np.zeros((A.shape[0], B.shape[1]), dtype=np.float32)
    for k in range(A.shape[1]):
        acc += A32[:, k:k + 1] * B32[k:k + 1, :]
    return acc.astype(np.float64)


@pytest.mark.parametrize("K", [64, 1024, 4096])
def test_tolerance_constant_against_simulated_binary32_accumulation_and_the_rigorous_bound(K):
    """C_TOL from both sides, with nothing of the GPU path involved.  Below: a simulated binary32
    accumulation (plain IEEE arithmetic in numpy) of a 32 x 64 region leaves a residual of the
    output summation against the exact checksum product that stays under a quarter of tau, for
    zero-mean and for same-sign operands.  Above: for same-sign operands tau is at most a tenth of
    the first-order worst-case bound K u sum|a||b| of Higham's analysis of recursive summation, so
    the comparison is a real test and not the trivial one; and tau is never below 8 u ||C||_F."""
    M, N = 32, 64
    u = 2.0 ** -24
    for da, db in (("normal", "normal"), ("uniform_pm1", "uniform_pm1"), ("uniform_01", "weights"), ("uniform_01", "uniform_01")):
        worst = 0.0
        for seed in range(6):
            A, B = wl.gemm_operands(M, N, K, "f16", seed=900 + seed, dist_a=da, dist_b=db)
            C32 = _accumulate_binary32(A, B)
            for scheme in (1, 2):
                tau = oracle.tolerance(K, oracle.frob(C32), "f16", scheme=scheme, l1_norm=oracle.l1norm(C32))
                chk = oracle.region_check(A, B, C32, "f16", 0, M, 0, N)
                worst = max(worst, abs(chk.residual) / tau)
                assert tau >= 8 * u * oracle.frob(C32)
                if da == "uniform_01" and db == "uniform_01" and K >= 1024:
                    assert tau <= 0.1 * K * u * oracle.s_abs(A, B, "f16")
        assert worst < 0.25, (da, db, worst)


def test_drift_term_is_a_thousandth_of_the_worst_case_for_same_sign_data():
    """C_BIAS: for operands of one sign sum|a||b| = ||C||_1, so the second term of the global
    tolerance is exactly 1e-3 of the first-order worst-case rounding bound K u ||C||_1."""
    K = 512
    A, B = wl.gemm_operands(16, 16, K, "f16", seed=3, dist_a="uniform_01", dist_b="uniform_01")
    C = oracle.gemm(A, B, "f16")
    l1 = oracle.l1norm(C)
    assert l1 == pytest.approx(oracle.s_abs(A, B, "f16"), rel=1e-12)
    drift = oracle.tolerance(K, 0.0, "f16", scheme=1, l1_norm=l1)
    assert drift == pytest.approx(1e-3 * K * 2.0 ** -24 * oracle.s_abs(A, B, "f16"), rel=1e-12)
    assert oracle.tolerance(K, 0.0, "f16", scheme=2, l1_norm=l1) == 0.0


def test_precision_of_a_checksum_handed_on_in_pieces():
    """U_CHI: a binary32 sum of a few fp16 values written as hi + 2^-11 lo with hi = fl16(s) and
    lo = fl16((s - hi) 2^11) is within 2^-22 |s| of s; a binary32 sum of bf16 values written as
    three bf16 pieces hi + mid + lo is within 2^-23 |s| (exact, in fact).  Plain numpy conversions."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(2, 5))
        v = wl.random_matrix((n, 4096), "f16", ("normal", "uniform_01", "weights")[trial % 3], 7000 + trial)
        s = v.astype(np.float32).sum(axis=0, dtype=np.float32)          # exact: a few fp16 values
        hi = s.astype(np.float16)
        lo = ((s - hi.astype(np.float32)) * np.float32(2048)).astype(np.float16)
        back = hi.astype(np.float64) + lo.astype(np.float64) / 2048.0
        big = np.abs(s) >= 2.0 ** -10          # (below that the low piece is a subnormal fp16)
        assert np.all(np.abs(back - s.astype(np.float64))[big] <= oracle.U_CHI["f16"] * np.abs(s.astype(np.float64))[big])
        b = wl.bf16_bits_to_f32(wl.random_matrix((n, 4096), "bf16", "normal", 8000 + trial))
        sb = b.sum(axis=0, dtype=np.float32)
        p0 = wl.bf16_bits_to_f32(wl.to_bf16_bits(sb))
        r1 = sb - p0
        p1 = wl.bf16_bits_to_f32(wl.to_bf16_bits(r1))
        p2 = wl.bf16_bits_to_f32(wl.to_bf16_bits(r1 - p1))
        backb = p0.astype(np.float64) + p1.astype(np.float64) + p2.astype(np.float64)
        assert np.all(np.abs(backb - sb.astype(np.float64)) <= oracle.U_CHI["bf16"] * np.abs(sb.astype(np.float64)))


@pytest.mark.parametrize("tile", [(32, 64), (32, 128), (64, 64), (128, 64)])
def test_tolerance_of_checksums_added_in_half_precision(tile):
    """The widened tolerance of the schemes that add their checksums in fp16 (Sec. 5.2.2's packed
    adds), against a simulation in plain numpy fp16 arithmetic: per k, the tile's B values are
    added up in fp16 within each class of columns 32 apart (the A values likewise for the
    two-sided scheme), everything after that exactly.  The residual against the tile's exact
    output summation stays under half the tolerance -- same-sign activations, where the error is
    largest, included -- while the exact scheme's tolerance would be overrun; and the integer
    identity of the two-sided definition holds exactly."""
    tm, tn = tile
    for two_sided in (False, True):
        over_exact = 0
        for K in (16, 64, 1024):
            for da, db in (("normal", "normal"), ("uniform_01", "weights"), ("uniform_01", "uniform_01")):
                for seed in range(4):
                    A, B = wl.gemm_operands(tm, tn, K, "f16", seed=50 + seed, dist_a=da, dist_b=db)
                    C = oracle.gemm(A, B, "f16")
                    chi = B[:, :32].copy()
                    for j in range(1, tn // 32):
                        chi = (chi + B[:, 32 * j:32 * j + 32]).astype(np.float16)
                    if two_sided:
                        a = A[:32].copy()
                        for i in range(1, tm // 32):
                            a = (a + A[32 * i:32 * i + 32]).astype(np.float16)
                        rhs = float((a.astype(np.float64) @ chi.astype(np.float64)).sum())
                    else:
                        rhs = float((A.astype(np.float64) @ chi.astype(np.float64)).sum())
                    chk = oracle.tile_check(A, B, C, "f16", 0, tm, 0, tn, two_sided=two_sided, operand_sums=tile)
                    assert abs(chk.lhs - rhs) <= 0.5 * chk.tau, (two_sided, K, da, db, abs(chk.lhs - rhs) / chk.tau)
                    exact = oracle.tile_check(A, B, C, "f16", 0, tm, 0, tn, two_sided=two_sided)
                    assert exact.tau < chk.tau and not exact.flag
                    over_exact += abs(chk.lhs - rhs) > exact.tau
        assert over_exact > 0
    Ai, Bi = wl.gemm_operands(tm, tn, 24, "i8", seed=9)
    two = oracle.tile_check(Ai, Bi, oracle.gemm(Ai, Bi, "i8"), "i8", 0, tm, 0, tn, two_sided=True)
    assert two.lhs == two.rhs and not two.flag


def test_fault_in_an_accumulator_that_holds_a_subset_of_k():
    """inject(k_set=...): with the set a contiguous range it is the k_begin / k_after form; with an
    interleaved set the corrupted value is flip(sum over the set below k_after) + every other
    product, checked against a direct evaluation over the integers."""
    M, N, K = 6, 7, 96
    for dtype in ("i8", "f16"):
        A, B = wl.gemm_operands(M, N, K, dtype, seed=15)
        C = oracle.gemm(A, B, dtype)
        a = oracle.inject(A, B, C, dtype, 5, 3, 30, k_after=48, k_begin=32)
        b = oracle.inject(A, B, C, dtype, 5, 3, 30, k_after=48, k_set=range(32, 96))
        assert np.allclose(a, b, rtol=1e-12, atol=1e-12, equal_nan=True)
        whole = oracle.inject(A, B, C, dtype, 0, 0, 3, k_set=range(K))
        assert np.allclose(whole, oracle.inject(A, B, C, dtype, 0, 0, 3), rtol=1e-12, atol=1e-12)
    A, B = wl.gemm_operands(M, N, K, "i8", seed=16)
    C = oracle.gemm(A, B, "i8")
    part = [k for k in range(K) if (k // 16) % 4 == 1]
    got = oracle.inject(A, B, C, "i8", 2, 4, 9, k_after=64, k_set=part)
    head = sum(int(A[2, k]) * int(B[k, 4]) for k in part if k < 64)
    want = C.copy()
    want[2, 4] = oracle.flip_bit(head, 9, "i8") + (int(C[2, 4]) - head)
    assert np.array_equal(got, want)
    assert oracle.part_of([part, [0]], 17) == 0


# ------------------------------------------------------------------ replication (Sec. 5.1)
@pytest.mark.parametrize("block_n", [32, 8, 5])
def test_replica_check_integer_identity_and_every_bit(block_n):
    """Single-accumulation replication over the integers: the replicated block sums to the
    tile's output summation exactly (ragged last block included), agrees with the one-sided
    tile check's checksum side, and every single-bit flip of every element is flagged."""
    M, N, K = 6, 13, 9
    A, B = wl.gemm_operands(M, N, K, "i8", seed=41)
    C = oracle.gemm(A, B, "i8")
    r0, r1, c0, c1 = 1, 6, 2, 13
    chk = oracle.replica_check(A, B, C, "i8", r0, r1, c0, c1, block_n=block_n)
    want = int((A.astype(np.int64)[r0:r1] @ B.astype(np.int64)[:, c0:c1]).sum())
    assert chk.lhs == chk.rhs == want and not chk.flag
    assert chk.rhs == oracle.tile_check(A, B, C, "i8", r0, r1, c0, c1).rhs
    for i in range(r0, r1):
        for j in range(c0, c1):
            for bit in (0, 7, 15, 31):
                Cb = C.copy()
                Cb[i, j] = oracle.flip_bit(int(C[i, j]), bit, "i8")
                assert oracle.replica_check(A, B, Cb, "i8", r0, r1, c0, c1, block_n=block_n).flag
    # an element outside the tile does not concern it
    Cb = C.copy()
    Cb[0, 0] += 1000
    assert not oracle.replica_check(A, B, Cb, "i8", r0, r1, c0, c1, block_n=block_n).flag


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_replica_check_fp_against_numpy_and_tolerance(dtype):
    M, N, K = 40, 70, 96
    A, B = wl.gemm_operands(M, N, K, dtype, seed=43)
    C = oracle.gemm(A, B, dtype)
    r0, r1, c0, c1 = 8, 40, 6, 70
    chk = oracle.replica_check(A, B, C, dtype, r0, r1, c0, c1)
    Aw, Bw = oracle.widen(A, dtype), oracle.widen(B, dtype)
    want = float((Aw[r0:r1] @ Bw[:, c0:c1]).sum())
    scale = float(np.abs(Aw[r0:r1]).sum(axis=0) @ np.abs(Bw[:, c0:c1]).sum(axis=1))
    assert abs(chk.rhs - want) <= 1e-13 * scale and abs(chk.lhs - want) <= 1e-13 * scale
    assert not chk.flag
    assert chk.tau == oracle.tolerance(K, oracle.frob(C, r0, r1, c0, c1), dtype, scheme=2)
    # a change well above the tolerance is seen, one well below is not
    for delta, seen in ((4 * chk.tau, True), (chk.tau / 4, False)):
        Cb = C.copy()
        Cb[r0 + 3, c0 + 40] += delta
        assert oracle.replica_check(A, B, Cb, dtype, r0, r1, c0, c1).flag == seen


# ------------------------------------------------- several checksums (Sec. 2.4, last paragraph)
def test_weighted_checks_hold_exactly_on_clean_integers_and_locate_every_single_fault():
    """Three independent checksum pairs per block: all hold exactly on clean integer data (checked
    against a direct evaluation), and a single wrong element is located exactly -- every element
    of a ragged block, several bits."""
    M, N, K = 11, 14, 9
    A, B = wl.gemm_operands(M, N, K, "i8", seed=61)
    C = oracle.gemm(A, B, "i8")
    r0, r1, c0, c1 = 2, 11, 3, 14
    wc = oracle.weighted_region_check(A, B, C, "i8", r0, r1, c0, c1)
    assert not wc.flag
    blk = C[r0:r1, c0:c1]
    assert wc.rows.lhs == sum((i + 1) * int(blk[i].sum()) for i in range(r1 - r0))
    assert wc.cols.lhs == sum((j + 1) * int(blk[:, j].sum()) for j in range(c1 - c0))
    assert wc.plain.rhs == int(A[r0:r1].astype(np.int64).sum(axis=0) @ B[:, c0:c1].astype(np.int64).sum(axis=1))
    assert wc.plain.lhs == wc.plain.rhs and wc.rows.lhs == wc.rows.rhs and wc.cols.lhs == wc.cols.rhs
    for i in range(r0, r1):
        for j in range(c0, c1):
            for bit in (0, 13, 31):
                Cf = oracle.inject(A, B, C, "i8", i, j, bit)
                bad = oracle.weighted_region_check(A, B, Cf, "i8", r0, r1, c0, c1)
                assert bad.flag
                assert oracle.locate(bad, "i8", r1 - r0, c1 - c0) == (i - r0, j - c0, int(Cf[i, j] - C[i, j]))


def test_weighted_checks_see_two_faults_that_cancel_in_the_plain_sum():
    """Two wrong elements with opposite errors leave the plain checksum intact; the weighted
    ones see them unless the two share both weights (the same element).  Exhaustive over pairs
    of a small block."""
    M, N, K = 5, 6, 7
    A, B = wl.gemm_operands(M, N, K, "i8", seed=62)
    C = oracle.gemm(A, B, "i8")
    cells = [(i, j) for i in range(M) for j in range(N)]
    for a in cells:
        for b in cells:
            if a == b:
                continue
            Cf = C.copy()
            Cf[a] += 1000
            Cf[b] -= 1000
            wc = oracle.weighted_region_check(A, B, Cf, "i8", 0, M, 0, N)
            assert not wc.plain.flag            # the single-checksum scheme is blind here
            assert wc.flag
            assert wc.rows.flag == (a[0] != b[0]) and wc.cols.flag == (a[1] != b[1])
            assert oracle.locate(wc, "i8", M, N) is None


def test_weighted_checks_in_floating_point():
    """fp16 operands: clean data passes all three comparisons (also for a binary32-accumulated C),
    a large single fault is located, and the weighted sums equal the definition."""
    M, N, K = 32, 64, 128
    for da, db in (("normal", "normal"), ("uniform_01", "weights"), ("uniform_01", "uniform_01")):
        A, B = wl.gemm_operands(M, N, K, "f16", seed=63, dist_a=da, dist_b=db)
        C = oracle.gemm(A, B, "f16")
        wc = oracle.weighted_region_check(A, B, C, "f16", 0, M, 0, N)
        assert not wc.flag
        w = (np.arange(M) + 1) / M
        assert wc.rows.lhs == pytest.approx(float((w[:, None] * C).sum()), rel=1e-12)
        assert wc.rows.rhs == pytest.approx(wc.rows.lhs, rel=1e-9, abs=1e-9)
        C32 = _accumulate_binary32(A, B)
        wc32 = oracle.weighted_region_check(A, B, C32, "f16", 0, M, 0, N)
        assert not wc32.flag
        assert max(abs(c.residual) / c.tau for c in (wc32.plain, wc32.rows, wc32.cols)) < 0.25
        Cf = oracle.inject(A, B, C, "f16", 17, 41, 27)
        bad = oracle.weighted_region_check(A, B, Cf, "f16", 0, M, 0, N)
        if abs(Cf[17, 41] - C[17, 41]) > 100 * bad.plain.tau:
            i, j, d = oracle.locate(bad, "f16", M, N)
            assert (i, j) == (17, 41) and d == pytest.approx(Cf[17, 41] - C[17, 41], rel=1e-6)
