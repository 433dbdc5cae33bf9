"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact for int8 -> int32; |dC| <= 1e-2|C| + 1e-2 rms(C) for fp16/bf16."""
import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl

pytestmark = pytest.mark.gpu

MODES = [B.NONE, B.GLOBAL, B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED]
WAVE_LEVEL = (B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED)   # one comparison per wavefront tile
# (M, N, K): one tile; several tiles with ragged edges; skinny; degenerate; unaligned K
# (K a whole number of 16-byte chunks but not of 128-byte k tiles: the streaming kernel's short last tile)
SHAPES = [(64, 64, 64), (200, 136, 264), (130, 70, 333), (1, 64, 13), (16, 1, 256), (1, 1, 1),
          (300, 520, 1024), (17, 260, 72), (512, 512, 128), (32, 32, 32), (96, 160, 48), (300, 520, 1040)]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", SHAPES)
def test_clean_parity(shape, mode, dtype):
    from gpu_util import run_gemm, c_close, normwise_error
    M, N, K = shape
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=100 + M + N + K)
    print(f"case shape={shape} mode={mode} dtype={dtype}", flush=True)
    res = run_gemm(A, Bm, dtype, mode)
    C_ref = oracle.gemm(A, Bm, dtype)
    assert c_close(res.C, C_ref, dtype), normwise_error(res.C, C_ref)
    if dtype != "i8":
        assert normwise_error(res.C, C_ref) < (2.0 ** -10 if dtype == "f16" else 2.0 ** -7)
    assert res.flag == 0
    dt = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}[dtype]
    aligned = K * (1 if dtype == "i8" else 2) % 16 == 0
    if mode == B.GLOBAL:
        rm, rn = B.abft_region_shape(M, N, K, dt, aligned)
        flag, checks = oracle.global_check_blocks(A, Bm, C_ref, dtype, rm, rn)
        assert not flag
        assert res.report.tiles == len(checks)
        # the reported region is the oracle's region of that index: same sides, same tolerance
        ref = checks[res.report.region - 1]
        if dtype == "i8":
            assert res.report.lhs == ref.lhs and res.report.rhs == ref.rhs and res.report.worst_ratio == 0.0
        else:
            # checksum side: fp32 weight checksums, products summed in fp32 within a k tile and
            # in fp64 above that; its rounding must stay a small part of the tolerance
            assert abs(res.report.rhs - ref.rhs) <= 0.1 * ref.tau + 1e-9
            assert abs(res.report.lhs - ref.lhs) <= ref.tau + 1e-300
            assert res.report.tau == pytest.approx(ref.tau, rel=1e-3)
            assert res.report.worst_ratio < 0.5
    if mode in WAVE_LEVEL:
        tm, tn, _ = B.abft_tile_shape(M, N, K, dt, aligned)
        # one comparison per wavefront register tile of the partition of C
        regions = list(oracle.tiles(M, N, tm, tn))
        assert res.report.tiles == len(regions)
        assert res.report.worst_ratio < 0.5
        # the reported tile is the oracle's tile of that index: same sides, same tolerance
        from gpu_util import wave_check
        ref = wave_check(mode, A, Bm, C_ref, dtype, regions[res.report.region - 1], (tm, tn))
        assert not ref.flag
        if dtype == "i8":
            assert res.report.lhs == ref.lhs and res.report.rhs == ref.rhs
        else:
            # both sides are fp32 accumulations on the device
            assert abs(res.report.rhs - ref.rhs) <= ref.tau + 1e-300
            assert abs(res.report.lhs - ref.lhs) <= ref.tau + 1e-300
            assert res.report.tau == pytest.approx(ref.tau, rel=1e-3)


# shapes chosen so that every tile configuration of the dispatcher runs under test:
# (shape, wavefront tile of the thread-level scheme, region of the global scheme)
CONFIG_SHAPES = [
    ((520, 1040, 512), (64, 64), (64, 64)),        # 64 x 64 streaming tile, ragged edges
    ((520, 1040, 128), (32, 128), (64, 128)),      # the same grid with a short k loop: 64 x 128 direct-to-LDS tile
    ((2304, 2304, 256), (32, 128), (128, 128)),    # 128 x 128 tile, more than one workgroup per compute unit: wide wavefront tiles for thread-level
    ((1536, 1536, 256), (64, 64), (128, 128)),     # at most one per compute unit: 2 x 2 wavefronts of 64 x 64 for every scheme
    ((16500, 64, 256), (32, 128), (128, 128)),     # narrow output: 128 x 128 tile of full-width wavefronts
    ((300, 520, 1024), (32, 32), (32, 32)),        # one round of 32 x 32 streaming tiles
    ((256, 1100, 512), (32, 64), (32, 64)),        # more than one round of those: 32 x 64 streaming tiles
]


@pytest.mark.parametrize("dtype", ["f16", "i8"])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", CONFIG_SHAPES)
def test_every_tile_configuration(case, mode, dtype):
    from gpu_util import run_gemm, c_close
    (M, N, K), wave_tile, region = case
    dt = {"f16": B.F16, "i8": B.I8}[dtype]
    tm, tn, ks = B.abft_tile_shape(M, N, K, dt)
    assert (tm, tn) == wave_tile and B.abft_region_shape(M, N, K, dt) == region
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=300 + M)
    print(f"case config shape={(M, N, K)} mode={mode} dtype={dtype}", flush=True)
    res = run_gemm(A, Bm, dtype, mode)
    C_ref = oracle.gemm(A, Bm, dtype)
    assert c_close(res.C, C_ref, dtype)
    assert res.flag == 0
    if mode == B.GLOBAL:
        bad, checks = oracle.global_check_blocks(A, Bm, C_ref, dtype, *region)
        assert not bad and res.report.tiles == len(checks) and res.report.worst_ratio < 0.5
    if mode in WAVE_LEVEL:
        assert res.report.worst_ratio < 0.5
    if mode != B.NONE:
        # a flipped exponent bit (sign bit for int8) in the last, ragged tile is seen: the exponent
        # bit that turns the value into an astronomically large one (bit 30 below 2.0, else bit 29)
        bit = 31 if dtype == "i8" else (30 if abs(C_ref[M - 1, N - 1]) < 2.0 else 29)
        hit = run_gemm(A, Bm, dtype, mode, inject=B.Fault(M - 1, N - 1, bit, -1))
        assert hit.flag == 1


@pytest.mark.parametrize("dtype", ["f16", "i8"])
@pytest.mark.parametrize("mode", MODES)
def test_layouts_strides_and_misalignment(mode, dtype):
    """Row-major K x N weights, padded leading dimensions and operands that are not
    16-byte aligned all go through the generic loader and must give the same C."""
    from gpu_util import run_gemm, c_close
    M, N, K = 96, 80, 136
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=7)
    C_ref = oracle.gemm(A, Bm, dtype)
    for kw in (dict(layout=B.B_KN), dict(lda_pad=8, ldb_pad=16, ldc_pad=3), dict(lda_pad=1),
               dict(misalign=1), dict(layout=B.B_KN, ldb_pad=5, misalign=3), dict(use_beta=True)):
        print(f"case mode={mode} dtype={dtype} {kw}", flush=True)
        res = run_gemm(A, Bm, dtype, mode, **kw)
        assert c_close(res.C, C_ref, dtype), kw
        assert res.flag == 0, kw


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_checksum_vectors(dtype):
    """alpha = 1^T A and beta = B 1 as the device computes them (Sec. 2.4 step 1)."""
    import torch
    from gpu_util import to_dev, DEV
    dt = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}[dtype]
    for (M, N, K) in [(64, 64, 64), (700, 33, 264), (5, 9, 13)]:
        A, Bm = wl.gemm_operands(M, N, K, dtype, seed=3)
        a_ref, b_ref = oracle.col_checksum(A, dtype), oracle.row_checksum(Bm, dtype)
        wide = torch.int64 if dtype == "i8" else torch.float64
        dA = to_dev(A, dtype)
        alpha = torch.zeros(K, dtype=wide, device=DEV)
        B.abft_activation_checksum(M, K, dA, K, dt, alpha)
        for layout, host in ((B.B_NK, np.ascontiguousarray(Bm.T)), (B.B_KN, Bm)):
            dB = to_dev(host, dtype)
            beta_raw = torch.zeros(B.abft_beta_bytes(K, N) // 8, dtype=wide, device=DEV)
            B.abft_weight_checksum(K, N, dB, host.shape[1], layout, dt, beta_raw)
            # per block of 16 columns: row checksums of the column blocks
            nb = -(-N // 16)
            beta_b_raw = torch.zeros(B.abft_beta_bytes(K, N, 16) // 8, dtype=wide, device=DEV)
            B.abft_weight_checksum(K, N, dB, host.shape[1], layout, dt, beta_b_raw, block_n=16)
            torch.cuda.synchronize()
            blocks = np.stack([oracle.row_checksum(np.ascontiguousarray(Bm[:, b * 16:(b + 1) * 16]), dtype)
                               for b in range(nb)])
            beta, beta_b = beta_raw.cpu().numpy()[:K], beta_b_raw.cpu().numpy()[:nb * K]
            # the second copy (what the product kernel reads): per block along k, at the next
            # multiple of 256 bytes; floats, or low / high base-256 digits for int8
            second = beta_b_raw.cpu().numpy().view(np.uint8)[-(-(nb * K * 8) // 256) * 256:]
            if dtype == "i8":
                assert np.array_equal(beta, b_ref)
                assert np.array_equal(beta_b.reshape(K, nb).T, blocks)
                digits = second[:nb * 2 * K].view(np.int8).astype(np.int64).reshape(nb, 2, K)
                assert np.array_equal(digits[:, 0] + 256 * digits[:, 1], blocks)
                # third copy: four planes of digits of the column-weighted checksum sum_j (j + 1) B[k][16 b + j]
                third = second[-(-(nb * K * 4) // 256) * 256:][:nb * K * 8].view(np.int8).astype(np.int64).reshape(nb, 8, K)
                wsum = np.stack([(Bm[:, b * 16:(b + 1) * 16].astype(np.int64) * (np.arange(min(16, N - b * 16)) + 1)).sum(axis=1)
                                 for b in range(nb)])
                assert np.array_equal(sum(third[:, q] * 256 ** q for q in range(4)), wsum)
            else:
                assert np.allclose(beta, b_ref, rtol=1e-12, atol=1e-12)
                assert np.allclose(beta_b.reshape(K, nb).T, blocks, rtol=1e-12, atol=1e-12)
                f32 = second[:nb * K * 4].view(np.float32).reshape(nb, K)
                assert np.array_equal(f32, blocks.astype(np.float32))
                if dtype == "f16":
                    # third copy: per block four planes of K halves: hi = fl16(beta), lo = fl16((beta - hi) 2^11),
                    # then the same two pieces of the column-weighted checksum sum_j (j + 1) / 16 B[k][16 b + j]
                    third = second[-(-(nb * K * 4) // 256) * 256:][:nb * K * 8].view(np.float16).reshape(nb, 4, K)
                    hi = f32.astype(np.float16)
                    lo = ((f32 - hi.astype(np.float32)) * np.float32(2048)).astype(np.float16)
                    assert np.array_equal(third[:, 0], hi) and np.array_equal(third[:, 1], lo)
                    Bw = oracle.widen(Bm, dtype)
                    wsum = np.stack([(Bw[:, b * 16:(b + 1) * 16] * ((np.arange(min(16, N - b * 16)) + 1) / 16.0)).sum(axis=1)
                                     for b in range(nb)]).astype(np.float32)
                    vhi = wsum.astype(np.float16)
                    assert np.array_equal(third[:, 2], vhi)
                    assert np.array_equal(third[:, 3], ((wsum - vhi.astype(np.float32)) * np.float32(2048)).astype(np.float16))
            # fourth copy: per block and k tile of the large-tile kernel (64 values of k; int8: 128) a
            # record of 1 KB behind the third copy: the tile's pieces / floats / digits of the second and third
            kt = 128 if dtype == "i8" else 64
            nrec = -(-K // kt)
            recs = second[-(-(nb * K * 4) // 256) * 256:][-(-(nb * K * 8) // 256) * 256:][:nb * nrec * 1024].reshape(nb, nrec, 1024)
            for b in range(nb):
                for t in range(nrec):
                    n_k = min(kt, K - t * kt)
                    ks = slice(t * kt, t * kt + n_k)
                    if dtype == "i8":
                        d = recs[b, t].view(np.int8).astype(np.int64)
                        assert np.array_equal(d[:n_k] + 256 * d[128:128 + n_k], blocks[b, ks])
                    else:
                        want = blocks[b, ks].astype(np.float32)
                        assert np.array_equal(recs[b, t][256:256 + 4 * n_k].view(np.float32), want)
                        if dtype == "f16":
                            h = want.astype(np.float16)
                            assert np.array_equal(recs[b, t][:2 * n_k].view(np.float16), h)
                            assert np.array_equal(recs[b, t][128:128 + 2 * n_k].view(np.float16),
                                                  ((want - h.astype(np.float32)) * np.float32(2048)).astype(np.float16))
        if dtype == "i8":
            assert np.array_equal(alpha.cpu().numpy(), a_ref)
        else:
            assert np.allclose(alpha.cpu().numpy(), a_ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("mode", [B.GLOBAL, B.THREAD, B.REPLICA, B.TWOSIDED])
@pytest.mark.parametrize("shape", [(64, 64, 64), (200, 136, 256), (96, 72, 304)])
def test_int8_injected_faults_always_flagged(shape, mode):
    """Every single-bit flip of an int32 accumulator changes the sum exactly: 100 % detection."""
    from gpu_util import run_gemm
    M, N, K = shape
    A, Bm = wl.gemm_operands(M, N, K, "i8", seed=21)
    C_ref = oracle.gemm(A, Bm, "i8")
    _, _, ks = B.abft_tile_shape(M, N, K, B.I8)
    rng = np.random.default_rng(22)
    parts = B.abft_k_parts(M, N, K, B.I8, mode)
    for t in range(40):
        i, j, bit = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(32))
        k_after = -1 if (t % 2 == 0 or K <= ks) else ks * int(rng.integers(1, K // ks))
        if k_after >= K:
            k_after = -1
        if t % 5 == 4:
            k_after = -2   # after the partial tiles of the wavefronts that share a tile have been added
        print(f"case shape={shape} mode={mode} fault=({i},{j},bit {bit},k_after {k_after}) parts={len(parts)}", flush=True)
        res = run_gemm(A, Bm, "i8", mode, inject=B.Fault(i, j, bit, k_after))
        # the accumulator that is hit belongs to the part of k that holds k_after - 1 (K - 1 for a
        # flip of the finished value) and holds that part's products with k < k_after; after the
        # addition of the parts it is the finished element itself
        if k_after == -2:
            C_bad = oracle.inject(A, Bm, C_ref, "i8", i, j, bit)
        else:
            part = parts[oracle.part_of(parts, (K if k_after < 0 else k_after) - 1)]
            C_bad = oracle.inject(A, Bm, C_ref, "i8", i, j, bit, k_after=k_after, k_set=part)
        want = ((C_bad + 2 ** 31) % 2 ** 32) - 2 ** 31  # the int32 register wraps
        assert np.array_equal(res.C, want)
        assert res.flag == 1


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(64, 64, 64), (192, 256, 512)])
@pytest.mark.parametrize("mode", [B.GLOBAL, B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED])
def test_fp_injected_faults_match_oracle_outside_band(mode, shape, dtype):
    """|delta| >= 2 tau must be flagged, |delta| <= tau/2 must not (don't-care in between);
    non-finite results must be flagged.  (The second shape runs on wavefront tiles of several MFMA
    blocks, where the schemes that add checksums in the operand type carry their wider tolerance.)"""
    import math
    from gpu_util import run_gemm, wave_check
    M, N, K = shape
    dt = B.F16 if dtype == "f16" else B.BF16
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=31)
    C_ref = oracle.gemm(A, Bm, dtype)
    tm, tn, ks = B.abft_tile_shape(M, N, K, dt)
    rng = np.random.default_rng(32)
    counts = {"must": 0, "mustnot": 0, "band": 0}
    parts = B.abft_k_parts(M, N, K, dt, mode)
    clean = run_gemm(A, Bm, dtype, mode)
    assert clean.flag == 0
    resid0 = clean.report.tau * clean.report.worst_ratio
    for t in range(60):
        i, j, bit = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(32))
        k_after = -2 if t % 3 == 2 else -1   # the finished partial accumulator, or the element after the addition
        print(f"case mode={mode} dtype={dtype} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        res = run_gemm(A, Bm, dtype, mode, inject=B.Fault(i, j, bit, k_after))
        # every scheme compares the finished tile: the oracle's check of the region that holds the
        # element, on the C the fault leaves behind
        if k_after == -2:
            C_bad = oracle.inject(A, Bm, C_ref, dtype, i, j, bit)
        else:
            C_bad = oracle.inject(A, Bm, C_ref, dtype, i, j, bit, k_set=parts[oracle.part_of(parts, K - 1)])
        if mode == B.GLOBAL:
            rm, rn = B.abft_region_shape(M, N, K, dt)
            r0, c0 = i // rm * rm, j // rn * rn
            chk = oracle.region_check(A, Bm, C_bad, dtype, r0, min(r0 + rm, M), c0, min(c0 + rn, N))
        else:
            r0, c0 = i // tm * tm, j // tn * tn
            chk = wave_check(mode, A, Bm, C_bad, dtype, (r0, min(r0 + tm, M), c0, min(c0 + tn, N)), (tm, tn))
        if not math.isfinite(C_bad[i, j]):
            assert res.flag == 1
            counts["must"] += 1
            continue
        delta = abs(chk.residual)
        # (the device's own clean residual: rounding of the accumulation and of the checksum sums)
        delta_lo, delta_hi = delta - resid0, delta + resid0
        if delta_lo >= 2 * chk.tau:
            assert res.flag == 1, (i, j, bit, delta, chk.tau)
            counts["must"] += 1
        elif delta_hi <= chk.tau / 2:
            assert res.flag == 0, (i, j, bit, delta, chk.tau)
            counts["mustnot"] += 1
        else:
            counts["band"] += 1
    assert counts["must"] > 5 and counts["mustnot"] > 5


def test_results_are_deterministic():
    from gpu_util import run_gemm
    A, Bm = wl.gemm_operands(300, 520, 1024, "f16", seed=41)
    first = run_gemm(A, Bm, "f16", B.GLOBAL)
    for _ in range(5):
        again = run_gemm(A, Bm, "f16", B.GLOBAL)
        assert np.array_equal(first.C, again.C)
        assert first.report.lhs == again.report.lhs and first.report.rhs == again.report.rhs


def test_auto_mode_follows_selector():
    from gpu_util import run_gemm, c_close
    A, Bm = wl.gemm_operands(64, 64, 64, "f16", seed=42)
    res = run_gemm(A, Bm, "f16", B.AUTO)
    # 64^3 is bandwidth bound -> thread-level: one comparison per wavefront tile, not per workgroup tile
    tm, tn, _ = B.abft_tile_shape(64, 64, 64, B.F16)
    assert res.flag == 0 and res.report.tiles == -(-64 // tm) * -(-64 // tn) and res.report.tau > 0
    assert res.report.l1 == 0.0   # the ||C||_1 term belongs to the global scheme only
    assert c_close(res.C, oracle.gemm(A, Bm, "f16"), "f16")


@pytest.mark.parametrize("shape", [(64, 1024, 4096), (200, 384, 512)])
@pytest.mark.parametrize("mode", [B.GLOBAL, B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_faults_where_wavefronts_share_a_tile_along_k(dtype, mode, shape):
    """Latency-bound products: four wavefronts share each register tile along k, their partial
    tiles are added in a fixed order (bit-reproducible) and every scheme compares the added-up
    tile.  A fault in any partial accumulator (mid-loop or finished) and a fault in the finished
    value after the addition are all seen by the one comparison of the tile that holds them."""
    import math
    from gpu_util import run_gemm, c_close
    M, N, K = shape
    dt = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}[dtype]
    parts = B.abft_k_parts(M, N, K, dt, mode)
    assert len(parts) == 4 and sorted(k for p in parts for k in p) == list(range(K))
    tm, tn, ks = B.abft_tile_shape(M, N, K, dt)
    if mode == B.GLOBAL:
        tm, tn = B.abft_region_shape(M, N, K, dt)
    fp = dtype != "i8"
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=55, dist_a="uniform_01" if fp else "int8",
                             dist_b="weights" if fp else "int8")
    C_ref = oracle.gemm(A, Bm, dtype)
    res = run_gemm(A, Bm, dtype, mode)
    assert c_close(res.C, C_ref, dtype) and res.flag == 0
    again = run_gemm(A, Bm, dtype, mode)
    assert np.array_equal(res.C, again.C)
    assert res.report.tiles == math.ceil(M / tm) * math.ceil(N / tn)
    assert res.report.worst_ratio < 0.5
    resid0 = res.report.tau * res.report.worst_ratio   # largest clean rounding residual of any tile
    rng = np.random.default_rng(56)
    seen = {"must": 0, "mustnot": 0}
    for t in range(15):
        i, j, bit = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(12, 32))
        k_after = (-1, -2, ks * int(rng.integers(1, K // ks)))[t % 3]
        print(f"case shared-k dtype={dtype} mode={mode} shape={shape} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        got = run_gemm(A, Bm, dtype, mode, inject=B.Fault(i, j, bit, k_after))
        if k_after == -2:
            C_bad = oracle.inject(A, Bm, C_ref, dtype, i, j, bit)
        else:
            part = parts[oracle.part_of(parts, (K if k_after < 0 else k_after) - 1)]
            C_bad = oracle.inject(A, Bm, C_ref, dtype, i, j, bit, k_after=k_after, k_set=part)
        if not fp:
            assert got.flag == 1
            assert np.array_equal(got.C, ((C_bad + 2 ** 31) % 2 ** 32) - 2 ** 31)
            seen["must"] += 1
            continue
        r0, c0 = i // tm * tm, j // tn * tn
        region = (r0, min(r0 + tm, M), c0, min(c0 + tn, N))
        if mode == B.GLOBAL:
            chk = oracle.region_check(A, Bm, C_bad, dtype, *region)
        else:
            from gpu_util import wave_check
            chk = wave_check(mode, A, Bm, C_bad, dtype, region, (tm, tn))
        if not math.isfinite(C_bad[i, j]):
            assert got.flag == 1
        elif abs(chk.residual) >= 2 * chk.tau + resid0:
            assert got.flag == 1, (abs(chk.residual), chk.tau)
            seen["must"] += 1
        elif abs(chk.residual) <= chk.tau / 2 - resid0:
            assert got.flag == 0, (abs(chk.residual), chk.tau)
            seen["mustnot"] += 1
    assert seen["must"] > 0


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_clean_runs_raise_no_false_alarm(dtype):
    """Zero false positives: 2500 clean runs per type (250 seeds x two shapes x the five protected schemes), over
    the value distributions of the benchmark configurations, including all-positive operands
    (where the accumulation's coherent bias shows): never a flag, residual below half the tolerance."""
    from gpu_util import run_gemm
    dists = [("uniform_pm1", "uniform_pm1"), ("uniform_01", "weights"), ("normal", "normal"), ("uniform_01", "uniform_01")]
    worst = 0.0
    for seed in range(250):
        da, db = dists[seed % len(dists)]
        for (M, N, K) in ((64, 64, 64), (200, 136, 256)):
            A, Bm = wl.gemm_operands(M, N, K, dtype, seed=7000 + seed, dist_a=da, dist_b=db)
            for mode in (B.GLOBAL, B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED):
                res = run_gemm(A, Bm, dtype, mode)
                assert res.flag == 0, (seed, da, db, (M, N, K), mode, res.report.worst_ratio)
                worst = max(worst, res.report.worst_ratio)
    print(f"worst residual / tolerance over the campaign ({dtype}): {worst:.3f}", flush=True)
    assert worst < 0.5


# ------------------------------------------- several checksums per tile (Sec. 2.4, last paragraph)
@pytest.mark.parametrize("dtype", ["i8", "f16"])
@pytest.mark.parametrize("shape", [(64, 64, 64), (200, 384, 512), (256, 1024, 1024), (96, 2048, 192), (512, 2048, 1024)])
def test_weighted_global_scheme_flags_and_locates(shape, dtype):
    """ABFT_GLOBAL_WEIGHTED on the latency-bound tiling: clean runs pass all three comparisons of
    every tile and leave C as the oracle's; a planted fault is flagged, and the reported position
    and size are those of the planted element (int8: always, exactly; fp16: whenever the fault
    is far outside the tolerance), equal to what the oracle's weighted check of that tile locates."""
    import math
    from gpu_util import DeviceGemm, c_close
    M, N, K = shape
    dt = {"f16": B.F16, "i8": B.I8}[dtype]
    g = DeviceGemm(M, N, K, dtype, seed=800 + M, dist_a="uniform_01" if dtype == "f16" else "int8",
                   dist_b="weights" if dtype == "f16" else "int8")
    assert g.rm <= 64 and g.rn <= 64          # the streaming tiles
    C_ref = oracle.gemm(g.A, g.Bm, dtype)
    flag, rep = g.run(B.GLOBAL_WEIGHTED)
    assert flag == 0 and c_close(g.C(), C_ref, dtype)
    assert rep.tiles == math.ceil(M / g.rm) * math.ceil(N / g.rn)
    assert rep.worst_ratio < 0.5 and rep.ratio_rows < 0.5 and rep.ratio_cols < 0.5
    assert (rep.fault_row, rep.fault_col) == (-1, -1)
    # every tile's three comparisons on the oracle's side as well
    for t in list(oracle.tiles(M, N, g.rm, g.rn))[:6]:
        assert not oracle.weighted_region_check(g.A, g.Bm, C_ref, dtype, *t, block_m=g.rm, block_n=g.rn).flag
    parts = B.abft_k_parts(M, N, K, dt, B.GLOBAL)
    rng = np.random.default_rng(M + N)
    located = 0
    for t in range(24):
        i, j = int(rng.integers(M)), int(rng.integers(N))
        bit = int(rng.integers(32)) if dtype == "i8" else (30, int(rng.integers(20, 30)), int(rng.integers(8, 20)))[t % 3]
        k_after = (-1, -2, g.k_step * int(rng.integers(1, max(2, K // g.k_step))))[t % 3]
        if k_after >= K:
            k_after = -1
        print(f"case weighted dtype={dtype} shape={shape} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        flag, rep = g.run(B.GLOBAL_WEIGHTED, inject=B.Fault(i, j, bit, k_after))
        if k_after == -2:
            C_bad = oracle.inject(g.A, g.Bm, C_ref, dtype, i, j, bit)
        else:
            C_bad = oracle.inject(g.A, g.Bm, C_ref, dtype, i, j, bit, k_after=k_after,
                                  k_set=parts[oracle.part_of(parts, (K if k_after < 0 else k_after) - 1)])
        r0, r1, c0, c1 = g.region_of(i, j, B.GLOBAL)
        wc = oracle.weighted_region_check(g.A, g.Bm, C_bad, dtype, r0, r1, c0, c1, block_m=g.rm, block_n=g.rn)
        if dtype == "i8":
            assert flag == 1 and wc.flag
            li, lj, delta = oracle.locate(wc, dtype, g.rm, g.rn)
            assert (r0 + li, c0 + lj) == (i, j)
            assert (rep.fault_row, rep.fault_col, rep.fault_delta) == (i, j, float(delta))
            assert np.array_equal(g.C(), ((C_bad + 2 ** 31) % 2 ** 32) - 2 ** 31)
            located += 1
            continue
        if not math.isfinite(C_bad[i, j]):
            assert flag == 1
            continue
        delta = abs(wc.plain.residual)
        if delta >= 2 * wc.plain.tau:
            assert flag == 1
        elif max(abs(c.residual) / c.tau for c in (wc.plain, wc.rows, wc.cols)) <= 0.4:
            assert flag == 0
        if delta >= 200 * wc.plain.tau:
            li, lj, d = oracle.locate(wc, dtype, g.rm, g.rn)
            assert (r0 + li, c0 + lj) == (i, j)
            assert (rep.fault_row, rep.fault_col) == (i, j)
            assert rep.fault_delta == pytest.approx(d, rel=1e-3)
            located += 1
    assert located > 3


def test_weighted_global_scheme_is_refused_where_it_does_not_exist():
    import torch
    from gpu_util import DEV
    t = torch.zeros(1 << 20, dtype=torch.float16, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = torch.zeros(1 << 24, dtype=torch.uint8, device=DEV)
    for (M, N, K, dt) in [(4096, 4096, 64, B.F16), (64, 64, 64, B.BF16)]:
        with pytest.raises(B.AbftError) as e:
            B.abft_gemm(M, N, K, t, K, t, K, B.B_NK, t, N, dt, B.GLOBAL_WEIGHTED, workspace=ws,
                        workspace_bytes=ws.numel(), fault_flag=flag)
        assert e.value.code == -9


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("shape", [32, 16])
def test_mfma_probe_runs_and_counts_its_operations(shape, dtype):
    """The measurement aid: launches, leaves its sink alone and reports the operations of one
    launch: compute units x 8 wavefronts x iterations x the register tile's 128 x 64 x depth x 2."""
    import torch
    from gpu_util import DEV
    dt = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}[dtype]
    src = torch.zeros(B.abft_mfma_probe_bytes(), dtype=torch.uint8, device=DEV)
    sink = torch.full((1,), 7.0, dtype=torch.float32, device=DEV)
    ops = B.abft_mfma_probe(shape, dt, 50, src, sink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    depth = (16 if shape == 32 else 32) * (2 if dtype == "i8" else 1)
    assert ops == cus * 8 * 50 * 128 * 64 * depth * 2
    assert float(sink.item()) == 7.0
