"""Parity at the benchmark's full sizes, in the launch configuration bench.py times:
sampled rows of C against the oracle, the checksum identity, and fault-injection
campaigns (seeded single-bit flips) whose verdicts must match the oracle's."""
import math

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl

pytestmark = pytest.mark.gpu
DT = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}


class Big:
    """Device-resident operands of one large GEMM (weights stored N x K)."""

    def __init__(self, M, N, K, dtype, seed, dist="normal"):
        import torch
        from gpu_util import to_dev, DEV
        self.M, self.N, self.K, self.dtype, self.dt = M, N, K, dtype, DT[dtype]
        self.A, self.Bm = wl.gemm_operands(M, N, K, dtype, seed, dist_a=dist, dist_b=dist)
        self.dA = to_dev(self.A, dtype)
        self.dB = to_dev(np.ascontiguousarray(self.Bm.T), dtype)
        c_t = torch.int32 if dtype == "i8" else (torch.float16 if dtype == "f16" else torch.bfloat16)
        self.dC = torch.zeros((M, N), dtype=c_t, device=DEV)
        self.flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        self.rep = torch.zeros(64, dtype=torch.uint8, device=DEV)
        self.wsb = max(B.abft_workspace_bytes(M, N, K, self.dt, m) for m in (B.NONE, B.GLOBAL, B.THREAD))
        self.ws = torch.zeros(max(self.wsb, 256), dtype=torch.uint8, device=DEV)
        self.rm, self.rn = B.abft_region_shape(M, N, K, self.dt, True)
        self.beta = torch.zeros(B.abft_beta_bytes(K, N, self.rn) // 8, dtype=torch.float64, device=DEV)
        B.abft_weight_checksum(K, N, self.dB, K, B.B_NK, self.dt, self.beta, block_n=self.rn)

    def run(self, mode, inject=None, want_report=True):
        import torch
        from gpu_util import read_report
        self.flag.zero_()
        self.rep.zero_()
        B.abft_gemm(self.M, self.N, self.K, self.dA, self.K, self.dB, self.K, B.B_NK, self.dC, self.N, self.dt,
                    mode, beta=self.beta, workspace=self.ws, workspace_bytes=self.wsb, fault_flag=self.flag,
                    report=self.rep if want_report else None, inject=inject)
        torch.cuda.synchronize()
        return int(self.flag.item()), (read_report(self.rep) if want_report else None)


@pytest.mark.parametrize("n,dtype", [(4096, "f16"), (4096, "bf16"), (8192, "f16"), (8192, "i8")])
def test_large_square_sampled_rows_and_identity(n, dtype):
    from gpu_util import c_to_host, c_close
    big = Big(n, n, n, dtype, seed=900 + n)
    rows = np.random.default_rng(n).choice(n, size=6, replace=False)
    ref = oracle.gemm_rows(big.A, big.Bm, dtype, rows)
    for mode in (B.GLOBAL, B.THREAD):
        print(f"case n={n} dtype={dtype} mode={mode}", flush=True)
        flag, rep = big.run(mode)
        got = c_to_host(big.dC[rows.tolist()], dtype)
        assert c_close(got, ref, dtype)
        assert flag == 0
        if mode == B.GLOBAL:
            assert rep.tiles == (n // big.rm) * (n // big.rn)
            if dtype == "i8":
                assert rep.worst_ratio == 0.0 and rep.lhs == rep.rhs   # exact identity in every region
            else:
                assert rep.worst_ratio < 0.5, rep.worst_ratio
        else:
            tm, tn, _ = B.abft_tile_shape(n, n, n, big.dt, True)
            assert rep.tiles == (n // tm) * (n // tn)
            assert rep.worst_ratio < 0.5, rep.worst_ratio


@pytest.mark.parametrize("dtype,trials", [("i8", 1000), ("f16", 1000)])
def test_fault_campaign_global_4096(dtype, trials):
    """1000 seeded single-bit flips across C and the running accumulators at 4096^3 under the
    scheme the selector picks (global): element uniform over C (fp16: uniform over 16 regions
    drawn once, whose oracle blocks are computed once each), bit uniform over all 32, half in the
    finished value and half in the running accumulator.  int8: every flip flagged.  fp16: the
    verdict equals the oracle's incremental evaluation outside the don't-care band; non-finite
    always flagged."""
    n = 4096
    big = Big(n, n, n, dtype, seed=77)
    _, _, ks = B.abft_tile_shape(n, n, n, big.dt, True)
    flag0, rep0 = big.run(B.GLOBAL)
    assert flag0 == 0
    rng = np.random.default_rng(78)
    must = mustnot = band = 0
    regions = [(int(rng.integers(n // big.rm)), int(rng.integers(n // big.rn))) for _ in range(16)]
    blocks = {}
    for t in range(trials):
        i, j, bit = int(rng.integers(n)), int(rng.integers(n)), int(rng.integers(32))
        if dtype != "i8":
            ri, rj = regions[t % len(regions)]
            i, j = ri * big.rm + i % big.rm, rj * big.rn + j % big.rn
        k_after = -1 if t % 2 == 0 else ks * int(rng.integers(1, n // ks))
        if t % 50 == 0:
            print(f"case {t} dtype={dtype} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        flag, rep = big.run(B.GLOBAL, inject=B.Fault(i, j, bit, k_after))
        if dtype == "i8":
            assert flag == 1
            must += 1
            continue
        # oracle, incremental: the corrupted element against its clean value
        kk = n if k_after < 0 else k_after
        # (row i of A and column j of B only: the oracle widens what it is handed)
        a_row, b_col = big.A[i:i + 1], np.ascontiguousarray(big.Bm[:, j:j + 1])
        head = oracle.partial_dot(a_row, b_col, dtype, 0, 0, 0, kk)
        tail = oracle.partial_dot(a_row, b_col, dtype, 0, 0, kk, n)
        bad = oracle.flip_bit(head, bit, dtype) + tail
        if not math.isfinite(bad):
            assert flag == 1
            must += 1
            continue
        delta = abs(bad - (head + tail))
        # tolerance of the region that holds the element, from the oracle's own block of C
        r0, c0 = i // big.rm * big.rm, j // big.rn * big.rn
        if (r0, c0) not in blocks:
            blk = oracle.gemm(big.A[r0:r0 + big.rm], np.ascontiguousarray(big.Bm[:, c0:c0 + big.rn]), dtype)
            blocks[(r0, c0)] = (blk, oracle.frob(blk) ** 2, oracle.l1norm(blk))
        blk, f2_clean, l1_clean = blocks[(r0, c0)]
        # norms of the block with the one corrupted element (the rest of the block is unchanged)
        clean = float(blk[i - r0, j - c0])
        frob_bad = math.sqrt(max(f2_clean - clean * clean + bad * bad, 0.0))
        l1_bad = l1_clean - abs(clean) + abs(bad)
        tau = oracle.tolerance(n, frob_bad, dtype, scheme=1, l1_norm=l1_bad)
        resid0 = rep0.tau * rep0.worst_ratio   # largest clean rounding residual of any region on the device
        if delta >= 2 * tau + resid0:
            assert flag == 1, (i, j, bit, delta, tau)
            must += 1
        elif delta <= tau / 2 - resid0:
            assert flag == 0, (i, j, bit, delta, tau)
            mustnot += 1
        else:
            band += 1
    assert must > 0
    if dtype != "i8":
        assert mustnot > 0


@pytest.mark.parametrize("mode", [B.THREAD, B.REPLICA])
@pytest.mark.parametrize("dtype,trials", [("i8", 400), ("f16", 400)])
def test_fault_campaign_wave_level_4096(dtype, trials, mode):
    """Seeded single-bit flips at 4096^3 under the two wavefront-level schemes (one-sided ABFT,
    replication): element uniform over 16 wavefront tiles drawn once (whose oracle blocks are
    computed once each), bit uniform over all 32, half in the finished value and half in the
    running accumulator.  int8: every flip flagged.  fp16: the verdict equals the oracle's outside
    the don't-care band around the tolerance of the tile that holds the element."""
    n = 4096
    big = Big(n, n, n, dtype, seed=79)
    tm, tn, ks = B.abft_tile_shape(n, n, n, big.dt, True)
    assert B.abft_k_ways(n, n, n, big.dt, mode)[0] == 1   # one wavefront per register tile: no k parts
    flag0, rep0 = big.run(mode)
    assert flag0 == 0 and rep0.tiles == (n // tm) * (n // tn)
    rng = np.random.default_rng(80)
    must = mustnot = 0
    tiles = [(int(rng.integers(n // tm)), int(rng.integers(n // tn))) for _ in range(16)]
    blocks = {}
    for t in range(trials):
        ti, tj = tiles[t % len(tiles)]
        i, j, bit = ti * tm + int(rng.integers(tm)), tj * tn + int(rng.integers(tn)), int(rng.integers(32))
        k_after = -1 if t % 2 == 0 else ks * int(rng.integers(1, n // ks))
        if t % 50 == 0:
            print(f"case {t} mode={mode} dtype={dtype} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        flag, _ = big.run(mode, inject=B.Fault(i, j, bit, k_after), want_report=False)
        if dtype == "i8":
            assert flag == 1
            must += 1
            continue
        kk = n if k_after < 0 else k_after
        a_row, b_col = big.A[i:i + 1], np.ascontiguousarray(big.Bm[:, j:j + 1])
        head = oracle.partial_dot(a_row, b_col, dtype, 0, 0, 0, kk)
        tail = oracle.partial_dot(a_row, b_col, dtype, 0, 0, kk, n)
        bad = oracle.flip_bit(head, bit, dtype) + tail
        if not math.isfinite(bad):
            assert flag == 1
            must += 1
            continue
        delta = abs(bad - (head + tail))
        r0, c0 = ti * tm, tj * tn
        if (r0, c0) not in blocks:
            blk = oracle.gemm(big.A[r0:r0 + tm], np.ascontiguousarray(big.Bm[:, c0:c0 + tn]), dtype)
            blocks[(r0, c0)] = (blk, oracle.frob(blk) ** 2)
        blk, f2_clean = blocks[(r0, c0)]
        clean = float(blk[i - r0, j - c0])
        frob_bad = math.sqrt(max(f2_clean - clean * clean + bad * bad, 0.0))
        tau = oracle.tolerance(n, frob_bad, dtype, scheme=2)
        resid0 = rep0.tau * rep0.worst_ratio   # largest clean rounding residual of any tile on the device
        if delta >= 2 * tau + resid0:
            assert flag == 1, (i, j, bit, delta, tau)
            must += 1
        elif delta <= tau / 2 - resid0:
            assert flag == 0, (i, j, bit, delta, tau)
            mustnot += 1
    assert must > 0
    if dtype != "i8":
        assert mustnot > 0


def test_ragged_large_uses_the_big_tile_and_matches():
    """M, N not multiples of the 256-wide tile: edge tiles read zeros, results and checksums
    are unaffected.  4000 x 3900 x 512 runs on the large-tile kernel (16 x 16 tiles: one full round of workgroups)."""
    from gpu_util import c_to_host, c_close
    M, N, K = 4000, 3900, 512
    big = Big(M, N, K, "f16", seed=5)
    assert (big.rm, big.rn) == (256, 256)
    rows = np.array([0, 255, 256, 3839, 3840, 3999])
    ref = oracle.gemm_rows(big.A, big.Bm, "f16", rows)
    for mode in (B.NONE, B.GLOBAL, B.THREAD):
        print(f"case ragged mode={mode}", flush=True)
        flag, rep = big.run(mode)
        assert c_close(c_to_host(big.dC[rows.tolist()], "f16"), ref, "f16")
        assert flag == 0
        if mode == B.GLOBAL:
            assert rep.tiles == 16 * 16 and rep.worst_ratio < 0.5
            # the reported region against the oracle's evaluation of the same block
            r = rep.region - 1
            r0, c0 = (r // 16) * 256, (r % 16) * 256
            chk = oracle.region_check(big.A[r0:r0 + 256], np.ascontiguousarray(big.Bm[:, c0:c0 + 256]),
                                      oracle.gemm(big.A[r0:r0 + 256], np.ascontiguousarray(big.Bm[:, c0:c0 + 256]), "f16"),
                                      "f16", 0, min(256, M - r0), 0, min(256, N - c0))
            assert abs(rep.rhs - chk.rhs) <= 0.1 * chk.tau + 1e-9
            assert rep.tau == pytest.approx(chk.tau, rel=1e-3)
    # injected fault in the last (clipped) tile row / column is still seen
    for mode in (B.GLOBAL, B.THREAD):
        flag, _ = big.run(mode, inject=B.Fault(3999, 3899, 29, -1))
        assert flag == 1


def test_large_conv_on_the_big_tile():
    """3x3 conv 64->256 on 56x56, batch 20 (M = 62720, K = 576): implicit GEMM through the
    direct-to-LDS kernel, sampled output pixels against the oracle's im2col product."""
    import ctypes
    import torch
    from gpu_util import to_dev, c_to_host, c_close, read_report, DEV
    c = wl.Conv(20, 56, 56, 64, 256, 3, 3, 1, 1)
    x, Wm = wl.conv_operands(c, "f16", seed=6)
    M, K, N = c.batch * c.OH * c.OW, 576, 256
    assert B.abft_region_shape(M, N, K, B.F16, True) == (256, 256)
    # oracle on sampled output pixels: lower two images only (pixels are independent per image)
    A2 = oracle.im2col(x[[0, 19]], "f16", 3, 3, 1, 1)
    rows2 = np.array([0, 55, 56 * 56 - 1, 56 * 56, 2 * 56 * 56 - 1, 3000])
    ref = oracle.gemm_rows(A2, Wm, "f16", rows2)
    rows = np.where(rows2 < 3136, rows2, rows2 - 3136 + 19 * 3136)
    dx, dB = to_dev(x, "f16"), to_dev(np.ascontiguousarray(Wm.T), "f16")
    dC = torch.zeros((M, N), dtype=torch.float16, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV)
    wsb = B.abft_workspace_bytes(M, N, K, B.F16, B.GLOBAL)
    ws = torch.zeros(wsb, dtype=torch.uint8, device=DEV)
    conv = B.Conv(c.batch, c.H, c.W, c.Cin, c.KH, c.KW, c.stride, c.pad)
    for mode in (B.NONE, B.GLOBAL, B.THREAD):
        print(f"case big conv mode={mode}", flush=True)
        flag.zero_(); rep.zero_(); dC.zero_()
        B.abft_conv(conv, N, dx, dB, K, B.B_NK, dC, N, B.F16, mode, workspace=ws, workspace_bytes=wsb,
                    fault_flag=flag, report=rep)
        torch.cuda.synchronize()
        assert c_close(c_to_host(dC[rows.tolist()], "f16"), ref, "f16")
        assert int(flag.item()) == 0
        if mode != B.NONE:
            assert read_report(rep).worst_ratio < 0.5
