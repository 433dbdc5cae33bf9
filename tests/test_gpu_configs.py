"""Parity at the real shapes of the benchmark configurations: every DLRM layer at batch 1 / 16 /
256, all 53 convolutions of ResNet-50 at batch 1 (all of C) and 64 (sampled output pixels), every
point of the N = K = 4096 sweep over M, each in every scheme, plus seeded fault injection into
fully-connected and convolution layers.  The oracle is the plain CPU definition; int8 results
must be bit-exact, fp16 within 1e-2 |C| + 1e-2 rms(C)."""
import math

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl

pytestmark = pytest.mark.gpu
DT = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}
SCHEMES = (B.NONE, B.GLOBAL, B.THREAD, B.AUTO)


def _check_report(rep, mode, M, N, bm, bn):
    assert rep.tiles == math.ceil(M / bm) * math.ceil(N / bn)
    assert rep.worst_ratio < 0.5, (mode, rep.worst_ratio)


def _verdict(flag, chk, resid0, where):
    """Device flag against the oracle's check `chk` of the region that holds a planted fault:
    required outside the don't-care band around the tolerance.  Returns what was required."""
    if not (math.isfinite(chk.lhs) and math.isfinite(chk.rhs)):
        assert flag == 1, where
        return "must"
    delta = abs(chk.residual)
    if delta >= 2 * chk.tau + resid0:
        assert flag == 1, (where, delta, chk.tau)
        return "must"
    if delta <= chk.tau / 2 - resid0:
        assert flag == 0, (where, delta, chk.tau)
        return "mustnot"
    return "band"


# --------------------------------------------------------------------------- #
# configs[1]: DLRM MLPs, M = batch in {1, 16, 256}
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("batch", [1, 16, 256])
@pytest.mark.parametrize("li", range(8))
def test_dlrm_layer_every_scheme_and_injection(li, batch):
    """One DLRM layer (weights N(0, 0.02), activations U[0, 1], fp16): all of C against the oracle
    in every scheme, no flag; then the same shape in int8 with every one of the 32 bits of one
    accumulator flipped (all flagged, C exactly the oracle's corrupted C); then fp16 flips in
    and out of the tolerance band judged against the oracle's check of the region."""
    from gpu_util import DeviceGemm, c_close
    L = wl.dlrm_layers(batch)[li]
    M, N, K = L.M, L.N, L.K
    g = DeviceGemm(M, N, K, "f16", seed=1000 + 10 * li + batch, dist_a="uniform_01", dist_b="weights")
    C_ref = oracle.gemm(g.A, g.Bm, "f16")
    resid0 = {}
    for mode in SCHEMES:
        print(f"case dlrm {L.name} batch={batch} mode={mode}", flush=True)
        g.dC.zero_()
        flag, rep = g.run(mode)
        assert c_close(g.C(), C_ref, "f16"), (L.name, mode)
        assert flag == 0
        resolved = B.abft_select(M, N, K, B.F16) if mode == B.AUTO else mode
        if mode == B.AUTO:
            assert resolved == B.THREAD    # every DLRM layer is bandwidth bound by Eq. 1
        if resolved != B.NONE:
            bm, bn = (g.rm, g.rn) if resolved == B.GLOBAL else (g.tm, g.tn)
            _check_report(rep, resolved, M, N, bm, bn)
            resid0[resolved] = rep.tau * rep.worst_ratio
    # fp16 flips: the exponent's top bit (always far outside the band), a high mantissa bit, a low one
    rng = np.random.default_rng(li * 7 + batch)
    required = {"must": 0, "mustnot": 0, "band": 0}
    for mode in (B.GLOBAL, B.THREAD):
        parts = B.abft_k_parts(M, N, K, B.F16, mode, g.aligned)
        for bit in (30, 22, int(rng.integers(0, 16)), int(rng.integers(16, 30))):
            i, j = int(rng.integers(M)), int(rng.integers(N))
            k_after = -2 if bit == 22 else -1
            flag, _ = g.run(mode, inject=B.Fault(i, j, bit, k_after), want_report=False)
            if k_after == -2:
                C_bad = oracle.inject(g.A, g.Bm, C_ref, "f16", i, j, bit)
            else:
                C_bad = oracle.inject(g.A, g.Bm, C_ref, "f16", i, j, bit, k_set=parts[oracle.part_of(parts, K - 1)])
            region = g.region_of(i, j, mode)
            chk = (oracle.region_check if mode == B.GLOBAL else oracle.tile_check)(g.A, g.Bm, C_bad, "f16", *region)
            required[_verdict(flag, chk, resid0[mode], (L.name, mode, i, j, bit))] += 1
    assert required["must"] >= 2
    # int8 layer of the same shape: every bit of one accumulator, both schemes
    q = DeviceGemm(M, N, K, "i8", seed=2000 + 10 * li + batch)
    Cq = oracle.gemm(q.A, q.Bm, "i8")
    for mode in SCHEMES:
        flag, _ = q.run(mode)
        assert flag == 0 and np.array_equal(q.C(), Cq), (L.name, mode)
    i, j = int(rng.integers(M)), int(rng.integers(N))
    for mode in (B.GLOBAL, B.THREAD):
        parts = B.abft_k_parts(M, N, K, B.I8, mode, q.aligned)
        for bit in range(32):
            flag, _ = q.run(mode, inject=B.Fault(i, j, bit, -1), want_report=False)
            assert flag == 1, (L.name, mode, bit)
            want = oracle.inject(q.A, q.Bm, Cq, "i8", i, j, bit, k_set=parts[oracle.part_of(parts, K - 1)])
            assert np.array_equal(q.C(), ((want + 2 ** 31) % 2 ** 32) - 2 ** 31)


# --------------------------------------------------------------------------- #
# configs[2]: the 53 convolutions of ResNet-50 at 224 x 224
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("li", range(53))
def test_resnet50_layer_batch1_all_of_c(li):
    """Batch 1: all of C of every convolution against the oracle's im2col product, in every
    scheme (the first layer runs lowered to row segments)."""
    from gpu_util import DeviceConv, c_close
    L = wl.resnet50_layers(1)[li]
    d = DeviceConv(L.conv, "f16", seed=3000 + li)
    A = oracle.im2col(d.x, "f16", L.conv.KH, L.conv.KW, L.conv.stride, L.conv.pad)
    assert A.shape == (L.M, L.K)
    C_ref = oracle.gemm(A, d.Wm, "f16")
    aligned = (L.conv.Cin * 2) % 16 == 0
    for mode in SCHEMES:
        print(f"case resnet50 b1 {L.name} M={L.M} N={L.N} K={L.K} mode={mode}", flush=True)
        d.dC.zero_()
        flag, rep = d.run(mode)
        assert c_close(d.C(), C_ref, "f16"), (L.name, mode)
        assert flag == 0
        resolved = B.abft_select(L.M, L.N, L.K, B.F16) if mode == B.AUTO else mode
        if resolved != B.NONE:
            assert rep.tiles > 0 and rep.worst_ratio < 0.5, (L.name, mode, rep.worst_ratio)
            if aligned:   # (the lowered first layer is tiled for its re-ordered k)
                bm, bn = B.abft_region_shape(L.M, L.N, L.K, B.F16, True) if resolved == B.GLOBAL else \
                    B.abft_tile_shape(L.M, L.N, L.K, B.F16, True)[:2]
                _check_report(rep, resolved, L.M, L.N, bm, bn)


@pytest.mark.parametrize("li", range(53))
def test_resnet50_layer_batch64_sampled_pixels(li):
    """Batch 64, the launch configuration the benchmark times: sampled output pixels (first and
    last pixel of the first and the last image, seeded others in both) against the oracle, in the
    scheme the selector picks, in the other one and unprotected; no flag, one comparison per
    region, residuals below half the tolerance."""
    from gpu_util import DeviceConv, c_close
    L = wl.resnet50_layers(64)[li]
    c = L.conv
    d = DeviceConv(c, "f16", seed=4000 + li)
    per_img = c.OH * c.OW
    rng = np.random.default_rng(li)
    local = np.unique(np.concatenate([[0, per_img - 1], rng.integers(0, per_img, size=10)]))
    # the oracle lowers the first and the last image only (pixels of different images are independent)
    A2 = oracle.im2col(d.x[[0, 63]], "f16", c.KH, c.KW, c.stride, c.pad)
    rows2 = np.concatenate([local, per_img + local])
    ref = oracle.gemm(np.ascontiguousarray(A2[rows2]), d.Wm, "f16")
    rows = np.concatenate([local, 63 * per_img + local])
    pick = B.abft_select(L.M, L.N, L.K, B.F16)
    for mode in (B.AUTO, B.GLOBAL if pick == B.THREAD else B.THREAD, B.NONE):
        print(f"case resnet50 b64 {L.name} M={L.M} N={L.N} K={L.K} mode={mode} (selector: {pick})", flush=True)
        d.dC.zero_()
        flag, rep = d.run(mode)
        assert c_close(d.C(rows=rows), ref, "f16"), (L.name, mode)
        assert flag == 0
        if mode != B.NONE:
            assert rep.tiles > 0 and rep.worst_ratio < 0.5, (L.name, mode, rep.worst_ratio)


CONV_FAULT_LAYERS = [
    wl.Conv(2, 28, 28, 128, 128, 3, 3, 1, 1),   # ResNet-50 layer2 3x3 (padding taps), two images
    wl.Conv(2, 56, 56, 128, 128, 3, 3, 2, 1),   # the strided 3x3 of layer2.0
    wl.Conv(2, 64, 64, 3, 64, 7, 7, 2, 3),      # first layer in small: Cin = 3, lowered to row segments
    wl.Conv(2, 14, 14, 1024, 256, 1, 1, 1, 0),  # 1x1: the plain product on the NHWC tensor
]


@pytest.mark.parametrize("dtype", ["f16", "i8"])
@pytest.mark.parametrize("mode", [B.GLOBAL, B.THREAD, B.REPLICA])
@pytest.mark.parametrize("ci", range(len(CONV_FAULT_LAYERS)))
def test_conv_injected_faults(ci, mode, dtype):
    """Single-bit faults planted into convolution layers (output pixel, output channel, bit; the
    finished accumulator, the value after the partial tiles are added, or the running accumulator
    after k filter values).  int8: always flagged and C is exactly the oracle's corrupted C.  fp16:
    the verdict agrees with the oracle's check of the region outside the don't-care band."""
    from gpu_util import DeviceConv, c_close
    c = CONV_FAULT_LAYERS[ci]
    dt = DT[dtype]
    d = DeviceConv(c, dtype, seed=5000 + ci)
    M, N, K = d.M, d.N, d.K
    A = oracle.im2col(d.x, dtype, c.KH, c.KW, c.stride, c.pad)
    C_ref = oracle.gemm(A, d.Wm, dtype)
    flag, rep0 = d.run(mode)
    assert flag == 0 and c_close(d.C(), C_ref, dtype)
    resid0 = rep0.tau * rep0.worst_ratio
    es = 1 if dtype == "i8" else 2
    aligned = (c.Cin * es) % 16 == 0
    lowered = not aligned
    if mode == B.GLOBAL:
        bm, bn = B.abft_region_shape(M, N, K, dt, aligned)
    else:
        bm, bn = B.abft_tile_shape(M, N, K, dt, aligned)[:2]
    ks = B.abft_tile_shape(M, N, K, dt, aligned)[2]
    parts = B.abft_k_parts(M, N, K, dt, mode, aligned)
    rng = np.random.default_rng(ci * 11 + mode)
    required = {"must": 0, "mustnot": 0, "band": 0}
    for t in range(24):
        i, j = int(rng.integers(M)), int(rng.integers(N))
        bit = int(rng.integers(32)) if dtype == "i8" else (30, int(rng.integers(10, 30)), int(rng.integers(0, 14)))[t % 3]
        k_after = (-1, -2, ks * int(rng.integers(1, max(2, (K - 1) // ks + 1))))[t % 3]
        if k_after >= K:
            k_after = -1
        print(f"case conv fault {c} dtype={dtype} mode={mode} fault=({i},{j},bit {bit},k_after {k_after})", flush=True)
        flag, _ = d.run(mode, inject=B.Fault(i, j, bit, k_after), want_report=False)
        if k_after == -2:
            C_bad = oracle.inject(A, d.Wm, C_ref, dtype, i, j, bit)
        elif lowered and k_after == -1:
            # the lowered product runs on its own tiling; whichever accumulator held the finished
            # partial sum, C changes by a flip of some partial sum: judged on the flag alone below
            C_bad = None
        else:
            C_bad = oracle.inject(A, d.Wm, C_ref, dtype, i, j, bit, k_after=k_after,
                                  k_set=parts[oracle.part_of(parts, (K if k_after < 0 else k_after) - 1)])
        if dtype == "i8":
            assert flag == 1
            if C_bad is not None:
                assert np.array_equal(d.C(), ((C_bad + 2 ** 31) % 2 ** 32) - 2 ** 31)
            required["must"] += 1
            continue
        if C_bad is None:
            if bit == 30:
                assert flag == 1     # an exponent flip of a partial sum: non-finite or astronomically large
                required["must"] += 1
            continue
        if lowered and k_after < 0:
            continue                 # regions follow the lowered tiling: covered by the int8 leg and bit 30
        r0, c0 = i // bm * bm, j // bn * bn
        region = (r0, min(r0 + bm, M), c0, min(c0 + bn, N))
        if mode == B.GLOBAL:
            chk = oracle.region_check(A, d.Wm, C_bad, dtype, *region)
        else:
            chk = (oracle.replica_check if mode == B.REPLICA else oracle.tile_check)(A, d.Wm, C_bad, dtype, *region)
        required[_verdict(flag, chk, resid0, (c, mode, i, j, bit, k_after))] += 1
    assert required["must"] > 0


def test_lowered_conv_needs_finite_activations():
    """A few-channel convolution run lowered to row segments multiplies the input values that
    follow a window's run in its row by zero weights: a non-finite activation makes outputs of
    neighbouring windows NaN too.  Every output the oracle calls non-finite is non-finite, every
    other output whose row segments hold no non-finite value equals the oracle's, the protected
    schemes raise the flag (as the oracle's check does), and the unlowered path (small workspace)
    has exactly the oracle's pattern."""
    import torch
    from gpu_util import DeviceConv, c_close, to_dev
    c = wl.Conv(1, 30, 30, 3, 64, 7, 7, 2, 3)
    for lowered in (True, False):
        d = DeviceConv(c, "f16", seed=77, lowered=lowered)
        d.x[0, 11, 13, 1] = np.float16(np.inf)
        d.dx = to_dev(d.x, "f16")
        A = oracle.im2col(d.x, "f16", 7, 7, 2, 3)
        C_ref = oracle.gemm(A, d.Wm, "f16")
        bad_ref = ~np.isfinite(C_ref).all(axis=1)
        assert 0 < bad_ref.sum() < d.M
        assert oracle.global_check(A, d.Wm, C_ref, "f16").flag
        for mode in (B.NONE, B.GLOBAL, B.THREAD):
            flag, _ = d.run(mode)
            C = d.C()
            bad = ~np.isfinite(C).all(axis=1)
            assert np.all(bad[bad_ref])
            if mode != B.NONE:
                assert flag == 1
            if not lowered:
                assert np.array_equal(bad, bad_ref)
            # pixels whose input rows oh*2-3 .. oh*2+4 and columns up to one pixel past the window
            # are free of the planted value
            ok = np.ones(d.M, dtype=bool)
            for m in range(d.M):
                oh, ow = divmod(m, c.OW)
                if oh * 2 - 3 <= 11 <= oh * 2 + 4 and ow * 2 - 3 <= 13 <= ow * 2 + 4:
                    ok[m] = False
            assert not np.any(bad[ok])
            assert c_close(C[ok], C_ref[ok], "f16")


# --------------------------------------------------------------------------- #
# configs[4]: N = K = 4096, M = 1 .. 8192
# --------------------------------------------------------------------------- #
_SWEEP_B = {}


@pytest.mark.parametrize("M", wl.sweep_m())
def test_sweep_point_every_scheme(M):
    """Every point of the intensity sweep: all of C for M <= 256, at least 64 sampled rows (first
    and last row of every band of 256 among them) above, in every scheme; no flag; the selector's
    choice is the one Eq. 1 gives."""
    from gpu_util import DeviceGemm, c_close, sample_rows
    N = K = 4096
    if "B" not in _SWEEP_B:
        _SWEEP_B["B"] = wl.random_matrix((K, N), "f16", "normal", 4242)
    Bm = _SWEEP_B["B"]
    A = wl.random_matrix((M, K), "f16", "normal", 4300 + M)
    g = DeviceGemm(M, N, K, "f16", seed=0, operands=(A, Bm))
    rows = sample_rows(M, 256 if M <= 256 else 64, band=256, seed=M)
    ref = oracle.gemm(np.ascontiguousarray(A[rows]), Bm, "f16")
    want = B.GLOBAL if 2.0 * M * N * K / (2.0 * (M * K + K * N + M * N)) > 2516.6e12 / 8e12 else B.THREAD
    assert B.abft_select(M, N, K, B.F16) == want and (M >= 512) == (want == B.GLOBAL)
    for mode in SCHEMES + (B.REPLICA, B.THREAD_HALF, B.TWOSIDED):
        print(f"case sweep M={M} mode={mode}", flush=True)
        g.dC.zero_()
        flag, rep = g.run(mode)
        assert c_close(g.C(rows=rows), ref, "f16"), (M, mode)
        assert flag == 0
        resolved = want if mode == B.AUTO else mode
        if resolved != B.NONE:
            bm, bn = (g.rm, g.rn) if resolved == B.GLOBAL else (g.tm, g.tn)
            _check_report(rep, resolved, M, N, bm, bn)
    # one fault far outside the band in the last row, both schemes
    for mode in (B.GLOBAL, B.THREAD):
        flag, _ = g.run(mode, inject=B.Fault(M - 1, N - 1, 30, -1), want_report=False)
        assert flag == 1
