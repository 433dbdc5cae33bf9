"""Chains of mid-size layers run layer by layer (abft_plan_run_chain) with the activation
checksums of a layer under the global scheme handed over by the epilogue of the layer before it
(Sec. 2.4 step 4): every layer against the oracle on the input it read, the device's comparison
of its worst region against the oracle's check of that region, the same results as the layers run
one by one, seeded single-bit faults in a layer that takes handed-over checksums and in one
that hands them over, and chains in which only some pairs of layers qualify."""
import ctypes
import math

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl
from test_gpu_chain import Chain, _storage, DT

pytestmark = pytest.mark.gpu

# every layer on the direct-to-LDS kernel; layers 1 (128 x 128 tiles, two workgroups per compute unit)
# and 2 (256 x 256 tiles) take handed-over sums, the last one (narrow: one round of 128 x 128 tiles on
# eight wavefronts each) forms its own in the loop
WIDTHS = [512, 1024, 1024, 2048, 512]
M_MID = 8192


def _reports(ch):
    import torch
    from gpu_util import DEV
    reps = [torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV) for _ in range(ch.nl)]
    for l, r in enumerate(reps):
        B.abft_plan_set_diagnostics(ch.plan, l, report=r)
    return reps


def _region(ch, l, a_in, region):
    """Row / column block of layer l's comparison region `region` (1-based, row-major) and the
    oracle's check of it, on the input a_in the device's layer read."""
    K, N = ch.widths[l], ch.widths[l + 1]
    bm, bn = B.abft_region_shape(ch.M, N, K, DT[ch.dtype], True)
    per_row = -(-N // bn)
    r0, c0 = (region - 1) // per_row * bm, (region - 1) % per_row * bn
    Ab, Bb = a_in[r0:r0 + bm], np.ascontiguousarray(ch.Ws[l][:, c0:c0 + bn])
    Cb = oracle.gemm(Ab, Bb, ch.dtype)
    return (r0, c0, bm, bn), oracle.region_check(Ab, Bb, Cb, ch.dtype, 0, Cb.shape[0], 0, Cb.shape[1]), Cb


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_handed_over_checksums_agree_with_the_oracle_and_with_layers_run_alone(dtype):
    import torch
    from gpu_util import read_report
    ch = Chain(M_MID, WIDTHS, dtype, seed=1200, modes=[B.GLOBAL] * 4)
    try:
        reps = _reports(ch)
        x, dx = ch.input(seed=1201)
        before = B.abft_handover_launches()
        print(f"case handover chain M={M_MID} widths={WIDTHS} dtype={dtype}", flush=True)
        ch.run(dx)
        torch.cuda.synchronize()
        # layers 1 and 2 read the output of a layer on the direct-to-LDS kernel and run on it themselves
        assert B.abft_handover_launches() - before == 2
        assert int(ch.flag.item()) == 0
        ch.check(x)
        chained = [c.clone() for c in ch.Cs]
        got = [read_report(r) for r in reps]
        a_in = x
        for l in range(ch.nl):
            K, N = ch.widths[l], ch.widths[l + 1]
            bm, bn = B.abft_region_shape(ch.M, N, K, DT[dtype], True)
            assert got[l].tiles == -(-ch.M // bm) * -(-N // bn), l
            _, ref, _ = _region(ch, l, a_in, got[l].region)
            assert not ref.flag
            assert abs(got[l].lhs - ref.lhs) <= ref.tau, l
            assert abs(got[l].rhs - ref.rhs) <= 0.1 * ref.tau, l
            assert got[l].tau == pytest.approx(ref.tau, rel=1e-3)
            assert got[l].worst_ratio < 0.5, (l, got[l].worst_ratio)
            a_in = _storage(ch.Cs[l], dtype)
        # the layers one by one form their activation checksums themselves: same C, bit for bit
        for r in reps:
            r.zero_()
        for l in range(ch.nl):
            a = dx if l == 0 else ch.Cs[l - 1]
            B.abft_plan_run(ch.plan, l, a, ch.widths[l], ch.Cs[l], ch.widths[l + 1], ch.flag)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 2
        assert int(ch.flag.item()) == 0
        for l in range(ch.nl):
            assert torch.equal(ch.Cs[l], chained[l]), l
            alone = read_report(reps[l])
            assert alone.tiles == got[l].tiles
            # (the worst region may differ between the two forms of the right-hand side; the tolerance may not)
            if alone.region == got[l].region:
                assert alone.lhs == got[l].lhs
                assert abs(alone.rhs - got[l].rhs) <= 0.1 * alone.tau
    finally:
        ch.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("layer", [1, 2])
def test_seeded_faults_in_a_chain_with_handed_over_checksums(dtype, layer):
    """Layer 1 takes checksums and hands some over, layer 2 only takes them.  Single-bit flips in
    finished accumulators of the layer: the verdict equals the oracle's incremental evaluation
    outside the don't-care band around the region's tolerance; the other layers stay silent."""
    import torch
    from gpu_util import read_report
    ch = Chain(M_MID, WIDTHS, dtype, seed=1300, modes=[B.GLOBAL] * 4)
    try:
        reps = _reports(ch)
        x, dx = ch.input(seed=1301)
        ch.run(dx)
        torch.cuda.synchronize()
        assert int(ch.flag.item()) == 0
        clean = read_report(reps[layer])
        resid0 = clean.tau * clean.worst_ratio
        a_in = _storage(ch.Cs[layer - 1], dtype)           # what the layer reads (a clean run's)
        K, N = ch.widths[layer], ch.widths[layer + 1]
        bm, bn = B.abft_region_shape(ch.M, N, K, DT[dtype], True)
        rng = np.random.default_rng(1302 + layer)
        blocks = {}
        must = mustnot = band = 0
        for t in range(48):
            i, j = int(rng.integers(ch.M)), int(rng.integers(N))
            bit = int(rng.integers(32)) if t % 3 else int(rng.integers(24, 31))
            print(f"case handover fault layer={layer} dtype={dtype} t={t} ({i},{j}) bit {bit}", flush=True)
            for r in reps:
                r.zero_()
            ch.flag.zero_()
            B.abft_plan_set_diagnostics(ch.plan, layer, report=reps[layer], inject=B.Fault(i, j, bit, -1))
            ch.run(dx)
            torch.cuda.synchronize()
            flag = int(ch.flag.item())
            others = [read_report(reps[l]).worst_ratio for l in range(ch.nl) if l != layer]
            a_row, b_col = a_in[i:i + 1], np.ascontiguousarray(ch.Ws[layer][:, j:j + 1])
            good = oracle.partial_dot(a_row, b_col, dtype, 0, 0, 0, K)
            bad = oracle.flip_bit(good, bit, dtype)
            if not math.isfinite(bad):
                assert flag == 1
                must += 1
                continue
            # (a corrupted output changes what the later layers read, consistently for both of
            # their sides: they stay silent unless it overflows there)
            if abs(bad) < 6e4:
                assert max(others) < 1.0, others
            r0, c0 = i // bm * bm, j // bn * bn
            if (r0, c0) not in blocks:
                blk = oracle.gemm(a_in[r0:r0 + bm], np.ascontiguousarray(ch.Ws[layer][:, c0:c0 + bn]), dtype)
                blocks[(r0, c0)] = (blk, oracle.frob(blk) ** 2, oracle.l1norm(blk))
            blk, f2, l1 = blocks[(r0, c0)]
            cl = float(blk[i - r0, j - c0])
            delta = abs(bad - good)
            tau = oracle.tolerance(K, math.sqrt(max(f2 - cl * cl + bad * bad, 0.0)), dtype, scheme=1,
                                   l1_norm=l1 - abs(cl) + abs(bad))
            if delta >= 2 * tau + resid0:
                assert flag == 1, (i, j, bit, delta, tau)
                must += 1
            elif delta <= tau / 2 - resid0:
                assert flag == 0, (i, j, bit, delta, tau)
                mustnot += 1
            else:
                band += 1
        print(f"handover faults layer {layer} {dtype}: {must} flagged, {mustnot} silent, {band} in the band", flush=True)
        assert must > 0 and mustnot > 0
    finally:
        B.abft_plan_set_diagnostics(ch.plan, layer)
        ch.close()


@pytest.mark.parametrize("modes,expect", [
    ([B.GLOBAL, B.THREAD, B.GLOBAL, B.GLOBAL], 1),   # layer 1 under another scheme still hands over to layer 2
    ([B.NONE, B.GLOBAL, B.NONE, B.GLOBAL], 1),       # an unprotected layer hands over; the streamed last layer takes none
    ([B.THREAD, B.THREAD, B.THREAD, B.THREAD], 0),
])
def test_chains_in_which_only_some_layers_qualify(modes, expect):
    import torch
    ch = Chain(M_MID, WIDTHS, "f16", seed=1400, modes=modes)
    try:
        x, dx = ch.input(seed=1401)
        before = B.abft_handover_launches()
        ch.run(dx)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == expect
        assert int(ch.flag.item()) == 0
        ch.check(x)
    finally:
        ch.close()


def test_ragged_batch_and_widths():
    """M not a multiple of 32, N not a multiple of the tile: the last row block's checksums cover
    the rows that exist, columns past N are never written."""
    import torch
    ch = Chain(6001, [512, 960, 1024, 640], "f16", seed=1500, modes=[B.GLOBAL] * 3)
    try:
        x, dx = ch.input(seed=1501)
        before = B.abft_handover_launches()
        ch.run(dx)
        torch.cuda.synchronize()
        assert int(ch.flag.item()) == 0
        ch.check(x)
        assert B.abft_handover_launches() - before >= 1
    finally:
        ch.close()


def test_handover_chain_under_graph_replay():
    """The second stream's comparison kernels are captured with the chain (fork after each product,
    join at the end of the call): every replay gives the eager outputs and a clean flag, and with a
    fault planted in a layer that takes handed-over checksums every replay raises the flag."""
    import torch
    ch = Chain(M_MID, WIDTHS, "f16", seed=1600, modes=[B.GLOBAL] * 4)
    try:
        x, dx = ch.input(seed=1601)
        ch.run(dx)
        torch.cuda.synchronize()
        assert int(ch.flag.item()) == 0
        eager = [c.clone() for c in ch.Cs]
        for planted in (False, True):
            if planted:
                B.abft_plan_set_diagnostics(ch.plan, 2, inject=B.Fault(100, 200, 29, -1))
            cap = torch.cuda.Stream()
            cap.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=cap):
                ch.run(dx, cap)
            for rep in range(3):
                for c in ch.Cs:
                    c.zero_()               # eager work between replays
                ch.flag.zero_()
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                print(f"case handover graph planted={planted} replay={rep}", flush=True)
                assert int(ch.flag.item()) == (1 if planted else 0), (planted, rep)
                if not planted:
                    for c, e in zip(ch.Cs, eager):
                        assert torch.equal(c, e), rep
    finally:
        B.abft_plan_set_diagnostics(ch.plan, 2)
        ch.close()


def test_bottleneck_pair_a_3x3_convolution_hands_over_to_a_1x1_convolution():
    """ResNet-50's conv2 -> conv3 of a bottleneck at 56 x 56, batch 16: the 3 x 3 convolution's epilogue
    leaves the column sums of its (ReLU) output, the 1 x 1 convolution behind it reads that output as a
    plain M x K matrix and takes them.  Outputs against the oracle (the second layer on the input it
    read), clean flag, the reported region against the oracle's check of it."""
    import torch
    from gpu_util import to_dev, c_to_host, c_close, read_report, DEV
    c2 = wl.Conv(16, 56, 56, 64, 64, 3, 3, 1, 1)
    c3 = wl.Conv(16, 56, 56, 64, 256, 1, 1, 1, 0)
    x, W2 = wl.conv_operands(c2, "f16", seed=1700)
    _, W3 = wl.conv_operands(c3, "f16", seed=1701)
    M, K2, K3 = 16 * 56 * 56, 9 * 64, 64
    dx = to_dev(x, "f16")
    dW2, dW3 = to_dev(np.ascontiguousarray(W2.T), "f16"), to_dev(np.ascontiguousarray(W3.T), "f16")
    layers = [B.Layer(M, 64, K2, B.F16, B.B_NK, 1, B.Conv(16, 56, 56, 64, 3, 3, 1, 1), dW2.data_ptr(), K2),
              B.Layer(M, 256, K3, B.F16, B.B_NK, 1, B.Conv(16, 56, 56, 64, 1, 1, 1, 0), dW3.data_ptr(), K3)]
    plan = B.abft_plan_create(layers)
    try:
        for l in range(2):
            B.abft_plan_set_mode(plan, l, B.GLOBAL)
        B.abft_plan_set_activation(plan, 0, B.ACT_RELU)
        Cs = [torch.zeros((M, 64), dtype=torch.float16, device=DEV), torch.zeros((M, 256), dtype=torch.float16, device=DEV)]
        flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV)
        B.abft_plan_set_diagnostics(plan, 1, report=rep)
        before = B.abft_handover_launches()
        print("case handover conv3x3 -> conv1x1", flush=True)
        B.abft_plan_run_chain(plan, 0, 2, dx, K2, Cs, [64, 256], flag)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 1
        assert int(flag.item()) == 0
        rows = np.arange(0, M, 97)
        A2 = oracle.im2col(x, "f16", 3, 3, 1, 1)
        ref2 = oracle.activation(oracle.gemm(A2[rows], W2, "f16"), "relu")
        assert c_close(c_to_host(Cs[0], "f16")[rows], ref2, "f16")
        a3 = Cs[0].cpu().numpy()                                   # what the second layer read
        assert c_close(c_to_host(Cs[1], "f16")[rows], oracle.gemm(a3[rows], W3, "f16"), "f16")
        got = read_report(rep)
        bm, bn = B.abft_region_shape(M, 256, K3, B.F16, True)
        per_row = -(-256 // bn)
        assert got.tiles == -(-M // bm) * per_row
        r0, c0 = (got.region - 1) // per_row * bm, (got.region - 1) % per_row * bn
        Ab, Bb = a3[r0:r0 + bm], np.ascontiguousarray(W3[:, c0:c0 + bn])
        Cb = oracle.gemm(Ab, Bb, "f16")
        ref = oracle.region_check(Ab, Bb, Cb, "f16", 0, Cb.shape[0], 0, Cb.shape[1])
        assert not ref.flag
        assert abs(got.lhs - ref.lhs) <= ref.tau and abs(got.rhs - ref.rhs) <= 0.1 * ref.tau
        assert got.worst_ratio < 0.5
    finally:
        B.abft_plan_destroy(plan)


def test_run_all_chains_layers_by_their_buffers():
    """abft_plan_run_all with layer l's output passed as layer l + 1's input hands the checksums
    over like abft_plan_run_chain; with inputs of their own the layers run independently."""
    import torch
    from gpu_util import to_dev
    ch = Chain(M_MID, WIDTHS, "f16", seed=1800, modes=[B.GLOBAL] * 4)
    try:
        x, dx = ch.input(seed=1801)
        io = B.PlanIO([dx] + ch.Cs[:-1], list(ch.widths[:-1]), ch.Cs, list(ch.widths[1:]))
        before = B.abft_handover_launches()
        B.abft_plan_run_all(ch.plan, io, ch.flag, -1)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 2
        assert int(ch.flag.item()) == 0
        ch.check(x)
        # the same layers on copies of their inputs: no pair is chained
        ins = [dx] + [c.clone() for c in ch.Cs[:-1]]
        io2 = B.PlanIO(ins, list(ch.widths[:-1]), ch.Cs, list(ch.widths[1:]))
        before = B.abft_handover_launches()
        B.abft_plan_run_all(ch.plan, io2, ch.flag, -1)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 0
        assert int(ch.flag.item()) == 0
        ch.check(x)
    finally:
        ch.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M,region", [(4096, (256, 256)), (2048, (256, 128))])
def test_handover_between_layers_on_the_256x256_tile(dtype, M, region):
    """Two M x 4096 x 4096 layers: 256 workgroup tiles each, of 256 x 256 (M = 4096) or 256 x 128
    (M = 2048): the tiles whose accumulators have the 16 x 16 layout.  Layer 0's epilogue forms the
    column sums from that layout, layer 1 takes them.  Sampled rows of both layers against the oracle on the input the device's
    layer read, the device's worst region against the oracle's check of that region, the same C bit
    for bit as the layers run one by one, and a seeded fault in the layer that takes the sums."""
    import torch
    from gpu_util import read_report, c_to_host, c_close, sample_rows
    widths = [4096, 4096, 4096]
    ch = Chain(M, widths, dtype, seed=1900, modes=[B.GLOBAL] * 2)
    try:
        reps = _reports(ch)
        x, dx = ch.input(seed=1901)
        before = B.abft_handover_launches()
        print(f"case handover on 256x256 tiles M={M} widths={widths} dtype={dtype}", flush=True)
        ch.run(dx)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 1
        assert int(ch.flag.item()) == 0
        chained = [c.clone() for c in ch.Cs]
        got = [read_report(r) for r in reps]
        rows = sample_rows(M, 24, band=256, seed=1902)
        a_in = x
        for l in range(ch.nl):
            K, N = widths[l], widths[l + 1]
            bm, bn = B.abft_region_shape(M, N, K, DT[dtype], True)
            assert (bm, bn) == region
            ref = oracle.activation(oracle.gemm_rows(a_in, ch.Ws[l], dtype, rows), ch.acts[l])
            assert c_close(c_to_host(ch.Cs[l], dtype)[rows], ref, dtype), l
            assert got[l].tiles == (M // bm) * (N // bn), l
            _, chk, _ = _region(ch, l, a_in, got[l].region)
            assert not chk.flag
            assert abs(got[l].lhs - chk.lhs) <= chk.tau, l
            assert abs(got[l].rhs - chk.rhs) <= 0.1 * chk.tau, l
            assert got[l].tau == pytest.approx(chk.tau, rel=1e-3)
            assert got[l].worst_ratio < 0.5, (l, got[l].worst_ratio)
            a_in = _storage(ch.Cs[l], dtype)
        # one by one: each layer forms its activation checksums itself
        for r in reps:
            r.zero_()
        for l in range(ch.nl):
            a = dx if l == 0 else ch.Cs[l - 1]
            B.abft_plan_run(ch.plan, l, a, widths[l], ch.Cs[l], widths[l + 1], ch.flag)
        torch.cuda.synchronize()
        assert B.abft_handover_launches() - before == 1
        assert int(ch.flag.item()) == 0
        for l in range(ch.nl):
            assert torch.equal(ch.Cs[l], chained[l]), l
        # single-bit flips in finished accumulators of layer 1: the verdict equals the oracle's
        # outside the don't-care band around the region's tolerance
        clean = got[1]
        resid0 = clean.tau * clean.worst_ratio
        a1 = _storage(chained[0], dtype)
        K, N = widths[1], widths[2]
        must = mustnot = 0
        for t, (i, j, bit) in enumerate(((1234, 2345, 30), (17, 4000, 28), (M - 1, 0, 30), (M // 2, 255, 2), (300, 3000, 5), (777, 1777, 26))):
            print(f"case handover fault on 256x256 tiles dtype={dtype} ({i},{j}) bit {bit}", flush=True)
            ch.flag.zero_()
            B.abft_plan_set_diagnostics(ch.plan, 1, report=reps[1], inject=B.Fault(i, j, bit, -1))
            ch.run(dx)
            torch.cuda.synchronize()
            flag = int(ch.flag.item())
            good = oracle.partial_dot(a1[i:i + 1], np.ascontiguousarray(ch.Ws[1][:, j:j + 1]), dtype, 0, 0, 0, K)
            bad = oracle.flip_bit(good, bit, dtype)
            if not math.isfinite(bad):
                assert flag == 1
                must += 1
                continue
            r0, c0 = i // region[0] * region[0], j // region[1] * region[1]
            blk = oracle.gemm(a1[r0:r0 + region[0]], np.ascontiguousarray(ch.Ws[1][:, c0:c0 + region[1]]), dtype)
            cl = float(blk[i - r0, j - c0])
            tau = oracle.tolerance(K, math.sqrt(max(oracle.frob(blk) ** 2 - cl * cl + bad * bad, 0.0)), dtype, scheme=1,
                                   l1_norm=oracle.l1norm(blk) - abs(cl) + abs(bad))
            delta = abs(bad - good)
            if delta >= 2 * tau + resid0:
                assert flag == 1, (i, j, bit, delta, tau)
                must += 1
            elif delta <= tau / 2 - resid0:
                assert flag == 0, (i, j, bit, delta, tau)
                mustnot += 1
        assert must > 0 and mustnot > 0
    finally:
        B.abft_plan_set_diagnostics(ch.plan, 1)
        ch.close()
