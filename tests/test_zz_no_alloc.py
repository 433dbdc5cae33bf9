"""The entry point that allocates nothing (abft_gemm_static): its scratch is an array inside the
library.  Two calls in a row, the second on a smaller input, against abft_gemm with a caller's
workspace on the same operands: C bit for bit, the same flag, the same reported sides."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl

pytestmark = pytest.mark.gpu

# first call, then a smaller one; shapes that take the scratch for the weight checksums (no beta
# given), for partial checksum dot products (unaligned K: the activation-checksum pass) or both
SEQUENCES = [
    [(1024, 1536, 1024), (200, 136, 264)],
    [(300, 520, 333), (130, 70, 77)],
    [(4096, 4096, 512), (64, 64, 64)],
]


def _both(M, N, K, dtype, mode, seed, inject=None):
    import torch
    from gpu_util import to_dev, read_report, c_to_host, DEV, DT
    dt = DT[dtype]
    A, Bm = wl.gemm_operands(M, N, K, dtype, seed=seed)
    dA, dB = to_dev(A, dtype), to_dev(np.ascontiguousarray(Bm.T), dtype)
    c_t = torch.int32 if dtype == "i8" else torch.float16
    out = []
    for static in (False, True):
        dC = torch.zeros((M, N), dtype=c_t, device=DEV)
        flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device=DEV)
        if static:
            B.abft_gemm_static(M, N, K, dA, K, dB, K, B.B_NK, dC, N, dt, mode, fault_flag=flag, report=rep,
                               inject=inject)
        else:
            wsb = B.abft_workspace_bytes(M, N, K, dt, mode)
            ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=DEV)
            B.abft_gemm(M, N, K, dA, K, dB, K, B.B_NK, dC, N, dt, mode, workspace=ws, workspace_bytes=wsb,
                        fault_flag=flag, report=rep, inject=inject)
        torch.cuda.synchronize()
        out.append((dC.clone(), int(flag.item()), read_report(rep)))
    return A, Bm, out


@pytest.mark.parametrize("dtype", ["f16", "i8"])
@pytest.mark.parametrize("mode", [B.GLOBAL, B.THREAD, B.NONE])
@pytest.mark.parametrize("si", range(len(SEQUENCES)))
def test_static_scratch_entry_point_matches_abft_gemm(si, mode, dtype):
    import torch
    from gpu_util import c_to_host, c_close
    assert B.abft_static_scratch_bytes() == 8 << 20
    for n, (M, N, K) in enumerate(SEQUENCES[si]):
        print(f"case static seq={si} call={n} shape={(M, N, K)} mode={mode} dtype={dtype}", flush=True)
        A, Bm, ((C0, f0, r0), (C1, f1, r1)) = _both(M, N, K, dtype, mode, seed=600 + si)
        assert torch.equal(C0, C1)
        assert f0 == 0 and f1 == 0
        assert (r0.lhs, r0.rhs, r0.tau, r0.tiles, r0.region) == (r1.lhs, r1.rhs, r1.tau, r1.tiles, r1.region)
        assert c_close(c_to_host(C1, dtype), oracle.gemm(A, Bm, dtype), dtype)
        if mode != B.NONE:
            # a planted fault is seen through the library's own scratch as well
            _, _, ((_, g0, _), (_, g1, _)) = _both(M, N, K, dtype, mode, seed=600 + si,
                                                   inject=B.Fault(M - 1, N - 1, 30, -1))
            assert g0 == 1 and g1 == 1


def test_static_scratch_rejects_what_does_not_fit():
    """A product whose scratch exceeds the array comes back as a workspace error; nothing runs."""
    import torch
    from gpu_util import DEV
    t = torch.zeros(64, dtype=torch.float16, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    n = 32768
    with pytest.raises(B.AbftError) as e:
        B.abft_gemm_static(n, n, n, t, n, t, n, B.B_NK, t, n, B.F16, B.GLOBAL, fault_flag=flag)
    assert e.value.code == -5
    assert int(flag.item()) == 0
