"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host logic (selector, intensity, argument validation) behaves.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2104_09455_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2104_09455_amd.build import build
        build()
    return B.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "abft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(abft_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 24
    for n in names:
        assert hasattr(lib, n), f"{n} declared in abft.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_version_and_strerror(lib):
    assert B.abft_version() >= 100
    assert B.abft_strerror(0) == "ok"
    for code in range(-8, 0):
        assert "unknown error code" not in B.abft_strerror(code)
    assert "unknown error code" in B.abft_strerror(-99)


def test_intensity_and_cmr(lib):
    for n in (32, 64, 2048):
        assert B.abft_arithmetic_intensity(n, n, n, B.F16) == pytest.approx(n / 3)
    # int8: 1-byte inputs, 4-byte outputs
    assert B.abft_arithmetic_intensity(2, 3, 5, B.I8) == pytest.approx(60 / (10 + 15 + 24))
    assert B.abft_cmr(B.F16) == pytest.approx(2516.6e12 / 8e12)
    assert B.abft_cmr(B.BF16) == B.abft_cmr(B.F16)
    assert B.abft_cmr(B.I8) == pytest.approx(5033.2e12 / 8e12)
    assert B.abft_arithmetic_intensity(0, 1, 1, B.F16) == 0.0


def test_selector_rule(lib):
    assert B.abft_select(8192, 8192, 8192, B.F16) == B.GLOBAL
    assert B.abft_select(4096, 4096, 4096, B.BF16) == B.GLOBAL
    assert B.abft_select(8192, 8192, 8192, B.I8) == B.GLOBAL
    assert B.abft_select(1, 1024, 1024, B.F16) == B.THREAD
    assert B.abft_select(256, 4096, 4096, B.F16) == B.THREAD
    assert B.abft_select(512, 4096, 4096, B.F16) == B.GLOBAL
    # strict inequality: intensity == CMR is not compute bound
    B.abft_set_cmr(B.F16, 200.0)
    try:
        assert B.abft_select(600, 600, 600, B.F16) == B.THREAD
        B.abft_set_cmr(B.F16, 199.9)
        assert B.abft_select(600, 600, 600, B.F16) == B.GLOBAL
    finally:
        B.abft_set_cmr(B.F16, 0.0)
    assert B.abft_cmr(B.F16) == pytest.approx(314.575)
    with pytest.raises(B.AbftError):
        B.abft_select(0, 1, 1, B.F16)
    with pytest.raises(B.AbftError):
        B.abft_select(1, 1, 1, 7)


def test_tile_shape_and_tolerance(lib):
    tm, tn, ks = B.abft_tile_shape(8192, 8192, 8192, B.F16)
    assert tm > 0 and tn > 0 and ks > 0 and 8192 % ks == 0
    tm1, tn1, _ = B.abft_tile_shape(1, 1024, 1024, B.F16)
    assert tm1 == 32  # aligned skinny product: the streaming tile
    tm2, tn2, _ = B.abft_tile_shape(1, 1024, 1021, B.F16, False)
    assert tm2 == 16  # unaligned skinny product: the generic 16-row tile
    _, _, ks8 = B.abft_tile_shape(64, 64, 64, B.I8)
    _, _, ks16 = B.abft_tile_shape(64, 64, 64, B.F16)
    assert ks8 == 2 * ks16  # the k tile is fixed in bytes
    c = B.abft_tolerance_coeff(64, B.F16, B.GLOBAL)
    assert c == pytest.approx(8 * 2.0 ** -24 * 8)
    assert B.abft_tolerance_coeff(64, B.F16, B.THREAD) == pytest.approx(8 * (2.0 ** -24 * 8 + 2.0 ** -22))
    assert B.abft_tolerance_coeff(64, B.BF16, B.THREAD) == pytest.approx(8 * (2.0 ** -24 * 8 + 2.0 ** -23))
    assert B.abft_tolerance_coeff(64, B.I8, B.GLOBAL) == 0.0
    assert B.abft_tolerance_bias_coeff(64, B.F16, B.GLOBAL) == pytest.approx(1e-3 * 2.0 ** -24 * 64)
    assert B.abft_tolerance_bias_coeff(64, B.F16, B.THREAD) == 0.0
    assert B.abft_tolerance_bias_coeff(64, B.I8, B.GLOBAL) == 0.0
    rm, rn = B.abft_region_shape(8192, 8192, 8192, B.F16)
    assert rm % tm == 0 and rn % tn == 0  # wavefront tiles nest inside workgroup tiles


def test_workspace_sizes(lib):
    assert B.abft_workspace_bytes(64, 64, 64, B.F16, B.NONE) == 0
    assert B.abft_workspace_bytes(64, 64, 64, B.F16, B.THREAD) == 0
    w = B.abft_workspace_bytes(64, 64, 64, B.F16, B.GLOBAL)
    assert w > 0 and w % 256 == 0
    assert B.abft_workspace_bytes(8192, 8192, 8192, B.F16, B.AUTO) == B.abft_workspace_bytes(
        8192, 8192, 8192, B.F16, B.GLOBAL)
    assert B.abft_workspace_bytes(1, 64, 64, B.F16, B.AUTO) == 0


def test_argument_validation_without_a_gpu(lib):
    """Bad arguments are rejected on the host before anything touches the device."""
    p = 0x1000  # never dereferenced: validation fails first
    g = lambda **kw: lib.abft_gemm(kw.get("M", 4), kw.get("N", 4), kw.get("K", 4), kw.get("A", p),
                                   kw.get("lda", 4), kw.get("B", p), kw.get("ldb", 4), kw.get("layout", 0),
                                   kw.get("C", p), kw.get("ldc", 4), kw.get("dtype", 0), kw.get("mode", 0),
                                   None, None, 0, kw.get("flag", p), None, None, None)
    assert g(M=0) == -2 and g(N=-1) == -2 and g(K=0) == -2
    assert g(A=None) == -1 and g(B=None) == -1 and g(C=None) == -1
    assert g(lda=3) == -3 and g(ldb=3) == -3 and g(ldc=3) == -3
    assert g(dtype=3) == -4 and g(mode=8) == -4 and g(mode=-1) == -4 and g(layout=2) == -4
    assert g(mode=1, flag=None) == -1
    assert g(mode=1) == -5  # global needs a workspace
    with pytest.raises(B.AbftError) as e:
        B.abft_plan_mode(None, 0)
    assert e.value.code == -8
    # plan calls without a plan
    assert lib.abft_plan_set_diagnostics(None, 0, None, None) == -8
    assert lib.abft_plan_run_chain(None, 0, 1, p, 4, None, None, p, None) == -8
    assert lib.abft_handover_launches() == 0   # nothing has run in this process
    # the measurement aid checks its arguments before it touches the device
    ops = ctypes.c_double(0.0)
    assert lib.abft_mfma_probe(24, 0, 10, p, p, ctypes.byref(ops), None) == -4
    assert lib.abft_mfma_probe(16, 3, 10, p, p, ctypes.byref(ops), None) == -4
    assert lib.abft_mfma_probe(16, 0, 10, None, p, ctypes.byref(ops), None) == -1
    assert lib.abft_mfma_probe(32, 0, 0, p, p, ctypes.byref(ops), None) == -2
    assert lib.abft_mfma_probe_bytes() % (512 * 256) == 0
    bad = B.Conv(1, 2, 2, 8, 3, 3, 1, 0)  # 3x3 filter on a 2x2 image without padding
    assert lib.abft_conv(ctypes.byref(bad), 4, p, p, 72, 0, p, 4, 0, 0, None, None, 0, p, None, None, None) == -2


def test_replication_mode_shares_the_thread_level_geometry(lib):
    """ABFT_REPLICA is checked per wavefront tile like ABFT_THREAD: same workspace, k partition
    and tolerance coefficient for every shape class the dispatcher knows."""
    for (M, N, K) in [(64, 64, 64), (256, 1024, 1024), (200, 136, 256), (1536, 1536, 128), (8192, 8192, 8192),
                      (1, 1024, 1021), (64, 1024, 4096)]:
        for dt in (B.F16, B.BF16, B.I8):
            al = (K * (1 if dt == B.I8 else 2)) % 16 == 0
            assert B.abft_workspace_bytes(M, N, K, dt, B.REPLICA) == B.abft_workspace_bytes(M, N, K, dt, B.THREAD)
            assert B.abft_k_ways(M, N, K, dt, B.REPLICA, al) == B.abft_k_ways(M, N, K, dt, B.THREAD, al)
            assert B.abft_tolerance_coeff(K, dt, B.REPLICA) == B.abft_tolerance_coeff(K, dt, B.THREAD)
            assert B.abft_tolerance_bias_coeff(K, dt, B.REPLICA) == 0.0
    assert B.MODE_NAMES[B.REPLICA] == "replica"


def test_operand_type_checksum_schemes_share_the_geometry_and_widen_the_tolerance(lib):
    """ABFT_THREAD_HALF and ABFT_TWOSIDED run on the thread-level scheme's tiles; their extra
    tolerance coefficient is 4 u_half sqrt(n_B tile_m + n_A tile_n) (0 for int8 and for the other
    schemes)."""
    import math
    for (M, N, K) in [(64, 64, 64), (256, 4096, 4096), (1536, 1536, 256), (8192, 8192, 8192)]:
        for mode in (B.THREAD_HALF, B.TWOSIDED):
            assert B.abft_k_ways(M, N, K, B.F16, mode) == B.abft_k_ways(M, N, K, B.F16, B.THREAD)
            assert B.abft_workspace_bytes(M, N, K, B.F16, mode) == 0
            assert B.abft_tolerance_coeff(K, B.F16, mode) == B.abft_tolerance_coeff(K, B.F16, B.THREAD)
    assert B.abft_tolerance_half_coeff(B.F16, B.THREAD_HALF, 32, 128) == pytest.approx(4 * 2.0 ** -11 * math.sqrt(3 * 32))
    assert B.abft_tolerance_half_coeff(B.F16, B.TWOSIDED, 64, 64) == pytest.approx(4 * 2.0 ** -11 * math.sqrt(64 + 64))
    assert B.abft_tolerance_half_coeff(B.BF16, B.THREAD_HALF, 64, 64) == pytest.approx(4 * 2.0 ** -8 * math.sqrt(64))
    assert B.abft_tolerance_half_coeff(B.F16, B.THREAD_HALF, 32, 32) == 0.0      # nothing is added up
    assert B.abft_tolerance_half_coeff(B.I8, B.TWOSIDED, 64, 64) == 0.0
    assert B.abft_tolerance_half_coeff(B.F16, B.THREAD, 64, 64) == 0.0
    assert B.MODE_NAMES[B.TWOSIDED] == "twosided" and B.MODE_NAMES[B.THREAD_HALF] == "thread_half"


def test_tile_choice_for_few_tiles(lib):
    """Documented choices of the dispatcher for latency-bound products (region = workgroup tile of
    the global scheme, tile = wavefront tile of the thread-level scheme)."""
    # one round of 32 x 32 streaming tiles, for every scheme
    assert B.abft_region_shape(256, 1024, 1024, B.F16) == (32, 32)
    assert B.abft_tile_shape(256, 1024, 1024, B.F16)[:2] == (32, 32)
    # more than 256 of those: 32 x 64 for everyone
    assert B.abft_region_shape(128, 4096, 4096, B.F16) == (32, 64)
    # more than 256 of those too: 64 x 64 streaming tiles, but only with a k loop of four tiles or more
    assert B.abft_region_shape(512, 4096, 4096, B.F16) == (64, 64)
    assert B.abft_region_shape(3136, 512, 128, B.F16) == (64, 128)
    # the chip is full: 128 x 128; about one 256 x 128 tile per compute unit with a long k loop: that tile
    # (the thread-level scheme keeps wavefront tiles of 32-row blocks); then 256 x 256
    assert B.abft_region_shape(12544, 768, 1024, B.F16) == (128, 128)
    assert B.abft_region_shape(12544, 512, 1024, B.F16) == (256, 128)
    assert B.abft_region_shape(12544, 512, 256, B.F16) == (128, 128)
    assert B.abft_tile_shape(12544, 512, 1024, B.F16)[:2] in ((32, 128), (64, 64))
    assert B.abft_region_shape(8192, 8192, 8192, B.F16) == (256, 256)
    # streaming tiles split k over four wavefronts
    assert B.abft_k_ways(256, 1024, 1024, B.F16, B.THREAD)[0] == 4
    assert B.abft_k_ways(8192, 8192, 8192, B.F16, B.THREAD)[0] == 1
