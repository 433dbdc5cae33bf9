"""A chain of fully-connected layers in one kernel launch (abft_plan_run_chain): every layer
against the oracle applied to the very input that layer read, the whole chain against the
oracle's chain, clean flags, fresh inputs on every call, HIP-graph replays, the layer-by-layer
form for chains that do not qualify, and the bounded waits' error path."""
import numpy as np
import pytest

import oracle
from paper_2104_09455_amd import binding as B
from paper_2104_09455_amd import workloads as wl

pytestmark = pytest.mark.gpu
DT = {"f16": B.F16, "bf16": B.BF16}


def _storage(t, dtype):
    import torch
    return t.cpu().numpy() if dtype == "f16" else t.view(torch.int16).cpu().numpy().view(np.uint16)


class Chain:
    def __init__(self, M, widths, dtype, seed, modes):
        import torch
        from gpu_util import to_dev, DEV
        self.M, self.widths, self.dtype, self.nl = M, widths, dtype, len(widths) - 1
        dt = DT[dtype]
        self.Ws, self.keep, layers = [], [], []
        for l in range(self.nl):
            K, N = widths[l], widths[l + 1]
            _, Wm = wl.gemm_operands(8, N, K, dtype, seed=seed + 10 + l, dist_a="uniform_01", dist_b="weights")
            self.Ws.append(Wm)
            dB = to_dev(np.ascontiguousarray(Wm.T), dtype)
            self.keep.append(dB)
            layers.append(B.Layer(M, N, K, dt, B.B_NK, 0, B.Conv(), dB.data_ptr(), K))
        self.acts = ["relu"] * (self.nl - 1) + [None]
        c_t = torch.float16 if dtype == "f16" else torch.bfloat16
        self.Cs = [torch.zeros((M, widths[l + 1]), dtype=c_t, device=DEV) for l in range(self.nl)]
        self.flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        self.plan = B.abft_plan_create(layers)
        for l in range(self.nl):
            B.abft_plan_set_mode(self.plan, l, modes[l])
            B.abft_plan_set_activation(self.plan, l, B.ACT_RELU if self.acts[l] else B.ACT_NONE)

    def input(self, seed):
        from gpu_util import to_dev
        x, _ = wl.gemm_operands(self.M, 8, self.widths[0], self.dtype, seed=seed, dist_a="uniform_01", dist_b="weights")
        return x, to_dev(x, self.dtype)

    def run(self, dx, stream=None):
        B.abft_plan_run_chain(self.plan, 0, self.nl, dx, self.widths[0], self.Cs, self.widths[1:], self.flag, stream)

    def check(self, x):
        """Every layer against the oracle on the input the device's layer read; the end of the chain
        against the oracle's own chain."""
        from gpu_util import c_to_host, c_close
        a = x
        for l in range(self.nl):
            ref = oracle.activation(oracle.gemm(a, self.Ws[l], self.dtype), self.acts[l])
            got = c_to_host(self.Cs[l], self.dtype)
            assert c_close(got, ref, self.dtype), l
            a = _storage(self.Cs[l], self.dtype)
        last = oracle.widen(oracle.mlp_forward(x, self.Ws, self.dtype, self.acts)[-1], self.dtype)
        got = c_to_host(self.Cs[-1], self.dtype)
        rms = float(np.sqrt(np.mean(last * last)))
        assert np.all(np.abs(got - last) <= 3e-2 * np.abs(last) + 3e-2 * rms)

    def close(self):
        B.abft_plan_destroy(self.plan)


def _modes(kind, nl):
    return {"none": [B.NONE] * nl, "global": [B.GLOBAL] * nl, "thread": [B.THREAD] * nl,
            "mixed": [(B.THREAD, B.GLOBAL, B.NONE)[l % 3] for l in range(nl)]}[kind]


TOP = [512, 1024, 1024, 512, 256, 1]        # DLRM top MLP
BOTTOM = [512, 256, 64]                     # DLRM bottom MLP behind its first (K = 13) layer


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("kind", ["none", "global", "thread", "mixed"])
@pytest.mark.parametrize("M,widths", [(1, TOP), (16, TOP), (256, TOP), (256, BOTTOM), (200, [128, 320, 64]),
                                      (1024, [256, 192, 64])])
def test_chain_in_one_launch_matches_the_oracle(M, widths, kind, dtype):
    """DLRM's MLPs at batch 1 / 16 / 256, a ragged batch and one of several tile rows per die."""
    import torch
    ch = Chain(M, widths, dtype, seed=500 + M, modes=_modes(kind, len(widths) - 1))
    try:
        for call in range(2):          # the second call reads new inputs through the same buffers
            x, dx = ch.input(seed=600 + M + call)
            print(f"case chain M={M} widths={widths} modes={kind} dtype={dtype} call={call}", flush=True)
            ch.run(dx)
            torch.cuda.synchronize()
            assert B.abft_plan_chain_status(ch.plan) == 0
            assert int(ch.flag.item()) == 0
            ch.check(x)
    finally:
        ch.close()


def test_chain_under_graph_replay():
    import torch
    ch = Chain(256, TOP, "f16", seed=700, modes=_modes("mixed", 5))
    try:
        x, dx = ch.input(seed=701)
        ch.run(dx)
        torch.cuda.synchronize()
        eager = [c.clone() for c in ch.Cs]
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=cap):
            ch.run(dx, cap)
        for rep in range(4):
            for c in ch.Cs:
                c.zero_()                   # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for c, e in zip(ch.Cs, eager):
                assert torch.equal(c, e), rep
            assert int(ch.flag.item()) == 0 and B.abft_plan_chain_status(ch.plan) == 0
        ch.check(x)
    finally:
        ch.close()


def test_chain_that_does_not_qualify_runs_layer_by_layer():
    """K = 13 in the first layer (DLRM's bottom MLP as it is): no single launch, same results."""
    import torch
    ch = Chain(64, [13, 512, 256, 64], "f16", seed=710, modes=_modes("thread", 3))
    try:
        x, dx = ch.input(seed=711)
        ch.run(dx)
        torch.cuda.synchronize()
        assert int(ch.flag.item()) == 0
        ch.check(x)
    finally:
        ch.close()


def test_chain_waits_are_bounded():
    """With no polls allowed, a wait that finds the previous layer unfinished gives up at once: the
    status word says so, the fault flag is raised, the kernel ends normally; after a reset the chain
    runs clean again."""
    import torch
    ch = Chain(256, TOP, "f16", seed=720, modes=_modes("thread", 5))
    try:
        x, dx = ch.input(seed=721)
        B.abft_plan_chain_reset(ch.plan, 0)
        ch.run(dx)
        torch.cuda.synchronize()
        status = B.abft_plan_chain_status(ch.plan)
        assert status in (0, 1)
        if status:
            assert int(ch.flag.item()) == 1
        else:
            ch.check(x)
        ch.flag.zero_()
        B.abft_plan_chain_reset(ch.plan, -1)
        ch.run(dx)
        torch.cuda.synchronize()
        assert B.abft_plan_chain_status(ch.plan) == 0 and int(ch.flag.item()) == 0
        ch.check(x)
    finally:
        ch.close()
