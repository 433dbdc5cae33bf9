"""Pins for the oracle's layer chain: activation function, storage rounding, MLP forward."""
import numpy as np
import pytest

import oracle


def test_relu_closed_form():
    x = np.random.default_rng(0).normal(size=(17, 9))
    r = oracle.activation(x, "relu")
    assert np.array_equal(r, (x + np.abs(x)) / 2)          # exact in binary arithmetic
    assert np.array_equal(r - oracle.activation(-x, "relu"), x)
    assert oracle.activation(x, None) is x


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_round_out_is_identity_on_every_representable_value(dtype):
    bits = np.arange(65536, dtype=np.uint16)
    store = bits.view(np.float16) if dtype == "f16" else bits
    wide = oracle.widen(store, dtype)
    fin = np.isfinite(wide)
    back = oracle.round_out(wide, dtype)
    back_bits = back.view(np.uint16) if dtype == "f16" else back
    # (+0 and -0 both survive; NaNs are excluded)
    assert np.array_equal(back_bits[fin], bits[fin])
    inf = np.isinf(wide)
    assert np.array_equal(back_bits[inf], bits[inf])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_round_out_ties_go_to_even_and_neighbours_win(dtype):
    # adjacent positive finite values a < b (bit patterns n, n + 1): the midpoint goes to the
    # even pattern, anything nearer one side goes to that side
    top = 0x7BFF if dtype == "f16" else 0x7F7F
    n = np.arange(0, top, dtype=np.uint16)
    lo_store = n.view(np.float16) if dtype == "f16" else n
    hi_store = (n + 1).astype(np.uint16)
    hi_store = hi_store.view(np.float16) if dtype == "f16" else hi_store
    a, b = oracle.widen(lo_store, dtype), oracle.widen(hi_store, dtype)
    as_bits = lambda s: s.view(np.uint16) if dtype == "f16" else s
    mid = as_bits(oracle.round_out((a + b) / 2, dtype))     # exact in fp64
    assert np.array_equal(mid, np.where(n % 2 == 0, n, n + 1))
    assert np.array_equal(as_bits(oracle.round_out(a + (b - a) * 0.25, dtype)), n)
    assert np.array_equal(as_bits(oracle.round_out(a + (b - a) * 0.75, dtype)), n + 1)
    # past the largest finite value by half a step or more: infinity
    big = oracle.widen(np.array([top], dtype=np.uint16).view(np.float16) if dtype == "f16"
                       else np.array([top], dtype=np.uint16), dtype)[0]
    step = big - oracle.widen(np.array([top - 1], dtype=np.uint16).view(np.float16) if dtype == "f16"
                              else np.array([top - 1], dtype=np.uint16), dtype)[0]
    out = as_bits(oracle.round_out(np.array([big + step / 2, big + step * 0.49]), dtype))
    assert out[0] == top + 1 and out[1] == top


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_mlp_forward_against_integer_chain(dtype):
    """Small integers make every product, sum and rounding exact: the chain equals the same
    chain in int64 with the integer max."""
    rng = np.random.default_rng(3)
    dims = [7, 5, 6, 4]
    x = rng.integers(-3, 4, size=(9, dims[0]))
    Ws = [rng.integers(-2, 3, size=(dims[i], dims[i + 1])) for i in range(3)]
    acts = ["relu", "relu", None]
    ref, a = [], x
    for W, act in zip(Ws, acts):
        a = a @ W
        if act:
            a = np.maximum(a, 0)
        ref.append(a)
    assert max(np.abs(r).max() for r in ref) <= 128           # exact in bf16's 8 bits too
    def store(v):
        h = v.astype(np.float16)
        if dtype == "f16":
            return h
        return (h.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)  # exact: small integers
    outs = oracle.mlp_forward(store(x), [store(W) for W in Ws], dtype, acts)
    for o, r in zip(outs, ref):
        assert np.array_equal(oracle.widen(o, dtype), r.astype(np.float64))
