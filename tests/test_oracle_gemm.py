"""Pins for the oracle's integer product and dequantizing epilogue."""
import json
import os

import numpy as np
import pytest

from oracle import stwq_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
F32 = np.float32


def test_k2_hand_case():
    with open(os.path.join(GOLD, "gemm_k2.json")) as f:
        g = json.load(f)
    q = np.array([g["stored"]], np.int8)
    wq = np.array([g["wq"]], np.int8)
    acc = O.gemm_i32(q, wq)
    assert acc.dtype == np.int32 and acc[0, 0] == g["acc"]
    wsum = np.array([g["wsum"]], np.int32)
    y = O.epilogue(acc, np.array([g["z"]], np.int32), wsum, np.array([g["delta"]], F32),
                   np.array([g["dw"]], F32), np.array([g["bias"]], F32), 1, 8)
    assert y[0, 0] == g["y"]
    corr = sum((c - g["z"]) * w for c, w in zip(g["codes"], g["wq"]))
    assert corr == g["corr"] == g["acc"] - (g["z"] - 128) * g["wsum"]


def test_gemm_against_python_loops_and_is_not_transposed():
    rng = np.random.default_rng(0)
    M, K, N = 5, 7, 3
    q = rng.integers(-128, 128, (M, K)).astype(np.int8)
    wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    acc = O.gemm_i32(q, wq)
    assert acc.shape == (M, N)
    for m in range(M):
        for o in range(N):
            assert acc[m, o] == sum(int(q[m, k]) * int(wq[o, k]) for k in range(K))


def test_gemm_extremes_and_integer_einsum():
    # worst-case magnitude the configurations can reach: K = 12288, all -128 * -128
    K = 12288
    q = np.full((2, K), -128, np.int8)
    wq = np.full((3, K), -128, np.int8)
    assert np.all(O.gemm_i32(q, wq) == K * 128 * 128)
    rng = np.random.default_rng(1)
    q = rng.integers(-128, 128, (130, 1024)).astype(np.int8)
    wq = rng.integers(-127, 128, (70, 1024)).astype(np.int8)
    ref = np.einsum("mk,ok->mo", q.astype(np.int64), wq.astype(np.int64))
    assert np.array_equal(O.gemm_i32(q, wq).astype(np.int64), ref)


def test_freivalds_on_a_larger_product():
    rng = np.random.default_rng(2)
    M, K, N = 700, 1024, 520
    q = rng.integers(-128, 128, (M, K)).astype(np.int8)
    wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    acc = O.gemm_i32(q, wq).astype(np.int64)
    for _ in range(3):
        r = rng.integers(-1000, 1000, N).astype(np.int64)
        assert np.array_equal(acc @ r, q.astype(np.int64) @ (wq.astype(np.int64).T @ r))


@pytest.mark.parametrize("bits", [6, 8])
def test_epilogue_equals_product_of_dequantized_operands(bits):
    rng = np.random.default_rng(3)
    L, n, K, N = 4, 3, 96, 20
    x = (rng.standard_normal((n * L, K)) * rng.uniform(0.5, 4, (1, K))).astype(F32)
    w = (rng.standard_normal((N, K)) * 0.02).astype(F32)
    b = (rng.standard_normal(N) * 0.01).astype(F32)
    s = rng.uniform(0.5, 4, K).astype(F32)
    pack = O.calibrate_layer(x, w, b, L, bits, bits, False, s=s)
    q, acc, y = O.forward(pack, x)
    t = np.arange(n * L) % L
    codes = q.astype(np.int64) + O.store_offset(bits)
    x_hat = pack["delta"].astype(np.float64)[t][:, None] * (codes - pack["z"][t][:, None])    # A.1 dequant
    w_hat = pack["dw"].astype(np.float64)[:, None] * pack["wq"]
    ref = x_hat @ w_hat.T + b.astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-9, atol=1e-12)
    # and it approximates the unquantized layer
    full = x.astype(np.float64) @ w.astype(np.float64).T + b
    assert np.linalg.norm(y - full) / np.linalg.norm(full) < (0.03 if bits == 8 else 0.15)


def test_zero_input_or_zero_weights_return_the_bias_exactly():
    rng = np.random.default_rng(4)
    L, K, N = 3, 32, 8
    xc = rng.standard_normal((4 * L, K)).astype(F32)
    w = (rng.standard_normal((N, K)) * 0.02).astype(F32)
    b = rng.standard_normal(N).astype(F32)
    pack = O.calibrate_layer(xc, w, b, L, 8, 8, True)
    _, _, y = O.forward(pack, np.zeros((2 * L, K), F32))
    assert np.array_equal(y, np.broadcast_to(b.astype(np.float64), y.shape))
    pack0 = O.calibrate_layer(xc, np.zeros_like(w), b, L, 8, 8, False)
    _, acc, y = O.forward(pack0, xc)
    assert not acc.any() and np.array_equal(y, np.broadcast_to(b.astype(np.float64), y.shape))


def test_invariances():
    rng = np.random.default_rng(6)
    L, K, N = 4, 64, 24
    xc = (rng.standard_normal((8 * L, K)) * 2).astype(F32)
    xt = (rng.standard_normal((3 * L, K)) * 2).astype(F32)
    w = (rng.standard_normal((N, K)) * 0.02).astype(F32)
    b = (rng.standard_normal(N) * 0.01).astype(F32)
    s = rng.uniform(0.5, 4, K).astype(F32)
    pack = O.calibrate_layer(xc, w, b, L, 8, 8, False, s=s)
    q, acc, y = O.forward(pack, xt)
    # permuting the input channels consistently leaves every accumulator unchanged
    p = rng.permutation(K)
    pack_p = O.calibrate_layer(xc[:, p], w[:, p], b, L, 8, 8, False, s=s[p])
    qp, accp, yp = O.forward(pack_p, xt[:, p])
    assert np.array_equal(qp, q[:, p]) and np.array_equal(accp, acc) and np.array_equal(yp, y)
    # permuting the outputs permutes y
    po = rng.permutation(N)
    pack_o = O.calibrate_layer(xc, w[po], b[po], L, 8, 8, False, s=s)
    _, acco, yo = O.forward(pack_o, xt)
    assert np.array_equal(acco, acc[:, po]) and np.array_equal(yo, y[:, po])
    # a row depends only on itself and its position
    _, acc1, y1 = O.forward(pack, xt[L:2 * L])
    assert np.array_equal(acc1, acc[L:2 * L]) and np.array_equal(y1, y[L:2 * L])
    # decode form: every row at position t0
    t0 = 2
    rows = xt[t0::L]
    _, accd, yd = O.forward(pack, rows, t0=t0)
    assert np.array_equal(accd, acc[t0::L]) and np.array_equal(yd, y[t0::L])


def test_bf16_rounding_helper():
    vals = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927], F32)
    bits = O.to_bf16_bits(vals)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: to even -> 1.0 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert bits[0] == 0x3F80 and bits[1] == 0x3F80 and bits[2] == 0x3F82
    back = O.bf16_bits_to_f64(bits)
    assert np.all(np.abs(back - vals) <= np.abs(vals) * 2.0 ** -8)
