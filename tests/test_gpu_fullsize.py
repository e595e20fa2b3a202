"""GPU parity at the full sizes of the build's configurations, in the launch configuration
bench.py times (auto schedule): every activation code and every offline quantity is compared;
accumulators and bf16 outputs are compared on a stratified row sample and, over the whole matrix,
through Freivalds' identity acc r = q (Wq^T r) in exact integer arithmetic."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import stwq_oracle as O

pytestmark = pytest.mark.gpu

import paper_2601_21238_amd as P            # noqa: E402
import gpu_common as G                       # noqa: E402


def sample_rows(spec, rng, n_random=1024):
    M, L = spec.M, spec.L
    rows = set()
    for b in range(spec.batch):                       # first and last row of every batch element
        rows.add(b * L)
        rows.add(b * L + L - 1)
    rows.update(range(min(256, M)))                   # all rows of the first and last 256-row tile
    rows.update(range(max(0, M - 256), M))
    rows.update(rng.integers(0, M, n_random).tolist())
    return np.array(sorted(rows))


def run_full(spec):
    rng = np.random.default_rng(spec.seed(9))
    w, b, xc, xt = G.make_case(spec)
    pack = G.oracle_pack(spec, xc, w, b)
    layer = G.gpu_layer(spec, xc, w, b, pack["s"])
    del xc
    G.check_calibration(layer, pack)
    if spec.gps:   # the library's own scale solve agrees with the oracle's
        s_gpu = layer.solve_scale(G.dev(wl.make_calibration(spec)), G.dev(w))
        assert np.allclose(G.host(s_gpu), pack["s"], rtol=1e-5, atol=0)
    xd = G.dev(xt)
    q = layer.quantize(xd)
    q_ref = O.quantize_act(xt, pack["inv_s"], pack["inv_delta"], pack["z"], spec.L, spec.a_bits)
    assert np.array_equal(G.host(q), q_ref), "activation codes differ"
    acc = torch.empty((spec.M, spec.N), dtype=torch.int32, device=G.DEV)
    y = layer.linear(q, acc_dbg=acc)                   # auto schedule, as in bench.py
    y2 = layer.linear(q)                               # and without the debug output
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    # sampled rows: per-row tables make the oracle's "row r sits at position r mod L" the identity
    rows = sample_rows(spec, rng)
    t = rows % spec.L
    sub = dict(pack, delta=pack["delta"][t], inv_delta=pack["inv_delta"][t], z=pack["z"][t], L=len(rows))
    _, acc_ref, y_ref = O.forward(sub, xt[rows])
    rows_d = torch.from_numpy(rows).to(G.DEV)
    assert np.array_equal(G.host(acc[rows_d]), acc_ref), "int32 accumulators differ on the sampled rows"
    G.check_bf16(y[rows_d], y_ref, f"{spec.name} sampled rows", pack["bias"])
    # whole matrix: Freivalds in int64 (|acc| < 2^31, |r| < 2^10, N < 2^14: no overflow)
    acc_h = G.host(acc).astype(np.int64)
    for _ in range(2):
        r = rng.integers(-1000, 1000, spec.N).astype(np.int64)
        lhs = acc_h @ r
        rhs = q_ref.astype(np.int64) @ (pack["wq"].astype(np.int64).T @ r)
        assert np.array_equal(lhs, rhs), "Freivalds check failed: some accumulator is wrong"


@pytest.mark.parametrize("name", ["qkv", "proj", "fc1", "fc2"])
def test_config2_full(name):
    """VAR-d16-shaped block at W8A8, M = 21760: the benchmark's workload."""
    spec = {s.name: s for s in wl.config_linears(2)}[name]
    run_full(spec)


def test_config3_qkv_w6a6_full():
    """VAR-d30-shaped qkv (1920 -> 5760, neither a multiple of 256), M = 43520, 6-bit codes held in int8.
    16 calibration samples instead of 64 keep the oracle's fp64 scale solve within the test budget."""
    spec = wl.shrink(wl.config_linears(3, bits=6)[0], n_calib=16)
    run_full(spec)


def test_config5_fc2_full():
    """3B-class fc2 (12288 -> 3072: the longest K of any configuration), M = 16384, W8A8, 4 calibration samples."""
    spec = wl.shrink(wl.config_linears(5)[3], n_calib=4)
    run_full(spec)


@pytest.mark.timeout(600)
def test_config4_decode_step_full():
    """The whole RAR-XXL-shaped decode step bench.py times: 24 blocks x (qkv, fc1, fc2), M = 128 rows at one token
    position per linear, one grouped quantization launch and one grouped linear launch on panel-packed weights
    (960 tiles on 256 compute units: the launch runs from the balanced per-workgroup tile lists).  Every offline
    quantity, activation code, accumulator and output of all 72 linears is compared with the oracle."""
    specs = wl.config_linears(4)
    assert len(specs) == 72
    qproblems, problems, refs, keep = [], [], [], []
    for spec in specs:
        w, b, xc, xt = G.make_case(spec)
        t0 = wl.decode_position(spec)
        pack = G.oracle_pack(spec, xc, w, b)
        layer = G.gpu_layer(spec, xc, w, b, pack["s"])
        G.check_calibration(layer, pack)
        q_ref, acc_ref, y_ref = O.forward(pack, xt, t0=t0)
        packed = torch.empty(P.stwq_packed_weight_bytes(spec.N, spec.K), dtype=torch.int8, device=G.DEV)
        P.stwq_pack_weights(layer.wq, packed)
        q = torch.zeros((spec.M, spec.K), dtype=torch.int8, device=G.DEV)
        qproblems.append(dict(x=G.dev(xt), L=1, inv_s=layer.inv_s, inv_delta=layer.inv_delta[t0:t0 + 1], zp=layer.zp[t0:t0 + 1],
                              a_bits=spec.a_bits, q=q))
        problems.append(dict(q=q, wq=packed, N=spec.N, w_layout=P.LAYOUT_PANEL32, dw=layer.dw, wsum=layer.wsum,
                             delta=layer.delta[t0:t0 + 1], zp=layer.zp[t0:t0 + 1], a_bits=spec.a_bits, bias=layer.bias, L=1,
                             y=torch.zeros((spec.M, spec.N), dtype=torch.bfloat16, device=G.DEV),
                             acc_dbg=torch.zeros((spec.M, spec.N), dtype=torch.int32, device=G.DEV)))
        refs.append((q_ref, acc_ref, y_ref, pack["bias"]))
        keep.append(layer)
        del w, xc
    _, lists = P.stwq_linear_grouped_plan([(s.M, s.K, s.N) for s in specs], 256)
    assert lists is not None and sum(len(l) for l in lists) == 960
    P.QuantizeGroup(qproblems).run()
    P.LinearGroup(problems).run()
    torch.cuda.synchronize()
    for spec, qp, pr, (q_ref, acc_ref, y_ref, bias) in zip(specs, qproblems, problems, refs):
        what = f"config 4, block {spec.layer}, {spec.name}"
        assert np.array_equal(G.host(qp["q"]), q_ref), f"{what}: activation codes differ"
        assert np.array_equal(G.host(pr["acc_dbg"]), acc_ref), f"{what}: accumulators differ"
        G.check_bf16(pr["y"], y_ref, what, bias)
