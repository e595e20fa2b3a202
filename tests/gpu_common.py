"""Shared plumbing of the GPU parity tests: run one layer through the HIP library and through
the oracle on the same seeded bytes, and compare to the bars of the build contract:
integer results bit-exact, bf16 output within 2e-3 relative or 1e-2 absolute of the oracle's
unrounded fp64 value."""
import numpy as np
import torch

import workloads as wl
from oracle import stwq_oracle as O
from paper_2601_21238_amd.layer import StwqLinear

REL_TOL, ABS_TOL = 2e-3, 1e-2
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def check_bf16(y_gpu: torch.Tensor, y_ref: np.ndarray, what=""):
    got = host(y_gpu.float()).astype(np.float64)
    err = np.abs(got - y_ref)
    ok = (err <= REL_TOL * np.abs(y_ref)) | (err <= ABS_TOL)
    assert ok.all(), (f"{what}: {np.count_nonzero(~ok)} of {ok.size} outputs outside tolerance; worst abs err "
                      f"{err.max():.4g}, worst rel {np.max(err / np.maximum(np.abs(y_ref), 1e-30)):.4g}")


def oracle_pack(spec, x_calib, w, bias, s=None):
    """Oracle calibration; the GPS scale is solved by the oracle unless given."""
    return O.calibrate_layer(x_calib, w, bias, spec.L, spec.a_bits, spec.w_bits, spec.gps and s is None, s=s)


def gpu_layer(spec, x_calib, w, bias, s):
    """Library calibration with the same scale vector."""
    layer = StwqLinear(spec.N, spec.K, spec.L, spec.a_bits, spec.w_bits, DEV)
    layer.calibrate(dev(x_calib), dev(w), None if s is None else dev(s), None if bias is None else dev(bias))
    return layer


def check_calibration(layer: StwqLinear, pack):
    """Every offline quantity is bit-exact."""
    assert np.array_equal(host(layer.wq), pack["wq"]), "weight codes differ"
    assert np.array_equal(host(layer.dw), pack["dw"]), "weight scales differ"
    assert np.array_equal(host(layer.wsum), pack["wsum"]), "weight row sums differ"
    if pack["inv_s"] is not None:
        assert np.array_equal(host(layer.inv_s), pack["inv_s"]), "1/s differs"
    assert np.array_equal(host(layer.pos_min), pack["pos_min"]), "pos_min differs"
    assert np.array_equal(host(layer.pos_max), pack["pos_max"]), "pos_max differs"
    assert np.array_equal(host(layer.delta), pack["delta"]), "delta differs"
    assert np.array_equal(host(layer.inv_delta), pack["inv_delta"]), "1/delta differs"
    assert np.array_equal(host(layer.zp), pack["z"]), "zero points differ"


def check_forward(layer: StwqLinear, pack, x, schedule, t0=None, what=""):
    q_ref, acc_ref, y_ref = O.forward(pack, x, t0=t0)
    xd = dev(x)
    q = layer.quantize(xd, t0=t0)
    assert np.array_equal(host(q), q_ref), f"{what}: activation codes differ"
    acc = torch.full((x.shape[0], layer.N), -7, dtype=torch.int32, device=DEV)
    y = layer.linear(q, acc_dbg=acc, t0=t0, schedule=schedule)
    torch.cuda.synchronize()
    assert np.array_equal(host(acc), acc_ref), f"{what}: int32 accumulators differ"
    check_bf16(y, y_ref, what)
    return q, acc, y


def make_case(spec):
    w, b = wl.make_weights(spec)
    xc = wl.make_calibration(spec)
    xt = wl.make_test_input(spec)
    return w, b, xc, xt
