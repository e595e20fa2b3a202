"""The synthetic input recipe: shapes, determinism and the structure the method relies on."""
import numpy as np

import workloads as wl


def test_config_shapes():
    c1 = wl.config_linears(1)
    assert len(c1) == 1 and (c1[0].M, c1[0].K, c1[0].N, c1[0].L) == (680, 1024, 1024, 680)
    c2 = {s.name: s for s in wl.config_linears(2)}
    assert [(s.K, s.N) for s in c2.values()] == [(1024, 3072), (1024, 1024), (1024, 4096), (4096, 1024)]
    assert all(s.M == 21760 for s in c2.values()) and c2["fc2"].gelu_input and c2["qkv"].gps and not c2["proj"].gps
    c3 = wl.config_linears(3, bits=6)
    assert c3[0].M == 43520 and c3[2].N == 7680 and c3[0].a_bits == 6 and c3[0].n_outliers == 16
    c4 = wl.config_linears(4)
    assert len(c4) == 72 and all(s.M == 128 and s.decode for s in c4)
    assert sum(s.N * s.K for s in c4) == 24 * (1280 * 3840 + 1280 * 5120 + 5120 * 1280)
    c5 = wl.config_linears(5)
    assert len(c5) == 120 and c5[0].M == 16384 and c5[3].K == 12288
    assert len({s.seed(r) for s in c2.values() for r in range(7)}) == 28


def test_recipe_is_seeded_and_structured():
    spec = wl.shrink(wl.config_linears(2)[0], K=64, N=32, L=20, batch=3, n_calib=6)
    w1, b1 = wl.make_weights(spec)
    w2, b2 = wl.make_weights(spec)
    assert np.array_equal(w1, w2) and np.array_equal(b1, b2) and w1.shape == (32, 64) and w1.dtype == np.float32
    xc = wl.make_calibration(spec)
    xt = wl.make_test_input(spec)
    assert xc.shape == (6 * 20, 64) and xt.shape == (3 * 20, 64)
    assert np.array_equal(xc, wl.make_calibration(spec)) and not np.array_equal(xc[:60], xt)
    out = wl.make_outliers(spec)
    assert len(out) == 8
    col = np.abs(xc).mean(axis=0)
    assert col[out].min() > 10 * np.delete(col, out).max()
    # chunked generation equals one-shot generation
    a = np.concatenate(list(wl.activation_chunks(spec, 6, wl.ROLE_CALIB, samples_per_chunk=4)))
    assert np.array_equal(a, xc)
    fc2 = wl.shrink(wl.config_linears(2)[3], K=64, N=32, L=20, batch=3, n_calib=6)
    xg = wl.make_calibration(fc2)
    assert xg.min() > -0.2 * 1.01 * 50 * 4 and xg.max() > 5     # GELU: bounded below, heavy positive tail
    dec = wl.shrink(wl.config_linears(4)[0], K=64, N=32)
    xd = wl.make_test_input(dec)
    assert xd.shape == (128, 64) and 0 <= wl.decode_position(dec) < 256
