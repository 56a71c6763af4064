"""Pins for the oracle's quantized-linear side: activation codes (Sections 3.1
and 3.3), weights, the grouped integer contraction and its dequantization."""
import os

import numpy as np
import pytest

import dgq_inputs as di

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _case(seed=21, B=2, N=96, C=320, O=48, G=64, bits=8, P=2, calib_self=False):
    run = di.linear_case(seed, B, N, C, O)
    cal = run if calib_self else di.linear_case(seed, B, N, C, O, calib=True)
    return run, cal


def test_linear_quantizer_worked_example(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "linear_quantizer_worked.txt"))
            if l.strip() and not l.startswith("#")]
    x = np.array([[float(r[0]) for r in rows]], np.float32)
    q_exp = np.array([int(r[2]) for r in rows])
    xdq_exp = np.array([float(r[3]) for r in rows])
    # calibrate on a one-row tensor with the same range: one group, s = 0.25, z = -1
    g = oracle.calibrate(x, 4, 64, 1)
    assert g.NG == 1 and g.s[0, 0] == 0.25 and g.z[0, 0] == -1.0
    r = oracle.quantize_act(g, x, want_dq=True)
    inv = np.argsort(g.perm[:g.glen[0]])
    assert np.array_equal(r["q"][0, :g.glen[0]][inv], q_exp)
    assert np.array_equal(r["xdq"][0], xdq_exp)


@pytest.mark.parametrize("bits", [4, 8])
def test_code_invariants(oracle, bits):
    run, cal = _case(bits=bits)
    g = oracle.calibrate(cal["X"], bits, 64, 2)
    X = run["X"]
    r = oracle.quantize_act(g, X, want_dq=True)
    q, cls, xdq, clip = r["q"], r["cls"], r["xdq"], r["clip"].astype(bool)
    assert q.max() <= 2 ** bits - 1
    # per-element scale in original channel order
    grp_of_pos = np.repeat(np.arange(g.NG), np.diff(g.goff))
    real = g.perm >= 0
    s_elem = np.zeros_like(X, dtype=np.float64)
    s_elem[:, g.perm[real]] = g.s[cls][:, grp_of_pos[real]]
    err = np.abs(X.astype(np.float64) - xdq)
    # |x - dequant(q(x))| <= s/2 on non-clipped elements (tiny slack for fp32 rounding of u)
    assert np.all(err[~clip] <= 0.5 * s_elem[~clip] * (1 + 1e-5))
    assert clip.any(), "the recipe is meant to produce run-time clipping"
    assert np.any(err[clip] > 0.5 * s_elem[clip])
    # padding positions hold 0
    assert np.all(q[:, ~real] == 0)
    # re-quantizing the dequantized tensor returns the same codes on non-clipped rows
    r2 = oracle.quantize_act(g, xdq.astype(np.float32))
    same_cls = r2["cls"] == cls
    assert same_cls.mean() > 0.9
    diff = (r2["q"] != q)[same_cls]
    assert diff.mean() < 1e-3  # float32 rounding of xdq may move exact ties only


def test_calibration_tensor_itself(oracle):
    """On the calibration data: min -> code 0 reproduced exactly, max clipped by
    at most s (divisor 2^b), everything else within s/2, classes identical."""
    run, _ = _case(calib_self=True)
    X = run["X"]
    g = oracle.calibrate(X, 8, 64, 2)
    r = oracle.quantize_act(g, X, want_dq=True)
    assert np.array_equal(r["cls"], g.cal_row_class)
    grp_of_pos = np.repeat(np.arange(g.NG), np.diff(g.goff))
    for p in range(2):
        rows = np.nonzero(r["cls"] == p)[0]
        for k in range(g.NG):
            ch = g.perm[g.goff[k]:g.goff[k] + g.glen[k]]
            cell = X[np.ix_(rows, ch)]
            dq = r["xdq"][np.ix_(rows, ch)]
            e = np.abs(cell - dq)
            assert e.max() <= g.s[p, k] * (1 + 1e-4)  # fp32 rounding of max - min
            i = np.unravel_index(np.argmin(cell), cell.shape)
            assert dq[i] == cell[i]  # x = min is reproduced exactly
            qq = r["q"][np.ix_(rows, np.arange(g.goff[k], g.goff[k] + g.glen[k]))]
            assert qq[i] == 0
            j = np.unravel_index(np.argmax(cell), cell.shape)
            assert qq[j] == 255 and r["clip"][rows[j[0]], ch[j[1]]] == 1


def test_monotone_in_x(oracle):
    x = np.linspace(-1, 3, 64, dtype=np.float32)[None, :]
    g = oracle.calibrate(x, 8, 64, 1)
    xs = np.sort(np.random.default_rng(0).uniform(-2, 4, (50, 64)).astype(np.float32), axis=0)
    r = oracle.quantize_act(g, xs)
    inv = np.argsort(g.perm[:64])
    q = r["q"][:, :64][:, inv].astype(int)
    assert np.all(np.diff(q, axis=0) >= 0)
    assert q.min() == 0 and q.max() == 255


@pytest.mark.parametrize("bits", [4, 8])
def test_layerwise_special_case(oracle, bits):
    """P = 1 and G = C (one group) is per-tensor min-max affine quantization,
    written here independently in NumPy (the paper's layer-wise granularity)."""
    rng = np.random.default_rng(4)
    X = rng.standard_normal((40, 128)).astype(np.float32)  # no outliers -> may still split
    X[:, :] = np.clip(X, -2.5, 2.5)
    X[0, :] = 2.5
    X[1, :] = -2.5  # every channel has the same width -> a single cluster
    g = oracle.calibrate(X, bits, 128, 1)
    assert g.NG == 1
    Y = rng.standard_normal((16, 128)).astype(np.float32) * np.float32(1.2)
    r = oracle.quantize_act(g, Y)
    s = np.float32(np.float32(X.max() - X.min()) / np.float32(2 ** bits))
    u = (Y - X.min()) * (np.float32(1) / s)
    q_np = np.clip(np.rint(u), 0, 2 ** bits - 1).astype(np.uint8)
    inv = np.argsort(g.perm[:128])
    assert np.array_equal(r["q"][:, :128][:, inv], q_np)


def test_outliers_keep_their_precision(oracle):
    """Grouping keeps outlier channels at their own scale and lowers the error
    of regular channels versus one layer-wise scale (the paper's claim about
    group-wise versus layer-wise quantizers, Figure 2 / Section 3.3)."""
    run, cal = _case(seed=33, C=640, G=128)
    X = run["X"]
    g = oracle.calibrate(cal["X"], 8, 128, 2)
    g1 = oracle.calibrate(np.concatenate([cal["X"], np.zeros((1, 640), np.float32)]), 8, 640, 1)
    r = oracle.quantize_act(g, X, want_dq=True)
    keep = (r["cls"] == 0)
    nc = ~r["clip"].astype(bool)
    reg = np.setdiff1d(np.arange(640), run["oc"])
    e = (X - r["xdq"])
    k_out = g.NG - 1
    assert np.all(np.abs(e[keep][:, run["oc"]])[nc[keep][:, run["oc"]]] <= 0.5 * g.s[0, k_out] * 1.00001)
    layer_s = (cal["X"].max() - cal["X"].min()) / 256.0
    assert g.s[0, :g.n_regular_groups].max() < layer_s / 30
    mse_grouped = np.mean(e[keep][:, reg] ** 2)
    assert mse_grouped < (layer_s ** 2 / 12) / 500


@pytest.mark.parametrize("w_bits", [4, 8])
def test_weight_quantizer(oracle, w_bits):
    rng = np.random.default_rng(8)
    W = (0.02 * rng.standard_normal((24, 100))).astype(np.float32)
    W[3] = 0
    wq, sw = oracle.quantize_weight(W, w_bits)
    qmax = 127 if w_bits == 8 else 7
    amax = np.abs(W).max(1)
    sw_np = np.where(amax > 0, amax / np.float32(qmax), np.float32(1)).astype(np.float32)
    assert np.array_equal(sw, sw_np)
    assert np.array_equal(wq, np.clip(np.rint(W / sw_np[:, None]), -qmax, qmax).astype(np.int8))
    assert np.abs(wq).max() == qmax and np.all(wq[3] == 0)
    assert np.all(np.abs(W - wq * sw[:, None]) <= 0.5 * sw[:, None] * 1.00001)


@pytest.mark.parametrize("bits", [4, 8])
def test_int32_accumulators_vs_int64_brute_force(oracle, bits):
    run, cal = _case(seed=5, B=1, N=24, C=200, O=12, bits=bits)
    g = oracle.calibrate(cal["X"], bits, 64, 2)
    r = oracle.quantize_act(g, run["X"])
    wq, sw = oracle.quantize_weight(run["W"], 8)
    y, acc = oracle.linear(g, r["q"], r["cls"], wq, sw, None, want_acc=True)
    off = 128 if bits == 8 else 0
    code = r["q"].astype(np.int64) - off
    for k in range(g.NG):
        pos = np.arange(g.goff[k], g.goff[k] + g.glen[k])
        ref = code[:, pos] @ wq[:, g.perm[pos]].astype(np.int64).T
        assert np.array_equal(acc[:, :, k].astype(np.int64), ref)
    # the groups tile K: their sum is the ungrouped dot product
    real = g.perm >= 0
    tot = code[:, real] @ wq[:, g.perm[real]].astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64).sum(-1), tot)
    # pure-Python big-int dot on a few entries
    for (i, o) in [(0, 0), (7, 3), (23, 11)]:
        ref = sum(int(code[i, j]) * int(wq[o, g.perm[j]]) for j in np.nonzero(real)[0])
        assert int(acc[i, o].sum()) == ref


@pytest.mark.parametrize("bits,w_bits", [(8, 8), (4, 8), (8, 4)])
def test_dequant_algebra(oracle, bits, w_bits):
    """Y == dequant(X) . dequant(W)^T + bias in double: pins z', wsum, the
    permutation, the padding and the class-dependent scales in one check."""
    run, cal = _case(seed=6, B=2, N=40, C=328, O=20, bits=bits)
    g = oracle.calibrate(cal["X"], bits, 64, 2)
    r = oracle.quantize_act(g, run["X"], want_dq=True)
    wq, sw = oracle.quantize_weight(run["W"], w_bits)
    bias = np.random.default_rng(1).standard_normal(20).astype(np.float32)
    y, _ = oracle.linear(g, r["q"], r["cls"], wq, sw, bias)
    wdq = wq.astype(np.float64) * sw.astype(np.float64)[:, None]
    ref = r["xdq"] @ wdq.T + bias.astype(np.float64)
    assert np.abs(y - ref).max() <= 2e-7 * np.abs(ref).max()
    y0, _ = oracle.linear(g, r["q"], r["cls"], wq, sw, None)
    assert np.abs((y0 + bias) - y).max() <= 1e-5 * np.abs(ref).max()


def test_closeness_to_full_precision(oracle):
    """On rows without clipping the error of Y against X.W^T matches the
    uniform-noise estimate sum s^2/12 W^2 + sum x^2 sw^2/12 within a factor 2."""
    run, cal = _case(seed=12, B=2, N=128, C=320, O=64)
    g = oracle.calibrate(cal["X"], 8, 64, 2)
    X = run["X"]
    r = oracle.quantize_act(g, X, want_dq=True)
    wq, sw = oracle.quantize_weight(run["W"], 8)
    y, _ = oracle.linear(g, r["q"], r["cls"], wq, sw, None)
    W = run["W"].astype(np.float64)
    ref = X.astype(np.float64) @ W.T
    ok = r["clip"].sum(1) == 0
    assert ok.mean() > 0.5
    grp_of_pos = np.repeat(np.arange(g.NG), np.diff(g.goff))
    real = g.perm >= 0
    s_ch = np.zeros((2, 320))
    s_ch[:, g.perm[real]] = g.s[:, grp_of_pos[real]]
    var = (s_ch[r["cls"][ok]] ** 2 / 12) @ (W ** 2).T + \
        (X[ok].astype(np.float64) ** 2) @ np.tile((sw.astype(np.float64) ** 2 / 12)[None, :], (320, 1))
    ratio = np.sqrt(((y[ok] - ref[ok]) ** 2).mean() / var.mean())
    assert 0.5 < ratio < 2.0, ratio
