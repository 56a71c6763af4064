"""Pins for the oracle's calibration side: exact 1-D 2-means, pixel classes,
D_d / d*, channel groups, cell parameters (Section 3.3)."""
import itertools
import os

import numpy as np
import pytest

import dgq_inputs as di

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _sse(a):
    a = np.asarray(a, dtype=np.float64)
    return float(((a - a.mean()) ** 2).sum()) if a.size else 0.0


def test_two_means_brute_force_tiny(oracle):
    """Against the definition: try every 2-colouring of up to 10 points."""
    rng = np.random.default_rng(7)
    for trial in range(40):
        n = int(rng.integers(2, 11))
        v = rng.standard_normal(n).astype(np.float32)
        if trial % 3 == 0:
            v[rng.integers(0, n)] += np.float32(20.0)
        best = None
        for mask in range(1, 2 ** n - 1):
            sel = np.array([(mask >> i) & 1 for i in range(n)], dtype=bool)
            sse = _sse(v[sel]) + _sse(v[~sel])
            if best is None or sse < best - 1e-12:
                best = sse
        k, tau, order = oracle.two_means(v)
        sv = v[order]
        got = _sse(sv[:k]) + _sse(sv[k:])
        assert got <= best * (1 + 1e-9) + 1e-12
        # the threshold reproduces the split on the data itself
        assert ((v > tau).sum()) == n - k
        assert np.all(np.diff(sv) >= 0)


def test_two_means_not_worse_than_lloyd(oracle):
    """A library K-means (Lloyd, random restarts) never beats the exact split."""
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(3)
    for n in (50, 400):
        v = np.concatenate([rng.standard_normal(n), 6 + 2 * rng.standard_normal(n // 10)])
        v = v.astype(np.float32)
        k, tau, order = oracle.two_means(v)
        sv = v[order].astype(np.float64)
        ours = _sse(sv[:k]) + _sse(sv[k:])
        km = KMeans(n_clusters=2, n_init=10, random_state=0).fit(v.reshape(-1, 1).astype(np.float64))
        assert ours <= km.inertia_ * (1 + 1e-9)
        assert abs(ours - km.inertia_) <= 1e-6 * km.inertia_


def test_two_means_degenerate(oracle):
    k, tau, _ = oracle.two_means(np.full(5, 2.5, np.float32))
    assert k == 5 and np.isinf(tau) and tau > 0
    k, tau, _ = oracle.two_means(np.array([1.0], np.float32))
    assert k == 1 and np.isinf(tau)
    # ties by index, split only between distinct values
    v = np.array([0, 0, 1, 1], np.float32)
    k, tau, order = oracle.two_means(v)
    assert k == 2 and list(order) == [0, 1, 2, 3] and 0 <= tau < 1


def test_variability_metric_worked_example(oracle):
    """Hand-computed 3x3 example of D_d and d* (golden fixture)."""
    vals = {}
    for line in open(os.path.join(GOLD, "variability_metric_worked.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        vals[k.strip()] = v.strip()
    X = np.array([float(t) for t in vals["X"].split()], np.float32).reshape(3, 3)
    g = oracle.calibrate(X, 8, 64, 1)
    assert g.D_channel == float(vals["D_channel"])
    assert g.D_pixel == float(vals["D_pixel"])
    assert g.dstar == (0 if vals["dstar"] == "channel" else 1)


def test_variability_metric_transpose_and_selection(oracle):
    rng = np.random.default_rng(11)
    X = rng.standard_normal((48, 64)).astype(np.float32)
    g = oracle.calibrate(X, 8, 64, 1)
    gt = oracle.calibrate(np.ascontiguousarray(X.T), 8, 64, 1)
    assert g.D_channel == gt.D_pixel and g.D_pixel == gt.D_channel
    # independent numpy expression of the metric
    def D(M, axis):
        mx, mn = M.max(axis=axis).astype(np.float64), M.min(axis=axis).astype(np.float64)
        return (mx.max() - mx.min()) + (mn.max() - mn.min())
    assert g.D_channel == D(X, 0) and g.D_pixel == D(X, 1)
    Xc = X.copy()
    Xc[:, 5] *= 50
    assert oracle.calibrate(Xc, 8, 64, 1).dstar == 0
    assert oracle.calibrate(np.ascontiguousarray(Xc.T), 8, 64, 1).dstar == 1


@pytest.mark.parametrize("B,N,C,G", [(2, 256, 1280, 128), (2, 512, 320, 64)])
def test_injected_outliers_are_recovered(oracle, B, N, C, G):
    """On the synthetic recipe the outlier clusters equal the injected sets."""
    cal = di.linear_case(5, B, N, C, calib=True, with_weight=False)
    g = oracle.calibrate(cal["X"], 8, G, 2)
    assert g.n_outlier_channels == len(cal["oc"])
    out_pos = np.arange(g.goff[g.n_regular_groups], g.Kp)
    found = np.sort(g.perm[out_pos][g.perm[out_pos] >= 0])
    assert np.array_equal(found, cal["oc"])
    assert np.array_equal(np.nonzero(g.cal_row_class)[0], cal["rows_ot"])
    assert g.n_class1_rows == len(cal["rows_ot"])


def test_group_structure(oracle):
    cal = di.linear_case(9, 2, 128, 320, calib=True, with_weight=False)
    X = cal["X"]
    g = oracle.calibrate(X, 8, 64, 2)
    # perm is a permutation of the channels plus padding
    real = g.perm[g.perm >= 0]
    assert np.array_equal(np.sort(real), np.arange(320))
    assert g.goff[0] == 0 and g.goff[-1] == g.Kp and np.all(g.goff % 64 == 0)
    assert np.all(np.diff(g.goff) == (g.glen + 63) // 64 * 64)
    assert g.glen.sum() == 320 and g.NG == 6
    for k in range(g.NG):
        seg = g.perm[g.goff[k]:g.goff[k + 1]]
        assert np.all(seg[:g.glen[k]] >= 0) and np.all(seg[g.glen[k]:] == -1)
    # channels are ordered by class-0 width inside each cluster
    c0 = X[g.cal_row_class == 0]
    w = c0.max(0) - c0.min(0)
    nr = g.glen[:g.n_regular_groups].sum()
    order = np.concatenate([g.perm[g.goff[k]:g.goff[k] + g.glen[k]] for k in range(g.NG)])
    assert np.all(np.diff(w[order[:nr]]) >= 0) and np.all(np.diff(w[order[nr:]]) >= 0)
    assert w[order[:nr]].max() < w[order[nr:]].min()
    # cell parameters: s = (max - min) / 2^b, z = min over the cell
    for p in range(2):
        rows = X[g.cal_row_class == p]
        for k in range(g.NG):
            ch = g.perm[g.goff[k]:g.goff[k] + g.glen[k]]
            cell = rows[:, ch]
            assert g.z[p, k] == cell.min()
            assert g.s[p, k] == np.float32((cell.max() - cell.min()) / np.float32(256))
            assert g.inv_s[p, k] == np.float32(1.0) / g.s[p, k]


def test_single_class_and_constant_cells(oracle):
    X = np.zeros((4, 64), np.float32)
    g = oracle.calibrate(X, 8, 64, 2)
    assert g.NG == 1 and np.isinf(g.tau_pix) and g.n_outlier_channels == 0
    assert g.s[0, 0] == 1.0 and g.z[0, 0] == 0.0
    assert g.s[1, 0] == g.s[0, 0]  # empty class copies class 0
    rng = np.random.default_rng(1)
    X = rng.standard_normal((32, 96)).astype(np.float32)
    g1 = oracle.calibrate(X, 4, 64, 1)
    assert np.isinf(g1.tau_pix) and g1.cal_row_class.sum() == 0
    assert np.array_equal(g1.s[0], g1.s[1]) and np.array_equal(g1.z[0], g1.z[1])


def test_parameter_table_bytes(oracle):
    """One (s, z) fp32 pair per cell: P * NG * 2 * 4 bytes per layer and timestep
    (cf. the parameter-memory estimate in Section 3.3)."""
    cal = di.linear_case(2, 2, 64, 320, calib=True, with_weight=False)
    g = oracle.calibrate(cal["X"], 8, 64, 2)
    assert g.s.nbytes + g.z.nbytes == 2 * g.NG * 2 * 4
