"""Pins for the oracle's single-dimension grouping (Section 3.3, Eq. 4-6): exact 1-D
K-means, the choice of the dimension, the groups and their (s_k, z_k)."""
import itertools

import numpy as np
import pytest


def _sse(a):
    a = np.asarray(a, dtype=np.float64)
    return float(((a - a.mean()) ** 2).sum()) if a.size else 0.0


def _partition_sse(sorted_v, bounds):
    return sum(_sse(sorted_v[bounds[c]:bounds[c + 1]]) for c in range(len(bounds) - 1))


def test_k_means_brute_force_tiny(oracle):
    """Against the definition: every assignment of up to 8 points to K <= 4 labels
    (non-contiguous ones included), each cluster scored around its own mean."""
    rng = np.random.default_rng(11)
    for trial in range(30):
        n = int(rng.integers(3, 9))
        K = int(rng.integers(2, 5))
        v = rng.standard_normal(n).astype(np.float32)
        if trial % 3 == 0:
            v[rng.integers(0, n)] += np.float32(15.0)
        if trial % 5 == 0:
            v[0] = v[-1]  # a duplicate
        best = None
        for lab in itertools.product(range(K), repeat=n):
            lab = np.array(lab)
            sse = sum(_sse(v[lab == c]) for c in range(K))
            if best is None or sse < best:
                best = sse
        k, bounds, taus, order = oracle.k_means(v, K)
        sv = v[order]
        assert k == min(K, np.unique(v).size)
        got = _partition_sse(sv, bounds)
        assert got <= best + 1e-9 * (1 + best)
        assert got >= best - 1e-9 * (1 + best)  # the optimum is attained, not beaten


def test_k_means_two_clusters_equal_two_means(oracle):
    """K = 2 is the split used for the pixel classes: same cut, same threshold bits."""
    rng = np.random.default_rng(5)
    for n in (2, 3, 17, 300):
        v = rng.standard_normal(n).astype(np.float32)
        v[: max(1, n // 10)] *= np.float32(12.0)
        k2, tau2, order2 = oracle.two_means(v)
        k, bounds, taus, order = oracle.k_means(v, 2)
        assert k == 2 and bounds[1] == k2
        assert taus[0].tobytes() == np.float32(tau2).tobytes()
        assert np.array_equal(order, order2)


def test_k_means_recovers_separated_blobs(oracle):
    rng = np.random.default_rng(2)
    centres = np.array([0.0, 10.0, 25.0, 60.0, 61.5])
    sizes = [40, 7, 19, 3, 11]
    v = np.concatenate([c + 0.1 * rng.standard_normal(m) for c, m in zip(centres, sizes)])
    perm = rng.permutation(v.size)
    v = v[perm].astype(np.float32)
    k, bounds, taus, order = oracle.k_means(v, 5)
    assert k == 5
    assert list(np.diff(bounds)) == sizes
    # thresholds sit between the blobs and class = number of thresholds below the value
    cls = (v[:, None] > taus[None, :]).sum(1)
    truth = np.repeat(np.arange(5), sizes)[perm]
    assert np.array_equal(cls, truth)


def test_k_means_thresholds_reproduce_partition_and_sse_monotone(oracle):
    rng = np.random.default_rng(9)
    v = np.abs(rng.standard_normal(500)).astype(np.float32) ** 3
    prev = None
    for K in range(1, 17):
        k, bounds, taus, order = oracle.k_means(v, K)
        assert k == K
        sv = v[order]
        cls_sorted = (sv[:, None] > taus[None, :]).sum(1) if K > 1 else np.zeros(v.size, int)
        want = np.repeat(np.arange(K), np.diff(bounds))
        assert np.array_equal(cls_sorted, want)
        assert np.all(np.diff(taus) > 0)
        sse = _partition_sse(sv, bounds)
        if prev is not None:
            assert sse <= prev * (1 + 1e-12)
        prev = sse
        # necessary condition of an optimum: every point is at least as close to its own
        # cluster's mean as to any other mean
        means = np.array([sv[bounds[c]:bounds[c + 1]].astype(np.float64).mean() for c in range(K)])
        d = np.abs(sv.astype(np.float64)[:, None] - means[None, :])
        assert np.all(d[np.arange(v.size), want] <= d.min(1) + 1e-9)


def test_k_means_not_worse_than_library_lloyd(oracle):
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(4)
    v = np.concatenate([rng.standard_normal(300), 8 + rng.standard_normal(40),
                        30 + 3 * rng.standard_normal(25)]).astype(np.float32)
    for K in (3, 8):
        k, bounds, taus, order = oracle.k_means(v, K)
        ours = _partition_sse(v[order], bounds)
        km = KMeans(n_clusters=K, n_init=20, random_state=0).fit(v.reshape(-1, 1).astype(np.float64))
        assert ours <= km.inertia_ * (1 + 1e-9)
    # K = 3 on three blobs: Lloyd finds the optimum too
    k, bounds, taus, order = oracle.k_means(v, 3)
    km = KMeans(n_clusters=3, n_init=20, random_state=0).fit(v.reshape(-1, 1).astype(np.float64))
    assert abs(_partition_sse(v[order], bounds) - km.inertia_) <= 1e-6 * km.inertia_


def test_k_means_degenerate(oracle):
    k, bounds, taus, _ = oracle.k_means(np.full(6, 1.5, np.float32), 4)
    assert k == 1 and list(bounds) == [0, 6]
    k, bounds, taus, order = oracle.k_means(np.array([3, 1, 3, 2, 1], np.float32), 8)
    assert k == 3 and list(np.diff(bounds)) == [2, 1, 2]  # one cluster per distinct value
    k, bounds, taus, _ = oracle.k_means(np.array([7.0], np.float32), 3)
    assert k == 1


def _channel_outlier_data(rng, rows=256, C=192):
    x = rng.standard_normal((rows, C)).astype(np.float32)
    oc = np.array([5, 77, 130])
    # outlier channels: wide, but every pixel sees one of them high and one low, so that
    # the per-pixel extremes vary little and the per-channel ranges a lot
    sign = np.where(np.arange(rows) % 2 == 0, 1, -1).astype(np.float32)
    x[:, oc[0]] += np.float32(40.0) * sign
    x[:, oc[1]] -= np.float32(40.0) * sign
    x[:, oc[2]] += np.float32(40.0) * sign
    return x, oc


def _pixel_outlier_data(rng, rows=256, C=192):
    x = rng.standard_normal((rows, C)).astype(np.float32)
    op = np.array([3, 100, 101, 200])
    x[op] *= np.float32(30.0)
    return x, op


def test_variability_metric_and_dimension(oracle):
    """Eq. 4-5 retyped with array reductions; the constructed outliers select the dimension."""
    rng = np.random.default_rng(21)
    for make, want in ((_channel_outlier_data, 0), (_pixel_outlier_data, 1)):
        x, _ = make(rng)
        g = oracle.calibrate_kmeans(x, 8, 8, -1)
        cmx, cmn = x.max(0).astype(np.float64), x.min(0).astype(np.float64)
        rmx, rmn = x.max(1).astype(np.float64), x.min(1).astype(np.float64)
        assert g.D_channel == (cmx.max() - cmx.min()) + (cmn.max() - cmn.min())
        assert g.D_pixel == (rmx.max() - rmx.min()) + (rmn.max() - rmn.min())
        assert g.dstar == want and g.mode == want
        # a forced dimension is honoured and reports the same metric
        g2 = oracle.calibrate_kmeans(x, 8, 8, 1 - want)
        assert g2.mode == 1 - want and g2.dstar == want


def test_channel_mode_groups_and_cells(oracle):
    rng = np.random.default_rng(22)
    x, oc = _channel_outlier_data(rng)
    for bits in (8, 4):
        g = oracle.calibrate_kmeans(x, bits, 4, 0)
        assert g.P == 1 and g.NG == 4 and g.mode == 0
        width = (x.max(0) - x.min(0)).astype(np.float32)
        k, bounds, taus, order = oracle.k_means(width, 4)
        real = g.perm[g.perm >= 0]
        assert sorted(real.tolist()) == list(range(x.shape[1]))   # a permutation
        for k_ in range(g.NG):
            members = g.perm[g.goff[k_]: g.goff[k_] + g.glen[k_]]
            assert np.array_equal(members, order[bounds[k_]: bounds[k_ + 1]])
            assert g.goff[k_] % 64 == 0
            assert np.all(g.perm[g.goff[k_] + g.glen[k_]: g.goff[k_ + 1]] == -1)
            xs = x[:, members]
            s = (np.float32(xs.max()) - np.float32(xs.min())) / np.float32(2 ** bits)
            assert g.s[0, k_] == s and g.z[0, k_] == xs.min()
            assert g.inv_s[0, k_] == np.float32(1.0) / s
        # the widest cluster is the constructed outlier set
        top = g.perm[g.goff[g.NG - 1]: g.goff[g.NG - 1] + g.glen[g.NG - 1]]
        assert sorted(top.tolist()) == sorted(oc.tolist())
        # relabelling the channels relabels the groups and changes nothing else
        p = rng.permutation(x.shape[1])
        gp = oracle.calibrate_kmeans(np.ascontiguousarray(x[:, p]), bits, 4, 0)
        assert np.array_equal(gp.glen, g.glen) and np.array_equal(gp.s, g.s) and np.array_equal(gp.z, g.z)
        for k_ in range(g.NG):
            a = set(p[gp.perm[gp.goff[k_]: gp.goff[k_] + gp.glen[k_]]].tolist())
            b = set(g.perm[g.goff[k_]: g.goff[k_] + g.glen[k_]].tolist())
            assert a == b


def test_pixel_mode_classes_and_cells(oracle):
    rng = np.random.default_rng(23)
    x, op = _pixel_outlier_data(rng, rows=300, C=100)
    g = oracle.calibrate_kmeans(x, 8, 6, 1)
    assert g.NG == 1 and g.P == 6 and g.Kp == 128 and g.glen[0] == 100
    assert np.array_equal(g.perm[:100], np.arange(100)) and np.all(g.perm[100:] == -1)
    width = (x.max(1) - x.min(1)).astype(np.float32)
    cls = (width[:, None] > g.taus[None, :]).sum(1)
    assert np.array_equal(cls, g.cal_row_class)
    k, bounds, taus, order = oracle.k_means(width, 6)
    assert np.array_equal(np.bincount(cls, minlength=6), np.diff(bounds))
    for p in range(6):
        xs = x[cls == p]
        s = (np.float32(xs.max()) - np.float32(xs.min())) / np.float32(256)
        assert g.s[p, 0] == s and g.z[p, 0] == xs.min()
    # the constructed outlier pixels sit in the upper classes
    assert cls[op].min() > np.median(cls)
    # run-time classes of the same tensor are the calibration classes
    r = oracle.quantize_act(g, x, want_dq=True)
    assert np.array_equal(r["cls"], cls)
    # s = range / 2^b puts a class's maximum at level 2^b, one above the last code: that
    # one element per class saturates (a whole step off), everything else is within half
    # a step of its reconstruction
    assert r["clip"].sum() == 6
    for p in range(6):
        rows_p = np.flatnonzero(cls == p)
        i, j = np.unravel_index(np.argmax(x[rows_p]), (rows_p.size, 100))
        assert r["clip"][rows_p[i], j] == 1
    step = g.s[cls, 0][:, None].astype(np.float64)
    err = np.abs(r["xdq"] - x.astype(np.float64))
    slack = 1e-6 * float(np.abs(x).max())  # fp32 rounding of s and of the range
    assert np.all(err[r["clip"] == 0] <= (0.5 * step + slack)[:, [0] * 100][r["clip"] == 0])
    assert np.all(err <= step + slack)


def test_single_cluster_is_the_per_tensor_quantizer(oracle):
    """K = 1 along either dimension: one (s, z) for the whole tensor, i.e. Eq. 1."""
    rng = np.random.default_rng(24)
    x = rng.standard_normal((64, 128)).astype(np.float32)
    for dim in (0, 1):
        g = oracle.calibrate_kmeans(x, 8, 1, dim)
        assert g.P == 1 and g.NG == 1
        s = (x.max() - x.min()) / np.float32(256)
        assert g.s[0, 0] == s and g.z[0, 0] == x.min()
        r = oracle.quantize_act(g, x)
        q = np.clip(np.rint((x - x.min()) * (np.float32(1) / s)), 0, 255).astype(np.uint8)
        assert np.array_equal(r["q"][:, :128], q[:, g.perm[:128]])  # position j holds channel perm[j]


def test_grouping_error_not_worse_than_per_tensor(oracle):
    """What the grouping is for: on tensors with outliers of the grouped kind the
    reconstruction error falls as K grows (K = 1 is the per-tensor quantizer)."""
    rng = np.random.default_rng(25)
    for make, dim in ((_channel_outlier_data, 0), (_pixel_outlier_data, 1)):
        x, _ = make(rng)
        errs = []
        for K in (1, 2, 8, 16):
            g = oracle.calibrate_kmeans(x, 8, K, dim)
            r = oracle.quantize_act(g, x, want_dq=True)
            errs.append(float(np.mean((r["xdq"] - x) ** 2)))
        assert errs[1] < 0.2 * errs[0]
        assert errs[3] <= errs[2] <= errs[1]
