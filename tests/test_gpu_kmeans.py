"""GPU parity of the single-dimension grouping of Section 3.3 (K clusters of channels or
of pixels by range, Eq. 4-6; one handle per timestep, Eq. 7) against the CPU oracle:
tables, thresholds, classes and codes bit-exact, fp32 outputs within 1e-4 * max|ref|.
All calls go through the C ABI (via the thin binding)."""
import numpy as np
import pytest

import dgq_inputs as di
from support import assert_close_fp32, codes_to_q

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2501_04304_amd as m
    m.lib()  # fails loudly if libdgq.so is missing
    return m


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _groups_equal(gg, og):
    inf = gg.info
    assert inf.channels == og.C and inf.act_bits == og.act_bits
    assert inf.n_groups == og.NG and inf.k_padded == og.Kp
    assert inf.n_pixel_classes == og.P
    assert inf.grouping == (1 if og.mode == 0 else 2)
    assert inf.dstar == og.dstar
    assert inf.d_channel == og.D_channel and inf.d_pixel == og.D_pixel
    assert inf.n_class1_rows == og.n_class1_rows
    assert inf.code_offset == (128 if og.act_bits == 8 else 0)
    t = gg.tables()
    assert np.array_equal(t["perm"], og.perm)
    assert np.array_equal(t["goff"], og.goff)
    assert np.array_equal(t["glen"], og.glen)
    assert np.array_equal(t["s"][:og.P].view(np.uint32), og.s.view(np.uint32))
    assert np.array_equal(t["z"][:og.P].view(np.uint32), og.z.view(np.uint32))
    if og.P > 1:
        assert np.array_equal(t["taus"].view(np.uint32), og.taus.view(np.uint32))


def _run(dgq, oracle, X, Xcal, W, act_bits, w_bits, K, dim, bias=None, sample_rows=None,
         check_acc=False):
    import torch
    og = oracle.calibrate_kmeans(Xcal, act_bits, K, dim)
    gg = dgq.dgq_calibrate_kmeans(_dev(Xcal), act_bits, K, dim)
    _groups_equal(gg, og)
    rows = X.shape[0]
    codes, cls = dgq.dgq_quantize_act(gg, _dev(X))
    torch.cuda.synchronize()
    oq = oracle.quantize_act(og, X)
    q_gpu = codes_to_q(codes.cpu().numpy(), act_bits, og.Kp, rows)
    real = og.perm >= 0
    assert np.array_equal(cls.cpu().numpy(), oq["cls"])
    assert np.array_equal(q_gpu[:, real], oq["q"][:, real])
    assert np.all(q_gpu[:, ~real] == (128 if act_bits == 8 else 0))
    wt = dgq.dgq_pack_weight(gg, _dev(W), None if bias is None else _dev(bias), w_bits)
    owq, osw = oracle.quantize_weight(W, w_bits)
    y = dgq.dgq_linear(gg, wt, codes, cls)
    torch.cuda.synchronize()
    y_np = y.cpu().numpy()
    sel = np.arange(rows) if sample_rows is None else np.asarray(sample_rows)
    oy, oacc = oracle.linear(og, oq["q"][sel], oq["cls"][sel], owq, osw, bias, want_acc=check_acc)
    assert_close_fp32(y_np[sel], oy, "y")
    if check_acc:
        O = W.shape[0]
        dump = torch.full((rows, O, og.NG), -7, dtype=torch.int32, device="cuda")
        y2 = dgq.dgq_linear(gg, wt, codes, cls, acc_dump=dump)
        torch.cuda.synchronize()
        assert np.array_equal(dump.cpu().numpy()[sel], oacc)
        assert_close_fp32(y2.cpu().numpy()[sel], oy, "y(dump)")
    res = dict(og=og, cls=oq["cls"], y=y_np, gg=gg, wt=wt, codes=codes, cls_dev=cls)
    return res


def _free(res):
    res["wt"].free()
    res["gg"].free()


SMALL = [
    # B, N, C, O, act_bits, w_bits, K, dim
    (2, 150, 328, 200, 8, 8, 8, 1),    # pixel grouping, ragged everything
    (2, 150, 328, 200, 4, 8, 16, 1),
    (2, 150, 328, 200, 8, 8, 8, 0),    # channel grouping, free-size groups
    (2, 150, 328, 200, 4, 4, 16, 0),
    (1, 77, 200, 130, 8, 4, 3, 1),
    (1, 5, 37, 3, 8, 8, 4, 1),         # C not a multiple of 4 (scalar loads), tiny
    (1, 5, 37, 3, 8, 8, 4, 0),
    (3, 129, 192, 257, 4, 8, 16, -1),  # the dimension chosen by D_d
    (2, 300, 640, 384, 8, 8, 2, 1),    # two pixel classes: the two-class kernels
    (2, 300, 640, 384, 8, 8, 1, 1),    # one cluster: the per-tensor quantizer
]


@pytest.mark.parametrize("B,N,C,O,ab,wb,K,dim", SMALL)
def test_small_layers(dgq, oracle, B, N, C, O, ab, wb, K, dim):
    seed = 700 + C + O + K
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    if N < 8:
        cal = run
    bias = np.random.default_rng(seed).standard_normal(O).astype(np.float32)
    res = _run(dgq, oracle, run["X"], cal["X"], run["W"], ab, wb, K, dim, bias=bias,
               check_acc=(dim == 0 or K <= 2))
    og = res["og"]
    if dim == 1 and K > 2 and B * N > 100:
        assert og.P == K and og.NG == 1 and len(np.unique(res["cls"])) > 2
    if dim == 0 and B * N > 100:
        assert og.P == 1 and og.NG == K
    _free(res)


@pytest.mark.parametrize("ab", [8, 4])
@pytest.mark.parametrize("B,N,C,O,K", [
    (2, 1111, 200, 1000, 8),    # the 64 x 128 tile shape, ragged
    (2, 2500, 136, 1700, 16),   # the 128 x 128 tile shape, ragged
])
def test_pixel_grouping_medium_and_large_tiles(dgq, oracle, B, N, C, O, K, ab):
    seed = 900 + C + O
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    M = B * N
    rng = np.random.default_rng(seed)
    edge = [0, 63, 64, 127, 128, M - 130, M - 65, M - 64, M - 2, M - 1]
    rows = np.unique(np.concatenate([rng.choice(M, 30, replace=False), run["rows_ot"][:6], edge]))
    bias = rng.standard_normal(O).astype(np.float32)
    res = _run(dgq, oracle, run["X"], cal["X"], run["W"], ab, 8, K, 1, bias=bias, sample_rows=rows)
    assert res["og"].P == K
    _free(res)


def test_pixel_grouping_uniform_and_mixed_wavefronts(dgq, oracle):
    """Rows sorted by range: most 32-row blocks then hold one class (the scalar path of
    the kernel), the blocks at the class boundaries several (the per-register path)."""
    run = di.linear_case(1234, 2, 1024, 320, 320)
    X = run["X"]
    order = np.argsort(X.max(1) - X.min(1), kind="stable")
    Xs = np.ascontiguousarray(X[order])
    res = _run(dgq, oracle, Xs, Xs, run["W"], 8, 8, 8, 1)
    cls = res["cls"].reshape(-1, 32)
    uniform = (cls.min(1) == cls.max(1))
    assert uniform.sum() > 10 and (~uniform).sum() >= 3
    assert len(np.unique(cls[uniform][:, 0])) >= 3   # uniform blocks of several classes
    _free(res)


def test_channel_grouping_config1(dgq, oracle):
    """16x16 latent, 512 x 1280 -> 1280: K = 16 channel clusters of whatever size the
    clustering gives (the largest has several hundred channels), accumulators exact."""
    run = di.linear_case(0, 2, 256, 1280, 1280)
    cal = di.linear_case(0, 2, 256, 1280, 1280, calib=True)
    res = _run(dgq, oracle, run["X"], cal["X"], run["W"], 8, 8, 16, 0, check_acc=True)
    og = res["og"]
    assert og.NG == 16 and og.glen.max() > 128 and og.glen.sum() == 1280
    _free(res)


@pytest.mark.parametrize("dim", [0, 1])
def test_sdxl_scale_sampled(dgq, oracle, dim):
    """A config-5 layer (65536 x 640 -> 640) in the launch configuration bench.py times,
    K = 16, calibrated on two of the sixteen batch elements; oracle on sampled rows."""
    B, N, C, O = 16, 4096, 640, 640
    run = di.linear_case(5000 + C + O, B, N, C, O)
    cal_full = di.linear_case(5000 + C + O, B, N, C, O, calib=True)
    cal = np.ascontiguousarray(cal_full["X"][: 2 * N])
    M = B * N
    rng = np.random.default_rng(2)
    rows = np.unique(np.concatenate([rng.choice(M, 24, replace=False), run["rows_ot"][:4],
                                     [0, M - 1]]))
    res = _run(dgq, oracle, run["X"], cal, run["W"], 8, 8, 16, dim, sample_rows=rows)
    _free(res)


def test_timestep_tables(dgq, oracle):
    """Eq. 7: one (S, Z) entry per denoising step.  Three steps whose activations differ in
    scale get their own handles; each step's tensor is coded with its own entry."""
    base = di.linear_case(77, 2, 200, 256, 128)
    scales = [1.0, 0.35, 2.5]
    handles, ogs = [], []
    for t, sc in enumerate(scales):
        Xt = (base["X"] * np.float32(sc)).astype(np.float32)
        handles.append(dgq.dgq_calibrate_kmeans(_dev(Xt), 8, 8, 1))
        ogs.append(oracle.calibrate_kmeans(Xt, 8, 8, 1))
        _groups_equal(handles[-1], ogs[-1])
    import torch
    for t, sc in enumerate(scales):
        Xt = (base["X"] * np.float32(sc)).astype(np.float32)
        codes, cls = dgq.dgq_quantize_act(handles[t], _dev(Xt))
        torch.cuda.synchronize()
        oq = oracle.quantize_act(ogs[t], Xt)
        q = codes_to_q(codes.cpu().numpy(), 8, ogs[t].Kp, Xt.shape[0])
        real = ogs[t].perm >= 0
        assert np.array_equal(q[:, real], oq["q"][:, real])
        assert np.array_equal(cls.cpu().numpy(), oq["cls"])
    # the entries differ: step 1's thresholds are step 0's scaled
    assert not np.array_equal(ogs[0].taus, ogs[1].taus)
    for h in handles:
        h.free()


def test_fewer_distinct_ranges_than_clusters(dgq, oracle):
    """Identical rows give one pixel class however many are asked for."""
    rng = np.random.default_rng(5)
    row = rng.standard_normal(128).astype(np.float32)
    X = np.tile(row, (40, 1))
    X[20:] *= np.float32(3.0)          # two distinct ranges
    W = rng.standard_normal((64, 128)).astype(np.float32)
    res = _run(dgq, oracle, X, X, W, 8, 8, 8, 1)
    assert res["og"].P == 2
    _free(res)
    X1 = np.tile(row, (40, 1))
    res = _run(dgq, oracle, X1, X1, W, 8, 8, 8, 1)
    assert res["og"].P == 1
    _free(res)


def test_unsupported_combinations(dgq):
    import torch
    run = di.linear_case(3, 2, 128, 256, 512)
    x = _dev(run["X"])
    g = dgq.dgq_calibrate_kmeans(x, 8, 8, 1)
    assert g.info.n_pixel_classes == 8
    w = dgq.dgq_pack_weight(g, _dev(run["W"]), None, 8)
    codes, cls = dgq.dgq_quantize_act(g, x)
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear_geglu(g, w, codes, cls)
    assert e.value.code == -4
    dump = torch.zeros((256, 512, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear(g, w, codes, cls, acc_dump=dump)
    assert e.value.code == -4
    # more rows than the former limit of the pixel dimension, all of one range: one class
    big = torch.zeros((40000, 64), dtype=torch.float32, device="cuda")
    gb = dgq.dgq_calibrate_kmeans(big, 8, 8, 1)
    assert gb.info.n_pixel_classes == 1
    gb.free()
    torch.cuda.synchronize()
    w.free()
    g.free()


@pytest.mark.parametrize("K", [8, 16])
def test_pixel_clustering_of_many_rows_against_the_definition(dgq, oracle, K):
    """The library clusters by divide and conquer over the monotone best cuts, the oracle by the
    O(K n^2) definition: thresholds, class sizes and cell tables of 12288 calibration rows
    (three 64 x 64 latents, heavy-tailed ranges with repeated values) must be equal bit for bit."""
    rng = np.random.default_rng(60 + K)
    n, C = 12288, 64
    X = rng.standard_normal((n, C)).astype(np.float32)
    X *= np.exp(rng.standard_normal((n, 1)) * 0.8).astype(np.float32)       # ranges over octaves
    X[rng.choice(n, 40, replace=False)] *= 25.0
    X[1000:1400] = X[1000]                                                  # repeated ranges
    og = oracle.calibrate_kmeans(X, 8, K, 1)
    gg = dgq.dgq_calibrate_kmeans(_dev(X), 8, K, dgq.DIM_PIXEL)
    _groups_equal(gg, og)
    gg.free()


def test_pixel_clustering_of_a_whole_calibration_set(dgq):
    """64 prompts x 4096 pixels = 262144 calibration rows (Section 4.1's calibration set; the
    O(n^2) definition would take hours): the clustering returns, the thresholds ascend, every
    class is populated at run time, and its cost is no worse than that of equal-count classes."""
    import torch
    rng = np.random.default_rng(61)
    n, C, K = 64 * 4096, 64, 16
    X = rng.standard_normal((n, C)).astype(np.float32)
    X *= np.exp(rng.standard_normal((n, 1)) * 0.7).astype(np.float32)
    X[rng.choice(n, 128, replace=False)] *= 25.0
    xd = _dev(X)
    gg = dgq.dgq_calibrate_kmeans(xd, 8, K, dgq.DIM_PIXEL)
    assert gg.info.n_pixel_classes == K
    taus = gg.tables()["taus"].astype(np.float64)
    assert np.all(np.diff(taus) > 0)
    width = (X.max(1) - X.min(1)).astype(np.float64)
    cls_ref = (width[:, None] > taus[None, :]).sum(1)
    codes, cls = dgq.dgq_quantize_act(gg, xd)
    torch.cuda.synchronize()
    assert np.array_equal(cls.cpu().numpy(), cls_ref.astype(np.uint8))
    assert np.bincount(cls_ref, minlength=K).min() > 0

    def sse(labels):
        return sum(((width[labels == c] - width[labels == c].mean()) ** 2).sum() for c in range(K))
    order = np.argsort(width, kind="stable")
    equal = np.empty(n, np.int64)
    equal[order] = np.arange(n) * K // n
    assert sse(cls_ref) <= sse(equal)
    gg.free()
