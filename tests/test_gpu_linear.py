"""GPU parity of calibration, the activation quantizer and the quantized linear
layer against the CPU oracle: integer results bit-exact, fp32 outputs within
1e-4 * max|ref|.  All calls go through the C ABI (via the thin binding)."""
import numpy as np
import pytest

import dgq_inputs as di
from support import assert_close_fp32, codes_to_q, gpu_groups_vs_oracle

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


def _run_layer(dgq, oracle, run, cal, act_bits, w_bits, G, P=2, bias=None, sample_rows=None,
               check_acc=True):
    """Calibrate, pack, quantize and contract on the GPU; compare every stage."""
    import torch
    og = oracle.calibrate(cal["X"], act_bits, G, P)
    gg = dgq.dgq_calibrate_groups(_dev(cal["X"]), act_bits, G, P)
    gpu_groups_vs_oracle(gg, og)

    X = run["X"]
    rows = X.shape[0]
    codes, cls = dgq.dgq_quantize_act(gg, _dev(X))
    torch.cuda.synchronize()
    oq = oracle.quantize_act(og, X)
    q_gpu = codes_to_q(codes.cpu().numpy(), act_bits, og.Kp, rows)
    real = og.perm >= 0
    assert np.array_equal(cls.cpu().numpy(), oq["cls"])
    assert np.array_equal(q_gpu[:, real], oq["q"][:, real])
    pad_val = 128 if act_bits == 8 else 0  # stored container 0
    assert np.all(q_gpu[:, ~real] == pad_val)

    W = run["W"]
    O = W.shape[0]
    wt = dgq.dgq_pack_weight(gg, _dev(W), None if bias is None else _dev(bias), w_bits)
    owq, osw = oracle.quantize_weight(W, w_bits)
    wtab = wt.tables()
    assert np.array_equal(wtab["wq"], owq)
    assert np.array_equal(wtab["sw"].view(np.uint32), osw.view(np.uint32))

    y = dgq.dgq_linear(gg, wt, codes, cls)
    torch.cuda.synchronize()
    sel = np.arange(rows) if sample_rows is None else np.asarray(sample_rows)
    sel_dev = torch.from_numpy(sel).cuda()
    y_sel = y[sel_dev].cpu().numpy()
    oy, oacc = oracle.linear(og, oq["q"][sel], oq["cls"][sel], owq, osw, bias, want_acc=check_acc)
    assert_close_fp32(y_sel, oy, "y")
    # the same bar per pixel class: the outlier rows are 25 times larger and would otherwise
    # set the scale of the tolerance for every regular row
    for p in np.unique(oq["cls"][sel]):
        m = oq["cls"][sel] == p
        assert_close_fp32(y_sel[m], oy[m], "y(class %d rows)" % p)
    if check_acc:
        # The accumulator dump runs the SAME tile shape as the plain launch (the launcher
        # picks the shape from the problem size alone), at full size: every int32 group
        # accumulator of the sampled rows against the oracle, and the dump launch's y
        # against the plain launch's y on the whole tensor, bit for bit (same fold order).
        dump = torch.full((rows, O, og.NG), -7, dtype=torch.int32, device="cuda")
        y2 = dgq.dgq_linear(gg, wt, codes, cls, acc_dump=dump)
        torch.cuda.synchronize()
        assert np.array_equal(dump[sel_dev].cpu().numpy(), oacc)
        assert torch.equal(y2.view(torch.int32), y.view(torch.int32))
        del dump, y2
    wt.free()
    gg.free()
    return og


def tile_rows(M, seed, extra=()):
    """One row of every 64-row tile (a random offset in each; the kernels' row tiles are 64 or
    128 rows), the tensor's first and last rows, and `extra`: a fault tied to a tile index
    cannot hide between the samples."""
    rng = np.random.default_rng(seed)
    starts = np.arange(0, M, 64)
    picks = np.minimum(starts + rng.integers(0, 64, size=len(starts)), M - 1)
    return np.unique(np.concatenate([picks, np.asarray(extra, dtype=np.int64), [0, M - 1]]))


SMALL = [
    # B, N, C, O, G, act_bits, w_bits, P
    (2, 150, 328, 200, 64, 8, 8, 2),   # ragged rows / channels / outputs
    (2, 150, 328, 200, 64, 4, 8, 2),
    (1, 77, 200, 130, 128, 8, 4, 2),
    (1, 5, 37, 3, 64, 8, 8, 2),        # C not a multiple of 4 (scalar loads), tiny
    (1, 1, 64, 1, 64, 4, 8, 1),        # single row, single class
    (2, 300, 640, 384, 128, 8, 8, 1),  # P = 1: the paper's pure channel grouping
    (3, 129, 192, 257, 64, 4, 4, 2),
]


@pytest.mark.parametrize("B,N,C,O,G,ab,wb,P", SMALL)
def test_small_layers(dgq, oracle, B, N, C, O, G, ab, wb, P):
    seed = 100 + C + O
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    if N < 8:  # too few tokens for the outlier-token recipe to leave a second class
        cal = run
    bias = np.random.default_rng(seed).standard_normal(O).astype(np.float32)
    _run_layer(dgq, oracle, run, cal, ab, wb, G, P, bias=bias)


@pytest.mark.parametrize("ab", [8, 4])
@pytest.mark.parametrize("B,N,C,O,G", [
    (2, 1111, 200, 1000, 64),   # 35 x 8 tiles of 64 x 128: the medium tile shape, ragged
    (2, 2500, 136, 1700, 64),   # 40 x 14 tiles of 128 x 128: the large tile shape, ragged
])
def test_ragged_medium_and_large_tiles(dgq, oracle, B, N, C, O, G, ab):
    """Row, channel and output counts that are no multiple of anything, at sizes where
    the launcher picks the 64 x 128 and the 128 x 128 tile (the small cases above all
    take the 64 x 64 one); oracle on sampled rows that include both ends of the edge tiles."""
    seed = 300 + C + O
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    M = B * N
    rng = np.random.default_rng(seed)
    edge = [0, 63, 64, 127, 128, M - 130, M - 65, M - 64, M - 2, M - 1]
    rows = np.unique(np.concatenate([rng.choice(M, 30, replace=False), run["rows_ot"][:6], edge]))
    bias = rng.standard_normal(O).astype(np.float32)
    _run_layer(dgq, oracle, run, cal, ab, 8, G, 2, bias=bias, sample_rows=rows)


def test_config1_full(dgq, oracle):
    """16x16 latent, 512 x 1280 -> 1280, G = 128, A8W8, seed 0; calibrated both
    on fresh data (clipping occurs) and on the tensor itself."""
    run = di.linear_case(0, 2, 256, 1280, 1280)
    cal = di.linear_case(0, 2, 256, 1280, 1280, calib=True)
    og = _run_layer(dgq, oracle, run, cal, 8, 8, 128)
    assert og.NG == 11 and og.Kp == 1344 and og.n_outlier_channels == 13
    _run_layer(dgq, oracle, run, run, 8, 8, 128, check_acc=False)


CFG2 = di.config2()


@pytest.mark.parametrize("li", range(len(CFG2["linears"])))
@pytest.mark.parametrize("mode", CFG2["modes"])
def test_config2_layers(dgq, oracle, li, mode):
    """64x64 latent: full-size GPU run, oracle on sampled rows (all outputs)."""
    name, M, B, N, C, O, G = CFG2["linears"][li]
    seed = di.layer_seed(CFG2["seed"], li)
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    rows = tile_rows(M, seed, np.concatenate([run["rows_ot"], [127, 128]]))
    _run_layer(dgq, oracle, run, cal, mode[0], mode[1], G, sample_rows=rows)


@pytest.mark.parametrize("mode", [(8, 8), (4, 8)])
@pytest.mark.parametrize("shape", [(16, 4096, 640, 640), (16, 4096, 640, 5120),
                                   (16, 4096, 2560, 640), (16, 1024, 1280, 1280),
                                   (16, 1024, 1280, 10240), (16, 1024, 5120, 1280),
                                   (16, 77, 2048, 640), (16, 77, 2048, 1280)])
def test_config5_sampled(dgq, oracle, shape, mode):
    """Every distinct launch shape of the SDXL-scale step bench.py times (q/k/v/out, ff.in
    and ff.out at both resolutions, the two projections of the 77-token prompt), both
    activation code widths, at full size; the oracle checks one row of every 128-row tile."""
    B, N, C, O = shape
    run = di.linear_case(5000 + C + O, B, N, C, O)
    cal = di.linear_case(5000 + C + O, B, N, C, O, calib=True)
    M = B * N
    rows = tile_rows(M, 1, run["rows_ot"][:4])
    _run_layer(dgq, oracle, run, cal, mode[0], mode[1], 128, sample_rows=rows)


def test_text_context_rows(dgq, oracle):
    """k/v projections of the text context: M = 2*77 rows (ragged tile), 768 -> 320."""
    run = di.linear_case(4105, 2, 77, 768, 320)
    cal = di.linear_case(4105, 2, 77, 768, 320, calib=True)
    _run_layer(dgq, oracle, run, cal, 8, 8, 64)


def test_error_paths(dgq):
    import torch
    run = di.linear_case(1, 1, 64, 128, 64)
    x = _dev(run["X"])
    g1 = dgq.dgq_calibrate_groups(x, 8, 64, 2)
    g2 = dgq.dgq_calibrate_groups(x, 8, 64, 2)
    w2 = dgq.dgq_pack_weight(g2, _dev(run["W"]), None, 8)
    codes, cls = dgq.dgq_quantize_act(g1, x)
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear(g1, w2, codes, cls)
    assert e.value.code == -3
    # misaligned input
    big = torch.zeros(64 * 128 + 4, dtype=torch.float32, device="cuda")
    xm = big[1:1 + 64 * 128].view(64, 128)
    with pytest.raises(dgq.DgqError) as e:
        dgq.lib().dgq_quantize_act  # noqa: B018
        dgq._check(dgq.lib().dgq_quantize_act(g1.handle, xm.data_ptr(), 64, codes.data_ptr(),
                                              cls.data_ptr(), None))
    assert e.value.code == -2
    torch.cuda.synchronize()


@pytest.mark.parametrize("ab", [8, 4])
@pytest.mark.parametrize("shape", [(2, 128, 320, 192, 64), (3, 333, 640, 200, 128), (4, 4096, 640, 1280, 128)])
def test_nibble_packed_weights(dgq, oracle, ab, shape):
    """4-bit weights stored two per byte: the same result, bit for bit, as the handle that
    keeps one weight per byte (which the tests above hold to the oracle), half the weight
    bytes, and the oracle's integer weights read back from the packed form."""
    import torch
    B, N, C, O, G = shape
    run = di.linear_case(9100 + C + O, B, N, C, O)
    cal = di.linear_case(9100 + C + O, min(B, 2), N, C, O, calib=True)
    og = oracle.calibrate(cal["X"], ab, G, 2)
    gg = dgq.dgq_calibrate_groups(_dev(cal["X"]), ab, G, 2)
    w = _dev(run["W"])
    bias = _dev(np.linspace(-1, 1, O).astype(np.float32))
    codes, cls = dgq.dgq_quantize_act(gg, _dev(run["X"]))
    wide = dgq.dgq_pack_weight(gg, w, bias, 4)
    packed = dgq.dgq_pack_weight(gg, w, bias, 4)
    b_wide = packed.device_bytes()
    assert dgq.dgq_linear_workspace_bytes(gg, packed, B * N) == 0
    packed.pack_nibbles()
    o_pad = (O + 127) // 128 * 128
    assert b_wide == o_pad * og.Kp + 12 * o_pad
    assert packed.device_bytes() == o_pad * og.Kp // 2 + 12 * o_pad
    need = dgq.dgq_linear_workspace_bytes(gg, packed, B * N)
    assert need == o_pad * og.Kp
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    y0 = dgq.dgq_linear(gg, wide, codes, cls)
    y1 = dgq.dgq_linear(gg, packed, codes, cls, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    # against the oracle directly, too (sampled rows on the large case)
    owq, osw = oracle.quantize_weight(run["W"], 4)
    t = packed.tables()
    assert np.array_equal(t["wq"], owq) and np.array_equal(t["sw"], osw)
    rows = B * N
    sel = np.arange(rows) if rows <= 2048 else tile_rows(rows, 5)
    oq = oracle.quantize_act(og, run["X"][sel])
    oy, _ = oracle.linear(og, oq["q"], oq["cls"], owq, osw, np.linspace(-1, 1, O).astype(np.float32))
    assert_close_fp32(y1[torch.from_numpy(sel).cuda()].cpu().numpy(), oy, "y")
    # a second call through the same workspace (another layer would reuse it)
    y2 = dgq.dgq_linear(gg, packed, codes, cls, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(y0, y2)
    # error paths: no or short workspace, other entry points, 8-bit weights, twice
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear(gg, packed, codes, cls)
    assert e.value.code == -6
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear(gg, packed, codes, cls, workspace=ws[:need - 16])
    assert e.value.code == -6
    with pytest.raises(dgq.DgqError) as e:
        packed.pack_nibbles()
    assert e.value.code == -3
    if O % 256 == 0:
        with pytest.raises(dgq.DgqError) as e:
            dgq.dgq_linear_geglu(gg, packed, codes, cls)
        assert e.value.code == -4
    w8 = dgq.dgq_pack_weight(gg, w, None, 8)
    with pytest.raises(dgq.DgqError) as e:
        w8.pack_nibbles()
    assert e.value.code == -4
