"""GPU parity of the contraction with the gated feed-forward activation fused into its
epilogue (dgq_linear_geglu) against the CPU oracle.

Two comparisons per case.  (1) The fused kernel forms y exactly as dgq_linear does (same
accumulators, same fold order, same scale/offset FMA), so against oracle.geglu applied to
the GPU's own unfused y only the activation differs: the kernel takes Phi from a rational
approximation of erfc (absolute error 1.5e-7 by construction, 3.2e-7 |t| on GELU(t) with its
fp32 arithmetic, checked on the CPU over [-12, 12]) and multiplies in fp32, i.e.
|err| <= 2e-6 |ref| + 5e-7 max|a| max|b|.  (2) Against the whole
oracle chain the 1e-4 * max|y| allowance of the contraction passes through the activation:
|err| <= 1e-4 max|y| (|GELU(b)| + 1.13 |a|) + the bound of (1), 1.13 being max |GELU'|.
"""
import numpy as np
import pytest

import dgq_inputs as di

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2501_04304_amd as m
    m.lib()  # fails loudly if libdgq.so is missing
    return m


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _gelu64(t):
    from math import erf, sqrt
    return np.array([x * 0.5 * (1.0 + erf(x / sqrt(2.0))) for x in t.ravel()]).reshape(t.shape)


def _run(dgq, oracle, B, N, C, O, G, act_bits, seed, sample_rows=None):
    import torch
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    X, W = run["X"], run["W"]
    rows = X.shape[0]
    bias = np.random.default_rng(seed).standard_normal(O).astype(np.float32)
    gg = dgq.dgq_calibrate_groups(_dev(cal["X"]), act_bits, G, 2)
    wt = dgq.dgq_pack_weight(gg, _dev(W), _dev(bias), 8)
    codes, cls = dgq.dgq_quantize_act(gg, _dev(X))
    y = dgq.dgq_linear(gg, wt, codes, cls)
    out = dgq.dgq_linear_geglu(gg, wt, codes, cls)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (rows, O // 2)
    y_np, out_np = y.cpu().numpy(), out.cpu().numpy().astype(np.float64)
    sel = np.arange(rows) if sample_rows is None else np.asarray(sample_rows)

    # (1) the activation alone
    ref1 = oracle.geglu(y_np[sel]).astype(np.float64)
    a, b = y_np[sel, :O // 2].astype(np.float64), y_np[sel, O // 2:].astype(np.float64)
    lim1 = 2e-6 * np.abs(ref1) + 5e-7 * np.abs(a).max() * np.abs(b).max()
    err1 = np.abs(out_np[sel] - ref1)
    assert (err1 <= lim1).all(), "activation: worst excess %.3e" % (err1 - lim1).max()

    # (2) the whole chain
    og = oracle.calibrate(cal["X"], act_bits, G, 2)
    oq = oracle.quantize_act(og, X[sel])
    owq, osw = oracle.quantize_weight(W, 8)
    oy, _ = oracle.linear(og, oq["q"], oq["cls"], owq, osw, bias)
    ref2 = oracle.geglu(oy).astype(np.float64)
    oa, ob = oy[:, :O // 2].astype(np.float64), oy[:, O // 2:].astype(np.float64)
    lim2 = 1e-4 * np.abs(oy).max() * (np.abs(_gelu64(ob)) + 1.13 * np.abs(oa)) + lim1
    err2 = np.abs(out_np[sel] - ref2)
    assert (err2 <= lim2).all(), "chain: worst excess %.3e" % (err2 - lim2).max()
    wt.free()
    gg.free()


@pytest.mark.parametrize("act_bits", [8, 4])
@pytest.mark.parametrize("B,N,C,O,G", [
    (2, 150, 328, 512, 64),     # 64 x 64 tiles, ragged rows and channels
    (1, 77, 200, 256, 128),     # a single pair of column tiles
    (2, 1111, 200, 1024, 64),   # 64 x 128 tiles, ragged rows
    (2, 2500, 136, 1792, 64),   # 128 x 128 tiles, ragged rows
])
def test_small_and_ragged(dgq, oracle, B, N, C, O, G, act_bits):
    M = B * N
    rows = None
    if M > 1000:
        rng = np.random.default_rng(O)
        rows = np.unique(np.concatenate([rng.choice(M, 30, replace=False),
                                         [0, 63, 64, 127, 128, M - 130, M - 65, M - 64, M - 1]]))
    _run(dgq, oracle, B, N, C, O, G, act_bits, 700 + C + O, rows)


@pytest.mark.parametrize("shape", [(16, 4096, 640, 5120), (16, 1024, 1280, 10240)])
def test_config5_feed_forward_sampled(dgq, oracle, shape):
    """The two gated projections of the SDXL-scale sweep at full size, sampled rows."""
    B, N, C, O = shape
    M = B * N
    rng = np.random.default_rng(2)
    rows = np.unique(np.concatenate([rng.choice(M, 16, replace=False), [0, M - 1]]))
    _run(dgq, oracle, B, N, C, O, 128, 8, 5200 + C, rows)


def test_rejects_widths_it_cannot_pair(dgq):
    run = di.linear_case(3, 1, 64, 128, 384)  # 384 is not a multiple of 256
    x = _dev(run["X"])
    gg = dgq.dgq_calibrate_groups(x, 8, 64, 2)
    wt = dgq.dgq_pack_weight(gg, _dev(run["W"]), None, 8)
    codes, cls = dgq.dgq_quantize_act(gg, x)
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear_geglu(gg, wt, codes, cls)
    assert e.value.code == -4
    wt.free()
    gg.free()
