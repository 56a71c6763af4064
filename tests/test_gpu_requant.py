"""GPU parity of two chained feed-forward layers (dgq_pack_weight_gated_for +
dgq_linear_geglu_requant): the gated layer's epilogue writes the following layer's codes.

What is computed is a composition of steps the oracle already has, each pinned on its own:
quantize (Section 3.1 / 3.3) -> grouped contraction -> a * GELU(b) -> the following layer's
quantizer.  The oracle chain gives fp32 h and the codes q2 = rne((h - z) / s) of the
following layer.  The GPU's h differs from the oracle's by fp32 rounding (the allowance of
the gated layer, with a tenth of the contraction's bar: 1e-5 max|y| (|GELU(b)| + 1.13 |a|)
+ the activation's own bound), and a code
is a rounding decision on h, so the comparison is the one used for the attention codes:

  * every code whose decision is at least that allowance (in units of the step) away
    from a half-integer must be equal, and those are nearly all codes;
  * the others may differ by one;
  * and, on the GPU alone, the fused codes are bit-identical to dgq_quantize_act applied
    to the fp32 output of dgq_linear_geglu (same kernel arithmetic up to the store), which
    pins the layout, the padding and the row handling for every element.
"""
import numpy as np
import pytest

import dgq_inputs as di
from support import codes_to_q, gpu_groups_vs_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2501_04304_amd as m
    m.lib()
    return m


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _gelu64(t):
    from math import erf, sqrt
    return np.array([x * 0.5 * (1.0 + erf(x / sqrt(2.0))) for x in t.ravel()]).reshape(t.shape)


def _oracle_h(oracle, og1, X, W, bias):
    oq = oracle.quantize_act(og1, X)
    owq, osw = oracle.quantize_weight(W, 8)
    oy, _ = oracle.linear(og1, oq["q"], oq["cls"], owq, osw, bias)
    return oy, oracle.geglu(oy)


def _run(dgq, oracle, B, N, C1, C2, G, act_bits, seed, next_kind, K=8, sample=None, cal_rows=256,
         next_bits=8, run_rows=None):
    """Layer 1: C1 -> 2 C2 (hybrid grid, two pixel classes, act_bits codes); layer 2 takes
    the C2 gated channels with 8-bit codes and channel groups only."""
    import torch
    O = 2 * C2
    run = di.linear_case(seed, B, N, C1, O)
    cal = di.linear_case(seed, B, N, C1, O, calib=True)
    X, W = run["X"], run["W"] * np.float32(8.0)   # pre-activations of order one, so GELU bends
    if run_rows is not None:                        # a few rows of the same layer
        X = np.ascontiguousarray(X[:run_rows])
    rows = X.shape[0]
    bias = (np.random.default_rng(seed).standard_normal(O) * 0.3).astype(np.float32)
    sel = np.arange(rows) if sample is None else np.asarray(sample)

    og1 = oracle.calibrate(cal["X"], act_bits, G, 2)
    g1 = dgq.dgq_calibrate_groups(_dev(cal["X"]), act_bits, G, 2)
    gpu_groups_vs_oracle(g1, og1)

    # the following layer is calibrated on the oracle's gated activation of calibration rows
    rng = np.random.default_rng(seed + 1)
    n_cal = cal["X"].shape[0]
    crow = np.sort(rng.choice(n_cal, min(cal_rows, n_cal), replace=False))
    _, hcal = _oracle_h(oracle, og1, cal["X"][crow], W, bias)
    if next_kind == "kmeans":
        og2 = oracle.calibrate_kmeans(hcal, next_bits, K, 0)
        g2 = dgq.dgq_calibrate_kmeans(_dev(hcal), next_bits, K, dgq.DIM_CHANNEL)
    else:
        og2 = oracle.calibrate(hcal, next_bits, 64, 1)
        g2 = dgq.dgq_calibrate_groups(_dev(hcal), next_bits, 64, 1)
    assert g2.info.n_pixel_classes == 1 and g2.info.k_padded == og2.Kp
    t2 = g2.tables()
    assert np.array_equal(t2["perm"], og2.perm)
    assert np.array_equal(t2["s"][:1].view(np.uint32), og2.s[:1].view(np.uint32))
    assert np.array_equal(t2["z"][:1].view(np.uint32), og2.z[:1].view(np.uint32))

    # GPU, fused
    codes1, cls1 = dgq.dgq_quantize_act(g1, _dev(X))
    wt_f = dgq.dgq_pack_weight_gated_for(g1, g2, _dev(W), _dev(bias), 8)
    shape2 = dgq.codes_shape(g2, rows)
    codes2 = torch.full(shape2, 0x55, dtype=torch.int8, device="cuda")
    cls2 = torch.full((rows,), 9, dtype=torch.uint8, device="cuda")
    dgq.dgq_linear_geglu_requant(g1, wt_f, codes1, cls1, g2, codes_next=codes2, row_class_next=cls2)
    # GPU, step by step
    wt = dgq.dgq_pack_weight(g1, _dev(W), _dev(bias), 8)
    h_gpu = dgq.dgq_linear_geglu(g1, wt, codes1, cls1)
    codes2s = torch.full(shape2, 0x55, dtype=torch.int8, device="cuda")
    codes2s, cls2s = dgq.dgq_quantize_act(g2, h_gpu, codes=codes2s)
    torch.cuda.synchronize()
    assert torch.equal(codes2, codes2s), "fused codes differ from quantize_act(geglu output)"
    assert torch.equal(cls2, cls2s) and int(cls2.max()) == 0

    # oracle chain on the selected rows
    oy, h = _oracle_h(oracle, og1, X[sel], W, bias)
    oq2 = oracle.quantize_act(og2, h)
    q_gpu = codes_to_q(codes2.cpu().numpy(), next_bits, og2.Kp, rows)[sel].astype(np.int64)
    real = og2.perm >= 0
    assert np.all(q_gpu[:, ~real] == (128 if next_bits == 8 else 0))   # stored 0 at padding positions
    q_ref = oq2["q"][:, real].astype(np.int64)
    q_got = q_gpu[:, real]
    # distance of each decision from a rounding boundary, in steps, from the oracle's h
    ch = og2.perm[real]
    grp = np.repeat(np.arange(og2.NG), og2.glen)     # group of each real position, in order
    assert grp.size == ch.size
    z = og2.z[0][grp].astype(np.float64)
    s = og2.s[0][grp].astype(np.float64)
    u = (h[:, ch].astype(np.float64) - z) / s
    margin = np.abs(u - np.floor(u) - 0.5)
    a, b = oy[:, :C2].astype(np.float64), oy[:, C2:].astype(np.float64)
    # the contraction's fp32 error is far inside its 1e-4 max|y| bar (a few 1e-6 measured):
    # a tenth of the bar is allowed here, so that "decided" covers nearly every code
    allow_h = 1e-5 * np.abs(oy).max() * (np.abs(_gelu64(b)) + 1.13 * np.abs(a)) \
        + 2e-6 * np.abs(h) + 5e-7 * np.abs(a).max() * np.abs(b).max()
    allow_u = allow_h[:, ch] / s
    inside = (u > -0.5) & (u < (1 << next_bits) - 0.5)   # outside, both sides saturate
    decided = (margin >= allow_u) | ~inside
    diff = q_got != q_ref
    assert not (diff & decided).any(), "%d decided codes differ" % int((diff & decided).sum())
    assert np.abs(q_got - q_ref).max() <= 1
    assert diff.mean() < 2e-3, "too many codes differ: %.2e" % diff.mean()
    if run_rows is None:
        assert np.unique(q_ref).size > (30 if next_bits == 8 else 8)  # not a trivial case
    for hnd in (wt_f, wt, g1, g2):
        hnd.free()
    return float(decided.mean()), float(diff.mean())


@pytest.mark.parametrize("next_kind", ["kmeans", "blocks"])
@pytest.mark.parametrize("B,N,C1,C2,G,ab", [
    (2, 150, 328, 256, 64, 8),     # 64 x 64 tiles (half a chunk per tile), ragged rows
    (1, 77, 200, 128, 128, 8),     # one column tile pair
    (2, 1111, 200, 640, 64, 4),    # 64 x 128 tiles, 4-bit codes in, ragged rows
    (2, 2500, 136, 896, 64, 8),    # 128 x 128 tiles, ragged rows
])
def test_small_and_ragged(dgq, oracle, B, N, C1, C2, G, ab, next_kind):
    M = B * N
    sample = None
    if M > 1000:
        rng = np.random.default_rng(C2)
        sample = np.unique(np.concatenate([rng.choice(M, 40, replace=False),
                                           [0, 15, 16, 63, 64, 127, 128, M - 130, M - 17, M - 16, M - 1]]))
    decided, _ = _run(dgq, oracle, B, N, C1, C2, G, ab, 900 + C1 + C2, next_kind, sample=sample)
    assert decided > 0.9


@pytest.mark.parametrize("next_kind", ["kmeans", "blocks"])
@pytest.mark.parametrize("B,N,C1,C2,G,ab", [
    (2, 150, 328, 256, 64, 8),
    (2, 1111, 200, 640, 64, 4),
    (2, 2500, 136, 896, 64, 8),
])
def test_four_bit_codes_for_the_following_layer(dgq, oracle, B, N, C1, C2, G, ab, next_kind):
    M = B * N
    sample = None
    if M > 1000:
        rng = np.random.default_rng(C2 + 1)
        sample = np.unique(np.concatenate([rng.choice(M, 40, replace=False),
                                           [0, 31, 32, 63, 64, 127, 128, M - 130, M - 33, M - 32, M - 1]]))
    decided, _ = _run(dgq, oracle, B, N, C1, C2, G, ab, 950 + C1 + C2, next_kind, sample=sample,
                      next_bits=4)
    assert decided > 0.99


@pytest.mark.parametrize("next_bits", [8, 4])
@pytest.mark.parametrize("rows", [1, 17, 33])
def test_a_few_rows(dgq, oracle, rows, next_bits):
    """Fewer rows than one code block of the following layer, and one more than a block."""
    _run(dgq, oracle, 2, 150, 328, 256, 64, 8, 1234, "kmeans", run_rows=rows, next_bits=next_bits)


def test_config5_feed_forward_sampled(dgq, oracle):
    """ff.in -> ff.out of the SDXL-scale sweep at full size (16384 x 1280 -> 2 x 5120 ->
    codes of the 5120-channel layer), sampled rows."""
    B, N, C1, C2 = 16, 1024, 1280, 5120
    M = B * N
    rng = np.random.default_rng(3)
    sample = np.unique(np.concatenate([rng.choice(M, 12, replace=False), [0, M - 1]]))
    _run(dgq, oracle, B, N, C1, C2, 128, 8, 5300, "kmeans", K=16, sample=sample, cal_rows=48)


def test_argument_errors(dgq):
    run = di.linear_case(3, 1, 64, 128, 512)
    x = _dev(run["X"])
    g1 = dgq.dgq_calibrate_groups(x, 8, 64, 2)
    h = _dev(np.random.default_rng(0).standard_normal((64, 256)).astype(np.float32))
    g2 = dgq.dgq_calibrate_kmeans(h, 8, 4, dgq.DIM_CHANNEL)
    g2p = dgq.dgq_calibrate_kmeans(h, 8, 4, dgq.DIM_PIXEL)       # needs a row statistic
    w = _dev(run["W"])
    for bad in (g2p,):
        with pytest.raises(dgq.DgqError) as e:
            dgq.dgq_pack_weight_gated_for(g1, bad, w, None, 8)
        assert e.value.code == -4
    with pytest.raises(dgq.DgqError) as e:                       # 128 channels, not 512 / 2
        dgq.dgq_pack_weight_gated_for(g1, g1, w, None, 8)
    assert e.value.code == -3
    wf = dgq.dgq_pack_weight_gated_for(g1, g2, w, None, 8)
    wp = dgq.dgq_pack_weight(g1, w, None, 8)
    codes, cls = dgq.dgq_quantize_act(g1, x)
    with pytest.raises(dgq.DgqError) as e:                       # a chained weight in the plain calls
        dgq.dgq_linear(g1, wf, codes, cls)
    assert e.value.code == -3
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_linear_geglu(g1, wf, codes, cls)
    assert e.value.code == -3
    with pytest.raises(dgq.DgqError) as e:                       # and a plain weight in the chained call
        dgq.dgq_linear_geglu_requant(g1, wp, codes, cls, g2)
    assert e.value.code == -3
    import torch
    torch.cuda.synchronize()
    for hnd in (wf, wp, g1, g2, g2p):
        hnd.free()
