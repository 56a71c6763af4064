"""GPU parity of the self-attention with log2-quantized probabilities (dgq_selfattn_logq)
against the CPU oracle.

A code is a rounding decision on -log2(A / s); the kernel evaluates that quantity in the log
domain in fp32, the oracle in double from the fp32 probability.  As for the cross-attention
codes the two must agree wherever the decision is at least DELTA = 2^-13 (log2 units) from
a rounding boundary and may differ by one elsewhere; the product is compared (1e-4 max|ref|)
on the rows that hold no such marginal code.  The scale is an input; scale_out (max A) is
compared to 1e-5 relative."""
import numpy as np
import pytest

import dgq_inputs as di
from support import assert_close_fp32

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


def _check(dgq, oracle, c, bits, s_in, sel=None, min_good=0.2):
    import torch
    from oracle.guard import DELTA
    B, N, H, d = c["Q"].shape
    codes = torch.full((B, H, N, N), 0xEE, dtype=torch.uint8, device="cuda")
    s_out = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
    out = dgq.dgq_selfattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]), bits, _dev(s_in),
                                scale_out=s_out, codes_dump=codes)
    # and without the optional outputs: the same product
    out2 = dgq.dgq_selfattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]), bits, _dev(s_in))
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    sel = np.arange(N) if sel is None else np.asarray(sel)
    ref = oracle.selfattn(c["Q"][:, sel], c["K"], c["V"], bits, s_in)
    got_codes = codes[:, :, torch.from_numpy(sel).cuda()].cpu().numpy()
    got_out = out.cpu().numpy()[:, sel]
    safe = ref["margin"] >= DELTA
    assert np.array_equal(got_codes[safe], ref["codes"][safe])
    assert np.abs(got_codes.astype(int) - ref["codes"].astype(int)).max() <= 1
    assert safe.mean() > 0.999
    good = np.transpose(safe.all(-1), (0, 2, 1))          # [B, Nsel, H]: rows without a marginal code
    assert good.mean() > min_good
    err = np.abs(got_out - ref["out"])[good]
    assert err.max() <= 1e-4 * np.abs(ref["out"]).max(), err.max() / np.abs(ref["out"]).max()
    if len(sel) == N:
        assert np.all(np.abs(s_out.cpu().numpy() - ref["s"]) <= 1e-5 * ref["s"])
    return ref


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("B,N,H,d", [
    (2, 200, 2, 40),    # ragged last key tile and last query block, head dim padded to 48
    (1, 64, 3, 64),
    (1, 33, 1, 8),      # one key in the second tile
    (2, 300, 2, 16),
    (1, 5, 2, 32),      # fewer keys than one lane half holds
    (1, 1, 1, 8),       # a single token: A = 1
    (1, 100, 2, 80),    # the 32 x 32 level's head width: five 16-dim steps, 256-byte key rows
    (1, 70, 2, 72),     # the same kernel with a padded last step
    (2, 90, 1, 160),    # the 16 x 16 and 8 x 8 levels' head width: ten steps, 384-byte key rows
    (1, 40, 1, 104),    # and a width in between (runs as ten steps)
])
def test_small_shapes(dgq, oracle, B, N, H, d, bits):
    c = di.selfattn_case(40 + N + d, B, N, H, d)
    s_in = np.array([1.0, 0.25][:B], np.float32)
    ref = _check(dgq, oracle, c, bits, s_in, min_good=0.5 if N > 1 else 0.0)
    if N >= 64 and bits == 8:
        assert np.unique(ref["codes"]).size > 10          # the codes span many octaves


def test_scale_at_the_maximum_and_below(dgq, oracle):
    """Given the call's own maximum the largest probability takes code 0; a smaller scale
    saturates everything above it; a scale of zero gives a zero product."""
    import torch
    c = di.selfattn_case(7, 2, 96, 2, 32)
    first = oracle.selfattn(c["Q"], c["K"], c["V"], 8, np.ones(2, np.float32))
    ref = _check(dgq, oracle, c, 8, first["s"])
    assert ref["codes"].min() == 0
    _check(dgq, oracle, c, 4, first["s"] * np.float32(0.125))
    out = dgq.dgq_selfattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]), 8,
                                _dev(np.zeros(2, np.float32)))
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0


def test_on_quantized_values(dgq, oracle):
    """A^ V^: the value tensor through dgq_quantize_value first (Section 3.3)."""
    import torch
    c = di.selfattn_case(11, 2, 128, 2, 40)
    vq = oracle.quantize_value(c["V"], 8)
    vhat, _, _ = dgq.dgq_quantize_value(_dev(c["V"]), 8)
    torch.cuda.synchronize()
    assert np.array_equal(vhat.cpu().numpy(), vq["vhat"])
    _check(dgq, oracle, dict(Q=c["Q"], K=c["K"], V=vq["vhat"]), 8, np.ones(2, np.float32))


def test_latent_64x64_sampled(dgq, oracle):
    """The 4096-token self-attention of the 64 x 64 latent (2 x 8 heads of 40), sampled
    queries: the oracle computes whole rows over all 4096 keys."""
    B, N, H, d = 2, 4096, 8, 40
    c = di.selfattn_case(4096, B, N, H, d)
    rng = np.random.default_rng(1)
    sel = np.unique(np.concatenate([rng.choice(N, 20, replace=False), [0, 31, 32, N - 33, N - 1]]))
    _check(dgq, oracle, c, 8, np.ones(B, np.float32), sel=sel, min_good=0.1)


def test_argument_errors(dgq):
    import torch
    q = torch.zeros((1, 8, 1, 8), dtype=torch.float32, device="cuda")
    s = torch.ones(1, dtype=torch.float32, device="cuda")
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_selfattn_logq(q, q, q, 5, s)
    assert e.value.code == -1
    for dbad in (168, 20):                                 # too wide; not a multiple of 8
        qb = torch.zeros((1, 8, 1, dbad), dtype=torch.float32, device="cuda")
        with pytest.raises(dgq.DgqError) as e:
            dgq.dgq_selfattn_logq(qb, qb, qb, 8, s)
        assert e.value.code == -4
    with pytest.raises(dgq.DgqError) as e:                 # workspace too small
        dgq.dgq_selfattn_logq(q, q, q, 8, s, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    assert dgq.dgq_selfattn_workspace_bytes(1, 8, 1, 168) == 0
