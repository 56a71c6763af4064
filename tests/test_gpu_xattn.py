"""GPU parity of the log2-quantized cross-attention against the CPU oracle.

Codes are compared bit-exactly on margin-guarded inputs (oracle/guard.py: no
rounding decision within 2^-13 log2 units of a boundary); on raw inputs every
element whose oracle margin is at least that large must still match and the
few others may differ by one step.  The prompt scale is an fp32 output: the
full-size configurations (config 3, config 5) are held to S_RTOL = 1e-6; the
small cases, whose maximum sits wherever a handful of rows put it, to the bar
support.scale_rtol derives from the magnitude of their logits (four fp32
roundings at that magnitude, 1.3e-6 to 5.3e-6; measured up to 2.2e-6).  The
product is held to 1e-4 * max|ref|."""
import numpy as np
import pytest

import dgq_inputs as di
from support import assert_close_fp32, scale_rtol

pytestmark = pytest.mark.gpu

S_RTOL = 1e-6


@pytest.fixture(scope="module")
def dgq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2501_04304_amd as m
    m.lib()
    return m


def _dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _gpu(dgq, c, bits, use_bias=True):
    import torch
    B, N, H, d = c["Q"].shape
    nk = c["K"].shape[1]
    codes = torch.full((B, H, N, nk - 1), 0xEE, dtype=torch.uint8, device="cuda")
    out, s = dgq.dgq_xattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]),
                                _dev(c["key_bias"]) if use_bias else None, bits,
                                codes_dump=codes)
    torch.cuda.synchronize()
    return out.cpu().numpy(), s.cpu().numpy(), codes.cpu().numpy()


def _compare(dgq, oracle, c, bits, exact=True, use_bias=True, s_rtol=None):
    from oracle.guard import DELTA
    ref = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"] if use_bias else None, bits)
    out, s, codes = _gpu(dgq, c, bits, use_bias)
    if s_rtol is None:
        s_rtol = scale_rtol(c, use_bias)
    assert np.all(np.abs(s - ref["s"]) <= s_rtol * ref["s"])
    safe = ref["margin"] >= DELTA
    assert np.array_equal(codes[safe], ref["codes"][safe])
    if exact:
        assert safe.all(), "guarded inputs must have no marginal element"
        assert np.array_equal(codes, ref["codes"])
        assert_close_fp32(out, ref["out"], "out")
    else:
        diff = np.abs(codes.astype(int) - ref["codes"].astype(int))
        assert diff.max() <= 1
        assert (~safe).mean() < 1e-3
    # codes without the dump buffer give the same product
    import torch
    out2, s2 = dgq.dgq_xattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]),
                                  _dev(c["key_bias"]) if use_bias else None, bits)
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy(), out) and np.array_equal(s2.cpu().numpy(), s)


SHAPES = [
    # B, N, H, d, nk
    (2, 300, 3, 40, 77),   # ragged query tile
    (1, 64, 2, 64, 77),
    (2, 70, 2, 37, 77),    # head dim not a multiple of 4
    (1, 33, 1, 160, 77),
    (1, 257, 2, 8, 10),    # few keys
    (1, 40, 2, 40, 100),   # more than 80 keys
    (3, 1, 1, 16, 2),      # one query, one quantized key
    (100, 100, 3, 16, 10), # 300 one-trip pairs on 150 ranges: a range holds two pairs, of two prompts every third time
]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("B,N,H,d,nk", SHAPES)
def test_guarded_shapes(dgq, oracle, B, N, H, d, nk, bits):
    from oracle.guard import guarded_attention_case
    c, _ = guarded_attention_case(700 + d + nk, B, N, H, d, nk=nk, bits_list=(bits,))
    _compare(dgq, oracle, c, bits, exact=True)


@pytest.mark.parametrize("bits", [4, 8])
def test_workgroup_ranges_cross_pairs(dgq, oracle, bits):
    """More 256-query trips than CUs and a trip count per (prompt, head) pair that the range
    length does not divide: workgroups walk from one pair into the next and stage its keys and
    values again; the last trip of every pair is ragged (2600 = 10 x 256 + 40)."""
    from oracle.guard import guarded_attention_case
    c, _ = guarded_attention_case(7700, 5, 2600, 9, 64, bits_list=(bits,))
    _compare(dgq, oracle, c, bits, exact=True)


@pytest.mark.parametrize("bits", [4, 8])
def test_least_workspace_gives_the_same_results(dgq, bits):
    """With the full workspace the maxima behind the prompt scale travel through it; with one
    float per (prompt, head, query) and nothing more they go through atomics on scale_out,
    cleared by a launch of its own.  Both must give the same scale, codes and product, on ranges
    that cross pairs and prompts (5 prompts x 9 heads, 11 trips per pair)."""
    import torch
    from oracle.guard import guarded_attention_case
    c, _ = guarded_attention_case(7701, 5, 2600, 9, 64, bits_list=(bits,))
    B, N, H, d = c["Q"].shape
    nk = c["K"].shape[1]
    dev = [_dev(c[n]) for n in ("Q", "K", "V", "key_bias")]
    res = []
    full = dgq.dgq_xattn_workspace_bytes(B, N, H, d, nk)
    least = (B * H * N * 4 + 255) // 256 * 256
    assert least < full
    for nbytes in (full, least):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        codes = torch.full((B, H, N, nk - 1), 0xEE, dtype=torch.uint8, device="cuda")
        s = torch.full((B,), 123.0, dtype=torch.float32, device="cuda")  # stale values must not survive
        out, s = dgq.dgq_xattn_logq(*dev, bits, scale_out=s, codes_dump=codes, workspace=ws)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), s.cpu().numpy(), codes.cpu().numpy()))
    for a, b in zip(res[0], res[1]):
        assert np.array_equal(a, b)
    with pytest.raises(dgq.DgqError):
        dgq.dgq_xattn_logq(*dev, bits, workspace=torch.empty(least - 256, dtype=torch.uint8, device="cuda"))


def test_without_key_bias(dgq, oracle):
    from oracle.guard import guarded_attention_case
    c, _ = guarded_attention_case(11, 2, 96, 2, 40, bits_list=(8,))
    c = dict(c)
    c["key_bias"] = np.zeros_like(c["key_bias"])
    # the guard ran with the boost; re-guard on the unboosted logits via the raw-input rule
    _compare(dgq, oracle, c, 8, exact=False, use_bias=False)


@pytest.mark.parametrize("bits", [4, 8])
def test_raw_inputs_only_marginal_elements_may_differ(dgq, oracle, bits):
    c = di.attention_case(12, 2, 512, 4, 40)
    _compare(dgq, oracle, c, bits, exact=False)


@pytest.mark.parametrize("bits", [4, 8])
def test_config3_full(dgq, oracle, bits):
    """64x64 latent: batch 2, 8 heads, 4096 queries x 77 keys, head dim 40."""
    from oracle.guard import guarded_attention_case
    name, B, N, H, d, nk, d_ctx = di.config3()["attention"][0]
    c, n_redrawn = guarded_attention_case(3000, B, N, H, d, nk=nk, d_ctx=d_ctx, bits_list=(4, 8))
    assert n_redrawn < 0.1 * B * N * H
    _compare(dgq, oracle, c, bits, exact=True, s_rtol=S_RTOL)


@pytest.mark.parametrize("bits", [4, 8])
def test_config5_shape_sampled(dgq, oracle, bits):
    """SDXL-scale launch shape (16 prompts, 10 heads, d = 64), both code widths bench.py
    times; the oracle checks two whole prompts, which is what a per-prompt scale allows."""
    import torch
    name, B, N, H, d, nk, d_ctx = di.config5()["attention"][0]
    c = di.attention_case(5000, B, N, H, d, nk=nk, d_ctx=d_ctx)
    from oracle.guard import DELTA
    out, s, codes = _gpu(dgq, c, bits)
    for b in (0, B - 1):
        sub = {k: (v[b:b + 1] if k != "key_bias" else v) for k, v in c.items()}
        ref = oracle.xattn(sub["Q"], sub["K"], sub["V"], sub["key_bias"], bits)
        assert abs(s[b] - ref["s"][0]) <= S_RTOL * ref["s"][0]
        safe = ref["margin"][0] >= DELTA
        assert np.array_equal(codes[b][safe], ref["codes"][0][safe])
        assert np.abs(codes[b].astype(int) - ref["codes"][0].astype(int)).max() <= 1
        # rows without a marginal element must match to the fp32 tolerance
        good = np.transpose(safe.all(-1), (1, 0))  # [N, H]
        err = np.abs(out[b] - ref["out"][0])[good]
        assert err.max() <= 1e-4 * np.abs(ref["out"][0]).max()
    torch.cuda.synchronize()


def test_scale_buffer_is_reset_between_calls(dgq, oracle):
    """The prompt maximum is accumulated with atomics; a second call with smaller
    probabilities must not see the first call's maximum."""
    import torch
    c1 = di.attention_case(21, 1, 64, 2, 40, start_boost=0.0)
    c2 = di.attention_case(22, 1, 64, 2, 40, start_boost=12.0)
    s_buf = torch.empty(1, dtype=torch.float32, device="cuda")
    for c in (c1, c2):
        out, s = dgq.dgq_xattn_logq(_dev(c["Q"]), _dev(c["K"]), _dev(c["V"]), _dev(c["key_bias"]),
                                    8, scale_out=s_buf)
        torch.cuda.synchronize()
        ref = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8)
        assert abs(s.item() - ref["s"][0]) <= scale_rtol(c) * ref["s"][0]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("B,N,H,d,nk", [(2, 300, 3, 40, 77), (1, 64, 2, 64, 77), (2, 70, 2, 37, 77),
                                        (1, 40, 2, 40, 100), (3, 1, 1, 16, 2)])
def test_given_scale_one_pass(dgq, oracle, B, N, H, d, nk, bits):
    """The log quantizer without dynamic quantization (a given prompt scale): against the
    oracle with the same scale; with the dynamic call's own scale it reproduces that call
    bit for bit; it reports the call's own maximum all the same."""
    import torch
    from oracle.guard import DELTA, guarded_attention_case
    c, _ = guarded_attention_case(700 + d + nk, B, N, H, d, nk=nk, bits_list=(bits,))
    out_dyn, s_dyn, codes_dyn = _gpu(dgq, c, bits)
    dev = [_dev(c[n]) for n in ("Q", "K", "V", "key_bias")]
    codes = torch.full((B, H, N, nk - 1), 0xEE, dtype=torch.uint8, device="cuda")
    s_own = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
    out, _ = dgq.dgq_xattn_logq_static(*dev, bits, _dev(s_dyn), scale_out=s_own, codes_dump=codes)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), codes_dyn)
    assert np.array_equal(out.cpu().numpy(), out_dyn)
    assert np.array_equal(s_own.cpu().numpy(), s_dyn)
    # a scale from elsewhere (here: 0.6 and 1.7 times the maximum), with and without the
    # request for the own maximum
    for f in (0.6, 1.7):
        s_in = (s_dyn * np.float32(f)).astype(np.float32)
        ref = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], bits, s_in=s_in)
        codes.fill_(0xEE)
        out, _ = dgq.dgq_xattn_logq_static(*dev, bits, _dev(s_in), codes_dump=codes)
        torch.cuda.synchronize()
        safe = ref["margin"] >= DELTA
        got = codes.cpu().numpy()
        assert np.array_equal(got[safe], ref["codes"][safe])
        assert np.abs(got.astype(int) - ref["codes"].astype(int)).max() <= 1
        good = np.transpose(safe.all(-1), (0, 2, 1))  # [B, N, H]: rows without a marginal code
        err = np.abs(out.cpu().numpy() - ref["out"])[good]
        assert err.size and err.max() <= 1e-4 * np.abs(ref["out"]).max()
        assert np.all(np.abs(ref["s"] - s_dyn) <= scale_rtol(c) * s_dyn)
