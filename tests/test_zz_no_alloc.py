"""dgq_xattn_logq_noalloc (the attention for callers that cannot allocate) against
dgq_xattn_logq: both run the same kernels, the first with the library's fixed device
array where the second takes a caller's workspace, so out, scale and codes must be
equal bit for bit.  Two calls in a row, the second on a smaller input (the array then
still holds the first call's values behind the part the second call uses); the oracle
comparison of the computation itself is in test_gpu_xattn.py.  Collected last on
purpose: a failure here must not hide the parity tests."""
import numpy as np
import pytest

import dgq_inputs as di
from support import scale_rtol

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


def _both(dgq, c, bits):
    import torch
    q, k, v, kb = _dev(c["Q"]), _dev(c["K"]), _dev(c["V"]), _dev(c["key_bias"])
    B, N, H, d = q.shape
    nk = k.shape[1]
    # every buffer of the new call exists before it runs: the call itself allocates nothing
    out = torch.full((B, N, H, d), float("nan"), device="cuda")
    s = torch.full((B,), float("nan"), device="cuda")
    codes = torch.full((B, H, N, nk - 1), 0xEE, dtype=torch.uint8, device="cuda")
    import gc
    gc.collect()   # tensors of earlier tests must not be released in the middle of the check
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    dgq.dgq_xattn_logq_noalloc(q, k, v, kb, bits, out, s, codes_dump=codes)
    assert torch.cuda.memory_allocated() <= before   # nothing was allocated through torch either
    codes_ref = torch.full_like(codes, 0xEE)
    out_ref, s_ref = dgq.dgq_xattn_logq(q, k, v, kb, bits, codes_dump=codes_ref)
    torch.cuda.synchronize()
    return (out.cpu().numpy(), s.cpu().numpy(), codes.cpu().numpy(),
            out_ref.cpu().numpy(), s_ref.cpu().numpy(), codes_ref.cpu().numpy())


def _same(got):
    out, s, codes, out_ref, s_ref, codes_ref = got
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(codes, codes_ref)
    assert np.array_equal(out.view(np.uint32), out_ref.view(np.uint32))
    assert np.isfinite(out).all()


@pytest.mark.parametrize("bits", [8, 4])
def test_two_calls_second_smaller(dgq, bits):
    big = di.attention_case(7001, 2, 1000, 8, 40)      # ragged query count, matrix-core path
    small = di.attention_case(7002, 1, 96, 2, 40)
    _same(_both(dgq, big, bits))
    _same(_both(dgq, small, bits))
    _same(_both(dgq, big, bits))                         # and back up again


def test_vector_path_needs_no_scratch(dgq):
    c = di.attention_case(7003, 1, 70, 2, 20, nk=9)     # d % 8 != 0: the fp32 per-thread kernels
    _same(_both(dgq, c, 8))


def test_against_oracle(dgq, oracle):
    from oracle.guard import guarded_attention_case
    c, _ = guarded_attention_case(7004, 2, 160, 2, 40, bits_list=(8,))
    out, s, codes, *_ = _both(dgq, c, 8)
    ref = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8)
    assert np.array_equal(codes, ref["codes"])
    assert np.all(np.abs(s - ref["s"]) <= scale_rtol(c) * ref["s"])
    assert np.abs(out - ref["out"]).max() <= 1e-4 * np.abs(ref["out"]).max()


def test_size_limit_is_an_error(dgq):
    import torch
    rows = dgq.XATTN_NOALLOC_MAX_ROWS
    B, H, d, nk = 1, 8, 8, 4
    N = rows // H + 32                                   # B * H * N just above the limit
    q = torch.zeros((B, N, H, d), device="cuda")
    kv = torch.zeros((B, nk, H, d), device="cuda")
    out = torch.full((B, N, H, d), 3.0, device="cuda")
    s = torch.full((B,), 3.0, device="cuda")
    with pytest.raises(dgq.DgqError) as e:
        dgq.dgq_xattn_logq_noalloc(q, kv, kv, None, 8, out, s)
    assert e.value.code == -6 and "DGQ_XATTN_NOALLOC_MAX_ROWS" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.min()) == 3.0 and float(s.min()) == 3.0   # nothing was enqueued
