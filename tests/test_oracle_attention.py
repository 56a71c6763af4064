"""Pins for the oracle's attention side: softmax scores (Section 3.2), log2
codes with a prompt-specific scale, the separate <start> column and the split
product (Section 3.3, attention-aware quantization)."""
import math
import os

import numpy as np
import pytest

import dgq_inputs as di

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_softmax_matches_library_and_sums_to_one(oracle):
    from scipy.special import softmax
    c = di.attention_case(1, 2, 24, 3, 40)
    A = oracle.attn_probs(c["Q"], c["K"], c["key_bias"])
    assert A.shape == (2, 3, 24, 77)
    L = np.einsum("bihd,bjhd->bhij", c["Q"].astype(np.float64), c["K"].astype(np.float64))
    L = L / math.sqrt(40) + c["key_bias"].astype(np.float64)
    ref = softmax(L, axis=-1)
    assert np.abs(A - ref).max() <= 1e-7
    assert np.abs(A.astype(np.float64).sum(-1) - 1).max() <= 1e-5
    # the boosted <start> column dominates, as in the paper's Figure 4(a)
    assert np.median(A[..., 0]) > 0.5


def test_softmax_uniform_when_keys_identical(oracle):
    c = di.attention_case(2, 1, 8, 2, 16, nk=11)
    K = np.repeat(c["K"][:, :1], 11, axis=1)
    A = oracle.attn_probs(c["Q"], K, None)
    assert np.allclose(A, 1.0 / 11, rtol=1e-6)


def test_log2_quantizer_worked_example(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "log2_quantizer_worked.txt"))
            if l.strip() and not l.startswith("#")]
    a = np.array([float(r[0]) for r in rows], np.float32)
    A = np.concatenate([[np.float32(0.9)], a]).reshape(1, 1, 1, -1)
    V = np.ones((1, A.shape[-1], 1, 4), np.float32)
    for col, bits in ((1, 4), (2, 8)):
        r = oracle.xattn_logq(A, V, bits)
        assert r["s"][0] == np.float32(0.5)
        assert list(r["codes"][0, 0, 0]) == [int(x[col]) for x in rows]


@pytest.mark.parametrize("bits", [4, 8])
def test_exact_powers_of_two(oracle, bits):
    """A = s * 2^-k gives code k, and every dequantized value is an exact
    power of two times s (frexp mantissa 0.5)."""
    qmax = 2 ** bits - 1
    ks = np.arange(0, min(qmax + 6, 140))
    s = np.float32(0.3125)
    a = (np.float64(s) * np.ldexp(1.0, -ks)).astype(np.float32)
    A = np.concatenate([[np.float32(0.5)], a]).reshape(1, 1, 1, -1)
    V = np.zeros((1, A.shape[-1], 1, 2), np.float32)
    r = oracle.xattn_logq(A, V, bits, want_ahat=True)
    assert r["s"][0] == s
    assert np.array_equal(r["codes"][0, 0, 0], np.minimum(ks, qmax))
    m, _ = np.frexp(r["ahat"][0, 0, 0, 1:] / np.float64(s))
    assert np.all(m == 0.5)
    assert r["ahat"][0, 0, 0, 0] == 0.5  # <start> column untouched


@pytest.mark.parametrize("bits", [4, 8])
def test_code_properties_on_recipe(oracle, bits):
    c = di.attention_case(3, 2, 64, 4, 40)
    r = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], bits, want_ahat=True)
    A, codes, s = r["A"], r["codes"].astype(int), r["s"]
    qmax = 2 ** bits - 1
    for b in range(2):
        assert s[b] == A[b, :, :, 1:].max()
        assert (codes[b] == 0).any()  # the maximum itself has code 0
    sb = s.astype(np.float64)[:, None, None, None]
    ah = r["ahat"]
    m, _ = np.frexp(ah[..., 1:] / sb)
    assert np.all(m == 0.5)
    assert np.array_equal(ah[..., 0], A[..., 0].astype(np.float64))  # bit-identical column 0
    t = -np.log2(A[..., 1:].astype(np.float64) / sb)
    notclip = t < qmax + 0.5
    assert np.all(np.abs(np.log2(ah[..., 1:] / A[..., 1:].astype(np.float64)))[notclip] <= 0.5 + 1e-12)
    assert np.all(codes[~notclip] == qmax)
    if bits == 4:
        assert (~notclip).any()
    # margins: distance to the nearest rounding boundary
    mg = r["margin"]
    frac = np.abs((t - np.floor(t)) - 0.5)
    inside = t < qmax - 0.5
    assert np.allclose(mg[inside], frac[inside], atol=1e-6)


def test_zero_probability_and_clamp(oracle):
    A = np.array([0.7, 0.3, 0.0, 1e-30, 3e-39], np.float32).reshape(1, 1, 1, 5)
    V = np.ones((1, 5, 1, 1), np.float32)
    r4 = oracle.xattn_logq(A, V, 4, want_ahat=True)
    assert list(r4["codes"][0, 0, 0]) == [0, 15, 15, 15]
    # never dequantized to zero
    assert np.all(r4["ahat"][0, 0, 0, 1:] >= 0.3 * 2.0 ** -15)
    r8 = oracle.xattn_logq(A, V, 8)
    assert list(r8["codes"][0, 0, 0]) == [0, 255, 98, 126]


def test_product_equals_full_precision_when_codes_are_zero(oracle):
    """If all non-<start> probabilities of a prompt are equal, every code is 0,
    A-hat == A and the output equals full-precision attention."""
    B, N, H, d, nk = 1, 6, 2, 8, 9
    rng = np.random.default_rng(0)
    A = np.empty((B, H, N, nk), np.float32)
    A[..., 0] = 0.6
    A[..., 1:] = np.float32(0.05)
    V = rng.standard_normal((B, nk, H, d)).astype(np.float32)
    r = oracle.xattn_logq(A, V, 4, want_ahat=True)
    assert np.all(r["codes"] == 0)
    ref = np.einsum("bhij,bjhd->bihd", A.astype(np.float64), V.astype(np.float64))
    assert np.abs(r["out"] - ref).max() <= 1e-7 * np.abs(ref).max()


@pytest.mark.parametrize("bits", [4, 8])
def test_product_definition_and_error_bound(oracle, bits):
    c = di.attention_case(4, 2, 32, 2, 40)
    r = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], bits, want_ahat=True)
    V = c["V"].astype(np.float64)
    ref_hat = np.einsum("bhij,bjhd->bihd", r["ahat"], V)
    assert np.abs(r["out"] - ref_hat).max() <= 2e-7 * np.abs(ref_hat).max()
    A = r["A"].astype(np.float64)
    ref_fp = np.einsum("bhij,bjhd->bihd", A, V)
    # |A-hat - A| <= (sqrt2 - 1) A off clipping; clipped entries are replaced by s*2^-qmax
    qmax = 2 ** bits - 1
    sb = r["s"].astype(np.float64)[:, None, None, None]
    dA = np.abs(r["ahat"] - A)
    bound_el = np.maximum((math.sqrt(2) - 1) * A, sb * 2.0 ** -qmax)
    bound_el[..., 0] = 0
    assert np.all(dA <= bound_el + 1e-15)
    bound = np.einsum("bhij,bjhd->bihd", bound_el, np.abs(V))
    assert np.all(np.abs(r["out"] - ref_fp) <= bound + 1e-6)


def test_scale_is_per_prompt(oracle):
    """Changing prompt 1 does not change prompt 0's scale or codes."""
    c = di.attention_case(5, 2, 16, 2, 40)
    r = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8)
    K2 = c["K"].copy()
    K2[1] *= 3
    r2 = oracle.xattn(c["Q"], K2, c["V"], c["key_bias"], 8)
    assert r["s"][0] == r2["s"][0] and r["s"][1] != r2["s"][1]
    assert np.array_equal(r["codes"][0], r2["codes"][0])
    assert np.array_equal(r["out"][0], r2["out"][0])


def test_redraw_changes_only_selected_queries():
    base = di.attention_case(6, 2, 8, 2, 16)
    red = np.zeros((2, 8, 2), np.int32)
    red[1, 3, 0] = 2
    c = di.attention_case(6, 2, 8, 2, 16, redraw=red)
    same = np.all(base["Q"] == c["Q"], axis=-1)
    assert not same[1, 3, 0] and same.sum() == same.size - 1
    assert np.array_equal(base["K"], c["K"]) and np.array_equal(base["V"], c["V"])


def test_given_scale(oracle):
    """The log quantizer without dynamic quantization: with the call's own maximum as the
    given scale nothing changes; a scale 2^k times larger shifts every unclamped code by k
    (log2 of a power of two is exact); probabilities above the scale saturate at the scale;
    the call's own maximum is reported whatever scale is used."""
    import dgq_inputs as di
    c = di.attention_case(606, 2, 48, 2, 16, nk=20, d_ctx=32)
    dyn = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8, want_ahat=True)
    same = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8, s_in=dyn["s"])
    assert np.array_equal(same["codes"], dyn["codes"]) and np.array_equal(same["out"], dyn["out"])
    for k in (1, 3):
        big = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8, s_in=dyn["s"] * np.float32(2 ** k))
        want = np.minimum(dyn["codes"].astype(int) + k, 255)
        assert np.array_equal(big["codes"].astype(int), want)
        assert np.array_equal(big["s"], dyn["s"])
    small = oracle.xattn(c["Q"], c["K"], c["V"], c["key_bias"], 8, s_in=dyn["s"] * np.float32(0.25),
                         want_ahat=True)
    assert np.array_equal(small["codes"].astype(int), np.maximum(dyn["codes"].astype(int) - 2, 0))
    B = c["Q"].shape[0]
    for b in range(B):
        s_in = float(dyn["s"][b]) * 0.25
        above = dyn["A"][b][..., 1:] > s_in
        assert above.any()
        assert np.all(small["codes"][b][above] == 0)
        assert np.all(small["ahat"][b][..., 1:][above] == np.float32(s_in))
        # the <start> column is never quantized
        assert np.array_equal(small["ahat"][b][..., 0], dyn["A"][b][..., 0].astype(np.float64))
