"""Pins for the oracle's self-attention with log2-quantized probabilities (Section 3.3:
the log quantizer of Section 3.1 on every attention score, given scale)."""
import numpy as np

import dgq_inputs as di


def _case(seed, B=2, N=48, H=2, d=16):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, N, H, d)).astype(np.float32)
    K = rng.standard_normal((B, N, H, d)).astype(np.float32)
    V = rng.standard_normal((B, N, H, d)).astype(np.float32)
    return Q, K, V


def test_uniform_attention_is_the_mean_of_v(oracle):
    """Q = 0 gives A = 1/nk for every key; with nk a power of two that is an exact power of
    two, the code is log2 nk, A^ = A, and the product is the plain mean of V."""
    _, K, V = _case(1, N=64)
    Q = np.zeros_like(K)
    one = np.ones(2, np.float32)
    for bits in (4, 8):
        r = oracle.selfattn(Q, K, V, bits, one, want_ahat=True)
        assert np.all(r["codes"] == 6)
        assert np.all(r["ahat"] == 1.0 / 64)
        assert np.all(r["s"] == np.float32(1.0 / 64))
        want = V.astype(np.float64).mean(axis=1)                 # [B,H,d]
        assert np.allclose(r["out"], want[:, None], rtol=0, atol=1e-6)
    # with the scale at the maximum itself the same probabilities take code 0
    r = oracle.selfattn(Q, K, V, 4, np.full(2, 1.0 / 64, np.float32))
    assert np.all(r["codes"] == 0)


def test_matches_the_cross_attention_quantizer_column_by_column(oracle):
    """The flag that sends column 0 through the quantizer changes nothing else: with the
    same given scale, columns 1.. carry the codes of the cross-attention definition, and the
    two products differ by exactly (A^_0 - A_0) V_0."""
    Q, K, V = _case(2)
    s = np.array([0.5, 0.25], np.float32)
    for bits in (4, 8):
        rs = oracle.selfattn(Q, K, V, bits, s, want_ahat=True)
        rx = oracle.xattn(Q, K, V, None, bits, want_ahat=True, s_in=s)
        assert np.array_equal(rs["codes"][..., 1:], rx["codes"])
        assert np.array_equal(rs["margin"][..., 1:], rx["margin"])
        assert np.array_equal(rs["ahat"][..., 1:], rx["ahat"][..., 1:])
        d0 = rs["ahat"][..., 0] - rx["A"][..., 0].astype(np.float64)        # [B,H,N]
        diff = np.einsum("bhn,bhd->bnhd", d0, V[:, 0].astype(np.float64))
        assert np.allclose(rs["out"].astype(np.float64) - rx["out"], diff, rtol=0, atol=2e-6)
        # column 0 itself: the same formula as any other column
        a0 = rs["A"][..., 0].astype(np.float64)
        q0 = np.clip(np.rint(-np.log2(a0 / s[:, None, None].astype(np.float64))), 0, (1 << bits) - 1)
        assert np.array_equal(rs["codes"][..., 0], q0.astype(np.uint8))


def test_power_of_two_error_and_clamps(oracle):
    Q, K, V = _case(3, N=40)
    Q *= 3.0                                      # peaked rows: a wide range of probabilities
    one = np.ones(2, np.float32)
    r8 = oracle.selfattn(Q, K, V, 8, one, want_ahat=True)
    A = r8["A"].astype(np.float64)
    ratio = r8["ahat"] / A
    assert ratio.max() <= 2 ** 0.5 * (1 + 1e-12) and ratio.min() >= 2 ** -0.5 * (1 - 1e-12)
    assert r8["codes"].max() > 15                 # so that four bits must clamp
    r4 = oracle.selfattn(Q, K, V, 4, one, want_ahat=True)
    assert np.array_equal(r4["codes"], np.minimum(r8["codes"], 15))
    assert np.all(r4["ahat"][r8["codes"] > 15] == 2.0 ** -15)
    assert np.array_equal(r4["s"], A.reshape(2, -1).max(axis=1).astype(np.float32))
    # a probability of exactly zero (the exponential underflows) takes the top code
    Qz = Q.copy()
    Qz[0, 0] *= 1e4
    rz = oracle.selfattn(Qz, K, V, 8, one)
    zero = rz["A"][0, :, 0, :] == 0
    assert zero.any() and np.all(rz["codes"][0, :, 0, :][zero] == 255)


def test_product_is_a_shift_and_add_of_integers(oracle):
    """With integer-valued V and 4-bit codes, out 2^15 / s = sum_j v_j << (15 - q_j) exactly
    (Section 3.1: the log quantizer turns the product into bit shifts)."""
    Q, K, _ = _case(4, B=1, N=24, H=1, d=8)
    rng = np.random.default_rng(5)
    V = rng.integers(-100, 100, size=(1, 24, 1, 8)).astype(np.float32)
    s = np.array([0.5], np.float32)
    r = oracle.selfattn(Q, K, V, 4, s)
    for i in range(24):
        sh = [15 - int(c) for c in r["codes"][0, 0, i]]
        for t in range(8):
            acc = sum(int(V[0, j, 0, t]) << sh[j] for j in range(24))
            assert float(r["out"][0, i, 0, t]) == np.float32(0.5 * acc / 32768.0)


def test_subset_of_queries(oracle):
    """Rows are independent: the oracle on a subset of the queries gives those rows."""
    Q, K, V = _case(6)
    s = np.array([1.0, 0.5], np.float32)
    full = oracle.selfattn(Q, K, V, 8, s)
    sel = [0, 7, 31, 47]
    part = oracle.selfattn(Q[:, sel], K, V, 8, s)
    assert np.array_equal(part["codes"], full["codes"][:, :, sel])
    assert np.array_equal(part["out"], full["out"][:, sel])
