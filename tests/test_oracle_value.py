"""Pins for the oracle's quantized value tensor V^ of the product A^ V^ (Section 3.3,
with the linear quantizer of Section 3.1 and the s_k / z_k form of its parameters)."""
import numpy as np
import pytest


def test_grid_points_are_reproduced(oracle):
    """A tensor that already lies on the quantizer's grid z + s k comes back unchanged,
    except the maximum, which level 2^b does not exist for."""
    rng = np.random.default_rng(1)
    for bits in (8, 4):
        L = 1 << bits
        s, z = np.float32(0.03125), np.float32(-1.75)     # exact in fp32, as is every z + s k
        k = rng.integers(0, L, size=(2, 11, 3, 8))
        k[:, 0, :, 0] = 0
        k[:, 1, :, 0] = L                                  # max - min = L s in every (prompt, head)
        V = (z + s * k.astype(np.float32)).astype(np.float32)
        r = oracle.quantize_value(V, bits)
        assert np.all(r["params"][..., 0] == s) and np.all(r["params"][..., 1] == z)
        assert np.array_equal(r["codes"], np.minimum(k, L - 1))
        inside = k < L
        assert np.array_equal(r["vhat"][inside], V[inside])
        assert np.all(r["vhat"][~inside] == V[~inside] - s)  # the clipped maximum: one step low


def test_equals_library_affine_quantizer_when_the_offset_is_a_whole_step(oracle):
    """With a power-of-two step and an offset of -128 steps the float-offset form
    (v - z) / s and the library's integer zero-point form v / s + 128 are the same map."""
    import torch
    rng = np.random.default_rng(2)
    s = np.float32(2.0 ** -5)
    V = (rng.standard_normal((1, 50, 2, 16)) * 1.2).astype(np.float32)
    V = np.clip(V, -128 * s, 128 * s).astype(np.float32)
    V[0, 0, :, 0] = -128 * s
    V[0, 1, :, 0] = 128 * s
    r = oracle.quantize_value(V, 8)
    assert np.all(r["params"][..., 0] == s) and np.all(r["params"][..., 1] == -128 * s)
    tq = torch.quantize_per_tensor(torch.from_numpy(V), float(s), 128, torch.quint8)
    assert np.array_equal(r["codes"], tq.int_repr().numpy())
    assert np.array_equal(r["vhat"], tq.dequantize().numpy())


def test_error_bound_monotone_and_idempotent(oracle):
    rng = np.random.default_rng(3)
    V = (rng.standard_normal((3, 77, 4, 40)) * rng.uniform(0.2, 5.0, size=(3, 1, 4, 1))).astype(np.float32)
    for bits in (8, 4):
        r = oracle.quantize_value(V, bits)
        s = r["params"][:, None, :, None, 0].astype(np.float64)
        err = np.abs(r["vhat"].astype(np.float64) - V)
        # s = range / 2^b: level 2^b does not exist, so the top half step saturates (error
        # up to a whole step); everything below it is within half a step
        z = r["params"][:, None, :, None, 1].astype(np.float64)
        top = (V - z) / s > (1 << bits) - 0.5
        assert top.any() and top.mean() < 0.1
        slack = 1e-6 * np.abs(V).max()
        assert np.all(err[~top] <= (0.5 * s + slack + 0 * err)[~top])
        assert np.all(err <= s + slack)
        # per (prompt, head): codes are monotone in the value
        for b in range(3):
            for h in range(4):
                v = V[b, :, h, :].ravel()
                c = r["codes"][b, :, h, :].ravel()
                o = np.argsort(v, kind="stable")
                assert np.all(np.diff(c[o].astype(int)) >= 0)
                assert c.min() == 0 and c.max() == (1 << bits) - 1
        # quantizing the reconstruction with the same grid changes nothing
        r2 = oracle.quantize_value(r["vhat"], bits)
        same_grid = np.all(r2["params"] == r["params"], axis=-1)   # max clipped: range shrinks by one step
        assert not same_grid.all() or np.array_equal(r2["vhat"], r["vhat"])
    # slices are independent: changing one (prompt, head) leaves the others alone
    V2 = V.copy()
    V2[1, :, 2, :] *= 3
    ra, rb = oracle.quantize_value(V, 8), oracle.quantize_value(V2, 8)
    mask = np.ones(V.shape, bool)
    mask[1, :, 2, :] = False
    assert np.array_equal(ra["vhat"][mask], rb["vhat"][mask])


def test_constant_slice(oracle):
    V = np.full((1, 5, 2, 8), 0.75, np.float32)
    r = oracle.quantize_value(V, 8)
    assert np.all(r["params"][..., 0] == 1.0) and np.all(r["codes"] == 0)
    assert np.array_equal(r["vhat"], V)


def test_product_is_a_shift_and_add_of_integers(oracle):
    """Section 3.1: the log quantizer turns the product into bit shifts.  With 4-bit
    attention codes q_a and 8-bit value codes q_v, every output is
        A_i0 v^_0 + s (s_v sum_j (q_v[j] << (15 - q_a[i,j])) + z_v sum_j (1 << (15 - q_a[i,j]))) / 2^15
    in exact integers; the oracle's floating-point product on V^ must land on it."""
    import dgq_inputs as di
    c = di.attention_case(4242, 2, 64, 3, 16, nk=20, d_ctx=48)
    vq = oracle.quantize_value(c["V"], 8)
    r = oracle.xattn(c["Q"], c["K"], vq["vhat"], c["key_bias"], 4)
    B, N, H, d = c["Q"].shape
    for b in range(B):
        s = float(r["s"][b])
        for h in range(H):
            sv, zv = (float(x) for x in vq["params"][b, h])
            qv = vq["codes"][b, :, h, :].astype(object)            # python ints
            for i in range(0, N, 7):
                qa = r["codes"][b, h, i].astype(int)               # keys 1 .. nk-1
                sh = [1 << (15 - int(q)) for q in qa]
                a0 = float(r["A"][b, h, i, 0])
                for t in range(d):
                    acc = sum(int(qv[j + 1, t]) * sh[j] for j in range(len(sh)))
                    ones = sum(sh)
                    want = a0 * float(vq["vhat"][b, 0, h, t]) + s * (sv * acc + zv * ones) / 32768.0
                    got = float(r["out"][b, i, h, t])
                    assert abs(got - want) <= 2e-6 * max(1.0, abs(want)), (b, h, i, t)


def test_integer_product_oracle(oracle):
    """oracle.xattn_intv (the shift-and-add product on V^'s codes) against three things it does
    not compute itself: python big integers on sampled outputs, the floating-point product of
    oracle.xattn on the reconstruction V^ (equal up to the fp32 rounding of V^), and the bound
    that keeps the sums inside an int32 accumulator."""
    import dgq_inputs as di
    c = di.attention_case(4243, 2, 48, 3, 16, nk=20, d_ctx=48)
    r = oracle.xattn_intv(c["Q"], c["K"], c["V"], c["key_bias"])
    vq = r["vq"]
    B, N, H, d = c["Q"].shape
    for (b, i, h, t) in [(0, 0, 0, 0), (1, 47, 2, 15), (0, 13, 1, 7), (1, 5, 0, 3)]:
        qa = [int(x) for x in r["codes"][b, h, i]]
        acc = sum(int(vq["codes"][b, j + 1, h, t]) << (15 - qa[j]) for j in range(len(qa)))
        ones = sum(1 << (15 - q) for q in qa)
        assert int(r["acc"][b, i, h, t]) == acc and int(r["zsum"][b, i, h]) == ones
    assert r["acc"].min() >= 0 and r["acc"].max() < 2 ** 31 and r["zsum"].max() < 2 ** 31
    ref = oracle.xattn(c["Q"], c["K"], vq["vhat"], c["key_bias"], 4)
    assert np.array_equal(ref["codes"], r["codes"])
    assert np.abs(r["out"] - ref["out"]).max() <= 1e-6 * np.abs(ref["out"]).max()
    # all codes 15 (weights 1): acc is the plain sum of the value codes
    vsum = vq["codes"][:, 1:].astype(np.int64).sum(1)              # [B,H,d]
    low = r["codes"].min(axis=-1) == 15                            # [B,H,N]
    for b, h, i in np.argwhere(low)[:4]:
        assert np.array_equal(r["acc"][b, i, h], vsum[b, h])
