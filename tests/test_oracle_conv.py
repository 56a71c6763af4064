"""Pins for the oracle's 3 x 3 convolution path: the unfolding (im2col3x3), the replicated
group tables (groups_for_conv3x3) and the quantized convolution they give together with the
already pinned quantizer and contraction (the paper quantizes every layer of the U-Net,
convolutions included, with the activation quantizer of Section 3.3)."""
import numpy as np

import dgq_inputs as di


def test_unfolding_gives_the_library_convolution(oracle):
    import torch
    rng = np.random.default_rng(1)
    B, H, W, Cc, O = 2, 5, 7, 6, 4
    X = rng.standard_normal((B * H * W, Cc))
    Wt = rng.standard_normal((O, 3, 3, Cc))                    # [o, dy, dx, c]
    got = oracle.im2col3x3(X, B, H, W) @ Wt.reshape(O, 9 * Cc).T
    ref = torch.nn.functional.conv2d(torch.from_numpy(X.reshape(B, H, W, Cc)).permute(0, 3, 1, 2),
                                     torch.from_numpy(Wt).permute(0, 3, 1, 2), padding=1)
    ref = ref.permute(0, 2, 3, 1).reshape(B * H * W, O).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-12)


def test_codes_of_the_unfolded_input_are_shifted_copies(oracle):
    """Quantizing the unfolded input with the replicated tables gives, tap by tap, the codes
    of the neighbouring pixel, and outside the image the code of the value 0."""
    B, H, W, Cc = 2, 6, 5, 72
    X = di.linear_case(5, B, H * W, Cc, 8)["X"]
    for bits in (8, 4):
        og = oracle.calibrate_kmeans(X, bits, 4, 0)
        og9 = oracle.groups_for_conv3x3(og)
        assert og9.Kp == 9 * og.Kp and og9.NG == 9 * og.NG and og9.C == 9 * Cc
        q1 = oracle.quantize_act(og, X)["q"].reshape(B, H, W, og.Kp)
        q0 = oracle.quantize_act(og, np.zeros((1, Cc), np.float32))["q"][0]      # codes of zero
        r9 = oracle.quantize_act(og9, oracle.im2col3x3(X, B, H, W), want_dq=True)
        assert np.all(r9["cls"] == 0)
        q9 = r9["q"].reshape(B, H, W, 9, og.Kp)
        for t, (dy, dx) in enumerate((a, b) for a in (-1, 0, 1) for b in (-1, 0, 1)):
            for h in range(H):
                for w in range(W):
                    hh, ww = h + dy, w + dx
                    want = q1[:, hh, ww] if 0 <= hh < H and 0 <= ww < W else np.broadcast_to(q0, (B, og.Kp))
                    assert np.array_equal(q9[:, h, w, t], want), (t, h, w)
        # the padding's code dequantizes to zero within half a step wherever zero lies in range
        real = og.perm >= 0
        grp = np.repeat(np.arange(og.NG), og.glen)
        s, z = og.s[0][grp].astype(np.float64), og.z[0][grp].astype(np.float64)
        inside = (z <= 0) & (z + s * ((1 << bits) - 1) >= 0)
        assert inside.any()
        dq0 = s * q0[real] + z
        assert np.all(np.abs(dq0[inside]) <= 0.5 * s[inside] * (1 + 1e-6))


def test_quantized_convolution_is_the_convolution_of_the_dequantized_operands(oracle):
    import torch
    B, H, W, Cc, O = 1, 6, 6, 40, 16
    c = di.linear_case(9, B, H * W, Cc, O)
    X = c["X"]
    rng = np.random.default_rng(2)
    Wt = (rng.standard_normal((O, 3, 3, Cc)) * 0.05).astype(np.float32)
    og = oracle.calibrate_kmeans(X, 8, 3, 0)
    og9 = oracle.groups_for_conv3x3(og)
    r9 = oracle.quantize_act(og9, oracle.im2col3x3(X, B, H, W), want_dq=True)
    wq, sw = oracle.quantize_weight(Wt.reshape(O, 9 * Cc), 8)
    y, _ = oracle.linear(og9, r9["q"], r9["cls"], wq, sw, None)
    # dequantized image: tap 4 is the pixel itself
    xdq = r9["xdq"][:, 4 * Cc:5 * Cc].reshape(B, H, W, Cc)
    # the padding is the dequantized code of zero, not zero: rebuild the padded image
    q0 = oracle.quantize_act(og, np.zeros((1, Cc), np.float32), want_dq=True)["xdq"][0]
    pad = np.broadcast_to(q0, (B, H + 2, W + 2, Cc)).copy()
    pad[:, 1:H + 1, 1:W + 1] = xdq
    wdq = (wq.astype(np.float64) * sw[:, None].astype(np.float64)).reshape(O, 3, 3, Cc)
    ref = torch.nn.functional.conv2d(torch.from_numpy(pad).permute(0, 3, 1, 2),
                                     torch.from_numpy(wdq).permute(0, 3, 1, 2))
    ref = ref.permute(0, 2, 3, 1).reshape(B * H * W, O).numpy()
    assert np.abs(y - ref).max() <= 1e-5 * np.abs(ref).max()
