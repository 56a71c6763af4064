"""Helpers shared by the GPU parity tests."""
from __future__ import annotations

import numpy as np


def gpu_groups_vs_oracle(gg, og):
    """Bit-exact comparison of a GPU group handle with the oracle's Groups."""
    inf = gg.info
    assert inf.channels == og.C and inf.act_bits == og.act_bits
    assert inf.n_groups == og.NG and inf.k_padded == og.Kp
    assert inf.n_outlier_channels == og.n_outlier_channels
    assert inf.n_regular_groups == og.n_regular_groups
    assert inf.dstar == og.dstar and inf.n_class1_rows == og.n_class1_rows
    assert np.float32(inf.tau_pix) == og.tau_pix or (np.isinf(inf.tau_pix) and np.isinf(og.tau_pix))
    assert inf.d_channel == og.D_channel and inf.d_pixel == og.D_pixel
    assert inf.code_offset == (128 if og.act_bits == 8 else 0)
    t = gg.tables()
    assert np.array_equal(t["perm"], og.perm)
    assert np.array_equal(t["goff"], og.goff)
    assert np.array_equal(t["glen"], og.glen)
    assert np.array_equal(t["s"].view(np.uint32), og.s.view(np.uint32))
    assert np.array_equal(t["z"].view(np.uint32), og.z.view(np.uint32))


def codes_to_q(codes_np, act_bits, kp):
    """Stored containers -> the unsigned codes q [rows, K'] the paper defines."""
    if act_bits == 8:
        return (codes_np.astype(np.int16) + 128).astype(np.uint8)
    b = codes_np.view(np.uint8).reshape(codes_np.shape[0], kp // 8, 4)
    q = np.empty((b.shape[0], kp // 8, 8), np.uint8)
    q[:, :, 0:4] = b & 0x0F   # byte i of a block: position i in the low nibble,
    q[:, :, 4:8] = b >> 4     # position i + 4 in the high nibble
    return q.reshape(b.shape[0], kp)


def assert_close_fp32(got, ref, what=""):
    """The fp32 tolerance of the build: max|err| <= 1e-4 * max|ref|."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref).max()
    lim = 1e-4 * np.abs(ref).max()
    assert err <= lim, "%s max|err| %.3e > %.3e" % (what, err, lim)
