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


def _swz64(t):
    return ((t >> 2) & 1) | ((((t >> 1) ^ (t >> 3)) & 1) << 1)


def codes_to_q(codes_np, act_bits, kp, rows):
    """Block-tiled containers -> the unsigned codes q [rows, K'] the paper defines.

    Layout (include/dgq.h): blocks of 1 KiB ordered [row block][chunk]; a block is one
    64-position chunk of 16 rows x 64 B (8 bit) or 32 rows x 32 B (4 bit); the 16-byte
    slots of row t are XOR-permuted (and, in 4-bit rows 16..31, the halves of a slot swapped)."""
    n_chunks = kp // 64
    b = codes_np.view(np.uint8).reshape(-1, n_chunks, 1024)
    if act_bits == 8:
        blk = b.reshape(-1, n_chunks, 16, 4, 16)          # [rb, ch, t, stored slot, byte]
        out = np.empty_like(blk)
        for t in range(16):
            for k in range(4):
                out[:, :, t, k] = blk[:, :, t, k ^ _swz64(t)]
        q = out.transpose(0, 2, 1, 3, 4).reshape(-1, kp)   # [rb*16, ch*64]
        return (q[:rows].astype(np.int8).astype(np.int16) + 128).astype(np.uint8)
    blk = b.reshape(-1, n_chunks, 32, 2, 16)
    out = np.empty_like(blk)
    for t in range(32):
        for h in range(2):
            out[:, :, t, h] = blk[:, :, t, h ^ ((t >> 3) & 1)]
    # rows 16..31 of a block keep the two 8-byte halves of every slot swapped
    out[:, :, 16:] = np.concatenate([out[:, :, 16:, :, 8:], out[:, :, 16:, :, :8]], axis=-1)
    packed = out.transpose(0, 2, 1, 3, 4).reshape(-1, kp // 8, 4)[:rows]  # groups of 8 positions
    q = np.empty((packed.shape[0], kp // 8, 8), np.uint8)
    q[:, :, 0:4] = packed & 0x0F   # byte i: position i in the low nibble,
    q[:, :, 4:8] = packed >> 4     # position i + 4 in the high nibble
    return q.reshape(packed.shape[0], kp)


def assert_close_fp32(got, ref, what=""):
    """The fp32 tolerance of the build: max|err| <= 1e-4 * max|ref|."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref).max()
    lim = 1e-4 * np.abs(ref).max()
    assert err <= lim, "%s max|err| %.3e > %.3e" % (what, err, lim)


def scale_rtol(c, use_bias=True):
    """Relative bar for the prompt scale of a cross-attention case, derived from fp32.

    The scale is 2^(S - lse2), with S a logit and lse2 the log-sum of its row, both fp32
    numbers in log2 units whose magnitude reaches L = max|logit| * log2(e).  Each carries
    about two roundings at that magnitude (the dot product, the scaling, the log-sum), the
    oracle none (it works in double), so the relative error of the scale is bounded by
    ln 2 * 4 * ulp32(L): 1.3e-6 for L in [4, 8), 2.6e-6 in [8, 16), 5.3e-6 in [16, 32).
    Never below 1e-6, the bar the full-size configurations are held to."""
    Q = c["Q"].astype(np.float64)
    K = c["K"].astype(np.float64)
    logits = np.einsum("bihd,bjhd->bhij", Q, K) / np.sqrt(Q.shape[-1])
    if use_bias and c.get("key_bias") is not None:
        logits = logits + c["key_bias"].astype(np.float64)
    big = np.abs(logits).max() * 1.4426950408889634
    return max(1e-6, float(np.log(2.0) * 4.0 * np.spacing(np.float32(big))))
