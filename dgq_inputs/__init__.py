"""Seeded synthetic inputs for the DGQ quantized-inference path.

This module only draws random tensors and lists layer shapes. It holds none of
the method's arithmetic (no quantizer, no softmax, no clustering), so both the
CPU oracle's tests and the HIP path's tests/bench may use it without sharing
any computation.

The tensors stand in for the Stable-Diffusion UNet activations the paper
measures on (Section 4.1): they take the transformer blocks' shapes and the
structure the paper reports in Section 3.2 -- a few outlier channels, a few
outlier pixels, and a dominant <start>-token column in cross-attention.
"""
from __future__ import annotations

import numpy as np

CALIB_SEED_OFFSET = 10 ** 6
N_TEXT_KEYS = 77


def n_outlier_channels(C: int) -> int:
    return max(1, int(round(0.01 * C)))


def n_outlier_tokens(N: int) -> int:
    return max(2, int(round(0.0005 * N)))


def linear_case(seed: int, B: int, N: int, C: int, O: int | None = None,
                calib: bool = False, with_weight: bool = True):
    """One linear layer's inputs.

    Draw order with Generator(PCG64(seed)): X ~ N(0,1) [B,N,C] fp32, outlier
    channel indices, outlier token indices, W ~ N(0, 0.02^2) [O,C] fp32.
    1 % of channels are scaled by 40 and max(2, 0.05 % of N) token positions
    (the same in every batch element) by 25.

    calib=True returns a tensor with the same outlier indices but fresh values
    (value generator seeded seed + 10^6), used as calibration data so that
    run-time clipping really occurs.

    Returns dict(X=[B*N, C] fp32, W=[O, C] fp32 or None, oc, ot, rows_ot).
    """
    rng = np.random.default_rng(np.random.PCG64(seed))
    X = rng.standard_normal((B, N, C), dtype=np.float32)
    oc = np.sort(rng.choice(C, min(C, n_outlier_channels(C)), replace=False))
    ot = np.sort(rng.choice(N, min(N, n_outlier_tokens(N)), replace=False))
    W = None
    if with_weight and O is not None:
        W = rng.standard_normal((O, C), dtype=np.float32)
        W *= np.float32(0.02)
    if calib:
        rng_c = np.random.default_rng(np.random.PCG64(seed + CALIB_SEED_OFFSET))
        X = rng_c.standard_normal((B, N, C), dtype=np.float32)
    X[:, :, oc] *= np.float32(40.0)
    X[:, ot, :] *= np.float32(25.0)
    rows_ot = np.sort((np.arange(B)[:, None] * N + ot[None, :]).ravel())
    return dict(X=X.reshape(B * N, C), W=W, oc=oc, ot=ot, rows_ot=rows_ot)


def attention_case(seed: int, B: int, N: int, H: int, d: int,
                   nk: int = N_TEXT_KEYS, d_ctx: int = 768,
                   start_boost: float = 8.0, redraw: np.ndarray | None = None):
    """Cross-attention inputs.

    Q ~ N(0,1) [B,N,H,d]; a text context ctx ~ N(0,1) [B,nk,d_ctx] is projected
    by Wk, Wv ~ N(0,1)/sqrt(d_ctx) (in double, rounded to fp32) so that K and V
    [B,nk,H,d] are ~N(0,1) and share the context across heads.  key_bias adds
    +start_boost to the logit of key 0, mimicking the dominant <start> column.

    redraw: optional int array [B,N,H]; a query vector whose entry is c > 0 is
    replaced by a fresh draw from a generator keyed by (seed, b, i, h, c).  The
    tests use this to move queries away from rounding boundaries of the log2
    code; which rows to redraw is decided by the caller.
    """
    rng = np.random.default_rng(np.random.PCG64(seed))
    Q = rng.standard_normal((B, N, H, d), dtype=np.float32)
    ctx = rng.standard_normal((B, nk, d_ctx), dtype=np.float32)
    Wk = rng.standard_normal((H * d, d_ctx), dtype=np.float32)
    Wv = rng.standard_normal((H * d, d_ctx), dtype=np.float32)
    inv = 1.0 / np.sqrt(float(d_ctx))
    K = (ctx.astype(np.float64) @ Wk.astype(np.float64).T * inv).astype(np.float32)
    V = (ctx.astype(np.float64) @ Wv.astype(np.float64).T * inv).astype(np.float32)
    K = np.ascontiguousarray(K.reshape(B, nk, H, d))
    V = np.ascontiguousarray(V.reshape(B, nk, H, d))
    key_bias = np.zeros(nk, dtype=np.float32)
    key_bias[0] = np.float32(start_boost)
    if redraw is not None:
        idx = np.argwhere(redraw > 0)
        for b, i, h in idx:
            c = int(redraw[b, i, h])
            r = np.random.default_rng(np.random.PCG64(
                np.random.SeedSequence([seed, int(b), int(i), int(h), c])))
            Q[b, i, h, :] = r.standard_normal(d, dtype=np.float32)
    return dict(Q=Q, K=K, V=V, key_bias=key_bias)


# ----------------------------------------------------------------------------
# Workload tables (shapes only).  A linear entry is
#   (name, M rows, B, N, C in, O out, group size G).
# ----------------------------------------------------------------------------

def selfattn_case(seed: int, B: int, N: int, H: int, d: int, sharp: float = 1.5):
    """Self-attention inputs: Q, K, V ~ N(0, 1) [B,N,H,d] fp32 drawn in that order with
    Generator(PCG64(seed)); Q is multiplied by `sharp`, so the logits q.k / sqrt(d) have
    standard deviation `sharp` and a row's probabilities span many octaves."""
    rng = np.random.Generator(np.random.PCG64(seed))
    Q = (rng.standard_normal((B, N, H, d)) * sharp).astype(np.float32)
    K = rng.standard_normal((B, N, H, d)).astype(np.float32)
    V = rng.standard_normal((B, N, H, d)).astype(np.float32)
    return dict(Q=Q, K=K, V=V)


def _block_linears(prefix, B, N, C, G, d_ctx, nk=N_TEXT_KEYS):
    M = B * N
    Mk = B * nk
    Gc = G if d_ctx % G == 0 else 64
    return [
        (prefix + "attn1.q", M, B, N, C, C, G),
        (prefix + "attn1.k", M, B, N, C, C, G),
        (prefix + "attn1.v", M, B, N, C, C, G),
        (prefix + "attn1.out", M, B, N, C, C, G),
        (prefix + "attn2.q", M, B, N, C, C, G),
        (prefix + "attn2.k", Mk, B, nk, d_ctx, C, Gc),
        (prefix + "attn2.v", Mk, B, nk, d_ctx, C, Gc),
        (prefix + "attn2.out", M, B, N, C, C, G),
        (prefix + "ff.in", M, B, N, C, 8 * C, G),
        (prefix + "ff.out", M, B, N, 4 * C, C, G),
    ]


def config1():
    """One DGQ linear at the 16x16 latent: M = 2*256, 1280 -> 1280, G = 128."""
    return dict(seed=0, linears=[("l0", 512, 2, 256, 1280, 1280, 128)],
                modes=[(8, 8)], attention=[])


def config2():
    """DGQ linears at the 64x64 latent, M = 2*4096, C = 320, G = 64."""
    B, N, C, G = 2, 4096, 320, 64
    M = B * N
    lin = [("q", M, B, N, C, C, G), ("k", M, B, N, C, C, G),
           ("v", M, B, N, C, C, G), ("out", M, B, N, C, C, G),
           ("ff.in", M, B, N, C, 8 * C, G), ("ff.out", M, B, N, 4 * C, C, G)]
    return dict(seed=2000, linears=lin, modes=[(8, 8), (4, 8)], attention=[])


def config3():
    """Cross-attention with log2-quantized probabilities at the 64x64 latent."""
    return dict(seed=3000, linears=[], modes=[],
                attention=[("xattn", 2, 4096, 8, 40, N_TEXT_KEYS, 768)],
                attn_bits=[4, 8])


# (tokens per sample, channels, number of transformer blocks at that stage)
SD14_STAGES = [(4096, 320, 5), (1024, 640, 5), (256, 1280, 5), (64, 1280, 1)]


def config4():
    """All DGQ linears and cross-attentions of one SD-v1.4 UNet step at 512x512.

    Block multiplicities 5/5/5/1 (2 down + 3 up per resolution, 1 mid) follow
    the public SD-v1.4 architecture; each distinct shape is listed once with a
    repeat count.
    """
    B = 2
    stages = []
    for si, (N, C, reps) in enumerate(SD14_STAGES):
        G = 64 if C == 320 else 128
        stages.append(dict(
            reps=reps,
            linears=_block_linears("s%d." % si, B, N, C, G, 768),
            attention=[("s%d.xattn" % si, B, N, 8, C // 8, N_TEXT_KEYS, 768)]))
    return dict(seed=4000, stages=stages, modes=[(8, 8), (8, 4)], attn_bits=[8])


def config5():
    """SDXL-scale sweep: 1024x1024 image, batch 8 x 2 (CFG), G = 128."""
    B = 16
    lin = []
    for tag, N, C in (("hi.", 4096, 640), ("lo.", 1024, 1280)):
        M = B * N
        lin += [(tag + "q", M, B, N, C, C, 128), (tag + "k", M, B, N, C, C, 128),
                (tag + "v", M, B, N, C, C, 128), (tag + "out", M, B, N, C, C, 128),
                (tag + "xk", B * N_TEXT_KEYS, B, N_TEXT_KEYS, 2048, C, 128),
                (tag + "xv", B * N_TEXT_KEYS, B, N_TEXT_KEYS, 2048, C, 128),
                (tag + "ff.in", M, B, N, C, 8 * C, 128),
                (tag + "ff.out", M, B, N, 4 * C, C, 128)]
    return dict(seed=5000, linears=lin, modes=[(8, 8), (4, 8)],
                attention=[("xattn", B, 4096, 10, 64, N_TEXT_KEYS, 2048)],
                attn_bits=[4, 8])


def layer_seed(cfg_seed: int, layer_index: int) -> int:
    return cfg_seed + layer_index
