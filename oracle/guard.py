"""Margin guard for the log2 attention codes (test infrastructure).

The code clamp(rne(-log2(A/s))) is discontinuous at half-integers, and a CPU
double evaluation and a GPU fp32 evaluation of the same probability differ in
the last bits.  For bit-exact comparisons the tests therefore use inputs on
which no decision lies within DELTA (in log2 units) of a rounding boundary:
query vectors whose row has such an element are re-drawn (dgq_inputs'
`redraw` counter) until the prompt scales and all margins are stable.  DELTA is
about 100x the fp32 evaluation error of the log-domain code.
"""
from __future__ import annotations

import numpy as np

import dgq_inputs as di

from . import attn_probs, xattn_logq

DELTA = 2.0 ** -13


def guarded_attention_case(seed, B, N, H, d, nk=77, d_ctx=768, bits_list=(4, 8), max_iter=40):
    """Returns (case dict, number of re-drawn query vectors)."""
    redraw = np.zeros((B, N, H), np.int32)
    for _ in range(max_iter):
        c = di.attention_case(seed, B, N, H, d, nk=nk, d_ctx=d_ctx, redraw=redraw)
        A = attn_probs(c["Q"], c["K"], c["key_bias"])
        bad = np.zeros((B, H, N), bool)
        for bits in bits_list:
            r = xattn_logq(A, c["V"], bits)
            bad |= (r["margin"] < DELTA).any(-1)
        if not bad.any():
            return c, int((redraw > 0).sum())
        redraw[np.transpose(bad, (0, 2, 1))] += 1
    raise RuntimeError("margin guard did not converge")
