"""GPU parity on the layer shapes of one SD-v1.4 UNet step at 512x512 (batch 2):
every distinct quantized linear of the four stages in both modes (A8W8, A8W4)
and the cross-attention of every stage with 8-bit codes.  Full-size GPU runs;
the oracle checks sampled rows of the linears (all outputs, all accumulators)
and whole prompts of the attention.  Head dims 40 and 80 run on the matrix
cores, 160 on the fp32 vector kernel."""
import numpy as np
import pytest

import dgq_inputs as di
from test_gpu_linear import _run_layer, tile_rows
from test_gpu_xattn import _compare

pytestmark = pytest.mark.gpu

CFG4 = di.config4()


@pytest.fixture(scope="module")
def dgq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2501_04304_amd as m
    m.lib()
    return m


def _distinct_linears():
    out, seen, li = [], set(), 0
    for st in CFG4["stages"]:
        for ent in st["linears"]:
            name, M, B, N, C, O, G = ent
            key = (M, C, O, G)
            if key not in seen:
                seen.add(key)
                out.append((li, ent))
            li += 1
    return out


LINEARS = _distinct_linears()


@pytest.mark.parametrize("mode", CFG4["modes"])
@pytest.mark.parametrize("li,ent", LINEARS, ids=[e[1][0] for e in LINEARS])
def test_config4_linears(dgq, oracle, li, ent, mode):
    name, M, B, N, C, O, G = ent
    seed = di.layer_seed(CFG4["seed"], li)
    run = di.linear_case(seed, B, N, C, O)
    cal = di.linear_case(seed, B, N, C, O, calib=True)
    rows = tile_rows(M, seed, run["rows_ot"][:4])
    _run_layer(dgq, oracle, run, cal, mode[0], mode[1], G, sample_rows=rows)


@pytest.mark.parametrize("si", range(len(CFG4["stages"])))
def test_config4_attention(dgq, oracle, si):
    from oracle.guard import guarded_attention_case
    name, B, N, H, d, nk, d_ctx = CFG4["stages"][si]["attention"][0]
    c, _ = guarded_attention_case(CFG4["seed"] + 900 + si, B, N, H, d, nk=nk, d_ctx=d_ctx,
                                  bits_list=(8,))
    # the prompt scale: 1e-6 on the three large stages; the 8 x 8 stage (64 queries, its
    # maximum decided by one row) takes the bar derived from its logits' magnitude
    _compare(dgq, oracle, c, 8, exact=True, s_rtol=1e-6 if N >= 256 else None)
