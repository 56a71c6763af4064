"""The hot calls only enqueue kernels (no allocation, no synchronisation, no memset
nodes), so a caller may capture them in a HIP graph.  One layer, one attention, a chained
gated layer and a self-attention are captured once and replayed several times, with eager work and synchronisations between
the replays; every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest

import dgq_inputs as di

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


def test_captured_step_replays_like_eager(dgq):
    import torch
    run = di.linear_case(31, 2, 700, 320, 384)
    cal = di.linear_case(31, 2, 700, 320, 384, calib=True)
    att = di.attention_case(32, 2, 500, 4, 40, nk=77, d_ctx=64)
    x = _dev(run["X"])
    g = dgq.dgq_calibrate_groups(_dev(cal["X"]), 8, 64, 2)
    w = dgq.dgq_pack_weight(g, _dev(run["W"]), None, 8)
    M, O = x.shape[0], run["W"].shape[0]
    # zeros, not empty: the rows of the last 32-row block beyond M are never written, and
    # the comparison below is over the whole buffer
    codes = torch.zeros(dgq.codes_shape(g, M), dtype=torch.int8, device="cuda")
    cls = torch.empty(M, dtype=torch.uint8, device="cuda")
    y = torch.empty((M, O), dtype=torch.float32, device="cuda")
    q, k, v, kb = (_dev(att[n]) for n in ("Q", "K", "V", "key_bias"))
    vhat = torch.empty_like(v)
    out = torch.empty_like(q)
    s = torch.empty(q.shape[0], dtype=torch.float32, device="cuda")
    ws = torch.empty(max(16, dgq.dgq_xattn_workspace_bytes(q.shape[0], q.shape[1], q.shape[2], q.shape[3], 77)),
                     dtype=torch.uint8, device="cuda")

    # the calls beside the timed step: a chained gated layer and a self-attention
    g2 = dgq.dgq_calibrate_kmeans(_dev(np.random.default_rng(1).standard_normal((256, O // 2)).astype(np.float32)),
                                  8, 4, dgq.DIM_CHANNEL)
    wf = dgq.dgq_pack_weight_gated_for(g, g2, _dev(run["W"]), None, 8)
    codes2 = torch.zeros(dgq.codes_shape(g2, M), dtype=torch.int8, device="cuda")
    cls2 = torch.empty(M, dtype=torch.uint8, device="cuda")
    sa = di.selfattn_case(33, 2, 200, 2, 40)
    sq, sk, sv = (_dev(sa[n]) for n in ("Q", "K", "V"))
    s_in = torch.ones(2, dtype=torch.float32, device="cuda")
    so = torch.empty_like(sq)
    smax = torch.empty(2, dtype=torch.float32, device="cuda")
    sws = torch.empty(dgq.dgq_selfattn_workspace_bytes(2, 200, 2, 40), dtype=torch.uint8, device="cuda")

    def step():
        dgq.dgq_quantize_act(g, x, codes=codes, row_class=cls)
        dgq.dgq_linear(g, w, codes, cls, y=y)
        dgq.dgq_quantize_value(v, 8, v_hat=vhat)
        dgq.dgq_xattn_logq(q, k, vhat, kb, 8, out=out, scale_out=s, workspace=ws)
        dgq.dgq_linear_geglu_requant(g, wf, codes, cls, g2, codes_next=codes2, row_class_next=cls2)
        dgq.dgq_selfattn_logq(sq, sk, sv, 8, s_in, out=so, scale_out=smax, workspace=sws)

    step()  # eager: also the one-time kernel attributes, which are no stream work
    torch.cuda.synchronize()
    want = [t.clone() for t in (codes, cls, y, vhat, out, s, codes2, cls2, so, smax)]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for rep in range(4):
        for t in (codes, cls, y, vhat, out, s, codes2, cls2, so, smax):
            t.zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("codes", "row_class", "y", "v_hat", "out", "scale", "codes_next",
                                   "row_class_next", "self_out", "self_max"),
                                  (codes, cls, y, vhat, out, s, codes2, cls2, so, smax), want):
            assert torch.equal(got, ref), "replay %d: %s differs from the eager result" % (rep, name)
        if rep == 1:                       # and an eager call in between
            step()
            torch.cuda.synchronize()
    wf.free()
    w.free()
    g.free()
    g2.free()
