"""A decode step is a fixed sequence of kernel launches on the caller's stream (no
allocation, no memset, no host synchronisation), so a token step through several layers
can be captured in a HIP graph and replayed.  Every replay is checked against the eager
result, with eager work and synchronisations between replays."""
import numpy as np
import pytest

import bct_synth as syn
from _util import make_pair, to_dev, to_np

pytestmark = pytest.mark.gpu


def test_captured_token_step_replays_exactly():
    import torch
    import paper_2411_15785_amd as P
    from oracle import bct_ref as R
    w = syn.Workload("graph", 3, 4, 8, 4, 128, 512, "bf16", 6)
    L = w.layers
    eager = [make_pair(w, R.RefCache, P.BctCache, layer=l)[1] for l in range(L)]
    graphed = [make_pair(w, R.RefCache, P.BctCache, layer=l)[1] for l in range(L)]
    # static input/output buffers of the captured step
    sq = [torch.empty((w.B, w.Hq, w.d), dtype=torch.bfloat16, device="cuda:0") for _ in range(L)]
    swq = [torch.empty((w.B, w.Hkv, w.d), dtype=torch.bfloat16, device="cuda:0") for _ in range(L)]
    swv = [torch.empty_like(a) for a in swq]
    sout = [torch.empty_like(a) for a in sq]

    def load_inputs(t):
        for l in range(L):
            q, wq, wv = (to_dev(a, w.dtype) for a in syn.make_step(w, t, l))
            sq[l].copy_(q), swq[l].copy_(wq), swv[l].copy_(wv)

    def token_step(caches, outs):
        for l in range(L):
            caches[l].decode_step(sq[l], swq[l], swv[l], outs[l])

    load_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream, as torch asks
        token_step(graphed, sout)
    torch.cuda.current_stream().wait_stream(side)
    eout = [torch.empty_like(a) for a in sq]
    token_step(eager, eout)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    load_inputs(1)
    with torch.cuda.graph(g):
        token_step(graphed, sout)
    # the capture itself ran nothing: the library's host-side step counters moved, the state did not
    for t in range(1, w.decode_steps):
        load_inputs(t)
        g.replay()
        token_step(eager, eout)
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(sout[l], eout[l]), f"replay of step {t}, layer {l}: out differs from eager"
            assert torch.equal(graphed[l].values_view(), eager[l].values_view()), f"step {t}, layer {l}: state"
        # unrelated eager work between replays
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)


def test_captured_stack_step_replays_exactly():
    """The whole decoder token-step (glue kernels and attention, the greedy ids fed back in place) as one graph:
    every replay gives the ids, logits and cache state of the eager stack."""
    import torch
    from paper_2411_15785_amd import model as M
    s = M.StackShape(n_layers=2, dim=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=320,
                     capacity_M=128, batch=3)
    w = syn.make_stack_weights(s, seed=8)

    def dev_weights():
        d = lambda a: to_dev(a, "bf16")
        return {"embed": d(w["embed"]), "final_norm": d(w["final_norm"]), "head": d(w["head"]),
                "layers": [{k: d(v) for k, v in lw.items()} for lw in w["layers"]], "keys": [d(k) for k in w["keys"]]}

    eager, graphed = M.BctStack(s, dev_weights()), M.BctStack(s, dev_weights())
    ids0 = torch.from_numpy(syn.make_token_ids(8, 0, s.batch, s.vocab)).cuda()
    e_ids, g_ids = ids0.clone(), ids0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on a side stream: allocates the activation buffers
        graphed.forward(g_ids, next_ids=g_ids)
    torch.cuda.current_stream().wait_stream(side)
    eager.forward(e_ids, next_ids=e_ids)
    torch.cuda.synchronize()
    assert torch.equal(e_ids, g_ids)

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        _, g_logits = graphed.forward(g_ids, next_ids=g_ids)
    for t in range(5):
        g.replay()
        _, e_logits = eager.forward(e_ids, next_ids=e_ids)
        torch.cuda.synchronize()
        assert torch.equal(g_ids, e_ids), f"replay {t}: greedy ids differ from eager"
        assert torch.equal(g_logits, e_logits), f"replay {t}: logits differ from eager"
        for l in range(s.n_layers):
            assert torch.equal(graphed.caches[l].values_view(), eager.caches[l].values_view()), f"replay {t}: state"
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)


def test_captured_prefill_chunk_replays_exactly():
    """A prefill chunk (transpose, statistics, state and read kernels; no allocation, no memset) captured as one
    graph: every replay, with the program's own eager chunk and unrelated work in between, gives the eager
    outputs and state bit for bit."""
    import torch
    import paper_2411_15785_amd as P
    from oracle import bct_ref as R
    w = syn.Workload("graph_pf", 1, 2, 4, 2, 128, 256, "bf16", 0)
    T = 200
    eager = make_pair(w, R.RefCache, P.BctCache, max_prefill_T=T)[1]
    graphed = make_pair(w, R.RefCache, P.BctCache, max_prefill_T=T)[1]
    sq = torch.empty((w.B, T, w.Hq, w.d), dtype=torch.bfloat16, device="cuda:0")
    swq = torch.empty((w.B, T, w.Hkv, w.d), dtype=torch.bfloat16, device="cuda:0")
    swv = torch.empty_like(swq)
    sout, eout = torch.empty_like(sq), torch.empty_like(sq)

    def load_inputs(k):
        q, wq, wv = (to_dev(a, w.dtype) for a in syn.make_step(w, k * T, 0, T=T))
        sq.copy_(q), swq.copy_(wq), swv.copy_(wv)

    load_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graphed.prefill(sq, swq, swv, T, sout)
    torch.cuda.current_stream().wait_stream(side)
    eager.prefill(sq, swq, swv, T, eout)
    torch.cuda.synchronize()
    assert torch.equal(sout, eout)

    g = torch.cuda.CUDAGraph()
    load_inputs(1)
    with torch.cuda.graph(g):
        graphed.prefill(sq, swq, swv, T, sout)
    for k in range(1, 5):
        load_inputs(k)
        g.replay()
        eager.prefill(sq, swq, swv, T, eout)
        torch.cuda.synchronize()
        assert torch.equal(sout, eout), f"replay of chunk {k}: out differs from eager"
        assert torch.equal(graphed.values_view(), eager.values_view()), f"chunk {k}: state"
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)


def test_captured_static_and_keyed_steps_replay_exactly():
    """The step that takes its scratch from the library's own device array (made for callers under graph
    capture) and the step that also moves per-sequence keys, captured together as one graph: each replay gives
    what the eager workspace step / eager keyed step give, bit for bit, state and keys included."""
    import torch
    import paper_2411_15785_amd as P
    from oracle import bct_ref as R
    w = syn.Workload("graph_sk", 1, 2, 4, 2, 128, 320, "bf16", 6)
    e_plain = make_pair(w, R.RefCache, P.BctCache, mv0=True)[1]
    g_static = make_pair(w, R.RefCache, P.BctCache, mv0=True)[1]
    e_keyed = make_pair(w, R.RefCache, P.BctCache, flags=1, mv0=True)[1]
    g_keyed = make_pair(w, R.RefCache, P.BctCache, flags=1, mv0=True)[1]
    bf = dict(dtype=torch.bfloat16, device="cuda:0")
    sq, swq = torch.empty((w.B, w.Hq, w.d), **bf), torch.empty((w.B, w.Hkv, w.d), **bf)
    swv, swk = torch.empty_like(swq), torch.empty_like(swq)
    kappa = torch.full((w.B, w.Hkv), 0.5, device="cuda:0")
    o_static, o_keyed, o_plain, o_ekeyed = (torch.empty_like(sq) for _ in range(4))

    def load_inputs(t):
        q, wq, wv = (to_dev(a, w.dtype) for a in syn.make_step(w, t))
        wk = to_dev(syn.pack(syn.normal(syn.layer_seed(0), 8, t, (w.B, w.Hkv, w.d)), w.dtype), w.dtype)
        sq.copy_(q), swq.copy_(wq), swv.copy_(wv), swk.copy_(wk)

    def graphed_steps():
        g_static.decode_step_static(sq, swq, swv, o_static)
        g_keyed.decode_step_keyed(sq, swq, swv, swk, out=o_keyed, key_gate=kappa)

    def eager_steps():
        e_plain.decode_step(sq, swq, swv, o_plain)
        e_keyed.decode_step_keyed(sq, swq, swv, swk, out=o_ekeyed, key_gate=kappa)

    load_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graphed_steps()
    torch.cuda.current_stream().wait_stream(side)
    eager_steps()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    load_inputs(1)
    with torch.cuda.graph(g):
        graphed_steps()
    for t in range(1, 6):
        load_inputs(t)
        g.replay()
        eager_steps()
        torch.cuda.synchronize()
        assert torch.equal(o_static, o_plain), f"replay of step {t}: static-scratch step differs from eager"
        assert torch.equal(g_static.values_view(), e_plain.values_view()), f"step {t}: state of the static-scratch step"
        assert torch.equal(o_keyed, o_ekeyed), f"replay of step {t}: keyed step differs from eager"
        assert torch.equal(g_keyed.values_view(), e_keyed.values_view()), f"step {t}: state of the keyed step"
        assert torch.equal(g_keyed.keys_view(), e_keyed.keys_view()), f"step {t}: keys of the keyed step"
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)
