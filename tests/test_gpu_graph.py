"""The library enqueues kernels only (no allocation, no synchronisation, no memset), so its calls can be
recorded into a HIP graph.  Replays are compared with eager calls on the same inputs, several times,
with eager work and synchronisations between the replays."""
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("split", [False, True])
def test_decode_step_in_a_graph(split):
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd import synth
    dev = torch.device(DEV)
    ws = gsa.alloc_decode_workspace(4, 2, 128, 128, 64, dev) if split else None   # two kernels per step
    x = synth.make_decode_inputs(4, 2, 128, 128, 64, 6, seed=31)
    q, k, v, g = (x[n].to(dev) for n in ("q", "k", "v", "g"))
    # eager reference: six steps
    Ke, Ve = x["K"].to(dev), x["V"].to(dev)
    ref = [gsa.gsa_decode_step(q[t], k[t], v[t], g[t], Ke, Ve, workspace=ws).clone() for t in range(6)]
    # graph: one step reading its inputs from static buffers
    Kg, Vg = x["K"].to(dev), x["V"].to(dev)
    qs, ks, vs, gs = q[0].clone(), k[0].clone(), v[0].clone(), g[0].clone()
    out = torch.empty_like(vs)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up outside the capture (first-use attribute calls)
        Kw, Vw = Kg.clone(), Vg.clone()
        gsa.gsa_decode_step(qs, ks, vs, gs, Kw, Vw, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gsa.gsa_decode_step(qs, ks, vs, gs, Kg, Vg, out=out, workspace=ws)
    for t in range(6):
        qs.copy_(q[t]); ks.copy_(k[t]); vs.copy_(v[t]); gs.copy_(g[t])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref[t]), "replay %d differs from the eager step" % t
        _ = (Kg.sum() + Vg.sum()).item()     # eager work between replays
    assert torch.equal(Kg, Ke) and torch.equal(Vg, Ve)


def test_forward_backward_in_a_graph():
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd.synth import GsaConfig, make_inputs
    dev = torch.device(DEV)
    cfg = GsaConfig("graph", B=2, T=200, H=2, d_k=128, d_v=64, m=32, dtype="bf16", seed=32)
    x = make_inputs(cfg)
    q, k, v, g, dO = (x[n].to(dev) for n in ("q", "k", "v", "g", "dO"))
    prob = gsa.make_problem(q, v, g, 1.0, None)
    ws = gsa.alloc_workspace(prob, True, dev)

    def step():
        o, z, _, _ = gsa.gsa_fwd(q, k, v, g, workspace=ws)
        return (o,) + tuple(gsa.gsa_bwd(q, k, v, g, z, dO, workspace=ws)[:4])

    ref = [t.clone() for t in step()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = step()
    for rep in range(3):
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got, want), "replay %d differs from the eager call" % rep
        _ = step()[0].float().sum().item()   # eager work on the same workspace between replays
