"""GPU parity of gsa_decode_step against the fp64 oracle (same seeded inputs)."""
import numpy as np
import pytest
import torch

from tests.util import check, to_np64

pytestmark = pytest.mark.gpu


def _run(oracle, B, H, d_k, d_v, m, steps, dtype, scale=1.0, seed=5, split=False, given=False, readout="softmax"):
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd import synth
    x = synth.make_decode_inputs(B, H, d_k, d_v, m, steps, state_std=0.1, seed=seed, dtype=dtype)
    dev = torch.device("cuda:0")
    Kg, Vg = x["K"].to(dev), x["V"].to(dev)
    q, k, v, g = (x[n].to(dev) for n in ("q", "k", "v", "g"))
    Ko, Vo = to_np64(x["K"]).copy(), to_np64(x["V"]).copy()
    qn, kn, vn, gn = (to_np64(x[n]) for n in ("q", "k", "v", "g"))
    ws = gsa.alloc_decode_workspace(B, H, d_k, d_v, m, dev) if split else None   # through gsa_decode_step_ws
    sg = sn = [None] * steps
    if given:     # write intensities of their own, around the tied value (through gsa_decode_step_ex)
        gen = torch.Generator().manual_seed(seed + 77)
        s_cpu = (2.0 * torch.rand(x["g"].shape, generator=gen) * -torch.expm1(x["g"])).float()
        sg, sn = s_cpu.to(dev), to_np64(s_cpu)
    outs = []
    for t in range(steps):
        outs.append(gsa.gsa_decode_step(q[t], k[t], v[t], g[t], Kg, Vg, scale=scale, workspace=ws, s=sg[t],
                                        readout=readout))
    torch.cuda.synchronize()
    worst = 0.0
    for t in range(steps):
        oo = oracle.decode_step(qn[t], kn[t], vn[t], gn[t], Ko, Vo, scale=scale, s=sn[t], readout=readout)
        r = check("o[step %d]" % t, to_np64(outs[t]), oo, dtype)[0]
        worst = max(worst, r)
    # memories are fp32 on the GPU whatever the I/O dtype
    check("K_state", to_np64(Kg), Ko, "f32" if dtype == "f32" else "bf16")
    check("V_state", to_np64(Vg), Vo, "f32" if dtype == "f32" else "bf16")
    assert np.max(np.abs(to_np64(Kg) - Ko)) / np.max(np.abs(Ko)) < 1e-5
    return worst


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,d_k,d_v,m", [(2, 2, 64, 64, 16), (3, 1, 128, 192, 32), (2, 3, 640, 576, 64),
                                           (1, 2, 1024, 64, 64), (1, 1, 256, 256, 128)])
def test_decode_small_shapes(oracle, B, H, d_k, d_v, m, dtype):
    _run(oracle, B, H, d_k, d_v, m, steps=5, dtype=dtype, scale=0.9)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,d_k,d_v,m", [(2, 2, 64, 64, 16), (3, 1, 128, 192, 32), (2, 3, 640, 576, 64),
                                           (1, 2, 1024, 64, 64), (1, 1, 256, 256, 128), (1, 4, 512, 512, 64),
                                           (32, 4, 128, 64, 32), (33, 4, 64, 64, 16), (17, 4, 192, 128, 64),
                                           (9, 8, 64, 1024, 128), (24, 3, 128, 64, 32)])
def test_decode_with_workspace(oracle, B, H, d_k, d_v, m, dtype):
    """gsa_decode_step_ws: memories spread over several workgroups up to 64 pairs; past that the call takes
    the one-workgroup form."""
    _run(oracle, B, H, d_k, d_v, m, steps=5, dtype=dtype, scale=0.9, split=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("readout,given", [("softmax", True), ("identity", False), ("swish", True), ("relu", True),
                                           ("relu2", False)])
def test_decode_variants(oracle, readout, given, split, dtype):
    """gsa_decode_step_ex: write intensity as an input of its own, element-wise read-outs; one workgroup per
    pair and the split form (6 pairs); 70 pairs with a workspace take the one-workgroup form."""
    _run(oracle, 3, 2, 128, 192, 32, steps=4, dtype=dtype, scale=0.9, split=split, given=given, readout=readout)
    if split:
        _run(oracle, 35, 2, 64, 64, 64, steps=2, dtype=dtype, scale=0.9, split=True, given=given, readout=readout)


def test_decode_with_workspace_matches_plain_step():
    """Both entry points on the same inputs: identical memories, outputs equal up to fp32 rounding order;
    the split form is reproducible."""
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd import synth
    dev = torch.device("cuda:0")
    B, H, d, m = 1, 4, 512, 64
    x = synth.make_decode_inputs(B, H, d, d, m, 3, seed=9, dtype="f32")
    q, k, v, g = (x[n].to(dev) for n in ("q", "k", "v", "g"))
    ws = gsa.alloc_decode_workspace(B, H, d, d, m, dev)
    assert ws.numel() >= B * H * (m // 4) * (d + 2) * 4
    runs = []
    for use_ws in (None, ws, ws):
        K, V = x["K"].to(dev), x["V"].to(dev)
        outs = [gsa.gsa_decode_step(q[t], k[t], v[t], g[t], K, V, workspace=use_ws).clone() for t in range(3)]
        runs.append((outs, K, V))
    for t in range(3):
        torch.testing.assert_close(runs[1][0][t], runs[0][0][t], rtol=1e-5, atol=1e-6)
        assert torch.equal(runs[1][0][t], runs[2][0][t])
    assert torch.equal(runs[0][1], runs[1][1]) and torch.equal(runs[0][2], runs[1][2])


def test_decode_workload_512_steps_batch64(oracle):
    """The decode workload: 512 steps at batch 64, H=4, m=64, d=512 from memories ~ N(0, 0.1^2)."""
    from paper_2409_07146_amd import synth
    d = synth.DECODE
    _run(oracle, d["B"], d["H"], d["d_k"], d["d_v"], d["m"], d["steps"], "bf16", seed=d["seed"])


def test_decode_extreme_gates(oracle):
    import paper_2409_07146_amd as gsa
    dev = torch.device("cuda:0")
    gen = torch.Generator().manual_seed(3)
    B, H, d, m = 2, 2, 128, 64
    K = torch.randn(B, H, m, d, generator=gen)
    V = torch.randn(B, H, m, d, generator=gen)
    q, k, v = (torch.randn(B, H, d, generator=gen) for _ in range(3))
    g = torch.zeros(B, H, m)
    g[0] = -100.0                     # full forget: o = v
    Kg, Vg = K.to(dev), V.to(dev)
    o = gsa.gsa_decode_step(q.to(dev), k.to(dev), v.to(dev), g.to(dev), Kg, Vg)
    Ko, Vo = to_np64(K).copy(), to_np64(V).copy()
    oo = oracle.decode_step(to_np64(q), to_np64(k), to_np64(v), to_np64(g), Ko, Vo)
    check("o", to_np64(o), oo, "f32")
    np.testing.assert_allclose(to_np64(o)[0], to_np64(v)[0], atol=1e-6)
    np.testing.assert_array_equal(to_np64(Kg)[1], to_np64(K)[1])   # g = 0 leaves memories untouched


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefill_then_decode(oracle, dtype):
    """The serving pattern of the paper's latency figure: gsa_fwd over a prompt hands its final
    memories to a loop of gsa_decode_step calls.  The whole thing must equal the recurrence run
    over prompt + generated tokens in one go (oracle forward over the concatenation)."""
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd.synth import GsaConfig, make_inputs
    B, P, N, H, d_k, d_v, m = 2, 150, 24, 2, 128, 64, 32
    cfg = GsaConfig("prefill", B=B, T=P + N, H=H, d_k=d_k, d_v=d_v, m=m, dtype=dtype, seed=21)
    x = make_inputs(cfg)
    dev = torch.device("cuda:0")
    q, k, v, g = (x[n].to(dev) for n in ("q", "k", "v", "g"))
    o_pre, _, KT, VT = gsa.gsa_fwd(q[:, :P].contiguous(), k[:, :P].contiguous(), v[:, :P].contiguous(),
                                   g[:, :P].contiguous(), scale=0.7, final_state=True)
    outs = [gsa.gsa_decode_step(q[:, P + t].contiguous(), k[:, P + t].contiguous(), v[:, P + t].contiguous(),
                                g[:, P + t].contiguous(), KT, VT, scale=0.7) for t in range(N)]
    torch.cuda.synchronize()
    ref = oracle.fwd(*(to_np64(x[n]) for n in ("q", "k", "v", "g")), scale=0.7)
    check("o[prompt]", to_np64(o_pre), ref["o"][:, :P], dtype)
    got = np.stack([to_np64(t) for t in outs], axis=1)
    check("o[generated]", got, ref["o"][:, P:], dtype)
    check("KT", to_np64(KT), ref["KT"], dtype)
    check("VT", to_np64(VT), ref["VT"], dtype)
