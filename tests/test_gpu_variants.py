"""GPU parity of gsa_fwd_ex / gsa_bwd_ex against the fp64 oracle: write intensity as an input of its
own (Algorithm 1's I; ABC when g = 0) and the read-outs of the paper's ablation table."""
import numpy as np
import pytest
import torch

from tests.util import check, suffix_mass, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
READOUTS = ["softmax", "identity", "swish", "relu", "relu2"]


def _inputs(B, T, H, d_k, d_v, m, dtype, seed, given, abc=False):
    from paper_2409_07146_amd import synth
    cfg = synth.GsaConfig("variant", B=B, T=T, H=H, d_k=d_k, d_v=d_v, m=m, dtype=dtype, seed=seed, init_state_std=0.5)
    x = synth.make_inputs(cfg)
    gen = torch.Generator().manual_seed(seed + 1000)
    s = None
    if abc:       # Eq. (abc_phi): a cumulative softmax over the tokens, no decay
        a = torch.exp(torch.randn(B, T, H, m, generator=gen))
        s = (a / torch.cumsum(a, dim=1)).float()
        x["g"] = torch.zeros_like(x["g"])
    elif given:   # independent of the gate, with the tied value 1 - exp(g) as its mean
        s = (2.0 * torch.rand(B, T, H, m, generator=gen) * -torch.expm1(x["g"])).float()
    x["s"] = s
    gs = torch.Generator().manual_seed(seed + 2000)
    x["dKT"] = torch.randn(x["K0"].shape, generator=gs) * 0.5
    x["dVT"] = torch.randn(x["V0"].shape, generator=gs) * 0.5
    return cfg, x


def _run_and_compare(oracle, cfg, x, readout, scale=1.0):
    import paper_2409_07146_amd as gsa
    dev = torch.device(DEV)
    put = lambda t: None if t is None else t.to(dev)
    d = {n: put(x[n]) for n in ("q", "k", "v", "g", "s", "dO", "K0", "V0", "dKT", "dVT")}
    o, z, KT, VT = gsa.gsa_fwd(d["q"], d["k"], d["v"], d["g"], K0=d["K0"], V0=d["V0"], scale=scale,
                               final_state=True, s=d["s"], readout=readout)
    n64 = lambda t: None if t is None else to_np64(t)
    a = {n: n64(x[n]) for n in ("q", "k", "v", "g", "s", "dO", "K0", "V0", "dKT", "dVT")}
    f = oracle.fwd(a["q"], a["k"], a["v"], a["g"], K0=a["K0"], V0=a["V0"], scale=scale, s=a["s"], readout=readout)
    z_bwd = z
    if readout == "relu":
        # ReLU's slope jumps at z = 0, and a score the two sides see on different sides of zero gives two
        # different (both valid) sub-gradients.  z_saved is an INPUT of the backward call, so here it is
        # the oracle's scores rounded to fp32 (the sign survives the rounding): both sides then decide
        # from the same numbers and the backward is compared on its own.  The kernel's z is checked
        # against the oracle's below like every other output.
        assert np.all(np.abs(f["z"]) > 1e-30)
        z_bwd = torch.from_numpy(f["z"]).float().to(dev)
    res = gsa.gsa_bwd(d["q"], d["k"], d["v"], d["g"], z_bwd, d["dO"], K0=d["K0"], V0=d["V0"], dKT=d["dKT"],
                      dVT=d["dVT"], scale=scale, initial_state_grad=True, s=d["s"], readout=readout)
    torch.cuda.synchronize()
    check("o", to_np64(o), f["o"], cfg.dtype)
    check("z", to_np64(z), f["z"], cfg.dtype)
    check("KT", to_np64(KT), f["KT"], cfg.dtype)
    check("VT", to_np64(VT), f["VT"], cfg.dtype)
    names = ["dq", "dk", "dv", "dg", "dK0", "dV0"] + (["ds"] if x["s"] is not None else [])
    r = oracle.bwd(a["q"], a["k"], a["v"], a["g"], a["dO"], K0=a["K0"], V0=a["V0"], dKT=a["dKT"], dVT=a["dVT"],
                   scale=scale, s=a["s"], readout=readout)
    for n, t in zip(names, res):
        check(n, to_np64(t), r[n], cfg.dtype, residue_of=_residue(n, a, r))


def _residue(name, a, r):
    """With the write intensity an input of its own, dg is the gradient through the decay alone: the suffix
    sum, over all later tokens of the sequence, of dGam_t = (z dz + p dp)_t - (s ds)_t, in which every
    (writer, reader) pair of later tokens enters once with each sign.  It comes out several times smaller
    than the tied gate gradient (which also holds -exp(g) ds) and than what is summed; its error is
    relative to the latter (tests.util.suffix_mass of the oracle's s * ds)."""
    if name == "dg" and a.get("s") is not None:
        return suffix_mass(a["s"] * r["ds"], axis=1)
    return None


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("readout", READOUTS)
@pytest.mark.parametrize("given", [False, True])
def test_variants_small(oracle, readout, given, dtype):
    if readout == "softmax" and not given:
        pytest.skip("that is gsa_fwd / gsa_bwd")
    cfg, x = _inputs(2, 150, 2, 128, 64, 32, dtype, seed=61, given=given)
    _run_and_compare(oracle, cfg, x, readout, scale=0.9)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m", [16, 64, 128])
def test_abc(oracle, m, dtype):
    """No decay, write intensities a cumulative softmax: Eqs. (abc_recurrent), (abc_phi)."""
    cfg, x = _inputs(1, 200, 2, 64, 128, m, dtype, seed=62, given=True, abc=True)
    _run_and_compare(oracle, cfg, x, "softmax")


@pytest.mark.parametrize("readout", ["softmax", "swish"])
def test_variants_at_the_layer_shape(oracle, readout):
    """d = 512, m = 64, bf16, ragged length (several chunks and a tail)."""
    cfg, x = _inputs(1, 333, 2, 512, 512, 64, "bf16", seed=63, given=True)
    _run_and_compare(oracle, cfg, x, readout)


def _sweep_case(seed):
    rng = np.random.default_rng(1000 + seed)
    B, T, H = int(rng.integers(1, 3)), int(rng.integers(1, 400)), int(rng.integers(1, 4))
    d_k, d_v = (int(64 * rng.integers(1, 5)) for _ in range(2))
    m = int(rng.choice([32, 64, 128]))
    dtype = ["bf16", "f32"][int(rng.integers(2))]
    readout = str(rng.choice(READOUTS))
    given = bool(rng.integers(2))
    abc = given and bool(rng.integers(3) == 0)
    if readout == "softmax" and not given:
        given = True
    return B, T, H, d_k, d_v, m, dtype, readout, given, abc, float(rng.choice([0.5, 1.0, 1.3]))


@pytest.mark.parametrize("seed", [10, 12, 28, 48, 56, 87, 97, 119])
def test_variant_sweep_seeds_with_a_small_decay_only_gate_gradient(oracle, seed):
    """Seeded random shapes and options on which a sweep measured the decay-only dg (given write
    intensities, bf16) at 5.1e-3 to 6.6e-3 of its own norm: it is several times smaller than the sums it
    is the difference of, and is held to the residue bar (_residue)."""
    B, T, H, d_k, d_v, m, dtype, readout, given, abc, scale = _sweep_case(seed)
    assert given and dtype == "bf16"
    cfg, x = _inputs(B, T, H, d_k, d_v, m, dtype, seed=seed, given=given, abc=abc)
    for n in ("K0", "V0", "dKT", "dVT"):
        x[n] = x[n] * 0.2
    _run_and_compare(oracle, cfg, x, readout, scale=scale)


def test_strong_writes_independent_of_the_gate(oracle):
    """s ~ U(0,1) against a decay of about 0.9 per token: writes ten times stronger than the tied
    1 - exp(g), the case in which the decay-only dg is the smallest next to its terms."""
    cfg, x = _inputs(2, 200, 2, 128, 64, 32, "bf16", seed=68, given=True)
    gen = torch.Generator().manual_seed(69)
    x["s"] = torch.rand(x["g"].shape, generator=gen).float()
    _run_and_compare(oracle, cfg, x, "softmax")


def test_given_tied_intensity_reproduces_the_plain_calls():
    """s = 1 - exp(g) handed over explicitly: same outputs as gsa_fwd/gsa_bwd, and the two gate gradients
    combine to the tied one by the chain rule."""
    import paper_2409_07146_amd as gsa
    cfg, x = _inputs(2, 130, 2, 128, 128, 64, "f32", seed=64, given=False)
    dev = torch.device(DEV)
    q, k, v, g, dO = (x[n].to(dev) for n in ("q", "k", "v", "g", "dO"))
    s = -torch.expm1(g)
    o0, z0, _, _ = gsa.gsa_fwd(q, k, v, g)
    o1, z1, _, _ = gsa.gsa_fwd(q, k, v, g, s=s)
    torch.testing.assert_close(o1, o0, rtol=2e-5, atol=2e-6)
    b0 = gsa.gsa_bwd(q, k, v, g, z0, dO)
    b1 = gsa.gsa_bwd(q, k, v, g, z1, dO, s=s)
    for i in range(3):
        torch.testing.assert_close(b1[i], b0[i], rtol=1e-4, atol=1e-5)
    torch.testing.assert_close(b1[3] - torch.exp(g) * b1[6], b0[3], rtol=1e-3, atol=2e-4)


def test_bad_readout_is_rejected():
    import ctypes
    from paper_2409_07146_amd import _lib
    lib = _lib.load()
    p = _lib.GsaProblem(B=1, T=64, H=1, d_k=64, d_v=64, m=16, dtype=1, scale=1.0, cu_seqlens=None, n_seqs=0)
    null = ctypes.c_void_p(None)
    assert lib.gsa_fwd_ex(ctypes.byref(p), 7, 0.0, 0, *([null] * 11), null, 0, null) == 2
    assert lib.gsa_bwd_ex(ctypes.byref(p), -1, 0.0, 0, *([null] * 18), null, 0, null) == 2
    assert lib.gsa_fwd_ex(ctypes.byref(p), 0, -1.0, 0, *([null] * 11), null, 0, null) == 2
    assert lib.gsa_fwd_ex(ctypes.byref(p), 0, float("nan"), 0, *([null] * 11), null, 0, null) == 2
    assert lib.gsa_fwd_ex(ctypes.byref(p), 0, 0.0, 2, *([null] * 11), null, 0, null) == 2     # unknown feature map
    assert lib.gsa_bwd_ex(ctypes.byref(p), 0, 0.0, -1, *([null] * 18), null, 0, null) == 2
    assert lib.gsa_decode_step_ex(1, 1, 64, 64, 16, 1, 1.0, 0, 0.0, 5, *([null] * 8), null, 0, null) == 2


def test_variant_on_a_long_sequence(oracle):
    """Given write intensities and an element-wise read-out on a sequence the scans walk in segments."""
    cfg, x = _inputs(1, 3300, 2, 64, 64, 16, "bf16", seed=65, given=True)
    _run_and_compare(oracle, cfg, x, "swish")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("readout,given", [("softmax", False), ("swish", True)])
def test_gate_logits_evaluated_inside(oracle, readout, given, dtype):
    """gate_tau > 0: the g argument holds gate logits u, the kernels use logsigmoid(u)/tau (the layer's
    alpha = sigmoid(W x)^(1/tau), Section 3.3) and dg comes back as the gradient with respect to u.  The oracle
    gets the log gate computed here in fp64, and its dg goes through the chain rule here as well."""
    import paper_2409_07146_amd as gsa
    from scipy.special import expit, log_expit
    tau = 8.0
    cfg, x = _inputs(2, 150, 2, 128, 64, 32, dtype, seed=66, given=given)
    gen = torch.Generator().manual_seed(67)
    u = (torch.randn(x["g"].shape, generator=gen) * 2.0).float()
    g64 = log_expit(to_np64(u)) / tau
    if given:
        x["s"] = (2.0 * torch.rand(u.shape, generator=gen) * -torch.expm1(torch.from_numpy(g64).float())).float()
    dev = torch.device(DEV)
    put = lambda t: None if t is None else t.to(dev)
    d = {n: put(x[n]) for n in ("q", "k", "v", "s", "dO", "K0", "V0", "dKT", "dVT")}
    ud = u.to(dev)
    o, z, KT, VT = gsa.gsa_fwd(d["q"], d["k"], d["v"], ud, K0=d["K0"], V0=d["V0"], final_state=True, s=d["s"],
                               readout=readout, gate_tau=tau)
    res = gsa.gsa_bwd(d["q"], d["k"], d["v"], ud, z, d["dO"], K0=d["K0"], V0=d["V0"], dKT=d["dKT"], dVT=d["dVT"],
                      initial_state_grad=True, s=d["s"], readout=readout, gate_tau=tau)
    torch.cuda.synchronize()
    a = {n: (None if x[n] is None else to_np64(x[n])) for n in ("q", "k", "v", "s", "dO", "K0", "V0", "dKT", "dVT")}
    f = oracle.fwd(a["q"], a["k"], a["v"], g64, K0=a["K0"], V0=a["V0"], s=a["s"], readout=readout)
    check("o", to_np64(o), f["o"], dtype)
    check("KT", to_np64(KT), f["KT"], dtype)
    r = oracle.bwd(a["q"], a["k"], a["v"], g64, a["dO"], K0=a["K0"], V0=a["V0"], dKT=a["dKT"], dVT=a["dVT"],
                   s=a["s"], readout=readout)
    r["dg"] = r["dg"] * (1.0 - expit(to_np64(u))) / tau
    names = ["dq", "dk", "dv", "dg", "dK0", "dV0"] + (["ds"] if given else [])
    for n, t in zip(names, res):
        check(n, to_np64(t), r[n], dtype)
    # decode step with the same option, continuing from the final memories
    q1, k1, v1, u1 = (t[:, -1].contiguous() for t in (d["q"], d["k"], d["v"], ud))
    s1 = None if d["s"] is None else d["s"][:, -1].contiguous()
    Kc, Vc = KT.clone(), VT.clone()
    o1 = gsa.gsa_decode_step(q1, k1, v1, u1, Kc, Vc, s=s1, readout=readout, gate_tau=tau)
    Ko, Vo = f["KT"].copy(), f["VT"].copy()
    oo = oracle.decode_step(a["q"][:, -1], a["k"][:, -1], a["v"][:, -1], g64[:, -1], Ko, Vo,
                            s=None if a["s"] is None else a["s"][:, -1], readout=readout)
    check("decode o", to_np64(o1), oo, dtype)
    check("decode K", to_np64(Kc), Ko, dtype)


def _feature_map_case(oracle, cfg, x, readout="softmax", cu=None, scale=1.0):
    """feature_map="swish": q, k, v are raw projections and the kernels apply phi(x) = x*sigmoid(x) (Section 3.3)
    as they load them.  The oracle gets phi of the same raw values computed here in fp64, and its dq, dk, dv go
    through phi's slope here as well."""
    import paper_2409_07146_amd as gsa
    from scipy.special import expit
    dev = torch.device(DEV)
    put = lambda t: None if t is None else t.to(dev)
    d = {n: put(x[n]) for n in ("q", "k", "v", "g", "s", "dO", "K0", "V0", "dKT", "dVT")}
    cud = None if cu is None else torch.tensor(cu, dtype=torch.int32, device=dev)
    o, z, KT, VT = gsa.gsa_fwd(d["q"], d["k"], d["v"], d["g"], K0=d["K0"], V0=d["V0"], scale=scale, cu_seqlens=cud,
                               final_state=True, s=d["s"], readout=readout, feature_map="swish")
    res = gsa.gsa_bwd(d["q"], d["k"], d["v"], d["g"], z, d["dO"], K0=d["K0"], V0=d["V0"], dKT=d["dKT"],
                      dVT=d["dVT"], scale=scale, cu_seqlens=cud, initial_state_grad=True, s=d["s"], readout=readout,
                      feature_map="swish")
    torch.cuda.synchronize()
    n64 = lambda t: None if t is None else to_np64(t)
    a = {n: n64(x[n]) for n in ("q", "k", "v", "g", "s", "dO", "K0", "V0", "dKT", "dVT")}
    phi = lambda u: u * expit(u)
    slope = lambda u: expit(u) * (1.0 + u * (1.0 - expit(u)))
    cun = None if cu is None else np.asarray(cu, dtype=np.int32)
    f = oracle.fwd(phi(a["q"]), phi(a["k"]), phi(a["v"]), a["g"], cu_seqlens=cun, K0=a["K0"], V0=a["V0"], scale=scale,
                   s=a["s"], readout=readout)
    for n, t in (("o", o), ("z", z), ("KT", KT), ("VT", VT)):
        check(n, to_np64(t), f[n], cfg.dtype)
    r = oracle.bwd(phi(a["q"]), phi(a["k"]), phi(a["v"]), a["g"], a["dO"], cu_seqlens=cun, K0=a["K0"], V0=a["V0"],
                   dKT=a["dKT"], dVT=a["dVT"], scale=scale, s=a["s"], readout=readout)
    for n in ("q", "k", "v"):
        r["d" + n] = r["d" + n] * slope(a[n])
    names = ["dq", "dk", "dv", "dg", "dK0", "dV0"] + (["ds"] if x["s"] is not None else [])
    for n, t in zip(names, res):
        check(n, to_np64(t), r[n], cfg.dtype)
    return d, a, f


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("readout,given", [("softmax", False), ("softmax", True), ("relu2", False)])
def test_feature_map_applied_inside(oracle, readout, given, dtype):
    import paper_2409_07146_amd as gsa
    from scipy.special import expit
    cfg, x = _inputs(2, 200, 2, 128, 192, 64, dtype, seed=81, given=given)
    for n in ("q", "k", "v"):      # raw projections: wider than the unit-variance inputs, both signs
        x[n] = (x[n].float() * 1.5).to(x[n].dtype)
    d, a, f = _feature_map_case(oracle, cfg, x, readout=readout, scale=0.7)
    # decode step with the same option, continuing from the final memories
    q1, k1, v1, g1 = (d[n][:, -1].contiguous() for n in ("q", "k", "v", "g"))
    s1 = None if d["s"] is None else d["s"][:, -1].contiguous()
    Kc, Vc = (torch.from_numpy(f[n]).float().to(DEV) for n in ("KT", "VT"))
    Ko, Vo = Kc.cpu().double().numpy().copy(), Vc.cpu().double().numpy().copy()
    o1 = gsa.gsa_decode_step(q1, k1, v1, g1, Kc, Vc, scale=0.7, s=s1, readout=readout, feature_map="swish")
    phi = lambda u: u * expit(u)
    oo = oracle.decode_step(phi(a["q"][:, -1]), phi(a["k"][:, -1]), phi(a["v"][:, -1]), a["g"][:, -1], Ko, Vo, scale=0.7,
                            s=None if a["s"] is None else a["s"][:, -1], readout=readout)
    check("decode o", to_np64(o1), oo, dtype)
    check("decode K", to_np64(Kc), Ko, dtype)
    check("decode V", to_np64(Vc), Vo, dtype)


@pytest.mark.parametrize("m", [32, 128])
def test_feature_map_other_slot_counts_packed(oracle, m):
    """ragged packed sequences (one of them long enough for the segmented scans), m = 32 and 128"""
    lens = [70, 1, 64 * 50 + 5, 129]
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    cfg, x = _inputs(1, cu[-1], 2, 64, 128, m, "bf16", seed=83, given=False)
    x["K0"] = x["K0"][:1].repeat(len(lens), 1, 1, 1) * 0.2
    x["V0"] = x["V0"][:1].repeat(len(lens), 1, 1, 1) * 0.2
    gs = torch.Generator().manual_seed(84)
    x["dKT"] = torch.randn(x["K0"].shape, generator=gs) * 0.1
    x["dVT"] = torch.randn(x["V0"].shape, generator=gs) * 0.1
    _feature_map_case(oracle, cfg, x, cu=cu)


def test_feature_map_at_the_layer_shape(oracle):
    """d = 512, m = 64, bf16, ragged length, several sequences' worth of chunks: the contraction length and
    the launch shape of the headline workload"""
    cfg, x = _inputs(2, 64 * 9 + 13, 2, 512, 512, 64, "bf16", seed=88, given=False)
    _feature_map_case(oracle, cfg, x)


def test_feature_map_through_autograd():
    """gsa_attention passes the option to both calls: same numbers as calling them directly"""
    import paper_2409_07146_amd as gsa
    cfg, x = _inputs(2, 100, 2, 64, 128, 32, "bf16", seed=89, given=False)
    dev = torch.device(DEV)
    q, k, v, g, dO = (x[n].to(dev) for n in ("q", "k", "v", "g", "dO"))
    leaves = [t.clone().requires_grad_(True) for t in (q, k, v, g)]
    o = gsa.gsa_attention(*leaves, feature_map="swish")
    (o.float() * dO.float()).sum().backward()
    o2, z2, _, _ = gsa.gsa_fwd(q, k, v, g, feature_map="swish")
    ref = gsa.gsa_bwd(q, k, v, g, z2, dO, feature_map="swish")
    assert torch.equal(o, o2)
    for leaf, r in zip(leaves, ref):
        assert torch.equal(leaf.grad, r)
    o3, _, _, _ = gsa.gsa_fwd(q, k, v, g)
    assert not torch.equal(o3, o2)      # the option does something


def test_feature_map_with_everything_else_on(oracle):
    """feature map + gate logits + given intensities + an element-wise read-out in one call"""
    import paper_2409_07146_amd as gsa
    from scipy.special import expit, log_expit
    tau = 8.0
    cfg, x = _inputs(2, 150, 2, 128, 64, 32, "bf16", seed=86, given=True)
    gen = torch.Generator().manual_seed(87)
    u = (torch.randn(x["g"].shape, generator=gen) * 2.0).float()
    g64 = log_expit(to_np64(u)) / tau
    x["s"] = (2.0 * torch.rand(u.shape, generator=gen) * -torch.expm1(torch.from_numpy(g64).float())).float()
    dev = torch.device(DEV)
    put = lambda t: None if t is None else t.to(dev)
    d = {n: put(x[n]) for n in ("q", "k", "v", "s", "dO", "K0", "V0", "dKT", "dVT")}
    ud = u.to(dev)
    kw = dict(s=d["s"], readout="swish", gate_tau=tau, feature_map="swish")
    o, z, KT, VT = gsa.gsa_fwd(d["q"], d["k"], d["v"], ud, K0=d["K0"], V0=d["V0"], final_state=True, **kw)
    res = gsa.gsa_bwd(d["q"], d["k"], d["v"], ud, z, d["dO"], K0=d["K0"], V0=d["V0"], dKT=d["dKT"], dVT=d["dVT"],
                      initial_state_grad=True, **kw)
    torch.cuda.synchronize()
    a = {n: to_np64(x[n]) for n in ("q", "k", "v", "s", "dO", "K0", "V0", "dKT", "dVT")}
    phi = lambda t: t * expit(t)
    slope = lambda t: expit(t) * (1.0 + t * (1.0 - expit(t)))
    f = oracle.fwd(phi(a["q"]), phi(a["k"]), phi(a["v"]), g64, K0=a["K0"], V0=a["V0"], s=a["s"], readout="swish")
    check("o", to_np64(o), f["o"], "bf16")
    check("VT", to_np64(VT), f["VT"], "bf16")
    r = oracle.bwd(phi(a["q"]), phi(a["k"]), phi(a["v"]), g64, a["dO"], K0=a["K0"], V0=a["V0"], dKT=a["dKT"],
                   dVT=a["dVT"], s=a["s"], readout="swish")
    r["dg"] = r["dg"] * (1.0 - expit(to_np64(u))) / tau
    for n in ("q", "k", "v"):
        r["d" + n] = r["d" + n] * slope(a[n])
    for n, t in zip(["dq", "dk", "dv", "dg", "dK0", "dV0", "ds"], res):
        check(n, to_np64(t), r[n], "bf16")
