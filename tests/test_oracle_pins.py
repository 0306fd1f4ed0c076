"""Pins the fp64 oracle to facts fixed by the paper and by mathematics, not by itself.

Each test states what it pins.  The independent forms used here (explicit
cumulative products, closed forms, a chunkwise evaluation, a library softmax,
finite differences) are written in numpy and never call into the oracle except
to obtain the value under test.  The paper prints no worked numeric example of
the operator, so there is no golden fixture from it.
"""
import numpy as np
import pytest
from scipy.special import expit as sp_expit
from scipy.special import softmax as sp_softmax


def _rand(rng, B, T, H, dk, dv, m, gate="paper", init=False):
    q = rng.standard_normal((B, T, H, dk)) / np.sqrt(dk)
    k = rng.standard_normal((B, T, H, dk)) / np.sqrt(dk)
    v = rng.standard_normal((B, T, H, dv))
    x = rng.standard_normal((B, T, H, m)) * 2.0
    g = -np.logaddexp(0.0, -x)            # log sigmoid
    if gate == "paper":
        g = g / 8.0
    K0 = rng.standard_normal((B, H, m, dk)) if init else None
    V0 = rng.standard_normal((B, H, m, dv)) if init else None
    return q, k, v, g, K0, V0


# ---------------------------------------------------------------- P1
_READOUT_NP = {                      # the read-outs of the ablation table, written with library functions
    "softmax": lambda z: sp_softmax(z),
    "identity": lambda z: z,
    "swish": lambda z: z * sp_expit(z),
    "relu": lambda z: np.maximum(z, 0.0),
    "relu2": lambda z: np.maximum(z, 0.0) ** 2,
}


def _brute_force(q, k, v, g, K0, V0, scale, s=None, readout="softmax"):
    """Quadratic form of the two-pass view (Eq. (gsa-2pass) unrolled as Eq.
    (gla-recurrent)): explicit products D(t,r,i) = prod_{j=r+1..t} alpha_j[i],
    no recurrence and no log-space arithmetic.  s: write intensities given as an
    input of their own (Algorithm 1's I), else 1 - alpha."""
    T, dk = q.shape
    dv, m = v.shape[1], g.shape[1]
    alpha = np.exp(g)
    o = np.zeros((T, dv))
    z = np.zeros((T, m))
    for t in range(T):
        w = np.zeros((t + 1, m))          # weight of write r in slot i as seen at t
        for r in range(t + 1):
            D = np.ones(m)
            for j in range(r + 1, t + 1):
                D = D * alpha[j]
            w[r] = D * ((1.0 - alpha[r]) if s is None else s[r])
        D0 = np.ones(m)
        for j in range(t + 1):
            D0 = D0 * alpha[j]
        for i in range(m):
            acc = 0.0
            for r in range(t + 1):
                acc += w[r, i] * float(k[r] @ q[t])
            if K0 is not None:
                acc += D0[i] * float(K0[i] @ q[t])
            z[t, i] = scale * acc
        if readout == "softmax":
            p = np.exp(z[t] - z[t].max())
            p = p / p.sum()
        else:
            p = _READOUT_NP[readout](z[t])
        for r in range(t + 1):
            o[t] += float(p @ w[r]) * v[r]
        if V0 is not None:
            o[t] += (p * D0) @ V0
    return o, z


@pytest.mark.parametrize("init,scale", [(False, 1.0), (True, 0.7)])
def test_p1_bruteforce_quadratic_form(oracle, init, scale):
    rng = np.random.default_rng(11)
    T, dk, dv, m = 19, 5, 7, 3
    q, k, v, g, K0, V0 = _rand(rng, 1, T, 1, dk, dv, m, gate="strong", init=init)
    out = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=scale)
    o_bf, z_bf = _brute_force(q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0],
                              None if K0 is None else K0[0, 0], None if V0 is None else V0[0, 0], scale)
    np.testing.assert_allclose(out["z"][0, :, 0], z_bf, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out["o"][0, :, 0], o_bf, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- P2
def test_p2_single_slot_closed_form(oracle):
    """m = 1: the softmax is identically 1, so o_t is the gate-weighted running
    average of v and does not depend on q or k (Eq. (gsa))."""
    rng = np.random.default_rng(12)
    T, dk, dv = 40, 6, 4
    q, k, v, g, _, V0 = _rand(rng, 2, T, 2, dk, dv, 1, init=True)
    out = oracle.fwd(q, k, v, g, V0=V0)
    alpha = np.exp(g[..., 0])                              # [B,T,H]
    exp = np.zeros_like(v)
    for t in range(T):
        acc = np.zeros((2, 2, dv))
        for r in range(t + 1):
            D = np.prod(alpha[:, r + 1:t + 1], axis=1)     # [B,H]
            acc += (D * (1 - alpha[:, r]))[..., None] * v[:, r]
        acc += np.prod(alpha[:, :t + 1], axis=1)[..., None] * V0[:, :, 0]
        exp[:, t] = acc
    np.testing.assert_allclose(out["o"], exp, rtol=1e-12, atol=1e-14)
    # constant v, zero start: o_t = c * (1 - prod_{j<=t} alpha_j)
    c = np.array([0.3, -1.2, 2.0, 0.5])
    vc = np.broadcast_to(c, v.shape).copy()
    oc = oracle.fwd(q, k, vc, g)["o"]
    expc = (1 - np.cumprod(alpha, axis=1))[..., None] * c
    np.testing.assert_allclose(oc, expc, rtol=1e-12, atol=1e-14)
    # and dq = dk = 0 exactly
    dO = rng.standard_normal(v.shape)
    gr = oracle.bwd(q, k, v, g, dO, V0=V0)
    assert np.all(gr["dq"] == 0.0)
    # dk gets gradient only through K memories, which feed only z; softmax grad is 0 at m=1
    assert np.max(np.abs(gr["dk"])) < 1e-15


# ---------------------------------------------------------------- P3
def _chunked_forward(q, k, v, g, C, scale=1.0):
    """Chunkwise evaluation (Appendix A, Eqs. (gla-chunk-gate), (gla-chunk), used twice
    as in Eq. (gsa-2pass)), written with chunk-local cumulative log gates.  One
    sequence, one head, zero initial memories."""
    T, dk = q.shape
    dv, m = v.shape[1], g.shape[1]
    s = -np.expm1(g)
    SK = np.zeros((m, dk))
    SV = np.zeros((m, dv))
    o = np.zeros((T, dv))
    for c0 in range(0, T, C):
        c1 = min(T, c0 + C)
        G = np.cumsum(g[c0:c1], axis=0)                    # [c,m]
        Q, K_, V_, S_ = q[c0:c1], k[c0:c1], v[c0:c1], s[c0:c1]
        n = c1 - c0
        mask = np.tril(np.ones((n, n)))
        # pass 1: gated on the slot (value) side
        decay = np.exp(G[:, None, :] - G[None, :, :])       # [t,r,m], used only where r<=t
        A = (Q @ K_.T) * mask
        z = np.exp(G) * (Q @ SK.T) + np.einsum("tr,tri,ri->ti", A, decay, S_)
        z = scale * z
        p = sp_softmax(z, axis=1)
        # pass 2: gated on the slot (key) side
        A2 = np.einsum("ti,tri,ri->tr", p, decay, S_) * mask
        o[c0:c1] = (p * np.exp(G)) @ SV + A2 @ V_
        # carry the memories across the chunk
        w = S_ * np.exp(G[-1][None, :] - G)                 # [r,m]
        SK = np.exp(G[-1])[:, None] * SK + w.T @ K_
        SV = np.exp(G[-1])[:, None] * SV + w.T @ V_
    return o


@pytest.mark.parametrize("C", [1, 7, 16, 64])
def test_p3_chunked_form_equals_recurrence(oracle, C):
    rng = np.random.default_rng(13)
    T, dk, dv, m = 50, 8, 6, 5
    q, k, v, g, _, _ = _rand(rng, 1, T, 1, dk, dv, m)
    o = oracle.fwd(q, k, v, g, scale=0.9)["o"][0, :, 0]
    oc = _chunked_forward(q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0], C, scale=0.9)
    np.testing.assert_allclose(o, oc, rtol=1e-10, atol=1e-12)


def test_p3_segment_and_packing_invariance(oracle):
    rng = np.random.default_rng(14)
    T, H, dk, dv, m = 37, 2, 6, 5, 4
    q, k, v, g, K0, V0 = _rand(rng, 1, T, H, dk, dv, m, init=True)
    full = oracle.fwd(q, k, v, g, K0=K0, V0=V0)
    for T1 in (1, 13, 36):
        a = oracle.fwd(q[:, :T1], k[:, :T1], v[:, :T1], g[:, :T1], K0=K0, V0=V0)
        b = oracle.fwd(q[:, T1:], k[:, T1:], v[:, T1:], g[:, T1:], K0=a["KT"], V0=a["VT"])
        np.testing.assert_allclose(np.concatenate([a["o"], b["o"]], 1), full["o"], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(b["KT"], full["KT"], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(b["VT"], full["VT"], rtol=1e-12, atol=1e-14)
    # packed run == separate runs (memories restart at each boundary)
    cu = np.array([0, 10, 10, 29, 37], dtype=np.int32)     # includes an empty sequence
    K0p = rng.standard_normal((4, H, m, dk))
    V0p = rng.standard_normal((4, H, m, dv))
    dO = rng.standard_normal(v.shape)
    dKT = rng.standard_normal((4, H, m, dk))
    dVT = rng.standard_normal((4, H, m, dv))
    pk = oracle.fwd(q, k, v, g, cu_seqlens=cu, K0=K0p, V0=V0p)
    pg = oracle.bwd(q, k, v, g, dO, cu_seqlens=cu, K0=K0p, V0=V0p, dKT=dKT, dVT=dVT)
    for s in range(4):
        a, b = cu[s], cu[s + 1]
        if a == b:
            np.testing.assert_array_equal(pk["KT"][s], K0p[s])
            np.testing.assert_array_equal(pg["dK0"][s], dKT[s])
            continue
        one = oracle.fwd(q[:, a:b], k[:, a:b], v[:, a:b], g[:, a:b], K0=K0p[s:s + 1], V0=V0p[s:s + 1])
        np.testing.assert_allclose(pk["o"][:, a:b], one["o"], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(pk["KT"][s], one["KT"][0], rtol=1e-13, atol=1e-15)
        og = oracle.bwd(q[:, a:b], k[:, a:b], v[:, a:b], g[:, a:b], dO[:, a:b], K0=K0p[s:s + 1],
                        V0=V0p[s:s + 1], dKT=dKT[s:s + 1], dVT=dVT[s:s + 1])
        for name in ("dq", "dk", "dv", "dg"):
            np.testing.assert_allclose(pg[name][:, a:b], og[name], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(pg["dK0"][s], og["dK0"][0], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(pg["dV0"][s], og["dV0"][0], rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- P4 / P5 / P6
def test_p4_zero_log_gate_is_softmax_attention_over_fixed_slots(oracle):
    rng = np.random.default_rng(15)
    q, k, v, g, K0, V0 = _rand(rng, 2, 9, 3, 7, 5, 6, init=True)
    g = np.zeros_like(g)                                   # alpha = 1: memories frozen
    out = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.5)
    scores = 0.5 * np.einsum("bthc,bhic->bthi", q, K0)
    exp = np.einsum("bthi,bhic->bthc", sp_softmax(scores, axis=-1), V0)
    np.testing.assert_allclose(out["o"], exp, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(out["KT"], K0)
    np.testing.assert_array_equal(out["VT"], V0)


def test_p5_full_forget_returns_current_value(oracle):
    rng = np.random.default_rng(16)
    q, k, v, g, K0, V0 = _rand(rng, 1, 12, 2, 4, 6, 5, init=True)
    g = np.full_like(g, -np.inf)                           # alpha = 0
    out = oracle.fwd(q, k, v, g, K0=K0, V0=V0)
    np.testing.assert_allclose(out["o"], v, rtol=1e-13, atol=1e-15)
    zr = out["z"] - out["z"][..., :1]
    assert np.max(np.abs(zr)) < 1e-14                      # uniform scores => p = 1/m
    # and a very negative finite gate behaves the same to rounding
    out2 = oracle.fwd(q, k, v, np.full_like(g, -60.0), K0=K0, V0=V0)
    np.testing.assert_allclose(out2["o"], v, rtol=0, atol=1e-12)


def test_p6_slot_uniform_gates_give_scalar_ema(oracle):
    rng = np.random.default_rng(17)
    B, T, H, dk, dv, m = 1, 30, 2, 5, 4, 6
    q, k, v, g, _, V0 = _rand(rng, B, T, H, dk, dv, m, init=True)
    g = np.repeat(g[..., :1], m, axis=-1)                  # same gate in every slot
    V0 = np.repeat(V0[:, :, :1], m, axis=2)                # same start row in every slot
    o = oracle.fwd(q, k, v, g, V0=V0)["o"]
    a = np.exp(g[..., 0])
    ema = V0[:, :, 0].copy()
    for t in range(T):
        ema = a[:, t][..., None] * ema + (1 - a[:, t])[..., None] * v[:, t]
        np.testing.assert_allclose(o[:, t], ema, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- P7 / P8
def test_p7_convexity(oracle):
    rng = np.random.default_rng(18)
    q, k, v, g, K0, V0 = _rand(rng, 2, 33, 2, 6, 5, 7, init=True)
    o = oracle.fwd(q, k, v, g, K0=K0, V0=V0)["o"]
    for b in range(2):
        for h in range(2):
            lo = np.minimum(np.minimum.accumulate(v[b, :, h], 0), V0[b, h].min(0))
            hi = np.maximum(np.maximum.accumulate(v[b, :, h], 0), V0[b, h].max(0))
            assert np.all(o[b, :, h] >= lo - 1e-12) and np.all(o[b, :, h] <= hi + 1e-12)
    c = rng.standard_normal(5)
    oc = oracle.fwd(q, k, np.broadcast_to(c, v.shape).copy(), g, K0=K0,
                    V0=np.broadcast_to(c, V0.shape).copy())["o"]
    np.testing.assert_allclose(oc, np.broadcast_to(c, oc.shape), rtol=1e-12, atol=1e-14)


def test_p8_symmetries(oracle):
    rng = np.random.default_rng(19)
    q, k, v, g, K0, V0 = _rand(rng, 1, 21, 2, 6, 5, 7, init=True)
    base = oracle.fwd(q, k, v, g, K0=K0, V0=V0)["o"]
    perm = rng.permutation(7)
    o2 = oracle.fwd(q, k, v, g[..., perm], K0=K0[:, :, perm], V0=V0[:, :, perm])["o"]
    np.testing.assert_allclose(o2, base, rtol=1e-12, atol=1e-14)
    # linear in (v, V0)
    v2 = rng.standard_normal(v.shape)
    V02 = rng.standard_normal(V0.shape)
    o3 = oracle.fwd(q, k, 2 * v - 3 * v2, g, K0=K0, V0=2 * V0 - 3 * V02)["o"]
    ob = oracle.fwd(q, k, v2, g, K0=K0, V0=V02)["o"]
    np.testing.assert_allclose(o3, 2 * base - 3 * ob, rtol=1e-11, atol=1e-12)
    # causal: changing tokens after t leaves o_t alone
    q4, k4, v4, g4 = q.copy(), k.copy(), v.copy(), g.copy()
    for x in (q4, k4, v4):
        x[:, 12:] += 1.0
    g4[:, 12:] *= 0.5
    o4 = oracle.fwd(q4, k4, v4, g4, K0=K0, V0=V0)["o"]
    np.testing.assert_array_equal(o4[:, :12], base[:, :12])
    assert np.max(np.abs(o4[:, 12:] - base[:, 12:])) > 1e-3


# ---------------------------------------------------------------- P9
def _loss(oracle, q, k, v, g, K0, V0, dO, dKT, dVT, cu, scale):
    f = oracle.fwd(q, k, v, g, cu_seqlens=cu, K0=K0, V0=V0, scale=scale)
    return float(np.sum(f["o"] * dO) + np.sum(f["KT"] * dKT) + np.sum(f["VT"] * dVT))


@pytest.mark.parametrize("packed", [False, True])
def test_p9_gradients_by_central_differences(oracle, packed):
    rng = np.random.default_rng(20)
    B, T, H, dk, dv, m = (1, 11, 2, 4, 3, 3) if packed else (2, 7, 1, 3, 4, 3)
    q, k, v, g, _, _ = _rand(rng, B, T, H, dk, dv, m, gate="strong")
    cu = np.array([0, 4, 11], dtype=np.int32) if packed else None
    n = 2
    K0 = rng.standard_normal((n, H, m, dk))
    V0 = rng.standard_normal((n, H, m, dv))
    dO = rng.standard_normal(v.shape)
    dKT = rng.standard_normal(K0.shape)
    dVT = rng.standard_normal(V0.shape)
    scale = 1.3
    gr = oracle.bwd(q, k, v, g, dO, cu_seqlens=cu, K0=K0, V0=V0, dKT=dKT, dVT=dVT, scale=scale)
    args = dict(q=q, k=k, v=v, g=g, K0=K0, V0=V0)
    names = dict(q="dq", k="dk", v="dv", g="dg", K0="dK0", V0="dV0")
    h = 1e-6
    for key, gname in names.items():
        x = args[key]
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + h
            lp = _loss(oracle, args["q"], args["k"], args["v"], args["g"], args["K0"], args["V0"],
                       dO, dKT, dVT, cu, scale)
            x[idx] = old - h
            lm = _loss(oracle, args["q"], args["k"], args["v"], args["g"], args["K0"], args["V0"],
                       dO, dKT, dVT, cu, scale)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.max(np.abs(num - gr[gname])) / max(1e-12, np.max(np.abs(num)))
        assert err < 2e-7, (key, err)


@pytest.mark.parametrize("readout", ["softmax", "swish"])
def test_p9_score_gradients_from_their_definitions(oracle, readout):
    """The two intermediates the backward can hand out: dp_t[i] = <Vt_t[i,:], dO_t> with Vt_t the value
    memory after token t's write (obtained here as the final memory of a forward over the first t tokens),
    and dz_t = J^T dp_t with J the read-out's Jacobian at z_t (written out with library functions).  The
    loss here has no final-memory term and one sequence, so both are direct."""
    rng = np.random.default_rng(29)
    B, T, H, dk, dv, m = 1, 9, 2, 4, 5, 3
    q, k, v, g, K0, V0 = _rand(rng, B, T, H, dk, dv, m, gate="strong", init=True)
    dO = rng.standard_normal(v.shape)
    gr = oracle.bwd(q, k, v, g, dO, K0=K0, V0=V0, scale=0.7, readout=readout, intermediates=True)
    f = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.7, readout=readout)
    for t in range(T):
        pre = oracle.fwd(q[:, :t + 1], k[:, :t + 1], v[:, :t + 1], g[:, :t + 1], K0=K0, V0=V0, scale=0.7,
                         readout=readout)
        for h in range(H):
            dp = pre["VT"][0, h] @ dO[0, t, h]
            np.testing.assert_allclose(gr["dp"][0, t, h], dp, rtol=1e-12, atol=1e-13)
            z = f["z"][0, t, h]
            if readout == "softmax":
                pz = sp_softmax(z)
                jac = np.diag(pz) - np.outer(pz, pz)
            else:
                sg = sp_expit(z)
                jac = np.diag(sg + z * sg * (1.0 - sg))
            np.testing.assert_allclose(gr["dz"][0, t, h], jac.T @ dp, rtol=1e-11, atol=1e-13)


def test_p9_gate_gradient_identity(oracle):
    """Cross-check of dg against the log-space identity behind the paper's dA line
    (Algorithm 1, backward driver; reading: it is a gradient with respect to log
    alpha and the reverse cumulative sum runs over the whole sequence):
        dg_j = sum_{t>=j} (z_t*dz_t + p_t*dp_t - s_t*ds_t) - a_j*ds_j
    where ds_t is the gradient with respect to the write intensity s_t = 1 - a_t
    taken as an independent input.  ds is obtained here by finite differences of
    a two-input recurrence written in numpy."""
    rng = np.random.default_rng(21)
    T, dk, dv, m = 9, 3, 4, 3
    q, k, v, g, _, _ = _rand(rng, 1, T, 1, dk, dv, m, gate="strong")
    dO = rng.standard_normal(v.shape)
    q1, k1, v1, g1, dO1 = q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0], dO[0, :, 0]

    def run(glog, s):
        K = np.zeros((m, dk)); V = np.zeros((m, dv)); L = 0.0
        zs, ps, dps = [], [], []
        for t in range(T):
            a = np.exp(glog[t])
            K = a[:, None] * K + s[t][:, None] * k1[t][None]
            V = a[:, None] * V + s[t][:, None] * v1[t][None]
            z = K @ q1[t]
            p = sp_softmax(z)
            L += float(dO1[t] @ (p @ V))
            zs.append(z); ps.append(p); dps.append(V @ dO1[t])
        return L, np.array(zs), np.array(ps), np.array(dps)

    s0 = -np.expm1(g1)
    _, z, p, dp = run(g1, s0)
    dz = p * (dp - np.sum(p * dp, axis=1, keepdims=True))
    h = 1e-6
    ds = np.zeros_like(s0)
    for t in range(T):
        for i in range(m):
            sp = s0.copy(); sp[t, i] += h
            sm = s0.copy(); sm[t, i] -= h
            ds[t, i] = (run(g1, sp)[0] - run(g1, sm)[0]) / (2 * h)
    dGam = z * dz + p * dp - s0 * ds
    dg_id = np.cumsum(dGam[::-1], axis=0)[::-1] - np.exp(g1) * ds
    dg = oracle.bwd(q, k, v, g, dO)["dg"][0, :, 0]
    np.testing.assert_allclose(dg, dg_id, rtol=2e-6, atol=2e-8)


# ---------------------------------------------------------------- variants
@pytest.mark.parametrize("readout", ["softmax", "identity", "swish", "relu", "relu2"])
def test_v1_bruteforce_with_given_write_intensity_and_readout(oracle, readout):
    """Write intensity as an input of its own (Algorithm 1 takes I beside A) and the read-outs of the
    ablation table, against the explicit-product quadratic form."""
    rng = np.random.default_rng(31)
    T, dk, dv, m = 17, 5, 6, 4
    q, k, v, g, K0, V0 = _rand(rng, 1, T, 1, dk, dv, m, gate="strong", init=True)
    s = rng.uniform(0.0, 1.0, size=g.shape)
    out = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.8, s=s, readout=readout)
    o_bf, z_bf = _brute_force(q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0], K0[0, 0], V0[0, 0], 0.8,
                              s=s[0, :, 0], readout=readout)
    np.testing.assert_allclose(out["z"][0, :, 0], z_bf, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out["o"][0, :, 0], o_bf, rtol=1e-10, atol=1e-12)
    # and the tied form is the special case s = 1 - exp(g)
    tied = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.8, readout=readout)
    same = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.8, s=-np.expm1(g), readout=readout)
    np.testing.assert_allclose(same["o"], tied["o"], rtol=1e-13, atol=1e-15)


def test_v2_abc_is_the_case_without_decay(oracle):
    """Eq. (abc_recurrent) with Eq. (abc_phi): memories are plain running sums of phi_t (x) k_t and
    phi_t (x) v_t, phi a cumulative softmax; written here with numpy prefix sums."""
    rng = np.random.default_rng(32)
    T, dk, dv, m = 23, 6, 5, 4
    q = rng.standard_normal((T, dk)); k = rng.standard_normal((T, dk)) / np.sqrt(dk)
    v = rng.standard_normal((T, dv))
    alpha = np.exp(rng.standard_normal((T, m)))
    phi = alpha / np.cumsum(alpha, axis=0)
    Kt = np.cumsum(phi[:, :, None] * k[:, None, :], axis=0)       # [T, m, dk]
    Vt = np.cumsum(phi[:, :, None] * v[:, None, :], axis=0)
    z = np.einsum("tmd,td->tm", Kt, q)
    o = np.einsum("tm,tmd->td", sp_softmax(z, axis=1), Vt)
    sh = lambda x: x[None, :, None]
    out = oracle.fwd(sh(q), sh(k), sh(v), np.zeros((1, T, 1, m)), s=sh(phi))
    np.testing.assert_allclose(out["o"][0, :, 0], o, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out["KT"][0, 0], Kt[-1], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("readout", ["softmax", "identity", "swish", "relu", "relu2"])
def test_v3_variant_gradients_by_central_differences(oracle, readout):
    rng = np.random.default_rng(33)
    B, T, H, dk, dv, m = 1, 8, 2, 3, 4, 3
    q, k, v, g, K0, V0 = _rand(rng, B, T, H, dk, dv, m, gate="strong", init=True)
    s = rng.uniform(0.1, 0.9, size=g.shape)
    dO = rng.standard_normal(v.shape)
    dKT = rng.standard_normal(K0.shape); dVT = rng.standard_normal(V0.shape)
    scale = 0.9
    gr = oracle.bwd(q, k, v, g, dO, K0=K0, V0=V0, dKT=dKT, dVT=dVT, scale=scale, s=s, readout=readout)
    args = dict(q=q, k=k, v=v, g=g, s=s, K0=K0, V0=V0)

    def loss():
        f = oracle.fwd(args["q"], args["k"], args["v"], args["g"], K0=args["K0"], V0=args["V0"], scale=scale,
                       s=args["s"], readout=readout)
        return float(np.sum(f["o"] * dO) + np.sum(f["KT"] * dKT) + np.sum(f["VT"] * dVT))

    h = 1e-6
    for key, gname in dict(q="dq", k="dk", v="dv", g="dg", s="ds", K0="dK0", V0="dV0").items():
        x = args[key]
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + h; lp = loss()
            x[idx] = old - h; lm = loss()
            x[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.max(np.abs(num - gr[gname])) / max(1e-12, np.max(np.abs(num)))
        assert err < 5e-7, (readout, key, err)


def test_v4_tied_gate_gradient_from_the_two_separate_ones(oracle):
    """With s = 1 - exp(g) tied, the chain rule gives dg_tied = dg - exp(g) * ds."""
    rng = np.random.default_rng(34)
    q, k, v, g, _, _ = _rand(rng, 2, 9, 2, 4, 3, 3, gate="strong")
    dO = rng.standard_normal(v.shape)
    tied = oracle.bwd(q, k, v, g, dO)
    sep = oracle.bwd(q, k, v, g, dO, s=-np.expm1(g))
    np.testing.assert_allclose(tied["dg"], sep["dg"] - np.exp(g) * sep["ds"], rtol=1e-11, atol=1e-13)
    for n in ("dq", "dk", "dv"):
        np.testing.assert_allclose(tied[n], sep[n], rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- decode
@pytest.mark.parametrize("readout,given", [("softmax", False), ("softmax", True), ("swish", True), ("relu2", False)])
def test_decode_step_matches_forward(oracle, readout, given):
    """The recurrent (decode) form is one step of Eq. (gsa): T calls equal a T-token forward (itself pinned
    above), also with the write intensity given and with an element-wise read-out."""
    rng = np.random.default_rng(22)
    B, T, H, dk, dv, m = 3, 6, 2, 5, 4, 4
    q, k, v, g, K0, V0 = _rand(rng, B, T, H, dk, dv, m, init=True)
    s = rng.uniform(0.0, 1.0, size=g.shape) if given else None
    full = oracle.fwd(q, k, v, g, K0=K0, V0=V0, scale=0.8, s=s, readout=readout)
    K, V = K0.copy(), V0.copy()
    for t in range(T):
        o = oracle.decode_step(q[:, t], k[:, t], v[:, t], g[:, t], K, V, scale=0.8,
                               s=None if s is None else s[:, t], readout=readout)
        np.testing.assert_allclose(o, full["o"][:, t], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(K, full["KT"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(V, full["VT"], rtol=1e-13, atol=1e-15)
