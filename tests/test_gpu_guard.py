"""Out-of-bounds canaries: every output and the workspace of a call sit inside sentinel-filled bands
of device memory, and the bands must be untouched afterwards.  The calls go straight through the C ABI
(the Python binding allocates its own outputs)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BAND = 4096          # bytes of sentinel on either side
SENTINEL = 0xA5


class Banded:
    """A device buffer of `nbytes` usable bytes (256-byte aligned) between two sentinel bands."""

    def __init__(self, nbytes):
        self.nbytes = int(nbytes)
        self.pad = (self.nbytes + 255) // 256 * 256
        self.raw = torch.full((BAND + self.pad + BAND,), SENTINEL, dtype=torch.uint8, device=DEV)
        assert self.raw.data_ptr() % 256 == 0
        self.ptr = ctypes.c_void_p(self.raw.data_ptr() + BAND)

    def view(self, dtype, shape):
        return self.raw[BAND:BAND + self.nbytes].view(dtype).view(*shape)

    def check(self, name):
        lo = self.raw[:BAND]
        hi = self.raw[BAND + self.nbytes:]      # the alignment padding after the buffer counts as band too
        assert bool((lo == SENTINEL).all()), "%s: bytes before the buffer were written" % name
        assert bool((hi == SENTINEL).all()), "%s: bytes after the buffer were written" % name


def _esz(dtype):
    return 2 if dtype == "bf16" else 4


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,T,H,d_k,d_v,m,cu", [
    (2, 150, 2, 64, 128, 16, None),                       # ragged tail, 16 slots
    (1, 333, 3, 128, 64, 128, None),                      # 128 slots, odd heads
    (1, 300, 2, 64, 64, 32, (0, 70, 70, 199, 300)),       # packed, with an empty sequence
    (1, 64 * 50 + 7, 1, 64, 64, 16, None),                # long enough for the segmented scans
])
def test_outputs_and_workspace_stay_inside_their_buffers(B, T, H, d_k, d_v, m, cu, dtype):
    from paper_2409_07146_amd import _lib, synth
    lib = _lib.load()
    cfg = synth.GsaConfig("guard", B=B, T=T, H=H, d_k=d_k, d_v=d_v, m=m, dtype=dtype, cu_seqlens=cu,
                          init_state_std=0.3, seed=91)
    x = synth.make_inputs(cfg)
    dev = torch.device(DEV)
    q, k, v, g, dO, K0, V0 = (x[n].to(dev) for n in ("q", "k", "v", "g", "dO", "K0", "V0"))
    cud = None if cu is None else x["cu_seqlens"].to(dev)
    n = cfg.n_seqs
    p = _lib.GsaProblem(B=B, T=T, H=H, d_k=d_k, d_v=d_v, m=m, dtype=1 if dtype == "bf16" else 0, scale=1.0,
                        cu_seqlens=None if cud is None else cud.data_ptr(), n_seqs=n)
    need = ctypes.c_size_t(0)
    assert lib.gsa_workspace_bytes(ctypes.byref(p), 1, ctypes.byref(need)) == 0
    e = _esz(dtype)
    tok = B * T * H
    bufs = dict(ws=Banded(need.value), o=Banded(tok * d_v * e), z=Banded(tok * m * 4),
                KT=Banded(n * H * m * d_k * 4), VT=Banded(n * H * m * d_v * 4),
                dq=Banded(tok * d_k * e), dk=Banded(tok * d_k * e), dv=Banded(tok * d_v * e),
                dg=Banded(tok * m * 4), dK0=Banded(n * H * m * d_k * 4), dV0=Banded(n * H * m * d_v * 4))
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    rc = lib.gsa_fwd(ctypes.byref(p), ptr(q), ptr(k), ptr(v), ptr(g), ptr(K0), ptr(V0), bufs["o"].ptr, bufs["z"].ptr,
                     bufs["KT"].ptr, bufs["VT"].ptr, bufs["ws"].ptr, need.value, st)
    assert rc == 0
    dKT = torch.randn(n, H, m, d_k, device=dev)
    dVT = torch.randn(n, H, m, d_v, device=dev)
    rc = lib.gsa_bwd(ctypes.byref(p), ptr(q), ptr(k), ptr(v), ptr(g), ptr(K0), ptr(V0), bufs["z"].ptr, ptr(dO),
                     ptr(dKT), ptr(dVT), bufs["dq"].ptr, bufs["dk"].ptr, bufs["dv"].ptr, bufs["dg"].ptr,
                     bufs["dK0"].ptr, bufs["dV0"].ptr, bufs["ws"].ptr, need.value, st)
    assert rc == 0
    torch.cuda.synchronize()
    for name, b in bufs.items():
        b.check(name)
    # and the call really wrote its outputs (no sentinel pattern left in them)
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32
    lens = [T] * B if cu is None else list(np.diff(cu))
    if all(l > 0 for l in lens):
        for name, d in (("o", d_v), ("dq", d_k), ("dk", d_k), ("dv", d_v)):
            assert bool(torch.isfinite(bufs[name].view(tt, (B, T, H, d)).float()).all()), name
        assert bool(torch.isfinite(bufs["dg"].view(torch.float32, (B, T, H, m))).all())


@pytest.mark.parametrize("B,H,d_k,d_v,m", [(64, 4, 128, 128, 64), (2, 2, 64, 192, 32), (1, 4, 512, 512, 64)])
def test_decode_step_stays_inside_its_buffers(B, H, d_k, d_v, m):
    """one workgroup per memory pair, and the split form with its workspace"""
    from paper_2409_07146_amd import _lib, synth
    lib = _lib.load()
    di = synth.make_decode_inputs(B, H, d_k, d_v, m, 1, seed=92)
    dev = torch.device(DEV)
    q, k, v, g = (di[n][0].to(dev) for n in ("q", "k", "v", "g"))
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    need = ctypes.c_size_t(0)
    assert lib.gsa_decode_workspace_bytes(B, H, d_k, d_v, m, ctypes.byref(need)) == 0
    for split in (False, True):
        K, V, o, ws = (Banded(B * H * m * d_k * 4), Banded(B * H * m * d_v * 4), Banded(B * H * d_v * 2),
                       Banded(max(need.value, 256)))
        K.view(torch.float32, (B, H, m, d_k)).copy_(di["K"])
        V.view(torch.float32, (B, H, m, d_v)).copy_(di["V"])
        if split:
            rc = lib.gsa_decode_step_ws(B, H, d_k, d_v, m, 1, 1.0, ptr(q), ptr(k), ptr(v), ptr(g), K.ptr, V.ptr, o.ptr,
                                        ws.ptr, max(need.value, 256), st)
        else:
            rc = lib.gsa_decode_step(B, H, d_k, d_v, m, 1, 1.0, ptr(q), ptr(k), ptr(v), ptr(g), K.ptr, V.ptr, o.ptr, st)
        assert rc == 0
        torch.cuda.synchronize()
        for name, b in (("K", K), ("V", V), ("o", o), ("ws", ws)):
            b.check(name)
        assert bool(torch.isfinite(o.view(torch.bfloat16, (B, H, d_v)).float()).all())
