"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, plans workspaces, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2409_07146_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        from paper_2409_07146_amd import build
        build.build()
    return _lib.load()


def _problem(**kw):
    from paper_2409_07146_amd._lib import GsaProblem
    p = GsaProblem()
    vals = dict(B=2, T=100, H=2, d_k=64, d_v=128, m=16, dtype=1, scale=1.0, cu_seqlens=None, n_seqs=0)
    vals.update(kw)
    for k, v in vals.items():
        setattr(p, k, v)
    return p


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "gsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(gsa_[a-z_]+)\s*\(", text))
    from paper_2409_07146_amd._lib import EXPORTS
    assert declared == set(EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.gsa_abi_version() == 2


def test_workspace_plan(lib):
    n = ctypes.c_size_t(0)
    p = _problem()
    assert lib.gsa_workspace_bytes(ctypes.byref(p), 0, ctypes.byref(n)) == 0
    chunks = 2 * 2                                   # B * ceil(100/64)
    state = chunks * 2 * 16 * (64 + 128) * 2         # chunk memories are kept in the I/O dtype (bf16 here)
    assert n.value >= state and n.value % 256 == 0
    fwd = n.value
    assert lib.gsa_workspace_bytes(ctypes.byref(p), 1, ctypes.byref(n)) == 0
    assert n.value >= fwd + state + 2 * (200 * 2 * 16 * 4)
    # packed form adds the chunk tables and one extra chunk slot per sequence
    p2 = _problem(B=1, T=200, cu_seqlens=0x1000, n_seqs=3)
    assert lib.gsa_workspace_bytes(ctypes.byref(p2), 0, ctypes.byref(n)) == 0
    assert n.value >= (200 // 64 + 3) * 2 * 16 * 192 * 2
    assert lib.gsa_workspace_bytes(ctypes.byref(p), 0, None) == 1


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), 2), (dict(H=0), 2), (dict(T=-1), 2), (dict(dtype=7), 2), (dict(scale=float("nan")), 2),
    (dict(B=2, cu_seqlens=0x1000, n_seqs=2), 2), (dict(B=1, cu_seqlens=0x1000, n_seqs=0), 2),
    (dict(d_k=48), 3), (dict(d_v=2048), 3), (dict(m=24), 3), (dict(m=256), 3),
])
def test_bad_problem_is_rejected(lib, kw, code):
    n = ctypes.c_size_t(0)
    p = _problem(**kw)
    assert lib.gsa_workspace_bytes(ctypes.byref(p), 0, ctypes.byref(n)) == code
    null = ctypes.c_void_p(None)
    assert lib.gsa_fwd(ctypes.byref(p), *([null] * 10), null, 0, null) == code


def test_null_and_workspace_errors_without_device(lib):
    null = ctypes.c_void_p(None)
    p = _problem()
    assert lib.gsa_fwd(None, *([null] * 10), null, 0, null) == 1
    assert lib.gsa_fwd(ctypes.byref(p), *([null] * 10), null, 0, null) == 1
    assert lib.gsa_bwd(ctypes.byref(p), *([null] * 16), null, 0, null) == 1
    fake = ctypes.c_void_p(0x10000)                   # never dereferenced: validation stops first
    args = [fake] * 4 + [null, null] + [fake] + [null] * 3
    assert lib.gsa_fwd(ctypes.byref(p), *args, null, 0, null) == 4            # no workspace
    assert lib.gsa_fwd(ctypes.byref(p), *args, ctypes.c_void_p(0x10010), 1 << 30, null) == 4   # misaligned
    assert lib.gsa_fwd(ctypes.byref(p), *args, fake, 16, null) == 4           # too small
    odd = ctypes.c_void_p(0x10004)
    assert lib.gsa_fwd(ctypes.byref(p), odd, fake, fake, fake, null, null, fake, null, null, null,
                       fake, 1 << 30, null) == 2                               # misaligned tensor
    # an output that overlaps an input (or another output, or the workspace) is refused
    at = lambda i: ctypes.c_void_p(0x10000000 * (i + 1))
    ok = [at(0), at(1), at(2), at(3), null, null, at(4), at(5), null, null]
    big = ctypes.c_void_p(0x10000000 * 9)
    for clash in (0, 1, 2, 3, 7):                                             # o on top of q, k, v, g, z_saved
        bad = list(ok)
        bad[6] = ctypes.c_void_p(bad[clash].value + 64)
        assert lib.gsa_fwd(ctypes.byref(p), *bad, big, 1 << 27, null) == 2
    bad = list(ok)
    bad[6] = ctypes.c_void_p(big.value + 4096)                                # o inside the workspace
    assert lib.gsa_fwd(ctypes.byref(p), *bad, big, 1 << 27, null) == 2
    # T = 0 is a no-op
    p0 = _problem(T=0)
    assert lib.gsa_fwd(ctypes.byref(p0), *([null] * 10), null, 0, null) == 0
    # decode step
    assert lib.gsa_decode_step(1, 1, 64, 64, 16, 1, 1.0, *([null] * 8)) == 1
    assert lib.gsa_decode_step(1, 1, 60, 64, 16, 1, 1.0, *([null] * 8)) == 3
    assert lib.gsa_decode_step(1, 0, 64, 64, 16, 1, 1.0, *([null] * 8)) == 2
    assert lib.gsa_decode_step(0, 1, 64, 64, 16, 1, 1.0, *([null] * 8)) == 0
    # decode step with a workspace: size query, then the workspace checks come after the shape checks
    n = ctypes.c_size_t(0)
    assert lib.gsa_decode_workspace_bytes(1, 4, 512, 512, 64, ctypes.byref(n)) == 0
    assert n.value >= 4 * 16 * 514 * 4 and n.value % 256 == 0
    assert lib.gsa_decode_workspace_bytes(64, 4, 512, 512, 64, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.gsa_decode_workspace_bytes(1, 4, 512, 500, 64, ctypes.byref(n)) == 3
    assert lib.gsa_decode_workspace_bytes(1, 4, 512, 512, 64, None) == 1
    assert lib.gsa_decode_step_ws(1, 1, 60, 64, 16, 1, 1.0, *([null] * 7), null, 0, null) == 3
    assert lib.gsa_decode_step_ws(1, 1, 64, 64, 16, 1, 1.0, *([null] * 7), null, 0, null) == 1
    assert lib.gsa_decode_step_ws(0, 1, 64, 64, 16, 1, 1.0, *([null] * 7), null, 0, null) == 0
    assert lib.gsa_decode_step_ws(1, 1, 64, 64, 16, 1, 1.0, *([fake] * 7), null, 0, null) == 4       # no workspace
    assert lib.gsa_decode_step_ws(1, 1, 64, 64, 16, 1, 1.0, *([fake] * 7), fake, 64, null) == 4      # too small
    assert lib.gsa_status_string(4).decode().startswith("workspace")


def test_python_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2409_07146_amd import _lib
    monkeypatch.setattr(_lib, "_lib", None)
    monkeypatch.setattr(_lib, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        _lib.load()
