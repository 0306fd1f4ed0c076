"""gsa_decode_step_static (the decode step for callers that cannot allocate: its split form works in an
array built into the library) against gsa_decode_step_ws on the same inputs, through the C ABI: two calls
in a row, the second on a smaller problem, so that the shared array still holds the first call's data."""
import ctypes

import pytest
import torch

from tests.util import check, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(B, H, d_k, d_v, m, dtype, seed):
    from paper_2409_07146_amd import synth
    di = synth.make_decode_inputs(B, H, d_k, d_v, m, 1, state_std=0.1, seed=seed, dtype=dtype)
    dev = torch.device(DEV)
    q, k, v = (di[n][0].to(dev) for n in ("q", "k", "v"))
    g = di["g"][0].to(dev)
    return q, k, v, g, di["K"].to(dev), di["V"].to(dev)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_matches_the_workspace_entry(dtype):
    import paper_2409_07146_amd as gsa
    # (B, H, d_k, d_v, m): split form with 64 pairs, then a smaller split problem, then above 64 pairs
    # (no scratch needed) -- the first two share the library's array back to back
    for seed, (B, H, d_k, d_v, m) in enumerate([(16, 4, 512, 512, 64), (1, 4, 128, 192, 32), (33, 2, 64, 64, 16)]):
        q, k, v, g, K, V = _case(B, H, d_k, d_v, m, dtype, 300 + seed)
        K1, V1, K2, V2 = K.clone(), V.clone(), K.clone(), V.clone()
        ws = gsa.alloc_decode_workspace(B, H, d_k, d_v, m, q.device)
        o1 = torch.empty_like(v)
        o2 = torch.full_like(v, float("nan"))
        gsa.gsa_decode_step(q, k, v, g, K1, V1, scale=0.9, out=o1, workspace=ws)
        gsa.gsa_decode_step_static(q, k, v, g, K2, V2, o2, scale=0.9)
        torch.cuda.synchronize()
        for name, a, b in (("o", o2, o1), ("K", K2, K1), ("V", V2, V1)):
            check(name, to_np64(a), to_np64(b), dtype)
            assert torch.equal(a, b), name     # same kernels, same order of operations


def test_static_scratch_entry_rejects_what_does_not_fit():
    from paper_2409_07146_amd import _lib
    lib = _lib.load()
    null = ctypes.c_void_p(None)
    # 64 pairs x 32 pieces x 1026 floats > 2^20 floats: refused before anything is touched
    assert lib.gsa_decode_step_static(16, 4, 64, 1024, 128, 1, 1.0, *([null] * 8)) == 4
    # bad shapes are still reported as such
    assert lib.gsa_decode_step_static(1, 1, 60, 64, 16, 1, 1.0, *([null] * 8)) == 3
    assert lib.gsa_decode_step_static(0, 4, 64, 64, 16, 1, 1.0, *([null] * 8)) == 0
