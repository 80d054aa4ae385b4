"""umas_policy_logprobs_static, the scoring entry point that allocates nothing, against umas_policy_logprobs.

Both run the same kernels; the static one keeps the per-tile partials in the library's file-scope device array
in place of a workspace.  Called through the C ABI with caller-made outputs, twice in a row, the second time on
a smaller input, so that whatever the first call left in the shared array must not leak into the second result.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2605_26646_amd as umas

pytestmark = pytest.mark.gpu


def abi(lib):
    lib.umas_policy_logprobs_static.restype = C.c_int
    lib.umas_policy_logprobs_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                                C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p]
    return lib.umas_policy_logprobs_static


def make_case(seed, n_rows, d, V, dtype, frac_sel):
    g = torch.Generator(device="cuda").manual_seed(seed)
    H = torch.randn(n_rows, d, device="cuda", generator=g)
    H = (H / H.pow(2).mean(dim=1, keepdim=True).sqrt()).to(dtype)
    W = (0.05 * torch.randn(V, d, device="cuda", generator=g)).to(dtype)
    ids = torch.randint(0, V, (n_rows,), device="cuda", generator=g, dtype=torch.int32)
    sel = None
    if frac_sel < 1.0:
        keep = torch.rand(n_rows, device="cuda", generator=g) < frac_sel
        sel = torch.nonzero(keep).flatten().to(torch.int32)
    return H, W, ids, sel


def call_static(fn, lib, H, W, ids, sel):
    n_rows, d = H.shape
    out = [torch.full((n_rows,), 7.0, dtype=torch.float32, device="cuda") for _ in range(3)]   # stale contents
    n_sel = n_rows if sel is None else sel.numel()
    st = fn(H.data_ptr(), W.data_ptr(), 1 if H.dtype == torch.bfloat16 else 0, n_rows, d, W.shape[0], ids.data_ptr(),
            None if sel is None else sel.data_ptr(), n_sel, out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(),
            torch.cuda.current_stream().cuda_stream)
    assert st == 0, lib.umas_last_error().decode()
    return out


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scoring_matches_the_workspace_entry_point_twice_in_a_row(dtype):
    lib = umas.load_library()
    fn = abi(lib)
    # the first call fills several row tiles and a ragged vocabulary tail, the second is smaller in rows and vocabulary
    shapes = [(1500, 128, 1000, 0.7), (300, 64, 520, 1.0)] if dtype == torch.bfloat16 else [(96, 64, 512, 0.7), (40, 32, 130, 1.0)]
    for k, (n_rows, d, V, frac) in enumerate(shapes):
        H, W, ids, sel = make_case(100 + k, n_rows, d, V, dtype, frac)
        got = call_static(fn, lib, H, W, ids, sel)
        want = umas.umas_policy_logprobs(H, W, ids, sel)
        torch.cuda.synchronize()
        for name, a, b in zip(("logp", "lse", "entropy"), got, want):
            assert torch.equal(a, b), f"call {k} {name}: max difference {(a - b).abs().max().item():.3g}"
        assert got[1].abs().max().item() > 0.0


def test_static_scoring_rejects_more_than_the_scratch_holds():
    lib = umas.load_library()
    fn = abi(lib)
    # host-side check only: the sizes are never touched
    V, d, n = 151936, 2048, 3329
    dummy = torch.zeros(64, dtype=torch.int32, device="cuda")
    st = fn(dummy.data_ptr(), dummy.data_ptr(), 1, n, d, V, dummy.data_ptr(), None, n, dummy.data_ptr(), dummy.data_ptr(),
            dummy.data_ptr(), None)
    assert st == -4 and "static scratch" in lib.umas_last_error().decode()
    assert lib.umas_policy_logprobs_workspace_bytes(3328, d, V, 1) <= umas.STATIC_SCRATCH_BYTES
