"""The entry point that allocates nothing: sd_lora_linear_fwd_static against sd_lora_linear_fwd
(same kernels, scratch in the library's own device array instead of a caller workspace).
Called through the C ABI with raw pointers, two calls in a row, the second on a smaller
input; no tensor is created between the two launches of a pair."""
import ctypes as C

import numpy as np
import pytest

from conftest import rel_err
from oracle import sdxl_block_oracle as O
from workloads import sdxl_inputs as G

pytestmark = pytest.mark.gpu

BF16_TOL = 1e-2


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_02031_amd import binding
    return binding


def _case(B, M, K, N, rank, seed, with_ln):
    import torch
    r = np.random.default_rng(seed)
    p = G.make_projection(r, N, K, bias=True, r=rank, scale=0.75, w_std=0.05, a_std=0.3, b_std=0.05)
    if with_ln:
        x = (r.standard_normal((M, K)) * 1.5 + 0.3).astype(np.float32)
        g = G.bf16_round((1 + 0.1 * r.standard_normal(K)).astype(np.float32))
        b = G.bf16_round((0.1 * r.standard_normal(K)).astype(np.float32))
        ref = O.lora_linear(O.layernorm(x, g, b), p["W"], p["b"], p["A"], p["B"], p["scale"])
        xd = torch.from_numpy(x).cuda()
        gd, bd = B.to_bf16(g), B.to_bf16(b)
    else:
        x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
        ref = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
        xd, gd, bd = B.to_bf16(x), None, None
    return xd, gd, bd, B.Proj.from_numpy(p), ref


def test_static_scratch_entry_point_matches_the_workspace_one(B):
    import torch
    L = B.lib()
    ptr = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first a large call (LayerNorm + rank-64 adapter, several row blocks on every XCD), then a
    # smaller one with another adapter: the array still holds the first call's down-projection
    # and flags when the second starts
    for (M, K, N, rank, seed, with_ln) in ((4096 + 37, 640, 640, 64, 5, True), (300, 328, 200, 8, 6, False)):
        xd, gd, bd, pd, ref = _case(B, M, K, N, rank, seed, with_ln)
        need = L.sd_lora_linear_workspace_bytes(M, N, K, rank, int(with_ln))
        assert need <= B.SD_STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        y_ws = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        y_st = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
        x_dt = 1 if with_ln else 0
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = L.sd_lora_linear_fwd(ptr(xd), x_dt, C.byref(pd.c), ptr(gd), ptr(bd), 1e-5, None, ptr(y_ws), 0, 0, M, N, K, ptr(ws), need, stream)
        assert rc == 0, L.sd_last_error()
        rc = L.sd_lora_linear_fwd_static(ptr(xd), x_dt, C.byref(pd.c), ptr(gd), ptr(bd), 1e-5, None, ptr(y_st), 0, 0, M, N, K, stream)
        assert rc == 0, L.sd_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        a, b = y_ws.view(torch.int16).cpu().numpy(), y_st.view(torch.int16).cpu().numpy()
        assert np.array_equal(a, b), "static-scratch call differs from the workspace call"
        assert rel_err(y_st.float().cpu().numpy(), ref) <= BF16_TOL
    assert B.gemm_dep_timeouts() == 0


def test_static_scratch_entry_point_rejects_what_does_not_fit(B):
    L = B.lib()
    p = B.sd_proj(0x1000, None, 0x5000, 0x6000, 64, 1.0)
    M, K, N = 1 << 20, 640, 640                     # 128 MiB of down-projection alone
    assert L.sd_lora_linear_workspace_bytes(M, N, K, 64, 0) > B.SD_STATIC_SCRATCH_BYTES
    rc = L.sd_lora_linear_fwd_static(0x1000, 0, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, M, N, K, None)
    assert rc == -3 and b"built-in array" in L.sd_last_error()
    # argument errors are the ordinary ones
    assert L.sd_lora_linear_fwd_static(None, 0, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 8, None) == -1
