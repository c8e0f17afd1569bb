"""ctypes binding of libswiftdiff.so: argument marshalling only.

Every function here has the name of the C-ABI entry point it calls (include/swiftdiff.h),
takes torch tensors that live on the GPU, passes their raw pointers and the current HIP
stream, and returns torch tensors.  torch is used for device memory and streams; no step
of the computation runs in torch or on the CPU.  If the library has not been built the
import fails: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SWIFTDIFF_LIB") or os.path.join(_HERE, "libswiftdiff.so")

SD_BF16, SD_F32 = 0, 1
SD_EPI_NONE, SD_EPI_GEGLU = 0, 1
_ERR = {-1: "SD_EINVAL", -2: "SD_EUNSUPPORTED", -3: "SD_EWORKSPACE", -4: "SD_EHIP"}


class SwiftDiffError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{_ERR.get(code, code)}: {text}")
        self.code = code


class sd_proj(C.Structure):
    _fields_ = [("W", C.c_void_p), ("bias", C.c_void_p), ("A", C.c_void_p), ("B", C.c_void_p),
                ("r", C.c_int32), ("scale", C.c_float)]


class sd_block_params(C.Structure):
    _fields_ = [("ln1_g", C.c_void_p), ("ln1_b", C.c_void_p),
                ("q1", sd_proj), ("k1", sd_proj), ("v1", sd_proj), ("o1", sd_proj),
                ("ln2_g", C.c_void_p), ("ln2_b", C.c_void_p),
                ("q2", sd_proj), ("k2", sd_proj), ("v2", sd_proj), ("o2", sd_proj),
                ("ln3_g", C.c_void_p), ("ln3_b", C.c_void_p),
                ("ff1", sd_proj), ("ff2", sd_proj)]


class sd_stack_params(C.Structure):
    _fields_ = [("gn_g", C.c_void_p), ("gn_b", C.c_void_p), ("proj_in", sd_proj), ("proj_out", sd_proj),
                ("blocks", C.POINTER(sd_block_params)), ("depth", C.c_int32)]


class sd_patch_desc(C.Structure):
    _fields_ = [("W", C.c_void_p), ("A", C.c_void_p), ("B", C.c_void_p), ("undo", C.c_void_p),
                ("out", C.c_int32), ("in_", C.c_int32), ("r", C.c_int32), ("scale", C.c_float)]


SD_PATCH_MAX_ADAPTERS = 4


class sd_patch_multi_desc(C.Structure):
    _fields_ = [("W", C.c_void_p), ("undo", C.c_void_p), ("serving", C.c_void_p),
                ("out", C.c_int32), ("in_", C.c_int32), ("n_adapters", C.c_int32), ("pad_", C.c_int32),
                ("A", C.c_void_p * SD_PATCH_MAX_ADAPTERS), ("B", C.c_void_p * SD_PATCH_MAX_ADAPTERS),
                ("r", C.c_int32 * SD_PATCH_MAX_ADAPTERS), ("scale", C.c_float * SD_PATCH_MAX_ADAPTERS)]


BAL_LOAD_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32)


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_02031_amd.build` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    i32, f32, vp, sz, i64 = C.c_int32, C.c_float, C.c_void_p, C.c_size_t, C.c_int64
    P = C.POINTER
    sig = {
        "sd_last_error": (C.c_char_p, []),
        "sd_version": (i32, []),
        "sd_gemm_dep_timeouts": (C.c_int, [P(i64)]),
        "sd_set_projection_fusion": (i32, [i32]),
        "sd_timing_enable": (C.c_int, [i32]),
        "sd_timing_collect": (C.c_int, [i32, P(f32), i32, P(i32)]),
        "sd_timing_disable": (C.c_int, []),
        "sd_ceiling_mfma_bf16": (C.c_int, [vp, i32, i32, P(C.c_double), vp]),
        "sd_ceiling_copy_f32": (C.c_int, [vp, vp, sz, vp]),
        "sd_ceiling_valu": (C.c_int, [vp, i32, i32, i32, P(C.c_double), P(C.c_double), vp]),
        "sd_ceiling_copy_1r2w_f32": (C.c_int, [vp, vp, vp, sz, vp]),
        "sd_lora_linear_workspace_bytes": (sz, [i32, i32, i32, i32, i32]),
        "sd_lora_linear_fwd": (C.c_int, [vp, i32, P(sd_proj), vp, vp, f32, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]),
        "sd_lora_linear_fwd_static": (C.c_int, [vp, i32, P(sd_proj), vp, vp, f32, vp, vp, i32, i32, i32, i32, i32, vp]),
        "sd_attn_block_workspace_bytes": (sz, [i32, i32, i32, i32, i32, i32]),
        "sd_attn_block_fwd": (C.c_int, [vp, vp, i32, vp, i32, i32, vp, vp, f32, P(sd_proj), P(sd_proj), P(sd_proj), P(sd_proj),
                                        i32, i32, i32, i32, vp, sz, vp]),
        "sd_attention_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "sd_attention_fwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]),
        "sd_ff_block_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "sd_ff_block_fwd": (C.c_int, [vp, vp, i32, vp, vp, f32, P(sd_proj), P(sd_proj), i32, i32, i32, vp, sz, vp]),
        "sd_groupnorm_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "sd_groupnorm_fwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, f32, vp, sz, vp]),
        "sd_groupnorm_silu_fwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, f32, vp, sz, vp]),
        "sd_spatial_transformer_workspace_bytes": (sz, [i32, i32, i32, i32, i32, i32]),
        "sd_spatial_transformer_fwd": (C.c_int, [vp, vp, P(sd_stack_params), vp, i32, i32, i32, i32, i32, i32, vp, sz, vp]),
        "sd_multi_lora_linear_workspace_bytes": (sz, [i32, i32]),
        "sd_multi_lora_linear_fwd": (C.c_int, [vp, vp, vp, P(vp), P(vp), P(i32), P(f32), P(i32), P(i32), i32, i32, vp,
                                               i32, i32, i32, vp, sz, vp]),
        "sd_patch_plan_bytes": (sz, [i32]),
        "sd_patch_plan_build": (C.c_int, [P(sd_patch_desc), i32, vp, sz, P(i64)]),
        "sd_lora_patch": (C.c_int, [vp, i32, i64, vp]),
        "sd_lora_unpatch": (C.c_int, [vp, i32, i64, vp]),
        "sd_patch_multi_plan_bytes": (sz, [i32]),
        "sd_patch_multi_plan_build": (C.c_int, [P(sd_patch_multi_desc), i32, vp, sz, P(i64)]),
        "sd_lora_patch_multi": (C.c_int, [vp, i32, i64, vp]),
        "sd_lora_unpatch_multi": (C.c_int, [vp, i32, i64, vp]),
        "sd_cfg_combine": (C.c_int, [vp, vp, f32, vp, sz, vp]),
        "sd_controlnet_residual_add": (C.c_int, [vp, C.POINTER(C.c_void_p), i32, vp, sz, vp]),
        "sd_bal_create": (vp, [i32, BAL_LOAD_FN, vp]),
        "sd_bal_start": (C.c_int, [vp]),
        "sd_bal_loaded": (C.c_int, [vp]),
        "sd_bal_before_step": (C.c_int, [vp, i32, i32, C.c_double, P(i32)]),
        "sd_bal_stats": (C.c_int, [vp, P(i32), P(C.c_double), P(C.c_double)]),
        "sd_bal_finish": (C.c_int, [vp, P(i32)]),
        "sd_bal_destroy": (None, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()
EXPORTS = ["sd_last_error", "sd_version", "sd_gemm_dep_timeouts", "sd_set_projection_fusion", "sd_timing_enable", "sd_timing_collect", "sd_timing_disable", "sd_ceiling_mfma_bf16", "sd_ceiling_copy_f32", "sd_ceiling_copy_1r2w_f32", "sd_ceiling_valu",
           "sd_lora_linear_workspace_bytes", "sd_lora_linear_fwd", "sd_lora_linear_fwd_static",
           "sd_attn_block_workspace_bytes", "sd_attn_block_fwd", "sd_attention_workspace_bytes", "sd_attention_fwd", "sd_ff_block_workspace_bytes",
           "sd_ff_block_fwd", "sd_groupnorm_workspace_bytes", "sd_groupnorm_fwd", "sd_groupnorm_silu_fwd",
           "sd_spatial_transformer_workspace_bytes", "sd_spatial_transformer_fwd",
           "sd_multi_lora_linear_workspace_bytes", "sd_multi_lora_linear_fwd", "sd_patch_plan_bytes",
           "sd_patch_plan_build", "sd_lora_patch", "sd_lora_unpatch", "sd_patch_multi_plan_bytes",
           "sd_patch_multi_plan_build", "sd_lora_patch_multi", "sd_lora_unpatch_multi", "sd_cfg_combine", "sd_controlnet_residual_add", "sd_bal_create", "sd_bal_start",
           "sd_bal_loaded", "sd_bal_before_step", "sd_bal_stats", "sd_bal_finish", "sd_bal_destroy"]


def lib() -> C.CDLL:
    return _lib


def set_projection_fusion(on: bool) -> bool:
    return bool(_lib.sd_set_projection_fusion(1 if on else 0))


def gemm_dep_timeouts() -> int:
    n = C.c_int64(-1)
    _check(_lib.sd_gemm_dep_timeouts(C.byref(n)))
    return int(n.value)


def _check(rc: int) -> None:
    if rc != 0:
        raise SwiftDiffError(rc, _lib.sd_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SD_BF16
    if t.dtype == torch.float32:
        return SD_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ws(nbytes: int, ws: Optional[torch.Tensor]) -> torch.Tensor:
    if ws is not None:
        return ws
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def to_bf16(a, device="cuda") -> Optional[torch.Tensor]:
    """numpy float32 (already bf16-representable) or None -> device bf16 tensor."""
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=torch.bfloat16).contiguous()


class Proj:
    """A projection's device tensors plus the C struct that points at them."""

    def __init__(self, W, bias=None, A=None, B=None, scale: float = 0.0):
        self.W, self.bias, self.A, self.B = W, bias, A, B
        self.r = int(A.shape[0]) if A is not None else 0
        self.scale = float(scale) if A is not None else 0.0
        self.c = sd_proj(_ptr(W), _ptr(bias), _ptr(A), _ptr(B), self.r, self.scale)

    @classmethod
    def from_numpy(cls, p: dict, device="cuda") -> "Proj":
        return cls(to_bf16(p["W"], device), to_bf16(p.get("b"), device), to_bf16(p.get("A"), device),
                   to_bf16(p.get("B"), device), p.get("scale", 0.0))


class StackParams:
    """Device copy of a stack's parameters and the host structs the C call reads."""

    _PROJS = ("q1", "k1", "v1", "o1", "q2", "k2", "v2", "o2", "ff1", "ff2")
    _LNS = ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "ln3_g", "ln3_b")

    def __init__(self, params: dict, device="cuda"):
        self.gn_g, self.gn_b = to_bf16(params["gn_g"], device), to_bf16(params["gn_b"], device)
        self.proj_in = Proj.from_numpy(params["proj_in"], device)
        self.proj_out = Proj.from_numpy(params["proj_out"], device)
        self.blocks: List[dict] = []
        depth = len(params["blocks"])
        self._cblocks = (sd_block_params * max(depth, 1))()
        self.r_max = 0
        for i, blk in enumerate(params["blocks"]):
            d = {}
            for n in self._LNS:
                d[n] = to_bf16(blk[n], device)
                setattr(self._cblocks[i], n, _ptr(d[n]))
            for n in self._PROJS:
                d[n] = Proj.from_numpy(blk[n], device)
                setattr(self._cblocks[i], n, d[n].c)
                self.r_max = max(self.r_max, d[n].r)
            self.blocks.append(d)
        self.c = sd_stack_params(_ptr(self.gn_g), _ptr(self.gn_b), self.proj_in.c, self.proj_out.c,
                                 C.cast(self._cblocks, C.POINTER(sd_block_params)), depth)


# ------------------------------------------------------------------------------------------
# entry points
# ------------------------------------------------------------------------------------------
def lora_linear_fwd(x: torch.Tensor, p: Proj, ln_gamma=None, ln_beta=None, ln_eps: float = 1e-5, residual=None,
                    out_dtype=torch.bfloat16, epilogue: int = SD_EPI_NONE, out=None, ws=None) -> torch.Tensor:
    M, K = x.shape
    n_rows = p.W.shape[0]
    N = n_rows // 2 if epilogue == SD_EPI_GEGLU else n_rows
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=x.device)
    need = _lib.sd_lora_linear_workspace_bytes(M, N, K, p.r, int(ln_gamma is not None))
    w = _ws(need, ws)
    _check(_lib.sd_lora_linear_fwd(_ptr(x), _dt(x), C.byref(p.c), _ptr(ln_gamma), _ptr(ln_beta), ln_eps, _ptr(residual),
                                   _ptr(y), _dt(y), epilogue, M, N, K, _ptr(w), w.numel(), _stream()))
    return y


SD_STATIC_SCRATCH_BYTES = 16 << 20


def lora_linear_fwd_static(x: torch.Tensor, p: Proj, ln_gamma=None, ln_beta=None, ln_eps: float = 1e-5, residual=None,
                           out_dtype=torch.bfloat16, epilogue: int = SD_EPI_NONE, out=None) -> torch.Tensor:
    """sd_lora_linear_fwd_static: no workspace argument.  The call itself allocates nothing when `out` is given."""
    M, K = x.shape
    n_rows = p.W.shape[0]
    N = n_rows // 2 if epilogue == SD_EPI_GEGLU else n_rows
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=x.device)
    _check(_lib.sd_lora_linear_fwd_static(_ptr(x), _dt(x), C.byref(p.c), _ptr(ln_gamma), _ptr(ln_beta), ln_eps, _ptr(residual),
                                          _ptr(y), _dt(y), epilogue, M, N, K, _stream()))
    return y


def attention_fwd(q: torch.Tensor, k: torch.Tensor, vt: torch.Tensor, heads: int, out=None, ws=None) -> torch.Tensor:
    Bn, Tq, Cc = q.shape
    Tk = k.shape[1]
    y = out if out is not None else torch.empty_like(q)
    w = _ws(_lib.sd_attention_workspace_bytes(Bn, Tq, Tk, heads), ws)
    _check(_lib.sd_attention_fwd(_ptr(q), _ptr(k), _ptr(vt), _ptr(y), Bn, Tq, Tk, Cc, heads, _ptr(w), w.numel(), _stream()))
    return y


def attn_block_fwd(x: torch.Tensor, ctx: Optional[torch.Tensor], ln_gamma, ln_beta, q: Proj, k: Proj, v: Proj, o: Proj,
                   heads: int, ln_eps: float = 1e-5, out=None, ws=None) -> torch.Tensor:
    Bn, T, Cc = x.shape
    Tc, Dc = (ctx.shape[1], ctx.shape[2]) if ctx is not None else (0, 0)
    y = out if out is not None else torch.empty_like(x)
    rmax = max(q.r, k.r, v.r, o.r)
    w = _ws(_lib.sd_attn_block_workspace_bytes(Bn, T, Cc, Tc, Dc, rmax), ws)
    _check(_lib.sd_attn_block_fwd(_ptr(x), _ptr(y), _dt(x), _ptr(ctx), Tc, Dc, _ptr(ln_gamma), _ptr(ln_beta), ln_eps,
                                  C.byref(q.c), C.byref(k.c), C.byref(v.c), C.byref(o.c), Bn, T, Cc, heads,
                                  _ptr(w), w.numel(), _stream()))
    return y


def ff_block_fwd(x: torch.Tensor, ln_gamma, ln_beta, ff1: Proj, ff2: Proj, ln_eps: float = 1e-5, out=None, ws=None) -> torch.Tensor:
    Cc = x.shape[-1]
    M = x.numel() // Cc
    F = ff2.W.shape[1]
    y = out if out is not None else torch.empty_like(x)
    w = _ws(_lib.sd_ff_block_workspace_bytes(M, Cc, F, max(ff1.r, ff2.r)), ws)
    _check(_lib.sd_ff_block_fwd(_ptr(x), _ptr(y), _dt(x), _ptr(ln_gamma), _ptr(ln_beta), ln_eps, C.byref(ff1.c), C.byref(ff2.c),
                                M, Cc, F, _ptr(w), w.numel(), _stream()))
    return y


def groupnorm_fwd(x: torch.Tensor, gamma, beta, groups: int = 32, eps: float = 1e-6, out=None, ws=None) -> torch.Tensor:
    Bn, T, Cc = x.shape
    y = out if out is not None else torch.empty_like(x)
    w = _ws(_lib.sd_groupnorm_workspace_bytes(Bn, T, Cc, groups), ws)
    _check(_lib.sd_groupnorm_fwd(_ptr(x), _ptr(y), _ptr(gamma), _ptr(beta), Bn, T, Cc, groups, eps, _ptr(w), w.numel(), _stream()))
    return y


def groupnorm_silu_fwd(x: torch.Tensor, gamma, beta, groups: int = 32, eps: float = 1e-6, out=None, ws=None) -> torch.Tensor:
    Bn, T, Cc = x.shape
    y = out if out is not None else torch.empty_like(x)
    w = _ws(_lib.sd_groupnorm_workspace_bytes(Bn, T, Cc, groups), ws)
    _check(_lib.sd_groupnorm_silu_fwd(_ptr(x), _ptr(y), _ptr(gamma), _ptr(beta), Bn, T, Cc, groups, eps, _ptr(w), w.numel(), _stream()))
    return y


def spatial_transformer_workspace_bytes(Bn, T, Cc, Tc, Dc, r_max) -> int:
    return int(_lib.sd_spatial_transformer_workspace_bytes(Bn, T, Cc, Tc, Dc, r_max))


def spatial_transformer_fwd(x: torch.Tensor, ctx: torch.Tensor, p: StackParams, heads: int, out=None, ws=None) -> torch.Tensor:
    Bn, T, Cc = x.shape
    Tc, Dc = ctx.shape[1], ctx.shape[2]
    y = out if out is not None else torch.empty_like(x)
    w = _ws(spatial_transformer_workspace_bytes(Bn, T, Cc, Tc, Dc, p.r_max), ws)
    _check(_lib.sd_spatial_transformer_fwd(_ptr(x), _ptr(ctx), C.byref(p.c), _ptr(y), Bn, T, Cc, heads, Tc, Dc,
                                           _ptr(w), w.numel(), _stream()))
    return y


def multi_lora_linear_fwd(x: torch.Tensor, W: torch.Tensor, bias, A_list: Sequence[torch.Tensor], B_list: Sequence[torch.Tensor],
                          scales: Sequence[float], seg_offsets: Sequence[int], seg_adapter: Sequence[int], out=None, ws=None) -> torch.Tensor:
    M, K = x.shape
    N = W.shape[0]
    na, ns = len(A_list), len(seg_adapter)
    y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    ranks = [int(a.shape[0]) for a in A_list]
    w = _ws(_lib.sd_multi_lora_linear_workspace_bytes(M, max(ranks) if ranks else 0), ws)
    Ap = (C.c_void_p * max(na, 1))(*[_ptr(a) for a in A_list])
    Bp = (C.c_void_p * max(na, 1))(*[_ptr(b) for b in B_list])
    rk = (C.c_int32 * max(na, 1))(*ranks)
    sc = (C.c_float * max(na, 1))(*[float(s) for s in scales])
    so = (C.c_int32 * (ns + 1))(*[int(v) for v in seg_offsets])
    sa = (C.c_int32 * max(ns, 1))(*[int(v) for v in seg_adapter])
    _check(_lib.sd_multi_lora_linear_fwd(_ptr(x), _ptr(W), _ptr(bias), Ap, Bp, rk, sc, so, sa, ns, na, _ptr(y), M, N, K,
                                         _ptr(w), w.numel(), _stream()))
    return y


class PatchPlan:
    """Descriptor list -> validated tile plan, uploaded once; reused by patch and unpatch.

    Each entry of `mats` is (W, A, B, undo, scale) with fp32 device tensors W [out, in],
    A [r, in], B [out, r], undo [out, in].
    """

    def __init__(self, mats: Sequence[tuple]):
        n = len(mats)
        self.n = n
        self._keep = list(mats)
        descs = (sd_patch_desc * max(n, 1))()
        for i, (W, A, B, undo, scale) in enumerate(mats):
            for t in (W, A, B, undo):
                assert t.dtype == torch.float32
            descs[i] = sd_patch_desc(_ptr(W), _ptr(A), _ptr(B), _ptr(undo), W.shape[0], W.shape[1], A.shape[0], float(scale))
        nbytes = int(_lib.sd_patch_plan_bytes(n))
        host = np.zeros(max(nbytes, 64), dtype=np.uint8)
        tiles = C.c_int64(0)
        _check(_lib.sd_patch_plan_build(descs, n, host.ctypes.data_as(C.c_void_p), host.nbytes, C.byref(tiles)))
        self.total_tiles = int(tiles.value)
        self.dev = torch.from_numpy(host).cuda()


class PatchMultiPlan:
    """Several adapters per matrix.  Each entry of `mats` is (W, undo, serving_or_None,
    [(A, B, scale), ...]) with fp32 device tensors W, undo [out, in], A_i [r_i, in],
    B_i [out, r_i] and an optional bf16 device tensor serving [out, in]."""

    def __init__(self, mats: Sequence[tuple]):
        n = len(mats)
        self.n = n
        self._keep = list(mats)
        descs = (sd_patch_multi_desc * max(n, 1))()
        for i, (W, undo, serving, adapters) in enumerate(mats):
            assert W.dtype == torch.float32 and undo.dtype == torch.float32
            assert serving is None or serving.dtype == torch.bfloat16
            d = sd_patch_multi_desc()
            d.W, d.undo, d.serving = _ptr(W), _ptr(undo), _ptr(serving)
            d.out, d.in_, d.n_adapters = W.shape[0], W.shape[1], len(adapters)
            for a, (A, Bm, scale) in enumerate(adapters[:SD_PATCH_MAX_ADAPTERS]):
                assert A.dtype == torch.float32 and Bm.dtype == torch.float32
                d.A[a], d.B[a], d.r[a], d.scale[a] = _ptr(A), _ptr(Bm), A.shape[0], float(scale)
            descs[i] = d
        nbytes = int(_lib.sd_patch_multi_plan_bytes(n))
        host = np.zeros(max(nbytes, 64), dtype=np.uint8)
        tiles = C.c_int64(0)
        _check(_lib.sd_patch_multi_plan_build(descs, n, host.ctypes.data_as(C.c_void_p), host.nbytes, C.byref(tiles)))
        self.total_tiles = int(tiles.value)
        self.dev = torch.from_numpy(host).cuda()


def lora_patch_multi(plan: PatchMultiPlan) -> None:
    _check(_lib.sd_lora_patch_multi(_ptr(plan.dev), plan.n, plan.total_tiles, _stream()))


def lora_unpatch_multi(plan: PatchMultiPlan) -> None:
    _check(_lib.sd_lora_unpatch_multi(_ptr(plan.dev), plan.n, plan.total_tiles, _stream()))


def cfg_combine(eps_uncond: torch.Tensor, eps_cond: torch.Tensor, guidance: float, out=None) -> torch.Tensor:
    y = out if out is not None else torch.empty_like(eps_uncond)
    _check(_lib.sd_cfg_combine(_ptr(eps_uncond), _ptr(eps_cond), float(guidance), _ptr(y), eps_uncond.numel(), _stream()))
    return y


def controlnet_residual_add(h: torch.Tensor, residuals: Sequence[torch.Tensor], out=None) -> torch.Tensor:
    y = out if out is not None else torch.empty_like(h)
    ptrs = (C.c_void_p * max(len(residuals), 1))(*[_ptr(r) for r in residuals])
    _check(_lib.sd_controlnet_residual_add(_ptr(h), ptrs, len(residuals), _ptr(y), h.numel(), _stream()))
    return y


class Bal:
    """One request's bounded asynchronous adapter loading.  `load(i)` runs on a loader thread of
    the library (one per adapter) and returns 0 on success; the denoising loop calls
    `before_step(step, k)` at every step boundary and patches when it returns True."""

    def __init__(self, n_adapters: int, load):
        self._cb = BAL_LOAD_FN(lambda _user, i: int(load(int(i)) or 0))   # kept alive with the handle
        self._h = _lib.sd_bal_create(n_adapters, self._cb, None)
        if not self._h:
            raise SwiftDiffError(-1, _lib.sd_last_error().decode())

    def start(self) -> None:
        _check(_lib.sd_bal_start(self._h))

    def loaded(self) -> bool:
        return bool(_lib.sd_bal_loaded(self._h))

    def before_step(self, step: int, k: int, timeout_s: float = 60.0) -> bool:
        now = C.c_int32(0)
        _check(_lib.sd_bal_before_step(self._h, step, k, float(timeout_s), C.byref(now)))
        return bool(now.value)

    def stats(self):
        st, stall, load = C.c_int32(0), C.c_double(0.0), C.c_double(0.0)
        _check(_lib.sd_bal_stats(self._h, C.byref(st), C.byref(stall), C.byref(load)))
        return {"patched_at_step": st.value, "stall_s": stall.value, "load_s": load.value}

    def finish(self) -> bool:
        due = C.c_int32(0)
        _check(_lib.sd_bal_finish(self._h, C.byref(due)))
        return bool(due.value)

    def close(self) -> None:
        if self._h:
            _lib.sd_bal_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


TIMING_TAGS = {"self_attention": 0, "cross_attention": 1, "qkv": 2, "attn_out": 3, "ff1": 4, "ff2": 5,
               "cross_q": 6, "proj_io": 7, "layernorm": 8, "groupnorm": 9}


def timing_enable(records_per_tag: int) -> None:
    _check(_lib.sd_timing_enable(records_per_tag))


def timing_collect(tag: str, capacity: int = 65536) -> List[float]:
    buf = (C.c_float * capacity)()
    n = C.c_int32(0)
    _check(_lib.sd_timing_collect(TIMING_TAGS[tag], buf, capacity, C.byref(n)))
    return [float(buf[i]) for i in range(n.value)]


def timing_disable() -> None:
    _check(_lib.sd_timing_disable())


def ceiling_mfma_bf16(out: torch.Tensor, workgroups: int, iters: int) -> float:
    """Enqueue the register-resident MFMA loop; returns the FLOPs of the launch."""
    fl = C.c_double(0.0)
    _check(_lib.sd_ceiling_mfma_bf16(_ptr(out), workgroups, iters, C.byref(fl), _stream()))
    return fl.value


def ceiling_valu(out: torch.Tensor, workgroups: int, iters: int, mode: int):
    """Enqueue the vector-ALU issue loop; returns (exponentials, FMAs) of the launch, in wavefront-wide instructions."""
    e, f = C.c_double(0.0), C.c_double(0.0)
    _check(_lib.sd_ceiling_valu(_ptr(out), workgroups, iters, mode, C.byref(e), C.byref(f), _stream()))
    return e.value, f.value


def ceiling_copy_1r2w_f32(src: torch.Tensor, dst0: torch.Tensor, dst1: torch.Tensor) -> None:
    _check(_lib.sd_ceiling_copy_1r2w_f32(_ptr(src), _ptr(dst0), _ptr(dst1), src.numel(), _stream()))


def ceiling_copy_f32(src: torch.Tensor, dst: torch.Tensor) -> None:
    _check(_lib.sd_ceiling_copy_f32(_ptr(src), _ptr(dst), src.numel(), _stream()))


def lora_patch(plan: PatchPlan) -> None:
    _check(_lib.sd_lora_patch(_ptr(plan.dev), plan.n, plan.total_tiles, _stream()))


def lora_unpatch(plan: PatchPlan) -> None:
    _check(_lib.sd_lora_unpatch(_ptr(plan.dev), plan.n, plan.total_tiles, _stream()))
