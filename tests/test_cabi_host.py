"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, answers workspace queries, and rejects bad arguments with error codes
before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2407_02031_amd", "libswiftdiff.so")


@pytest.fixture(scope="module")
def B():
    if not os.path.exists(LIB):
        from paper_2407_02031_amd import build
        build.build(verbose=False)
    from paper_2407_02031_amd import binding
    return binding


def test_header_symbols_are_exported(B):
    text = open(os.path.join(ROOT, "include", "swiftdiff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sd_[a-z0-9_]+)\s*\(", text))
    assert {"sd_lora_linear_fwd", "sd_attn_block_fwd", "sd_lora_patch", "sd_lora_unpatch",
            "sd_multi_lora_linear_fwd", "sd_spatial_transformer_fwd", "sd_groupnorm_fwd"} <= declared
    raw = C.CDLL(LIB)
    for name in declared:
        assert hasattr(raw, name), f"{name} declared in the header but not exported"
    assert declared == set(B.EXPORTS)
    assert B.lib().sd_version() == 1


def test_struct_layouts_match_the_header(B):
    assert C.sizeof(B.sd_proj) == 40
    assert C.sizeof(B.sd_patch_desc) == 48
    assert C.sizeof(B.sd_patch_multi_desc) == 3 * 8 + 4 * 4 + 4 * 8 + 4 * 8 + 4 * 4 + 4 * 4
    assert C.sizeof(B.sd_block_params) == 6 * 8 + 10 * 40
    assert B.lib().sd_patch_plan_bytes(310) == 310 * 64


def test_workspace_queries(B):
    L = B.lib()
    assert L.sd_lora_linear_workspace_bytes(512, 320, 320, 8, 1) >= 512 * 320 * 2 + 512 * 8 * 2
    assert L.sd_lora_linear_workspace_bytes(0, 0, 0, 0, 0) == 256
    big = L.sd_spatial_transformer_workspace_bytes(2, 4096, 640, 77, 2048, 64)
    # fp32 stream + LN out + q, k, v^T, attention out + GEGLU activations dominate
    assert big >= 8192 * 640 * (4 + 2 * 6) + 8192 * 2560 * 2
    assert big < 400 * 2 ** 20
    assert L.sd_groupnorm_workspace_bytes(2, 4096, 640, 32) >= 2 * 128 * 32 * 2 * 4


def test_patch_plan_build_validates_on_host(B):
    L = B.lib()
    descs = (B.sd_patch_desc * 2)()
    descs[0] = B.sd_patch_desc(0x1000, 0x2000, 0x3000, 0x4000, 300, 200, 32, 1.0)
    descs[1] = B.sd_patch_desc(0x5000, 0x6000, 0x7000, 0x8000, 128, 128, 8, 0.5)
    host = np.zeros(128, np.uint8)
    tiles = C.c_int64(-1)
    assert L.sd_patch_plan_build(descs, 2, host.ctypes.data_as(C.c_void_p), host.nbytes, C.byref(tiles)) == 0
    assert tiles.value == 10 * 1 + 4 * 1     # workgroup tiles of 32 rows x 256 columns
    plan = host.view(np.int64).reshape(2, 8)
    assert plan[0, 6] == 0 and plan[1, 6] == 10
    # buffer too small
    assert L.sd_patch_plan_build(descs, 2, host.ctypes.data_as(C.c_void_p), 64, C.byref(tiles)) == -3
    # null undo, misaligned pointer, bad rank, undo aliasing W
    for bad in (B.sd_patch_desc(0x1000, 0x2000, 0x3000, 0, 8, 8, 8, 1.0),
                B.sd_patch_desc(0x1004, 0x2000, 0x3000, 0x4000, 8, 8, 8, 1.0),
                B.sd_patch_desc(0x1000, 0x2000, 0x3000, 0x4000, 8, 8, 0, 1.0),
                B.sd_patch_desc(0x1000, 0x2000, 0x3000, 0x1000, 8, 8, 8, 1.0)):
        descs[1] = bad
        assert L.sd_patch_plan_build(descs, 2, host.ctypes.data_as(C.c_void_p), host.nbytes, C.byref(tiles)) == -1
        assert b"desc 1" in L.sd_last_error()
    assert L.sd_patch_plan_build(None, 0, None, 0, C.byref(tiles)) == 0 and tiles.value == 0
    # several adapters per matrix
    md = (B.sd_patch_multi_desc * 1)()
    md[0].W, md[0].undo, md[0].serving = 0x1000, 0x4000, 0x8008
    md[0].out, md[0].in_, md[0].n_adapters = 300, 200, 2
    md[0].A[0], md[0].B[0], md[0].r[0], md[0].scale[0] = 0x2000, 0x3000, 32, 1.0
    md[0].A[1], md[0].B[1], md[0].r[1], md[0].scale[1] = 0x5000, 0x6000, 7, 0.5
    mhost = np.zeros(int(L.sd_patch_multi_plan_bytes(1)), np.uint8)
    assert L.sd_patch_multi_plan_build(md, 1, mhost.ctypes.data_as(C.c_void_p), mhost.nbytes, C.byref(tiles)) == 0 and tiles.value == 10
    md[0].n_adapters = 5
    assert L.sd_patch_multi_plan_build(md, 1, mhost.ctypes.data_as(C.c_void_p), mhost.nbytes, C.byref(tiles)) == -1
    md[0].n_adapters = 2
    md[0].B[1] = None
    assert L.sd_patch_multi_plan_build(md, 1, mhost.ctypes.data_as(C.c_void_p), mhost.nbytes, C.byref(tiles)) == -1
    md[0].B[1] = 0x6000
    md[0].serving = 0x8004      # not 8-byte aligned
    assert L.sd_patch_multi_plan_build(md, 1, mhost.ctypes.data_as(C.c_void_p), mhost.nbytes, C.byref(tiles)) == -1
    # the two-destination copy ceiling: null / misaligned pointers, n not a multiple of 4
    assert L.sd_ceiling_copy_1r2w_f32(None, None, None, 16, None) == -1
    assert L.sd_ceiling_copy_1r2w_f32(0x1000, 0x2000, 0x3004, 16, None) == -1
    assert L.sd_ceiling_copy_1r2w_f32(0x1000, 0x2000, 0x3000, 6, None) == -1
    assert L.sd_ceiling_copy_1r2w_f32(0x1000, 0x2000, 0x3000, 0, None) == 0
    # cfg_combine: null pointers with n > 0
    assert L.sd_cfg_combine(None, None, 7.5, None, 16, None) == -1
    assert L.sd_cfg_combine(None, None, 7.5, None, 0, None) == 0
    # controlnet_residual_add: count out of range, null pointers with n > 0, nothing to do with n == 0
    assert L.sd_controlnet_residual_add(None, None, 9, None, 16, None) == -1
    assert L.sd_controlnet_residual_add(None, None, -1, None, 0, None) == -1
    assert L.sd_controlnet_residual_add(None, None, 2, None, 16, None) == -1
    assert L.sd_controlnet_residual_add(None, None, 2, None, 0, None) == 0
    two = (C.c_void_p * 2)(0x1000, None)
    assert L.sd_controlnet_residual_add(0x1000, two, 2, 0x2000, 16, None) == -1 and b"residual 1" in L.sd_last_error()


def test_forward_calls_reject_bad_arguments_before_touching_the_device(B):
    L = B.lib()
    p = B.sd_proj(0x1000, None, None, None, 0, 0.0)
    # null x
    assert L.sd_lora_linear_fwd(None, 0, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 8, 0x3000, 1 << 20, None) == -1
    # K not a multiple of 8
    assert L.sd_lora_linear_fwd(0x1000, 0, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 12, 0x3000, 1 << 20, None) == -2
    # rank not a multiple of 8
    p4 = B.sd_proj(0x1000, None, 0x5000, 0x6000, 4, 1.0)
    assert L.sd_lora_linear_fwd(0x1000, 0, C.byref(p4), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 8, 0x3000, 1 << 20, None) == -2
    # fp32 x without LayerNorm
    assert L.sd_lora_linear_fwd(0x1000, 1, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 8, 0x3000, 1 << 20, None) == -1
    # workspace too small
    assert L.sd_lora_linear_fwd(0x1000, 0, C.byref(p), None, None, 1e-5, None, 0x2000, 0, 0, 4, 8, 8, 0x3000, 16, None) == -3
    # GEGLU with residual
    assert L.sd_lora_linear_fwd(0x1000, 0, C.byref(p), None, None, 1e-5, 0x7000, 0x2000, 0, 1, 4, 8, 8, 0x3000, 1 << 20, None) == -1
    # head dim != 64
    assert L.sd_attention_fwd(0x1000, 0x2000, 0x3000, 0x4000, 2, 16, 16, 96, 2, None, 0, None) == -2
    assert b"head dim" in L.sd_last_error()
    # empty problems succeed without a device
    assert L.sd_lora_linear_fwd(None, 0, C.byref(p), None, None, 1e-5, None, None, 0, 0, 0, 8, 8, None, 0, None) == 0
    assert L.sd_attention_fwd(None, None, None, None, 0, 0, 0, 64, 1, None, 0, None) == 0
    assert L.sd_lora_patch(None, 0, 0, None) == 0
    # multi-LoRA: segments must cover [0, M)
    so = (C.c_int32 * 2)(0, 5)
    sa = (C.c_int32 * 1)(-1)
    assert L.sd_multi_lora_linear_fwd(0x1000, 0x2000, None, None, None, None, None, so, sa, 1, 0, 0x3000, 8, 8, 8, 0x4000, 1 << 20, None) == -1
    assert b"cover" in L.sd_last_error()


def test_projection_fusion_switch_is_host_state(B):
    L = B.lib()
    assert L.sd_set_projection_fusion(0) == 1      # on by default; returns the previous setting
    assert L.sd_set_projection_fusion(1) == 0
    assert L.sd_set_projection_fusion(1) == 1
    assert L.sd_gemm_dep_timeouts(None) == -1       # null count is rejected before touching the device
