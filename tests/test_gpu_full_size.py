"""GPU parity at the full sizes of the five benchmark configurations, in the launch
configuration bench.py times (same entry points, same workspace sizes).  The oracle runs the
whole stack in float64 on the host (seconds to tens of seconds per configuration)."""
import numpy as np
import pytest

from conftest import rel_err
from oracle import sdxl_block_oracle as O
from workloads import sdxl_inputs as G

pytestmark = pytest.mark.gpu

BF16_TOL = 1e-2
PATCH_TOL = 1e-5


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_02031_amd import binding
    return binding


def host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


@pytest.mark.parametrize("cfg", [G.SDXL64, G.SDXL32], ids=lambda c: c.name)
def test_full_stack_matches_oracle(B, cfg):
    import torch
    print(f"\n[case] stack {cfg.name} seed 0", flush=True)
    p = G.make_stack_inputs(cfg, seed=0)
    sp = B.StackParams(p)
    x, ctx = B.to_bf16(p["x"]), B.to_bf16(p["ctx"])
    ws = torch.empty(B.spatial_transformer_workspace_bytes(cfg.Bn, cfg.T, cfg.C, cfg.Tc, cfg.Dc, sp.r_max), dtype=torch.uint8, device="cuda")
    y = B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, ws=ws)
    got = host(y)
    assert np.isfinite(got).all()
    ref = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
    e_full = rel_err(got, ref)
    e_upd = rel_err(got - p["x"], ref - p["x"])
    print(f"[result] {cfg.name}: rel err {e_full:.3e}, update-only {e_upd:.3e}", flush=True)
    assert e_full <= BF16_TOL
    # what the stack adds to x, normalised by its own maximum; this one includes the bf16
    # rounding of the output y itself (|y| up to ~5 against an update of ~1.5), hence 3x
    assert e_upd <= 3 * BF16_TOL
    # the adapters' effect on the whole stack is small at these weight scales (about 1.2 % of
    # max|y|), but still several times the GPU path's error: a dropped adapter would be seen.
    # The sharper check is per sub-layer, below.
    if cfg is G.SDXL64:
        # This size cuts 128 attention tiles in half and runs five rounds of GEMM tiles: with the
        # in-launch mechanisms off (two launches per projection, a merge kernel after the
        # attention) the stack must give the same bits.
        try:
            B.set_projection_fusion(False)
            y2 = B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, ws=ws)
            torch.cuda.synchronize()
        finally:
            B.set_projection_fusion(True)
        assert torch.equal(y, y2)
        assert B.gemm_dep_timeouts() == 0
        nol = dict(p, blocks=[{k: (dict(v, A=None, B=None) if isinstance(v, dict) else v) for k, v in blk.items()} for blk in p["blocks"]])
        assert rel_err(O.spatial_transformer(p["x"], p["ctx"], nol, cfg.heads, dtype=np.float32), ref) > 3 * e_full


def test_full_sdxl64_sublayers_match_oracle(B):
    """Per-call parity at the 64x64-latent size: each sub-layer's update normalised by its
    own maximum, so a broken attention cannot hide under the residual stream."""
    import torch
    cfg = G.SDXL64
    print(f"\n[case] sub-layers {cfg.name} seed 1", flush=True)
    p = G.make_stack_inputs(G.with_overrides(cfg, depth=1), seed=1)
    blk = p["blocks"][0]
    h = np.random.default_rng(11).standard_normal((cfg.Bn, cfg.T, cfg.C)).astype(np.float32)
    hd = torch.from_numpy(h).cuda()
    P = B.Proj.from_numpy
    d = B.to_bf16
    for name, ctx, keys in (("self", None, ("ln1_g", "ln1_b", "q1", "k1", "v1", "o1")), ("cross", p["ctx"], ("ln2_g", "ln2_b", "q2", "k2", "v2", "o2"))):
        g, b, pq, pk, pv, po = (blk[k] for k in keys)
        ref = O.attn_sublayer(h, ctx, g, b, pq, pk, pv, po, cfg.heads)
        y = B.attn_block_fwd(hd, d(ctx) if ctx is not None else None, d(g), d(b), P(pq), P(pk), P(pv), P(po), cfg.heads)
        e = rel_err(host(y) - h, ref - h)
        print(f"[result] {name}-attention update rel err {e:.3e}", flush=True)
        assert e <= BF16_TOL
    ref = O.ff_sublayer(h, blk["ln3_g"], blk["ln3_b"], blk["ff1"], blk["ff2"])
    y = B.ff_block_fwd(hd, d(blk["ln3_g"]), d(blk["ln3_b"]), P(blk["ff1"]), P(blk["ff2"]))
    e = rel_err(host(y) - h, ref - h)
    print(f"[result] feed-forward update rel err {e:.3e}", flush=True)
    assert e <= BF16_TOL


def test_full_patch_sweep(B):
    """310 fp32 matrices, 830,668,800 elements, rank 32: one grouped patch launch, then one
    grouped unpatch launch.  Every matrix is checked element by element against the oracle
    (streamed, one matrix at a time) and, after the unpatch, for bit-exact restoration."""
    import torch
    print("\n[case] patch sweep, 310 matrices, seed 0", flush=True)
    mats = G.make_patch_inputs(seed=0)
    assert len(mats) == 310
    dm = []
    for m in mats:
        W = torch.from_numpy(m["W"]).cuda()
        dm.append((W, torch.from_numpy(m["A"]).cuda(), torch.from_numpy(m["B"]).cuda(), torch.empty_like(W), m["scale"]))
    plan = B.PatchPlan(dm)
    B.lora_patch(plan)
    torch.cuda.synchronize()
    worst, identical = 0.0, 0
    for i in range(310):
        ref, _ = O.lora_patch(mats[i]["W"], mats[i]["A"], mats[i]["B"], mats[i]["scale"])
        got = dm[i][0].cpu().numpy()
        identical += int(got.tobytes() == ref.tobytes())
        e = rel_err(got, ref)
        assert e <= PATCH_TOL, f"matrix {i}: rel err {e:.3e}"
        worst = max(worst, e)
        # the undo record holds W's bits from before the patch
        if i % 31 == 0:
            assert dm[i][3].cpu().numpy().tobytes() == mats[i]["W"].tobytes(), f"undo record of matrix {i}"
    print(f"[result] patch worst rel err over all 310 matrices {worst:.3e}; {identical} of them bit-identical to the oracle", flush=True)
    # every matrix changed, and its undo record holds the original bits
    for i in range(0, 310, 7):
        assert not torch.equal(dm[i][0], torch.from_numpy(mats[i]["W"]).cuda())
    B.lora_unpatch(plan)
    torch.cuda.synchronize()
    for i, m in enumerate(mats):
        assert dm[i][0].cpu().numpy().tobytes() == m["W"].tobytes(), f"matrix {i} not restored bit-exactly"


def test_full_multi_lora(B):
    """8 requests x 4096 tokens, C = 640, adapters of rank 16/32/64/64 in guidance-pair order."""
    import torch
    cfg = G.MULTI_LORA
    print(f"\n[case] {cfg.name} seed 0", flush=True)
    p = G.make_multi_lora_inputs(cfg, seed=0, n_proj=4)
    x = B.to_bf16(p["x"])
    for j, pr in enumerate(p["projs"]):
        y = B.multi_lora_linear_fwd(x, B.to_bf16(pr["W"]), None, [B.to_bf16(a) for a in pr["A"]], [B.to_bf16(b) for b in pr["B"]],
                                    pr["scales"], p["seg_offsets"], p["seg_adapter"])
        ref = O.multi_lora_linear(p["x"], pr["W"], None, pr["A"], pr["B"], pr["scales"], p["seg_offsets"], p["seg_adapter"])
        e = rel_err(host(y), ref)
        print(f"[result] projection {j}: rel err {e:.3e}", flush=True)
        assert e <= BF16_TOL
        if j == 0:
            # sorted order [0,0,1,1,2,2,3,3] is a different assignment and must differ
            other = O.multi_lora_linear(p["x"], pr["W"], None, pr["A"], pr["B"], pr["scales"], p["seg_offsets"], [0, 0, 1, 1, 2, 2, 3, 3], dtype=np.float32)
            assert rel_err(other, ref) > BF16_TOL
