"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs, element
by element, at sizes that span several tiles and ragged tails.  Tolerances are the ones the
task states: max|d|/max|ref| <= 1e-2 for bf16 paths, <= 1e-5 for fp32 patching, unpatch
bit-exact.  Each call's output is normalised by its own maximum (for residual sub-layers:
the update, not the residual stream), and negative controls show the check can fail."""
import time

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


def dev(a, B):
    return B.to_bf16(a)


def host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


def rng(seed):
    return np.random.default_rng(seed)


def mkproj(r, N, K, rank, bias=True, scale=1.0, w_std=0.05):
    return G.make_projection(r, N, K, bias=bias, r=rank, scale=scale, w_std=w_std, a_std=0.3 if rank else 0.0, b_std=0.05)


# ------------------------------------------------------------------- lora_linear_fwd
@pytest.mark.parametrize("M,K,N,rank,scale", [
    (300, 328, 200, 8, 0.5),      # ragged in every dimension, K not a multiple of 64
    (512, 320, 320, 8, 1.0),      # the tiny config's projection
    (1000, 640, 1920, 64, 1.0),   # several 256-row tiles
    (77, 2048, 320, 16, 2.0),     # text-context projection shape
    (130, 64, 136, 0, 0.0),       # no adapter
    (1, 8, 8, 8, 1.0),            # smallest legal shape
])
def test_lora_linear_matches_oracle(B, M, K, N, rank, scale):
    r = rng(M + K + N)
    p = mkproj(r, N, K, rank, bias=True, scale=scale)
    x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
    ref = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
    y = B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(p))
    assert y.shape == (M, N)
    assert rel_err(host(y), ref) <= BF16_TOL
    if rank:
        # negative control: the adapter term is well above the tolerance, so dropping it
        # (or its scale) would be seen
        base = O.linear(x, p["W"], p["b"])
        assert rel_err(base, ref) > 3 * BF16_TOL
        # merged-weight path: plain linear on W' agrees with the unmerged call
        Wm = G.bf16_round(O.merged_weight(p["W"], p["A"], p["B"], p["scale"]).astype(np.float32))
        pm = dict(p, W=Wm, A=None, B=None)
        ym = B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(pm))
        assert rel_err(host(ym), ref) <= 2 * BF16_TOL     # W' itself is rounded to bf16 here


def test_lora_linear_same_workspace_new_inputs(B):
    """The base GEMM's tiles read the down-projection that other tiles of the same launch
    wrote moments before, possibly on another XCD with its own L2.  Reusing one workspace with
    changing inputs and adapters would serve a stale down-projection (the previous call's, still
    cached) if those reads and writes were not of device scope; a tile that did not wait at all
    would read the previous call's too.  Large enough that every XCD runs tiles of both kinds."""
    import torch
    M, K, N, rank = 4096 + 37, 640, 640, 64
    r = rng(99)
    need = B.lib().sd_lora_linear_workspace_bytes(M, N, K, rank, 0)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    for trial in range(4):
        p = mkproj(r, N, K, rank, bias=True, scale=1.0 + trial)
        x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
        ref = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
        base = O.linear(x, p["W"], p["b"])
        assert rel_err(base, ref) > 10 * BF16_TOL          # the adapter term carries most of the output
        xd, pd = dev(x, B), B.Proj.from_numpy(p)
        for rep in range(3):
            y = B.lora_linear_fwd(xd, pd, ws=ws)
            assert rel_err(host(y), ref) <= BF16_TOL, (trial, rep)
    assert B.gemm_dep_timeouts() == 0


def test_lora_linear_random_shapes(B):
    """Seeded sweep over ragged shapes and ranks (rank > 64: two column tiles of down-projection
    per row block, so a base tile waits for a count of 2; rank not a multiple of 64; one-row and
    one-tile problems; more row blocks than CUs) through the single-launch projection."""
    r = rng(2024)
    shapes = [(1, 64, 8, 8), (63, 72, 40, 128), (64, 64, 64, 64), (65, 136, 264, 72), (129, 200, 136, 128),
              (700, 640, 640, 96), (2100, 320, 136, 24), (20000, 64, 136, 8), (333, 1288, 72, 200)]
    for _ in range(6):
        shapes.append((int(r.integers(1, 900)), 8 * int(r.integers(1, 60)), 8 * int(r.integers(1, 60)), 8 * int(r.integers(1, 20))))
    for (M, K, N, rank) in shapes:
        p = mkproj(r, N, K, rank, bias=True, scale=0.7)
        x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
        ref = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
        y = B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(p))
        assert rel_err(host(y), ref) <= BF16_TOL, (M, K, N, rank)
    assert B.gemm_dep_timeouts() == 0


def test_lora_linear_layernorm_residual_fp32(B):
    import torch
    r = rng(7)
    M, K, N = 260, 320, 320
    p = mkproj(r, N, K, 16, bias=True, scale=0.5)
    x = (r.standard_normal((M, K)) * 2 + 0.5).astype(np.float32)
    g, b = G.bf16_round((1 + 0.1 * r.standard_normal(K)).astype(np.float32)), G.bf16_round((0.1 * r.standard_normal(K)).astype(np.float32))
    res = r.standard_normal((M, N)).astype(np.float32)
    upd = O.lora_linear(O.layernorm(x, g, b), p["W"], p["b"], p["A"], p["B"], p["scale"])
    xd, resd = torch.from_numpy(x).cuda(), torch.from_numpy(res).cuda()
    y = B.lora_linear_fwd(xd, B.Proj.from_numpy(p), ln_gamma=dev(g, B), ln_beta=dev(b, B), residual=resd, out_dtype=torch.float32)
    assert y.dtype == torch.float32
    assert rel_err(host(y) - res, upd) <= BF16_TOL
    # in place on the residual buffer
    B.lora_linear_fwd(xd, B.Proj.from_numpy(p), ln_gamma=dev(g, B), ln_beta=dev(b, B), residual=resd, out=resd)
    assert np.array_equal(host(resd), host(y))


@pytest.mark.parametrize("M,C,F,rank", [(200, 64, 96, 8), (512, 320, 1280, 0), (384, 640, 2560, 64),
                                        # narrow outputs (F <= 64: no wider than one down-projection tile)
                                        (150, 64, 32, 0), (150, 64, 32, 8), (300, 128, 64, 0), (300, 128, 64, 16), (70, 72, 8, 8)])
def test_lora_linear_geglu_epilogue(B, M, C, F, rank):
    r = rng(M + F)
    p = mkproj(r, 2 * F, C, rank, bias=True, scale=1.0, w_std=0.08)
    x = G.bf16_round(r.standard_normal((M, C)).astype(np.float32))
    ref = O.geglu(O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"]))
    y = B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(p), epilogue=B.SD_EPI_GEGLU)
    assert y.shape == (M, F)
    assert rel_err(host(y), ref) <= BF16_TOL
    # negative control: value/gate halves swapped is a different function
    u = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
    assert rel_err(O.geglu(np.concatenate([u[:, F:], u[:, :F]], 1)), ref) > 10 * BF16_TOL


@pytest.mark.parametrize("M,C,F,rank", [(8192 + 77, 328, 2560 + 8, 16), (8192, 328, 2560 - 8, 16), (8192 - 100, 64, 2560, 0)])
def test_lora_linear_geglu_large_ragged(B, M, C, F, rank):
    """Enough tiles for the 256-row GEGLU tile body (two rounds of the chip or more), with ragged
    last row and column tiles and a K that is not a multiple of 64; with and without an adapter
    (without one the launch has no down-projection tiles ahead of the 256x256 ones)."""
    r = rng(M + F)
    p = mkproj(r, 2 * F, C, rank, bias=True, scale=0.5, w_std=0.08)
    x = G.bf16_round(r.standard_normal((M, C)).astype(np.float32))
    ref = O.geglu(O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"]))
    y = B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(p), epilogue=B.SD_EPI_GEGLU)
    got = host(y)
    assert got.shape == (M, F)
    assert rel_err(got, ref) <= BF16_TOL
    # corners and an interior band, each on its own scale
    for rows, cols in ((slice(0, 256), slice(0, 128)), (slice(M - 77, M), slice(F - 8, F)), (slice(M - 77, M), slice(0, 128)),
                       (slice(0, M), slice(2048 - 64, 2048 + 64)), (slice(M - 130, M), slice(2048, F))):
        assert rel_err(got[rows, cols], ref[rows, cols]) <= BF16_TOL
    assert B.gemm_dep_timeouts() == 0


@pytest.mark.parametrize("M,N,K,rank", [(8192 + 77, 2048 + 8, 2048 + 8, 16), (8192, 2048, 2048, 0)])
def test_lora_linear_large_plain_projection(B, M, N, K, rank):
    """One plain projection large enough for the 256x256 tile body (two rounds of the chip or more,
    K >= 2048): ragged last row and column tiles and a ragged K with an adapter, exact tiles without."""
    r = rng(M + N + K)
    p = mkproj(r, N, K, rank, bias=True, scale=0.5, w_std=0.03)
    x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
    ref = O.lora_linear(x, p["W"], p["b"], p["A"], p["B"], p["scale"])
    got = host(B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(p)))
    assert got.shape == (M, N)
    assert rel_err(got, ref) <= BF16_TOL
    for rows, cols in ((slice(0, 256), slice(0, 256)), (slice(M - 77, M), slice(N - 8, N)), (slice(M - 77, M), slice(0, 256)),
                       (slice(0, M), slice(1024 - 64, 1024 + 64)), (slice(4096 - 3, 4096 + 3), slice(0, N))):
        assert rel_err(got[rows, cols], ref[rows, cols]) <= BF16_TOL
    assert B.gemm_dep_timeouts() == 0


# ---------------------------------------------------------------------- attention_fwd
def vt_layout(v, B):
    """[Bn, Tk, C] -> the transposed, per-sample padded layout [C, Bn * Tkp]."""
    Bn, Tk, C = v.shape
    Tkp = (Tk + 7) // 8 * 8
    vt = np.full((C, Bn * Tkp), np.nan, np.float32)      # padding is garbage on purpose
    for b in range(Bn):
        vt[:, b * Tkp:b * Tkp + Tk] = v[b].T
    return dev(vt, B)


@pytest.mark.parametrize("Bn,Tq,Tk,heads,qscale", [
    (2, 300, 300, 2, 1.0),      # ragged self-attention, several key tiles
    (2, 256, 77, 5, 1.0),       # cross-attention shape, Tk = 77
    (1, 2048, 640, 1, 3.0),     # the 256-query kernel, peaky softmax
    (2, 130, 1, 1, 1.0),        # single key
    (1, 64, 200, 3, 8.0),       # scores with std ~ 8: online-softmax rescaling exercised
])
def test_attention_matches_oracle(B, Bn, Tq, Tk, heads, qscale):
    r = rng(Tq + Tk)
    C = heads * 64
    q = G.bf16_round((qscale * r.standard_normal((Bn, Tq, C))).astype(np.float32))
    k = G.bf16_round(r.standard_normal((Bn, Tk, C)).astype(np.float32))
    v = G.bf16_round(r.standard_normal((Bn, Tk, C)).astype(np.float32))
    if Tk > 100:
        k[:, Tk - 3] *= 8.0      # a planted large-score key in the last tile (x8 keeps bf16 values exact)
    ref = O.attention(q, k, v, heads)
    out = B.attention_fwd(dev(q, B), dev(k, B), vt_layout(v, B), heads)
    got = host(out)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= BF16_TOL
    if Tk > 1:
        # negative control: values paired with the wrong keys move the result far beyond tolerance
        assert rel_err(O.attention(q, k, np.roll(v, 1, axis=1), heads), ref) > 10 * BF16_TOL


def test_attention_cut_tiles(B):
    """640 query tiles on a 256-CU part: the launch cuts the key range of 128 tiles in half and
    merges the halves afterwards (odd number of key tiles, ragged last one, peaky scores so the
    two halves of a tile end with different running maxima)."""
    Bn, Tq, Tk, heads = 1, 4096, 520, 20
    r = rng(4096 + 520)
    C = heads * 64
    q = G.bf16_round((2.0 * r.standard_normal((Bn, Tq, C))).astype(np.float32))
    k = G.bf16_round(r.standard_normal((Bn, Tk, C)).astype(np.float32))
    v = G.bf16_round(r.standard_normal((Bn, Tk, C)).astype(np.float32))
    k[:, 100] *= 4.0
    k[:, Tk - 2] *= 4.0
    assert B.lib().sd_attention_workspace_bytes(Bn, Tq, Tk, heads) > 256   # this shape does take the cut path
    ref = O.attention(q, k, v, heads)
    got = host(B.attention_fwd(dev(q, B), dev(k, B), vt_layout(v, B), heads))
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= BF16_TOL
    # per query tile too: a wrong merge of one cut tile must not hide behind the global maximum
    per_tile = np.abs(got - ref).reshape(Bn, Tq // 128, 128, C).max(axis=(2, 3)) / np.abs(ref).max()
    assert per_tile.max() <= BF16_TOL


def test_attention_large_scores_in_alternate_key_octets(B):
    """Keys whose index has bit 3 set score ~+770, the others ~-770: a running maximum taken
    over only part of a tile's keys would overflow the exponentials (the kernel holds the two
    octets of every 16 keys in different half-wavefronts and must exchange their maxima)."""
    Bn, Tq, Tk, heads = 1, 96, 160, 1
    r = rng(77)
    q = G.bf16_round((1.0 + 0.0625 * r.integers(-2, 3, size=(Bn, Tq, 64))).astype(np.float32))
    sign = np.where((np.arange(Tk) & 8) != 0, 1.0, -1.0).astype(np.float32)
    k = G.bf16_round((12.0 * sign)[None, :, None] * np.ones((Bn, Tk, 64), np.float32))
    v = G.bf16_round(r.standard_normal((Bn, Tk, 64)).astype(np.float32))
    ref = O.attention(q, k, v, heads)
    got = host(B.attention_fwd(dev(q, B), dev(k, B), vt_layout(v, B), heads))
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= BF16_TOL
    # and the mirrored pattern
    k2 = -k
    ref2 = O.attention(q, k2, v, heads)
    got2 = host(B.attention_fwd(dev(q, B), dev(k2, B), vt_layout(v, B), heads))
    assert np.isfinite(got2).all()
    assert rel_err(got2, ref2) <= BF16_TOL


# ------------------------------------------------------- attn_block_fwd / ff_block_fwd
def small_cfg(**kw):
    base = dict(name="t", Bn=2, T=200, C=128, heads=2, depth=1, r=8, alpha=4.0, lora_ff=True, Tc=77, Dc=256,
                w_std=0.08, ctx_std=1.0, a_std=0.3, b_std=0.08)
    base.update(kw)
    return G.StackConfig(**base)


@pytest.mark.parametrize("cross", [False, True])
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_attn_block_matches_oracle(B, cross, io):
    import torch
    cfg = small_cfg()
    p = G.make_stack_inputs(cfg, seed=3)
    blk = p["blocks"][0]
    names = ("q2", "k2", "v2", "o2", "ln2_g", "ln2_b") if cross else ("q1", "k1", "v1", "o1", "ln1_g", "ln1_b")
    pq, pk, pv, po, g, b = (blk[n] for n in names)
    h = p["x"] if io == "bf16" else rng(5).standard_normal(p["x"].shape).astype(np.float32)
    ctx = p["ctx"] if cross else None
    ref = O.attn_sublayer(h, ctx, g, b, pq, pk, pv, po, cfg.heads)
    hd = dev(h, B) if io == "bf16" else torch.from_numpy(h).cuda()
    y = B.attn_block_fwd(hd, dev(ctx, B) if cross else None, dev(g, B), dev(b, B), B.Proj.from_numpy(pq), B.Proj.from_numpy(pk),
                         B.Proj.from_numpy(pv), B.Proj.from_numpy(po), cfg.heads)
    got = host(y)
    if io == "f32":
        # the update alone, normalised by its own maximum
        assert rel_err(got - h, ref - h) <= BF16_TOL
        # negative controls on the update: no adapter, or a zeroed context, is visible
        nol = [dict(q, A=None, B=None) for q in (pq, pk, pv, po)]
        assert rel_err(O.attn_sublayer(h, ctx, g, b, *nol, cfg.heads) - h, ref - h) > 3 * BF16_TOL
        if cross:
            assert rel_err(O.attn_sublayer(h, np.zeros_like(ctx), g, b, pq, pk, pv, po, cfg.heads) - h, ref - h) > 3 * BF16_TOL
    else:
        assert rel_err(got, ref) <= BF16_TOL


@pytest.mark.parametrize("Bn,T,Tc,C,heads,rank", [(1, 1, 1, 64, 1, 8), (3, 70, 5, 64, 1, 16), (2, 129, 100, 128, 2, 72),
                                                   (1, 600, 77, 192, 3, 128), (2, 257, 130, 128, 2, 8)])
def test_attn_block_ragged_sizes(B, Bn, T, Tc, C, heads, rank):
    """Self- and cross-attention sub-layers at ragged token counts, including ranks above 64 and
    context lengths that are not multiples of 8: the v^T projection is a transposed problem whose
    tiles wait for the down-projection row blocks that cover their token columns."""
    import torch
    # alpha fixed: the adapter's share of q and k, and with it the score scale, does not grow with the rank
    cfg = small_cfg(Bn=Bn, T=T, Tc=Tc, C=C, heads=heads, r=rank, alpha=8.0, Dc=72)
    p = G.make_stack_inputs(cfg, seed=T + Tc)
    blk = p["blocks"][0]
    h = rng(T).standard_normal(p["x"].shape).astype(np.float32)
    for cross in (False, True):
        names = ("q2", "k2", "v2", "o2", "ln2_g", "ln2_b") if cross else ("q1", "k1", "v1", "o1", "ln1_g", "ln1_b")
        pq, pk, pv, po, g, b = (blk[n] for n in names)
        ctx = p["ctx"] if cross else None
        ref = O.attn_sublayer(h, ctx, g, b, pq, pk, pv, po, cfg.heads)
        args = (torch.from_numpy(h).cuda(), dev(ctx, B) if cross else None, dev(g, B), dev(b, B), B.Proj.from_numpy(pq),
                B.Proj.from_numpy(pk), B.Proj.from_numpy(pv), B.Proj.from_numpy(po), cfg.heads)
        y = B.attn_block_fwd(*args)
        assert rel_err(host(y) - h, ref - h) <= BF16_TOL, (cross,)
        try:        # the same call as two launches per projection: same bits
            B.set_projection_fusion(False)
            y2 = B.attn_block_fwd(*args)
        finally:
            B.set_projection_fusion(True)
        assert torch.equal(y, y2), (cross,)
    assert B.gemm_dep_timeouts() == 0


@pytest.mark.parametrize("T,Tc", [(256, 128), (200, 77)])
def test_attn_block_with_biased_q_k_v(B, T, Tc):
    """A projection record may carry a bias whatever its role.  With one on k the keys cannot leave
    their projection pre-multiplied by the softmax scale (the attention kernel scales the scores
    itself), and one on v is a per-row bias of the transposed v^T problem; T = 256 gives tiles that
    lie inside the output, T = 200 ragged ones."""
    import torch
    cfg = small_cfg(Bn=2, T=T, Tc=Tc, C=128, heads=2, r=16)
    p = G.make_stack_inputs(cfg, seed=11)
    blk = p["blocks"][0]
    r = rng(T + 1)
    h = r.standard_normal(p["x"].shape).astype(np.float32)
    for cross in (False, True):
        names = ("q2", "k2", "v2", "o2", "ln2_g", "ln2_b") if cross else ("q1", "k1", "v1", "o1", "ln1_g", "ln1_b")
        pq, pk, pv, po, g, b = (blk[n] for n in names)
        pq, pk, pv = (dict(q, b=G.bf16_round((0.5 * r.standard_normal(q["W"].shape[0])).astype(np.float32))) for q in (pq, pk, pv))
        ctx = p["ctx"] if cross else None
        ref = O.attn_sublayer(h, ctx, g, b, pq, pk, pv, po, cfg.heads)
        y = B.attn_block_fwd(torch.from_numpy(h).cuda(), dev(ctx, B) if cross else None, dev(g, B), dev(b, B), B.Proj.from_numpy(pq),
                             B.Proj.from_numpy(pk), B.Proj.from_numpy(pv), B.Proj.from_numpy(po), cfg.heads)
        assert rel_err(host(y) - h, ref - h) <= BF16_TOL, (cross,)
        # the q and v biases matter at this tolerance; a k bias shifts every score of a query by
        # the same amount, which softmax removes (so the GPU's scaling of biased keys is what is tested)
        for drop in range(3):
            qs = [pq, pk, pv]
            qs[drop] = dict(qs[drop], b=None)
            e = rel_err(O.attn_sublayer(h, ctx, g, b, *qs, po, cfg.heads) - h, ref - h)
            assert (e < 1e-9) if drop == 1 else (e > 3 * BF16_TOL), (cross, drop, e)


def test_ff_block_matches_oracle(B):
    import torch
    cfg = small_cfg(T=150, C=192, heads=3)
    p = G.make_stack_inputs(cfg, seed=4)
    blk = p["blocks"][0]
    h = rng(6).standard_normal((cfg.M, cfg.C)).astype(np.float32)
    ref = O.ff_sublayer(h, blk["ln3_g"], blk["ln3_b"], blk["ff1"], blk["ff2"])
    y = B.ff_block_fwd(torch.from_numpy(h).cuda(), dev(blk["ln3_g"], B), dev(blk["ln3_b"], B),
                       B.Proj.from_numpy(blk["ff1"]), B.Proj.from_numpy(blk["ff2"]))
    assert rel_err(host(y) - h, ref - h) <= BF16_TOL


# ---------------------------------------------------------------------- groupnorm_fwd
@pytest.mark.parametrize("Bn,T,C", [(2, 256, 320), (1, 70, 64), (2, 1000, 640), (1, 33, 1280)])
def test_groupnorm_matches_oracle(B, Bn, T, C):
    r = rng(T + C)
    x = G.bf16_round((r.standard_normal((Bn, T, C)) * 1.5 + r.standard_normal((Bn, 1, C)) * 2).astype(np.float32))
    g = G.bf16_round((1 + 0.1 * r.standard_normal(C)).astype(np.float32))
    b = G.bf16_round((0.1 * r.standard_normal(C)).astype(np.float32))
    ref = O.groupnorm(x, g, b)
    y = B.groupnorm_fwd(dev(x, B), dev(g, B), dev(b, B))
    assert rel_err(host(y), ref) <= BF16_TOL
    # the fused GroupNorm + SiLU operator of the ResNet blocks
    ref_s = O.groupnorm_silu(x, g, b)
    ys = B.groupnorm_silu_fwd(dev(x, B), dev(g, B), dev(b, B))
    assert rel_err(host(ys), ref_s) <= BF16_TOL
    assert rel_err(ref, ref_s) > 10 * BF16_TOL          # the activation is visible at this tolerance


# ------------------------------------------------------------ spatial_transformer_fwd
def run_stack(B, cfg, seed=0):
    p = G.make_stack_inputs(cfg, seed)
    sp = B.StackParams(p)
    y = B.spatial_transformer_fwd(dev(p["x"], B), dev(p["ctx"], B), sp, cfg.heads)
    return p, host(y)


def test_stack_small_ragged(B):
    cfg = small_cfg(T=200, depth=2)
    p, got = run_stack(B, cfg, seed=1)
    ref = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
    assert rel_err(got, ref) <= BF16_TOL
    assert rel_err(got - p["x"], ref - p["x"]) <= 2 * BF16_TOL     # what the stack adds, bf16 output rounding included


def test_stack_with_biased_q_k_v(B):
    """SDXL's q, k, v carry no bias, but a projection record may: the stack takes them too (the
    text keys / values projected ahead inside the self-attention launches included)."""
    cfg = small_cfg(T=200, depth=2)
    p = G.make_stack_inputs(cfg, seed=4)
    r = rng(40)
    for blk in p["blocks"]:
        for name in ("q1", "k1", "v1", "q2", "k2", "v2"):
            blk[name] = dict(blk[name], b=G.bf16_round((0.5 * r.standard_normal(blk[name]["W"].shape[0])).astype(np.float32)))
    got = host(B.spatial_transformer_fwd(dev(p["x"], B), dev(p["ctx"], B), B.StackParams(p), cfg.heads))
    ref = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
    assert rel_err(got - p["x"], ref - p["x"]) <= 2 * BF16_TOL
    # without the value biases the oracle's result is far away
    for blk in p["blocks"]:
        blk["v1"] = dict(blk["v1"], b=None)
        blk["v2"] = dict(blk["v2"], b=None)
    e = rel_err(O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads) - p["x"], ref - p["x"])
    assert e > 6 * BF16_TOL, e


def test_stack_tiny_config(B):
    # configs[0]: batch 2, 16x16 latent, C = 320, rank 8 on the attention projections
    p, got = run_stack(B, G.TINY, seed=0)
    ref = O.spatial_transformer(p["x"], p["ctx"], p, G.TINY.heads)
    assert rel_err(got, ref) <= BF16_TOL
    # batch independence (Section 3.3): sample b alone gives the same bits
    import torch
    sp = B.StackParams(p)
    for b in range(2):
        yb = B.spatial_transformer_fwd(dev(p["x"][b:b + 1], B), dev(p["ctx"][b:b + 1], B), sp, G.TINY.heads)
        assert rel_err(host(yb), ref[b:b + 1]) <= BF16_TOL
    # run-to-run determinism
    y1 = B.spatial_transformer_fwd(dev(p["x"], B), dev(p["ctx"], B), sp, G.TINY.heads)
    y2 = B.spatial_transformer_fwd(dev(p["x"], B), dev(p["ctx"], B), sp, G.TINY.heads)
    assert torch.equal(y1, y2)


# --------------------------------------------------------------- multi_lora_linear_fwd
def test_multi_lora_small(B):
    cfg = G.MultiLoraConfig(name="s", requests=5, T=150, C=128, ranks=(8, 16, 32), request_adapter=(2, 0, 1, 0, 2), std=0.08, x_std=1.0)
    p = G.make_multi_lora_inputs(cfg, seed=2, n_proj=1, bias=True)
    pr = p["projs"][0]
    offs = [0, 150, 150, 290, 450, 601, 750]           # ragged, one empty segment
    adp = [2, 1, 0, -1, 1, 2]
    ref = O.multi_lora_linear(p["x"], pr["W"], pr["b"], pr["A"], pr["B"], [0.5, 1.0, 2.0], offs, adp)
    y = B.multi_lora_linear_fwd(dev(p["x"], B), dev(pr["W"], B), dev(pr["b"], B), [dev(a, B) for a in pr["A"]],
                                [dev(b, B) for b in pr["B"]], [0.5, 1.0, 2.0], offs, adp)
    assert rel_err(host(y), ref) <= BF16_TOL
    wrong = O.multi_lora_linear(p["x"], pr["W"], pr["b"], pr["A"], pr["B"], [0.5, 1.0, 2.0], offs, [0, 1, 0, -1, 1, 2])
    assert rel_err(wrong, ref) > 3 * BF16_TOL


# ------------------------------------------------------------- lora_patch / lora_unpatch
def patch_roundtrip(B, mats):
    import torch
    dm = []
    for m in mats:
        W = torch.from_numpy(m["W"]).cuda()
        dm.append((W, torch.from_numpy(m["A"]).cuda(), torch.from_numpy(m["B"]).cuda(), torch.zeros_like(W), m["scale"]))
    plan = B.PatchPlan(dm)
    B.lora_patch(plan)
    patched = [t[0].cpu().numpy().copy() for t in dm]
    B.lora_unpatch(plan)
    restored = [t[0].cpu().numpy() for t in dm]
    return patched, restored


def test_patch_small_ragged_and_roundtrip(B):
    groups = ((2, 300, 200), (1, 128, 128), (1, 33, 1027), (3, 640, 640), (1, 1, 4))
    mats = G.make_patch_inputs(groups, r=32, alpha=16.0, seed=5)
    mats += G.make_patch_inputs(((1, 70, 72),), r=5, alpha=5.0, seed=6)       # odd rank
    patched, restored = patch_roundtrip(B, mats)
    for m, Wp, Wr in zip(mats, patched, restored):
        ref, _ = O.lora_patch(m["W"], m["A"], m["B"], m["scale"])
        assert rel_err(Wp, ref) <= PATCH_TOL
        assert not np.array_equal(Wp, m["W"])
        assert Wr.tobytes() == m["W"].tobytes()                                  # bit-exact
        # the arithmetic inverse would not have restored the bits
    sub = O.lora_unpatch_by_subtraction(patched[3], mats[3]["A"], mats[3]["B"], mats[3]["scale"])
    assert sub.tobytes() != mats[3]["W"].tobytes()


def test_patch_exact_integers(B):
    r = rng(9)
    W = r.integers(-8, 9, (256, 384)).astype(np.float32)
    A = r.integers(-3, 4, (32, 384)).astype(np.float32)
    Bm = r.integers(-3, 4, (256, 32)).astype(np.float32)
    patched, restored = patch_roundtrip(B, [{"W": W, "A": A, "B": Bm, "scale": 2.0}])
    ref, _ = O.lora_patch(W, A, Bm, 2.0)
    assert np.array_equal(patched[0], ref)           # exactly representable -> identical bits
    assert np.array_equal(restored[0], W)


def test_patch_several_adapters_one_pass(B):
    """Two and three adapters per matrix in one pass: the oracle's successive-patch chain, the
    bits of successive single-adapter launches, the bf16 serving copy, and the exact restore."""
    import torch
    # (rank 32 throughout on tiles that lie inside the matrix takes a pipelined path of its own for
    # one and for two adapters: 96 x 512 and 300 x 200 / 160 x 768 reach it)
    shapes = ((300, 200), (128, 128), (33, 1027), (640, 640), (64, 256), (96, 512), (160, 768))
    ranks = ((32, 32), (32, 8, 5), (32,), (16, 32), (32, 32, 32, 32), (32,), (32, 32))
    r = rng(21)
    host, devm, single = [], [], []
    for (o, i), rks in zip(shapes, ranks):
        W = (0.02 * r.standard_normal((o, i))).astype(np.float32)
        ads = [((0.02 * r.standard_normal((rk, i))).astype(np.float32), (0.02 * r.standard_normal((o, rk))).astype(np.float32), sc)
               for rk, sc in zip(rks, (1.0, 0.5, 2.0, -1.0))]
        host.append((W, ads))
        Wd = torch.from_numpy(W).cuda()
        devm.append((Wd, torch.empty_like(Wd), torch.empty(Wd.shape, dtype=torch.bfloat16, device="cuda"),
                     [(torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), sc) for A, Bm, sc in ads]))
    plan = B.PatchMultiPlan(devm)
    B.lora_patch_multi(plan)
    torch.cuda.synchronize()
    for (W, ads), (Wd, undo, serving, dads) in zip(host, devm):
        ref, ref_undo, ref_serving = O.lora_patch_multi(W, ads, serving=True)
        got = Wd.cpu().numpy()
        assert rel_err(got, ref) <= PATCH_TOL
        assert undo.cpu().numpy().tobytes() == W.tobytes()
        # the serving copy is the rounding of what the GPU itself stored, bit for bit
        assert serving.float().cpu().numpy().tobytes() == O.bf16_rne(got).tobytes()
        assert rel_err(serving.float().cpu().numpy(), ref_serving) <= 2.0 ** -7
        # dropping the last adapter is visible at this tolerance (the check is not vacuous)
        if len(ads) > 1:
            assert rel_err(O.lora_patch_multi(W, ads[:-1])[0], ref) > 100 * PATCH_TOL
        # successive single-adapter launches on a fresh copy give the same bits
        Ws = torch.from_numpy(W).cuda()
        for A, Bm, sc in dads:
            one = B.PatchPlan([(Ws, A, Bm, torch.empty_like(Ws), sc)])
            B.lora_patch(one)
        torch.cuda.synchronize()
        assert Ws.cpu().numpy().tobytes() == got.tobytes()
    B.lora_unpatch_multi(plan)
    torch.cuda.synchronize()
    for (W, ads), (Wd, undo, serving, dads) in zip(host, devm):
        assert Wd.cpu().numpy().tobytes() == W.tobytes()
        assert serving.float().cpu().numpy().tobytes() == O.bf16_rne(W).tobytes()


def test_cfg_combine_bit_exact(B):
    import torch
    r = rng(31)
    for n, g in ((1, 7.5), (7, 1.0), (4096, 7.5), (2 * 4 * 128 * 128 + 3, 5.0), (65536, 0.0)):
        eu = G.bf16_round(r.standard_normal(n).astype(np.float32))
        ec = G.bf16_round(r.standard_normal(n).astype(np.float32))
        got = B.cfg_combine(dev(eu, B), dev(ec, B), g)
        assert host(got).tobytes() == O.cfg_combine(eu, ec, g).tobytes()
    # batch-of-two layout: the two halves of one buffer, unaligned second half, in place
    n = 1001
    x = G.bf16_round(r.standard_normal(2 * n).astype(np.float32))
    xd = dev(x, B)
    out = B.cfg_combine(xd[:n], xd[n:], 3.0, out=xd[:n])
    assert host(out).tobytes() == O.cfg_combine(x[:n], x[n:], 3.0).tobytes()


def test_controlnet_residual_add_bit_exact(B):
    """Section 2, "ControlNet": the summed ControlNet outputs added to a skip-connection tensor."""
    import torch
    r = rng(37)
    for n, nres in ((1, 1), (7, 3), (4096, 2), (2 * 320 * 64 * 64 + 5, 3), (65536, 8), (2049, 0)):
        h = G.bf16_round(r.standard_normal(n).astype(np.float32))
        rs = [G.bf16_round(r.standard_normal(n).astype(np.float32)) for _ in range(nres)]
        got = B.controlnet_residual_add(dev(h, B), [dev(x, B) for x in rs])
        assert host(got).tobytes() == O.controlnet_residual_add(h, rs).tobytes(), (n, nres)
    # in place on the backbone tensor, residuals at unaligned offsets of one buffer
    n = 1001
    x = G.bf16_round(r.standard_normal(3 * n).astype(np.float32))
    xd = dev(x, B)
    out = B.controlnet_residual_add(xd[:n], [xd[n:2 * n], xd[2 * n:]], out=xd[:n])
    assert host(out).tobytes() == O.controlnet_residual_add(x[:n], [x[n:2 * n], x[2 * n:]]).tobytes()
    # more ControlNets than the entry point takes
    with pytest.raises(B.SwiftDiffError):
        B.controlnet_residual_add(xd[:n], [xd[n:2 * n]] * 9)


def test_empty_inputs_are_no_ops(B):
    """Zero rows, zero tokens, zero samples: every forward call returns without touching its
    outputs (which are empty) and without an error; a later ordinary call still works."""
    import torch
    r = rng(7)
    p = B.Proj.from_numpy(mkproj(r, 64, 32, 8, bias=True, scale=1.0))
    e = torch.empty((0, 32), dtype=torch.bfloat16, device="cuda")
    assert B.lora_linear_fwd(e, p).shape == (0, 64)
    g = torch.ones(32, dtype=torch.bfloat16, device="cuda")
    assert B.lora_linear_fwd(e, p, ln_gamma=g, ln_beta=g).shape == (0, 64)
    C_, heads = 128, 2
    pq, pk, pv, po = (B.Proj.from_numpy(mkproj(r, C_, C_, 8, bias=False, scale=1.0)) for _ in range(4))
    gc = torch.ones(C_, dtype=torch.bfloat16, device="cuda")
    for shape in ((0, 64, C_), (2, 0, C_)):
        xe = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
        assert B.attn_block_fwd(xe, None, gc, gc, pq, pk, pv, po, heads).shape == shape
        assert B.groupnorm_fwd(xe, gc, gc, 32).shape == shape
    qe = torch.empty((2, 0, C_), dtype=torch.bfloat16, device="cuda")      # no queries against eight keys
    k8 = torch.zeros((2, 8, C_), dtype=torch.bfloat16, device="cuda")
    assert B.attention_fwd(qe, k8, torch.zeros((C_, 16), dtype=torch.bfloat16, device="cuda"), heads).shape == (2, 0, C_)
    f1 = B.Proj.from_numpy(mkproj(r, 2 * 4 * C_, C_, 8, bias=True, scale=1.0))
    f2 = B.Proj.from_numpy(mkproj(r, C_, 4 * C_, 8, bias=True, scale=1.0))
    xe = torch.empty((0, C_), dtype=torch.bfloat16, device="cuda")
    assert B.ff_block_fwd(xe, gc, gc, f1, f2).shape == (0, C_)
    W = torch.zeros((64, 32), dtype=torch.bfloat16, device="cuda")
    A = torch.zeros((8, 32), dtype=torch.bfloat16, device="cuda")
    Bm = torch.zeros((64, 8), dtype=torch.bfloat16, device="cuda")
    assert B.multi_lora_linear_fwd(e, W, None, [A], [Bm], [1.0], [0], [], out=None).shape == (0, 64)
    torch.cuda.synchronize()
    # and the library is in working order afterwards
    x = G.bf16_round(r.standard_normal((40, 32)).astype(np.float32))
    pn = mkproj(r, 64, 32, 8, bias=True, scale=1.0)
    ref = O.lora_linear(x, pn["W"], pn["b"], pn["A"], pn["B"], pn["scale"])
    assert rel_err(host(B.lora_linear_fwd(dev(x, B), B.Proj.from_numpy(pn))), ref) <= BF16_TOL


def test_ceiling_copies_copy(B):
    """The streaming-ceiling kernels of the benchmark are plain copies: every byte arrives, sizes
    that are not a multiple of the grid's stride included."""
    import torch
    for n in (4, 1028, 128 * 4 * 131072 + 4 * 77):
        src = torch.arange(n, device="cuda", dtype=torch.float32)
        d0, d1, d2 = (torch.full((n,), -1.0, device="cuda") for _ in range(3))
        B.ceiling_copy_f32(src, d0)
        B.ceiling_copy_1r2w_f32(src, d1, d2)
        assert torch.equal(d0, src) and torch.equal(d1, src) and torch.equal(d2, src), n


def test_ceiling_valu_loop_runs_and_counts(B):
    """The vector-ALU ceiling loop: instruction counts as documented, and a finite result in every
    lane (2^-|a| chains stay in (0, 1], the FMA chains converge to 1)."""
    import torch
    out = torch.full((8 * 256,), float("nan"), device="cuda")
    for mode, (e, f) in enumerate(((1, 0), (0, 4), (1, 4), (2, 0))):
        exps, fmas = B.ceiling_valu(out, 8, 100, mode)
        assert exps == e * 8 * 4 * 100 * 8 and fmas == f * 8 * 4 * 100 * 8
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())
    with pytest.raises(Exception):
        B.ceiling_valu(out, 8, 100, 4)


def test_bal_orders_the_patch_inside_a_denoising_loop(B):
    """The serving loop of Section 4.2 in miniature: a projection reads the bf16 serving copy of an
    fp32 master weight; two adapters load in the background (gated so that they arrive during
    step 3 of 8); the loop early-starts unpatched, patches when the scheduler says so, and patches
    off after the request.  Steps before the order equal the base projection, steps after it the
    patched one, and the master weight ends with its original bits."""
    import threading
    import torch
    r = rng(41)
    M, K, N, k_bound, n_steps = 192, 256, 320, 6, 8
    W = (0.05 * r.standard_normal((N, K))).astype(np.float32)
    ads_h = [((0.3 * r.standard_normal((rk, K))).astype(np.float32), (0.05 * r.standard_normal((N, rk))).astype(np.float32), sc)
             for rk, sc in ((32, 1.0), (16, 0.5))]
    x = G.bf16_round(r.standard_normal((M, K)).astype(np.float32))
    Wd = torch.from_numpy(W).cuda()
    undo = torch.empty_like(Wd)
    serving = Wd.to(torch.bfloat16)
    stage = [(torch.empty(A.shape, dtype=torch.float32).pin_memory(), torch.empty(Bm.shape, dtype=torch.float32).pin_memory()) for A, Bm, _ in ads_h]
    dev_ads = [(torch.empty(A.shape, dtype=torch.float32, device="cuda"), torch.empty(Bm.shape, dtype=torch.float32, device="cuda"), sc) for A, Bm, sc in ads_h]
    plan = B.PatchMultiPlan([(Wd, undo, serving, dev_ads)])
    gate = threading.Event()

    def load(i):                      # loader thread: "disk" -> pinned host memory
        if not gate.wait(10.0):
            return 1
        stage[i][0].copy_(torch.from_numpy(ads_h[i][0]))
        stage[i][1].copy_(torch.from_numpy(ads_h[i][1]))
        return 0

    bal = B.Bal(len(ads_h), load)
    bal.start()
    xd = dev(x, B)
    outs, ordered = [], None
    for step in range(1, n_steps + 1):
        if step == 4:                 # the adapters arrived during step 3
            gate.set()
            t0 = time.time()
            while not bal.loaded():
                assert time.time() - t0 < 5.0
                time.sleep(0.001)
        if bal.before_step(step, k_bound):
            ordered = step
            for (hA, hB), (dA, dB, _) in zip(stage, dev_ads):
                dA.copy_(hA, non_blocking=True)
                dB.copy_(hB, non_blocking=True)
            B.lora_patch_multi(plan)
        outs.append(host(B.lora_linear_fwd(xd, B.Proj(serving))))
    assert ordered == 4 and bal.stats()["stall_s"] == 0.0
    base = O.linear(x, O.bf16_rne(W), None)
    Wp, _, Wserv = O.lora_patch_multi(W, ads_h, serving=True)
    patched = O.linear(x, Wserv, None)
    assert rel_err(patched, base) > 10 * BF16_TOL            # the adapters matter at this tolerance
    for step, y in enumerate(outs, start=1):
        assert rel_err(y, base if step < ordered else patched) <= BF16_TOL
    assert rel_err(Wd.cpu().numpy(), Wp) <= PATCH_TOL
    assert bal.finish() is True
    B.lora_unpatch_multi(plan)
    torch.cuda.synchronize()
    assert Wd.cpu().numpy().tobytes() == W.tobytes()
    assert rel_err(host(B.lora_linear_fwd(xd, B.Proj(serving))), base) <= BF16_TOL
    bal.close()


# ------------------------------------------------------------------ HIP graph replay
def test_stack_graph_replay_matches_eager(B):
    """The stack call only enqueues kernels, so it can be captured into a HIP graph.  Every
    replay, with eager work and synchronisations in between, must give the eager bits."""
    import torch
    cfg = small_cfg(T=200, depth=1)
    p = G.make_stack_inputs(cfg, seed=2)
    sp = B.StackParams(p)
    x, ctx = dev(p["x"], B), dev(p["ctx"], B)
    ws = torch.empty(B.spatial_transformer_workspace_bytes(cfg.Bn, cfg.T, cfg.C, cfg.Tc, cfg.Dc, sp.r_max), dtype=torch.uint8, device="cuda")
    y_eager = B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, ws=ws).clone()
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, out=y, ws=ws)
    for i in range(4):
        y.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {i} differs from the eager result"
        # eager work between replays
        again = B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, ws=ws)
        assert torch.equal(again, y_eager)


def test_projections_as_one_launch_or_two_give_the_same_bits(B):
    """A projection runs as one launch (base-GEMM tiles wait for the down-projection tiles of the
    same grid) or, with the diagnostic switch off, as two; the arithmetic is the same, so the
    whole stack and a many-segment multi-LoRA batch must agree bit for bit."""
    import torch
    cfg = small_cfg(T=200, depth=2)
    p = G.make_stack_inputs(cfg, seed=5)
    sp = B.StackParams(p)
    x, ctx = dev(p["x"], B), dev(p["ctx"], B)
    # 20 segments of 3 adapters: more projections than one launch's group holds
    mcfg = G.MultiLoraConfig(name="m", requests=20, T=70, C=128, ranks=(8, 16, 32), request_adapter=tuple(i % 3 for i in range(20)),
                             std=0.08, x_std=1.0)
    mp = G.make_multi_lora_inputs(mcfg, seed=3, n_proj=1, bias=True)
    pr = mp["projs"][0]
    offs = [70 * i for i in range(21)]
    adp = [(-1 if i % 7 == 6 else i % 3) for i in range(20)]
    margs = (dev(mp["x"], B), dev(pr["W"], B), dev(pr["b"], B), [dev(a, B) for a in pr["A"]], [dev(b, B) for b in pr["B"]],
             [0.5, 1.0, 2.0], offs, adp)
    mref = O.multi_lora_linear(mp["x"], pr["W"], pr["b"], pr["A"], pr["B"], [0.5, 1.0, 2.0], offs, adp)
    outs = {}
    try:
        for on in (False, True):
            B.set_projection_fusion(on)
            y = B.spatial_transformer_fwd(x, ctx, sp, cfg.heads)
            my = B.multi_lora_linear_fwd(*margs)
            torch.cuda.synchronize()
            outs[on] = (y.clone(), my.clone())
    finally:
        B.set_projection_fusion(True)
    assert torch.equal(outs[False][0], outs[True][0])
    assert torch.equal(outs[False][1], outs[True][1])
    assert rel_err(host(outs[True][1]), mref) <= BF16_TOL
    assert B.gemm_dep_timeouts() == 0


def test_zz_no_tile_gave_up_waiting(B):
    """Runs last in this file: across everything above, no base-GEMM tile ran out of spins
    while waiting for a down-projection tile of its own launch."""
    assert B.gemm_dep_timeouts() == 0


@pytest.mark.parametrize("boost", [1.0, 4.0])
def test_attn_block_scores_that_climb_from_key_tile_to_key_tile(B, boost):
    """Inside the block the attention kernel first tries without measuring the maximum of the
    key tiles between a segment's first and last: the exponentials are formed against the first
    tile's maximum, which is exact as long as nothing overflows, and a workgroup whose row sums
    or accumulators end up non-finite runs again in the measured form.  Cross-attention with keys
    under the caller's control (W_k picks the context's leading channels): the scores of
    successive 64-key tiles step up, fall back, stay level and step up again.  boost = 1: the
    steps (up to 2^68 above the first tile) stay in range, the first attempt stands.  boost = 4:
    they reach 2^270, the first attempt overflows and the measured form must take over.  Half of
    the queries see the mirrored, falling sequence, so both kinds share wavefronts.  Ragged last
    tile."""
    import torch
    Bn, T, Tc, C, Dc = 2, 200, 64 * 6 + 23, 64, 64
    r = rng(4242)
    n0 = r.standard_normal(C).astype(np.float32)
    n0 = (n0 - n0.mean()) / n0.std()                       # what LayerNorm makes of a row along n0
    sign = np.where(r.random((Bn, T, 1)) < 0.5, 1.0, -1.0).astype(np.float32)
    h = (sign * n0 * (1.0 + 0.05 * r.standard_normal((Bn, T, 1))) + 0.15 * r.standard_normal((Bn, T, C))).astype(np.float32)
    # natural-log score of key j for a query along +n0: level[j // 64] (+ noise); the head-room is 8 in log2 = 5.5
    level = boost * np.array([0.0, 14.0, 3.0, 3.5, 30.0, 29.0, 47.0], np.float32)
    a = level[np.arange(Tc) // 64] + 0.5 * r.standard_normal(Tc).astype(np.float32)
    ctx = np.zeros((Bn, Tc, Dc), np.float32)
    ctx[:, :, :C] = (a[None, :, None] * n0[None, None, :] / C * 8.0)
    ctx += 0.05 * r.standard_normal(ctx.shape).astype(np.float32)
    ctx = G.bf16_round(ctx)
    eye = np.eye(C, dtype=np.float32)
    mk = lambda W, bias: {"W": G.bf16_round(W), "b": bias, "A": G.bf16_round(0.05 * r.standard_normal((8, W.shape[1])).astype(np.float32)),
                          "B": G.bf16_round(0.02 * r.standard_normal((W.shape[0], 8)).astype(np.float32)), "scale": 0.5}
    pq, pk = mk(eye, None), mk(eye, None)
    pv = mk(0.3 * r.standard_normal((C, Dc)).astype(np.float32), None)
    po = mk(0.3 * r.standard_normal((C, C)).astype(np.float32), G.bf16_round(0.1 * r.standard_normal(C).astype(np.float32)))
    g, b = np.ones(C, np.float32), np.zeros(C, np.float32)
    ref = O.attn_sublayer(h, ctx, g, b, pq, pk, pv, po, 1)
    # the test is what it says: scores (in powers of two) of a +n0 query climb from tile to tile, past 2^100 with the boost
    qn = O.proj(O.layernorm(h, g, b), pq)
    kn = O.proj(ctx, pk)
    i_pos = int(np.argmax(sign[0, :, 0] > 0))
    s_row = (qn[0, i_pos] @ kn[0].T) / 8.0 * 1.4426950408889634
    tile_max = [s_row[i:i + 64].max() for i in range(0, Tc, 64)]
    assert tile_max[1] - tile_max[0] > 8 and tile_max[2] < tile_max[1] and tile_max[4] - tile_max[3] > 8 and tile_max[6] - tile_max[5] > 8
    assert (tile_max[6] - tile_max[0] > 140) == (boost > 1) and tile_max[6] - tile_max[0] < (300 if boost > 1 else 100)
    y = B.attn_block_fwd(torch.from_numpy(h).cuda(), dev(ctx, B), dev(g, B), dev(b, B), B.Proj.from_numpy(pq), B.Proj.from_numpy(pk),
                         B.Proj.from_numpy(pv), B.Proj.from_numpy(po), 1)
    got = host(y)
    assert np.isfinite(got).all()
    assert rel_err(got - h, ref - h) <= BF16_TOL
    # negative control: the output depends on which keys win (attention to the first tile only is far away)
    ref_first = O.attn_sublayer(h, ctx[:, :64], g, b, pq, pk, pv, po, 1)
    assert rel_err(ref_first - h, ref - h) > 10 * BF16_TOL
