"""Pins of the CPU oracle against things other than itself: brute-force loops on tiny
inputs, closed forms, invariants and special cases that reduce to a textbook result.
A plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, wrong half of GEGLU, wrong group layout) fails at least one test here."""
import math

import numpy as np
import pytest

from conftest import rel_err
from oracle import sdxl_block_oracle as O
from workloads import sdxl_inputs as G


def rng(seed=0):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------- projections
def test_linear_brute_force_integers():
    r = rng(1)
    M, K, N = 3, 5, 4
    x = r.integers(-4, 5, (M, K)).astype(np.float64)
    W = r.integers(-4, 5, (N, K)).astype(np.float64)
    b = r.integers(-4, 5, (N,)).astype(np.float64)
    ref = [[sum(x[m][k] * W[n][k] for k in range(K)) + b[n] for n in range(N)] for m in range(M)]
    assert np.array_equal(O.linear(x, W, b), np.array(ref))
    # non-square on purpose: a transposed W would not even have the right shape, and
    # a square case with a transposed W must differ
    Wsq = r.integers(-4, 5, (K, K)).astype(np.float64)
    assert not np.array_equal(O.linear(x, Wsq), x @ Wsq)


def test_lora_linear_brute_force_and_scale():
    r = rng(2)
    M, K, N, rk = 3, 5, 4, 2
    x = r.integers(-3, 4, (M, K)).astype(np.float64)
    W = r.integers(-3, 4, (N, K)).astype(np.float64)
    b = r.integers(-3, 4, (N,)).astype(np.float64)
    A = r.integers(-3, 4, (rk, K)).astype(np.float64)
    B = r.integers(-3, 4, (N, rk)).astype(np.float64)
    s = 0.5  # alpha = 1, r = 2: scale must not be dropped
    ref = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = b[n]
            for k in range(K):
                acc += x[m, k] * W[n, k]
            for j in range(rk):
                t = 0.0
                for k in range(K):
                    t += x[m, k] * A[j, k]
                acc += s * t * B[n, j]
            ref[m, n] = acc
    got = O.lora_linear(x, W, b, A, B, s)
    assert np.array_equal(got, ref)
    assert not np.array_equal(got, O.lora_linear(x, W, b, A, B, 1.0))


def test_merged_equals_unmerged():
    # Section 2, "Low-Rank Adaptation": the adapter's whole effect is W' = W + s B A
    r = rng(3)
    M, K, N, rk = 37, 96, 80, 8
    x, W, b = r.standard_normal((M, K)), r.standard_normal((N, K)), r.standard_normal(N)
    A, B = r.standard_normal((rk, K)), r.standard_normal((N, rk))
    s = 4.0 / 8.0
    y_unmerged = O.lora_linear(x, W, b, A, B, s)
    y_merged = O.linear(x, O.merged_weight(W, A, B, s), b)
    assert np.abs(y_unmerged - y_merged).max() <= 1e-12 * np.abs(y_merged).max()
    # fp32 mode agrees with fp64 mode to fp32 round-off
    y32 = O.lora_linear(x, W, b, A, B, s, dtype=np.float32)
    assert np.abs(y32 - y_unmerged).max() <= 2e-5 * np.abs(y_unmerged).max()


def test_multi_lora_matches_per_segment_and_special_cases():
    r = rng(4)
    K, N = 24, 16
    ranks = (2, 4, 8)
    x = r.standard_normal((50, K))
    W, b = r.standard_normal((N, K)), r.standard_normal(N)
    As = [r.standard_normal((q, K)) for q in ranks]
    Bs = [r.standard_normal((N, q)) for q in ranks]
    sc = [1.0, 0.5, 2.0]
    offs = [0, 7, 7, 20, 33, 50]          # one empty segment
    adp = [2, 0, -1, 1, 2]
    y = O.multi_lora_linear(x, W, b, As, Bs, sc, offs, adp)
    for i, a in enumerate(adp):
        lo, hi = offs[i], offs[i + 1]
        ref = O.linear(x[lo:hi], W, b) if a < 0 else O.lora_linear(x[lo:hi], W, b, As[a], Bs[a], sc[a])
        assert np.array_equal(y[lo:hi], ref)
    # one adapter for all rows == plain lora_linear; adapter -1 == plain linear
    assert np.array_equal(O.multi_lora_linear(x, W, b, As, Bs, sc, [0, 50], [1]),
                          O.lora_linear(x, W, b, As[1], Bs[1], sc[1]))
    assert np.array_equal(O.multi_lora_linear(x, W, b, As, Bs, sc, [0, 50], [-1]), O.linear(x, W, b))
    # brute force for one row of an adapted segment
    m = 25  # segment 3, adapter 1
    a = 1
    for n in range(N):
        acc = b[n] + sum(x[m, k] * W[n, k] for k in range(K))
        acc += sc[a] * sum(sum(x[m, k] * As[a][j, k] for k in range(K)) * Bs[a][n, j] for j in range(ranks[a]))
        assert abs(acc - y[m, n]) < 1e-12 * max(1.0, abs(acc))


# --------------------------------------------------------------- normalisation
def test_layernorm_properties_and_brute_force():
    r = rng(5)
    x = r.standard_normal((6, 40)) * 3 + 1.5
    g, b = r.standard_normal(40), r.standard_normal(40)
    y = O.layernorm(x, np.ones(40), np.zeros(40), eps=0.0)
    assert np.abs(y.mean(-1)).max() < 1e-12
    assert np.abs((y * y).mean(-1) - 1).max() < 1e-12
    # shift invariance
    assert np.allclose(O.layernorm(x + 100.0, g, b), O.layernorm(x, g, b), atol=1e-9)
    # brute force one row with eps and affine
    row = x[2]
    mu = sum(row) / 40
    var = sum((v - mu) ** 2 for v in row) / 40
    ref = [(row[i] - mu) / math.sqrt(var + 1e-5) * g[i] + b[i] for i in range(40)]
    assert np.allclose(O.layernorm(x, g, b)[2], ref, rtol=1e-12, atol=1e-12)


def test_groupnorm_group_layout_and_special_cases():
    r = rng(6)
    Bn, T, C, Gr = 2, 5, 12, 3
    x = r.standard_normal((Bn, T, C)) * 2 + 0.3
    g, b = r.standard_normal(C), r.standard_normal(C)
    y = O.groupnorm(x, g, b, groups=Gr, eps=1e-6)
    # brute force: group j holds channels [j*C/G, (j+1)*C/G), statistics over all tokens
    cpg = C // Gr
    for n in range(Bn):
        for j in range(Gr):
            vals = [x[n, t, c] for t in range(T) for c in range(j * cpg, (j + 1) * cpg)]
            mu = sum(vals) / len(vals)
            var = sum((v - mu) ** 2 for v in vals) / len(vals)
            for t in range(T):
                for c in range(j * cpg, (j + 1) * cpg):
                    ref = (x[n, t, c] - mu) / math.sqrt(var + 1e-6) * g[c] + b[c]
                    assert abs(ref - y[n, t, c]) < 1e-12
    # one group over one sample == LayerNorm of the flattened sample
    one = O.groupnorm(x[:1], np.ones(C), np.zeros(C), groups=1, eps=1e-5)
    flat = O.layernorm(x[:1].reshape(1, -1), np.ones(T * C), np.zeros(T * C), eps=1e-5)
    assert np.allclose(one.reshape(1, -1), flat, atol=1e-12)
    # samples are independent
    assert np.array_equal(O.groupnorm(x, g, b, groups=Gr)[1:], O.groupnorm(x[1:], g, b, groups=Gr))
    # T = 1 and groups = C: every element is its own group -> output is beta exactly (x - mean = 0)
    x1 = r.standard_normal((1, 1, C))
    assert np.allclose(O.groupnorm(x1, g, b, groups=C), b.reshape(1, 1, C), atol=1e-12)


# ------------------------------------------------------------------- attention
def test_softmax_rows_sum_to_one_and_shift_invariance():
    S = rng(7).standard_normal((9, 33)) * 10
    P = O.softmax_rows(S)
    assert (P >= 0).all()
    assert np.abs(P.sum(-1) - 1).max() < 1e-12
    assert np.allclose(O.softmax_rows(S + 1000.0), P, atol=1e-12)
    # huge scores do not overflow
    assert np.isfinite(O.softmax_rows(S * 1e3)).all()


def test_attention_brute_force_tiny():
    r = rng(8)
    Bn, Tq, Tk, heads, d = 2, 4, 3, 2, 2
    C = heads * d
    q, k, v = r.standard_normal((Bn, Tq, C)), r.standard_normal((Bn, Tk, C)), r.standard_normal((Bn, Tk, C))
    out = O.attention(q, k, v, heads)
    for b in range(Bn):
        for h in range(heads):
            for i in range(Tq):
                s = [sum(q[b, i, h * d + e] * k[b, j, h * d + e] for e in range(d)) / math.sqrt(d) for j in range(Tk)]
                mx = max(s)
                w = [math.exp(t - mx) for t in s]
                z = sum(w)
                for e in range(d):
                    ref = sum(w[j] / z * v[b, j, h * d + e] for j in range(Tk))
                    assert abs(ref - out[b, i, h * d + e]) < 1e-12


def test_attention_special_cases():
    r = rng(9)
    Bn, Tq, Tk, heads = 1, 5, 7, 2
    C = heads * 64
    q, k, v = r.standard_normal((Bn, Tq, C)), r.standard_normal((Bn, Tk, C)), r.standard_normal((Bn, Tk, C))
    # all-equal scores (q = 0) -> mean of V
    assert np.allclose(O.attention(np.zeros_like(q), k, v, heads), np.broadcast_to(v.mean(1, keepdims=True), q.shape), atol=1e-12)
    # single key -> output is that value row
    assert np.allclose(O.attention(q, k[:, :1], v[:, :1], heads), np.broadcast_to(v[:, :1], q.shape), atol=1e-12)
    # one dominant key -> its value row (scores are q.k/8: make key 3 parallel to every query's sum direction)
    kd = k.copy()
    qd = np.abs(q) + 1.0
    kd[:, 3] = 50.0
    kd[:, [0, 1, 2, 4, 5, 6]] = 0.0
    out = O.attention(qd, kd, v, heads)
    assert np.allclose(out, np.broadcast_to(v[:, 3:4], q.shape), atol=1e-9)
    # permuting keys and values together changes nothing
    perm = r.permutation(Tk)
    assert np.allclose(O.attention(q, k[:, perm], v[:, perm], heads), O.attention(q, k, v, heads), atol=1e-12)
    # heads are independent: changing head 1's keys leaves head 0's output unchanged
    k2 = k.copy()
    k2[..., 64:] = r.standard_normal(k2[..., 64:].shape)
    o1, o2 = O.attention(q, k, v, heads), O.attention(q, k2, v, heads)
    assert np.array_equal(o1[..., :64], o2[..., :64]) and not np.allclose(o1[..., 64:], o2[..., 64:])
    # the 1/sqrt(d) scale is 1/8 for d = 64: doubling q equals scores scaled by 2
    S = np.einsum("bqd,bkd->bqk", q[..., :64], k[..., :64]) / 8.0
    ref = np.einsum("bqk,bkd->bqd", O.softmax_rows(S), v[..., :64])
    assert np.allclose(o1[..., :64], ref, atol=1e-12)


# ------------------------------------------------------------------------ GEGLU
def test_gelu_closed_forms_and_geglu_halves():
    assert O.gelu(np.array([0.0]))[0] == 0.0
    z = np.array([0.3, 1.7, 4.0])
    assert np.allclose(O.gelu(-z), O.gelu(z) - z, atol=1e-15)          # gelu(-z) = gelu(z) - z
    assert abs(O.gelu(np.array([12.0]))[0] - 12.0) < 1e-12             # -> z for large z
    for t in (-2.5, -0.1, 0.7, 3.0):                                   # vs math.erf
        assert abs(O.gelu(np.array([t]))[0] - 0.5 * t * (1 + math.erf(t / math.sqrt(2)))) < 1e-15
    # tanh approximation is a different function (guards the flavour)
    t = 1.0
    tanh_form = 0.5 * t * (1 + math.tanh(math.sqrt(2 / math.pi) * (t + 0.044715 * t ** 3)))
    assert abs(O.gelu(np.array([t]))[0] - tanh_form) > 1e-5
    u = rng(10).standard_normal((4, 10))
    out = O.geglu(u)
    assert out.shape == (4, 5)
    assert np.allclose(out, u[:, :5] * O.gelu(u[:, 5:]))
    swapped = np.concatenate([u[:, 5:], u[:, :5]], axis=1)
    assert not np.allclose(O.geglu(swapped), out)


# ------------------------------------------------------------ block / stack
def _small_stack(depth=1, r=4, seed=0, lora_ff=True):
    cfg = G.StackConfig("t", Bn=2, T=6, C=128, heads=2, depth=depth, r=r, alpha=2.0, lora_ff=lora_ff, Tc=5, Dc=32)
    return cfg, G.make_stack_inputs(cfg, seed)


def test_block_identity_when_output_projections_vanish():
    cfg, p = _small_stack()
    blk = p["blocks"][0]
    for name in ("o1", "o2", "ff2"):
        blk[name]["W"][:] = 0
        blk[name]["b"][:] = 0
        blk[name]["B"][:] = 0
    h = rng(11).standard_normal((2, 6, 128))
    assert np.array_equal(O.block(h, p["ctx"], blk, cfg.heads), h)


def test_block_zero_adapter_equals_no_adapter_and_adapter_matters():
    cfg, p = _small_stack()
    blk = p["blocks"][0]
    h = rng(12).standard_normal((2, 6, 128))
    y_lora = O.block(h, p["ctx"], blk, cfg.heads)
    nolora = {k: (dict(v, A=None, B=None) if isinstance(v, dict) else v) for k, v in blk.items()}
    zeroB = {k: (dict(v, B=np.zeros_like(v["B"])) if isinstance(v, dict) else v) for k, v in blk.items()}
    y0 = O.block(h, p["ctx"], nolora, cfg.heads)
    assert np.array_equal(O.block(h, p["ctx"], zeroB, cfg.heads), y0)
    assert np.abs(y_lora - y0).max() > 1e-6
    # merged weights give the same block
    merged = {k: (dict(v, W=O.merged_weight(v["W"], v["A"], v["B"], v["scale"]), A=None, B=None)
                  if isinstance(v, dict) else v) for k, v in blk.items()}
    ym = O.block(h, p["ctx"], merged, cfg.heads)
    assert np.abs(ym - y_lora).max() < 1e-11 * np.abs(y_lora).max()


def test_block_cross_attention_reads_the_context():
    cfg, p = _small_stack()
    blk = p["blocks"][0]
    h = rng(13).standard_normal((2, 6, 128))
    ctx2 = p["ctx"].copy()
    ctx2[1] *= 50.0
    y1, y2 = O.block(h, p["ctx"], blk, cfg.heads), O.block(h, ctx2, blk, cfg.heads)
    assert np.array_equal(y1[0], y2[0])          # sample 0 does not see sample 1's context
    assert np.abs(y1[1] - y2[1]).max() > 1e-6


def test_stack_batch_independence_and_depth_composition():
    # Section 3.3: the two latents of the guidance pair have no dependency
    cfg, p = _small_stack(depth=3)
    y = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
    for b in range(2):
        yb = O.spatial_transformer(p["x"][b:b + 1], p["ctx"][b:b + 1], p, cfg.heads)
        assert np.array_equal(y[b:b + 1], yb)
    # depth-n is n applications of block between the wrapper ops
    h = O.proj(O.groupnorm(p["x"], p["gn_g"], p["gn_b"]), p["proj_in"])
    for blk in p["blocks"]:
        h = O.block(h, p["ctx"], blk, cfg.heads)
    assert np.array_equal(O.proj(h, p["proj_out"]) + p["x"], y)
    # outer residual: zero proj_out -> output is the input
    p["proj_out"]["W"][:] = 0
    p["proj_out"]["b"][:] = 0
    assert np.array_equal(O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads), p["x"].astype(np.float64))


def test_fp32_mode_is_close_to_fp64_mode():
    cfg, p = _small_stack(depth=2)
    y64 = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
    y32 = O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads, dtype=np.float32)
    assert y32.dtype == np.float32
    assert np.abs(y32 - y64).max() <= 1e-5 * np.abs(y64).max()


# ---------------------------------------------------------------------- patch
def test_patch_exact_integer_case():
    r = rng(14)
    out_f, in_f, rk = 6, 10, 3
    W = r.integers(-8, 9, (out_f, in_f)).astype(np.float32)
    A = r.integers(-3, 4, (rk, in_f)).astype(np.float32)
    B = r.integers(-3, 4, (out_f, rk)).astype(np.float32)
    Wp, undo = O.lora_patch(W, A, B, 2.0)
    ref = np.array([[W[n, k] + 2.0 * sum(B[n, j] * A[j, k] for j in range(rk)) for k in range(in_f)] for n in range(out_f)], dtype=np.float32)
    assert np.array_equal(Wp, ref)
    assert np.array_equal(undo, W)
    # with exactly representable values the arithmetic inverse is exact as well
    assert np.array_equal(O.lora_unpatch_by_subtraction(Wp, A, B, 2.0), W)
    assert O.lora_unpatch(Wp, undo).tobytes() == W.tobytes()


def test_patch_against_fp64_and_roundtrip_bits():
    m = G.make_patch_inputs(((1, 256, 192),), r=32, alpha=16.0, seed=3)[0]   # scale 0.5
    Wp, undo = O.lora_patch(m["W"], m["A"], m["B"], m["scale"])
    ref = O.merged_weight(m["W"], m["A"], m["B"], m["scale"])
    assert Wp.dtype == np.float32
    assert np.abs(Wp - ref).max() <= 1e-6 * np.abs(ref).max()
    assert not np.array_equal(Wp, m["W"])
    assert O.lora_unpatch(Wp, undo).tobytes() == m["W"].tobytes()


def test_subtraction_does_not_restore_the_weights():
    # the negative control behind the undo record: fl32(fl32(W + d) - d) != W in general
    m = G.make_patch_inputs(((1, 320, 320),), r=32, alpha=32.0, seed=0)[0]
    Wp, undo = O.lora_patch(m["W"], m["A"], m["B"], m["scale"])
    back = O.lora_unpatch_by_subtraction(Wp, m["A"], m["B"], m["scale"])
    frac = float((back.view(np.uint32) != m["W"].view(np.uint32)).mean())
    assert frac > 0.01
    assert O.lora_unpatch(Wp, undo).tobytes() == m["W"].tobytes()


# ------------------------------------------------------------ input generator
def test_patch_multi_is_successive_single_patches_and_exact_on_integers():
    r = np.random.default_rng(11)
    out_f, in_f = 6, 5
    W = r.integers(-8, 9, size=(out_f, in_f)).astype(np.float32)
    ads = [(r.integers(-3, 4, size=(rk, in_f)).astype(np.float32), r.integers(-3, 4, size=(out_f, rk)).astype(np.float32), sc)
           for rk, sc in ((2, 1.0), (3, 2.0), (1, -1.0))]
    Wp, undo = O.lora_patch_multi(W, ads)
    # integers: every intermediate is exact, so the plain definition W + sum_i s_i B_i A_i by loops
    for n in range(out_f):
        for k in range(in_f):
            acc = float(W[n, k])
            for A, B, sc in ads:
                acc += sc * sum(float(B[n, j]) * float(A[j, k]) for j in range(A.shape[0]))
            assert Wp[n, k] == acc
    assert undo.tobytes() == W.tobytes()
    # one adapter: the single-patch function, bit for bit
    W1, _ = O.lora_patch(W, *ads[0])
    assert O.lora_patch_multi(W, ads[:1])[0].tobytes() == W1.tobytes()
    # real-valued: equals successive single patches bit for bit, and the fp64 sum within 1e-6
    Wr = (0.02 * r.standard_normal((40, 24))).astype(np.float32)
    adr = [((0.02 * r.standard_normal((rk, 24))).astype(np.float32), (0.02 * r.standard_normal((40, rk))).astype(np.float32), sc)
           for rk, sc in ((8, 1.0), (4, 0.5))]
    Wm, _ = O.lora_patch_multi(Wr, adr)
    step = Wr
    for A, B, sc in adr:
        step, _ = O.lora_patch(step, A, B, sc)
    assert Wm.tobytes() == step.tobytes()
    ref = Wr.astype(np.float64) + sum(sc * (B.astype(np.float64) @ A.astype(np.float64)) for A, B, sc in adr)
    assert rel_err(Wm, ref) <= 1e-6
    # dropping an adapter or its scale is visible
    assert rel_err(O.lora_patch_multi(Wr, adr[:1])[0], ref) > 1e-4
    assert rel_err(O.lora_patch_multi(Wr, [adr[0], (adr[1][0], adr[1][1], 1.0)])[0], ref) > 1e-4


def test_bf16_rounding_of_the_serving_copy():
    import torch
    # ties go to the even mantissa; one ulp above the tie goes up
    cases = {0x3F808000: 0x3F80, 0x3F818000: 0x3F82, 0x3F808001: 0x3F81, 0xBF808000: 0xBF80, 0x3F7FFFFF: 0x3F80, 0x00000000: 0x0000}
    for bits, want in cases.items():
        x = np.array([bits], dtype=np.uint32).view(np.float32)
        got = O.bf16_rne(x).view(np.uint32)[0] >> 16
        assert got == want, (hex(bits), hex(got), hex(want))
    r = np.random.default_rng(5)
    x = (r.standard_normal(4096) * np.exp(r.uniform(-20, 20, 4096))).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()      # an independent implementation
    assert O.bf16_rne(x).tobytes() == lib.tobytes()
    Wr = (0.02 * r.standard_normal((16, 8))).astype(np.float32)
    A, B = (0.02 * r.standard_normal((4, 8))).astype(np.float32), (0.02 * r.standard_normal((16, 4))).astype(np.float32)
    Wp, undo, Wb = O.lora_patch_multi(Wr, [(A, B, 1.0)], serving=True)
    assert Wb.tobytes() == O.bf16_rne(Wp).tobytes() and np.abs(Wb - Wp).max() <= np.abs(Wp).max() * 2.0 ** -8


def test_cfg_combine_special_cases():
    r = np.random.default_rng(9)
    eu = G.bf16_round(r.standard_normal((4, 33)).astype(np.float32))
    ec = G.bf16_round(r.standard_normal((4, 33)).astype(np.float32))
    assert O.cfg_combine(eu, ec, 0.0).tobytes() == eu.tobytes()          # g = 0: the unconditional latent
    assert O.cfg_combine(eu, ec, 1.0, out_bf16=False).tobytes() == (eu + (ec - eu)).astype(np.float32).tobytes()
    assert np.abs(O.cfg_combine(eu, ec, 1.0) - ec).max() <= np.abs(ec).max() * 2.0 ** -7   # g = 1: the conditional one
    g = 7.5
    out = O.cfg_combine(eu, ec, g, out_bf16=False)
    for i in range(4):
        for j in range(33):
            want = float(eu[i, j]) + g * (float(ec[i, j]) - float(eu[i, j]))
            assert abs(float(out[i, j]) - want) <= 1e-6 * max(1.0, abs(want))
    # the two latents are not interchangeable, and the weight is not dropped
    assert rel_err(O.cfg_combine(ec, eu, g, out_bf16=False), out) > 0.1
    assert rel_err(O.cfg_combine(eu, ec, 1.0, out_bf16=False), out) > 0.1
    # exact on small integers
    eu_i = np.array([[1.0, -2.0, 3.0]], np.float32); ec_i = np.array([[2.0, 2.0, -1.0]], np.float32)
    assert O.cfg_combine(eu_i, ec_i, 3.0, out_bf16=False).tolist() == [[4.0, 10.0, -9.0]]


def test_silu_closed_forms_and_groupnorm_silu_composition():
    assert O.silu(np.array([0.0]))[0] == 0.0
    z = np.array([-30.0, -2.0, -0.5, 0.5, 2.0, 30.0])
    want = [v / (1.0 + math.exp(-v)) for v in z]
    assert np.allclose(O.silu(z), want, rtol=1e-14, atol=0)
    assert np.allclose(O.silu(z) - O.silu(-z), z, rtol=1e-13)          # silu(z) - silu(-z) = z
    assert abs(O.silu(np.array([30.0]))[0] - 30.0) < 1e-11 and abs(O.silu(np.array([-30.0]))[0]) < 1e-11
    assert O.silu(np.array([-1.278]))[0] == pytest.approx(-0.27846, abs=1e-5)   # the minimum of z*sigmoid(z)
    r = np.random.default_rng(3)
    x = r.standard_normal((2, 9, 64)); g = 1 + 0.1 * r.standard_normal(64); b = 0.1 * r.standard_normal(64)
    y = O.groupnorm_silu(x, g, b)
    n = O.groupnorm(x, g, b)
    for idx in ((0, 0, 0), (1, 8, 63), (0, 4, 31)):
        assert y[idx] == pytest.approx(n[idx] / (1.0 + math.exp(-n[idx])), rel=1e-13)
    assert rel_err(O.groupnorm(x, g, b), y) > 0.1                        # the activation is not a no-op


def test_bal_timeline_closed_forms():
    d, S, k = 0.1, 50, 20
    # already loaded: patched before the first step, nothing waits, latency = S steps + the patch
    assert O.bal_timeline(0.0, d, S, k, patch_time=0.03) == (1, 0.0, pytest.approx(S * d + 0.03))
    # loaded during step 11 (10 steps done at t = 1.0): the first boundary at or after is before step 12
    pb, stall, total = O.bal_timeline(1.05, d, S, k)
    assert (pb, stall) == (12, 0.0) and total == pytest.approx(S * d)
    # exactly on a boundary counts as loaded
    assert O.bal_timeline(1.0 + 1e-12, d, S, k)[0] == 12 and O.bal_timeline(1.0 - 1e-9, d, S, k)[0] == 11
    # slower than the bound: the loop reaches the boundary before step k at (k-1) d and waits
    pb, stall, total = O.bal_timeline(3.0, d, S, k)
    assert pb == k and stall == pytest.approx(3.0 - (k - 1) * d) and total == pytest.approx(3.0 + (S - k + 1) * d)
    # k = 1 is synchronous loading: everything waits, no step runs unpatched
    pb, stall, total = O.bal_timeline(3.0, d, S, 1)
    assert (pb, stall) == (1, pytest.approx(3.0)) and total == pytest.approx(3.0 + S * d)
    # never loaded within the run and no bound inside it: never patched
    assert O.bal_timeline(1e9, d, S, S + 1)[0] is None
    # latency saved against load-then-run is min(load, time before the bound)
    for load in (0.2, 1.0, 1.9, 2.5, 7.0):
        sync = load + S * d
        assert sync - O.bal_timeline(load, d, S, k)[2] == pytest.approx(min(load, (k - 1) * d), abs=d)


def test_bf16_helpers_roundtrip_and_rne():
    bits = np.arange(0, 0x7F80, 7, dtype=np.uint16)          # positive finite bf16 values
    assert np.array_equal(G.bf16_bits(G.bf16_widen(bits)), bits)
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: ties to even -> 1.0
    assert G.bf16_round(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 1.0
    assert G.bf16_round(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == np.float32(1.0 + 2.0 ** -6)
    x = rng(15).standard_normal(1000).astype(np.float32)
    assert np.abs(G.bf16_round(x) - x).max() <= np.abs(x).max() * 2.0 ** -8


def test_generator_is_seeded_and_shaped():
    a = G.make_stack_inputs(G.TINY, seed=0)
    b = G.make_stack_inputs(G.TINY, seed=0)
    c = G.make_stack_inputs(G.TINY, seed=1)
    assert np.array_equal(a["x"], b["x"]) and not np.array_equal(a["x"], c["x"])
    assert a["x"].shape == (2, 256, 320) and a["ctx"].shape == (2, 77, 2048)
    blk = a["blocks"][0]
    assert blk["k2"]["W"].shape == (320, 2048) and blk["ff1"]["W"].shape == (2560, 320)
    assert blk["q1"]["A"].shape == (8, 320) and blk["q1"]["B"].shape == (320, 8)
    assert blk["ff1"]["A"] is None and blk["q1"]["scale"] == 1.0
    assert np.array_equal(G.bf16_round(blk["q1"]["W"]), blk["q1"]["W"])
    n = sum(c for c, _, _ in G.PATCH_SWEEP)
    elems = sum(c * o * i for c, o, i in G.PATCH_SWEEP)
    assert n == 310 and elems == 830_668_800


def test_controlnet_residual_add_special_cases():
    # Section 2, "ControlNet": several ControlNets' outputs are summed, then applied to the backbone tensor
    rng = np.random.default_rng(11)
    h = O.bf16_rne(rng.standard_normal((5, 33)).astype(np.float32))
    rs = [O.bf16_rne(rng.standard_normal((5, 33)).astype(np.float32)) for _ in range(3)]
    assert O.controlnet_residual_add(h, []).tobytes() == h.tobytes()                       # nothing to add
    assert O.controlnet_residual_add(h, [np.zeros_like(h)] * 3).tobytes() == h.tobytes()
    one = O.controlnet_residual_add(h, rs[:1], out_bf16=False)
    assert one.tobytes() == (h + rs[0]).astype(np.float32).tobytes()                        # one ControlNet: a plain add
    # against float64: three float32 additions of O(1) values
    ref = h.astype(np.float64) + sum(r.astype(np.float64) for r in rs)
    got = O.controlnet_residual_add(h, rs, out_bf16=False)
    assert np.abs(got - ref).max() <= 4 * 2.0 ** -23 * np.abs(ref).max()
    # small integers are exact whatever the order
    hi = np.array([[1.0, -2.0, 8.0]], np.float32)
    assert O.controlnet_residual_add(hi, [np.array([[2.0, 2.0, -3.0]], np.float32), np.array([[4.0, 1.0, -5.0]], np.float32)],
                                     out_bf16=False).tolist() == [[7.0, 1.0, 0.0]]
    # the ControlNets' outputs are summed first: 2^24 + (1 + 1) is exact, (2^24 + 1) + 1 is not
    big = np.array([2.0 ** 24], np.float32)
    u = np.array([1.0], np.float32)
    assert O.controlnet_residual_add(big, [u, u], out_bf16=False)[0] == np.float32(2.0 ** 24 + 2)
    # a dropped term or a flipped sign is seen
    assert rel_err(O.controlnet_residual_add(h, rs[:2], out_bf16=False), got) > 0.1
    assert rel_err(O.controlnet_residual_add(h, [rs[0], rs[1], -rs[2]], out_bf16=False), got) > 0.1


# ------------------------------------- sub-layer composition, by brute force in plain Python
# The block's equations (pre-LayerNorm self-attention, cross-attention to the text context,
# GEGLU feed-forward, each added to the stream) written out with nested loops and the math
# module only: no numpy contraction, no call into the oracle.  `mut` plants one mistake in
# this reference, so that the test can show each of them would be seen:
#   "q_from_h"      the query projected from the un-normalised stream
#   "kv_from_h"     self-attention keys / values projected from h instead of LN(h)
#   "ff_no_ln"      the feed-forward sub-layer without its LayerNorm
#   "gamma_beta"    LayerNorm's gamma and beta exchanged
#   "cross_first"   cross-attention before self-attention
#   "no_residual"   a sub-layer's output replacing the stream instead of being added to it
#   "gate_first"    GEGLU taking the first half as the gate
def _py_matvec_rows(X, W, b=None):
    return [[sum(x[k] * w[k] for k in range(len(x))) + (b[n] if b is not None else 0.0) for n, w in enumerate(W)] for x in X]


def _py_proj(X, p):
    Y = _py_matvec_rows(X, p["W"], p.get("b"))
    if p.get("A") is not None:
        Tm = _py_matvec_rows(X, p["A"])
        U = _py_matvec_rows(Tm, p["B"])
        Y = [[y + p["scale"] * u for y, u in zip(yr, ur)] for yr, ur in zip(Y, U)]
    return Y


def _py_layernorm(X, g, b, eps=1e-5):
    out = []
    for x in X:
        mu = sum(x) / len(x)
        var = sum((v - mu) ** 2 for v in x) / len(x)
        out.append([(v - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, v in enumerate(x)])
    return out


def _py_attention(Q, K, V, heads):
    C = len(Q[0])
    d = C // heads
    out = [[0.0] * C for _ in Q]
    for h in range(heads):
        for i, q in enumerate(Q):
            s = [sum(q[h * d + e] * k[h * d + e] for e in range(d)) / math.sqrt(d) for k in K]
            mx = max(s)
            w = [math.exp(v - mx) for v in s]
            z = sum(w)
            for e in range(d):
                out[i][h * d + e] = sum(w[j] / z * V[j][h * d + e] for j in range(len(K)))
    return out


def _py_attn_sublayer(H, ctx, g, b, pq, pk, pv, po, heads, mut):
    if mut == "gamma_beta":
        g, b = b, g
    Nrm = _py_layernorm(H, g, b)
    src = Nrm if ctx is None else ctx
    if mut == "kv_from_h" and ctx is None:
        src = H
    Q = _py_proj(H if mut == "q_from_h" else Nrm, pq)
    Kk, Vv = _py_proj(src, pk), _py_proj(src, pv)
    U = _py_proj(_py_attention(Q, Kk, Vv, heads), po)
    if mut == "no_residual":
        return U
    return [[h + u for h, u in zip(hr, ur)] for hr, ur in zip(H, U)]


def _py_ff_sublayer(H, g, b, p1, p2, mut):
    if mut == "gamma_beta":
        g, b = b, g
    Nrm = H if mut == "ff_no_ln" else _py_layernorm(H, g, b)
    U = _py_proj(Nrm, p1)
    F = len(U[0]) // 2
    if mut == "gate_first":
        G_ = [[u[F + i] * (0.5 * u[i] * (1.0 + math.erf(u[i] / math.sqrt(2.0)))) for i in range(F)] for u in U]
    else:
        G_ = [[u[i] * (0.5 * u[F + i] * (1.0 + math.erf(u[F + i] / math.sqrt(2.0)))) for i in range(F)] for u in U]
    Y = _py_proj(G_, p2)
    return [[h + y for h, y in zip(hr, yr)] for hr, yr in zip(H, Y)]


def _py_block(H, ctx, blk, heads, mut=None):
    """H [Bn][T][C], ctx [Bn][Tc][Dc] as nested lists; every sample on its own."""
    out = []
    for hb, cb in zip(H, ctx):
        def self_attn(h):
            return _py_attn_sublayer(h, None, blk["ln1_g"], blk["ln1_b"], blk["q1"], blk["k1"], blk["v1"], blk["o1"], heads, mut)

        def cross_attn(h):
            return _py_attn_sublayer(h, cb, blk["ln2_g"], blk["ln2_b"], blk["q2"], blk["k2"], blk["v2"], blk["o2"], heads, mut)
        h = cross_attn(hb) if mut == "cross_first" else self_attn(hb)
        h = self_attn(h) if mut == "cross_first" else cross_attn(h)
        out.append(_py_ff_sublayer(h, blk["ln3_g"], blk["ln3_b"], blk["ff1"], blk["ff2"], mut))
    return out


def _toy_block(seed=21):
    """Bn=2, T=3, Tc=2, C=4, 2 heads of 2, Dc=3, F=16, rank 2, scale 0.5; every projection
    biased (also q, k, v: a dropped bias would otherwise hide), gamma away from 1, beta
    away from 0, unit-scale weights so that softmax is far from uniform."""
    r = rng(seed)
    C, Dc, F, rk = 4, 3, 16, 2

    def pr(n_out, n_in):
        return {"W": r.standard_normal((n_out, n_in)), "b": r.standard_normal(n_out), "A": r.standard_normal((rk, n_in)),
                "B": r.standard_normal((n_out, rk)), "scale": 0.5}
    blk = {}
    for i in (1, 2, 3):
        blk[f"ln{i}_g"] = 1.5 + 0.5 * r.standard_normal(C)
        blk[f"ln{i}_b"] = 0.7 * r.standard_normal(C) + 0.3
    blk.update(q1=pr(C, C), k1=pr(C, C), v1=pr(C, C), o1=pr(C, C), q2=pr(C, C), k2=pr(C, Dc), v2=pr(C, Dc), o2=pr(C, C),
               ff1=pr(2 * F, C), ff2=pr(C, F))
    h = r.standard_normal((2, 3, C)) * 1.3 + 0.4
    ctx = r.standard_normal((2, 2, Dc))
    return h, ctx, blk


def _to_lists(blk):
    return {k: ({kk: (vv.tolist() if isinstance(vv, np.ndarray) else vv) for kk, vv in v.items()} if isinstance(v, dict) else v.tolist())
            for k, v in blk.items()}


def test_sublayers_and_block_against_plain_python_loops():
    h, ctx, blk = _toy_block()
    L = _to_lists(blk)
    heads = 2
    # each sub-layer on its own, both samples
    for b in range(2):
        hb, cb = h[b].tolist(), ctx[b].tolist()
        ref = _py_attn_sublayer(hb, None, L["ln1_g"], L["ln1_b"], L["q1"], L["k1"], L["v1"], L["o1"], heads, None)
        got = O.attn_sublayer(h[b:b + 1], None, blk["ln1_g"], blk["ln1_b"], blk["q1"], blk["k1"], blk["v1"], blk["o1"], heads)
        assert np.abs(got[0] - np.array(ref)).max() <= 1e-12 * np.abs(np.array(ref)).max()
        ref = _py_attn_sublayer(hb, cb, L["ln2_g"], L["ln2_b"], L["q2"], L["k2"], L["v2"], L["o2"], heads, None)
        got = O.attn_sublayer(h[b:b + 1], ctx[b:b + 1], blk["ln2_g"], blk["ln2_b"], blk["q2"], blk["k2"], blk["v2"], blk["o2"], heads)
        assert np.abs(got[0] - np.array(ref)).max() <= 1e-12 * np.abs(np.array(ref)).max()
        ref = _py_ff_sublayer(hb, L["ln3_g"], L["ln3_b"], L["ff1"], L["ff2"], None)
        got = O.ff_sublayer(h[b:b + 1], blk["ln3_g"], blk["ln3_b"], blk["ff1"], blk["ff2"])
        assert np.abs(got[0] - np.array(ref)).max() <= 1e-12 * np.abs(np.array(ref)).max()
    # the whole block: order self -> cross -> feed-forward
    got = O.block(h, ctx, blk, heads)
    ref = np.array(_py_block(h.tolist(), ctx.tolist(), L, heads))
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 1e-12 * scale
    # every planted mistake moves the reference far away from the oracle: this pin sees them
    for mut in ("q_from_h", "kv_from_h", "ff_no_ln", "gamma_beta", "cross_first", "no_residual", "gate_first"):
        bad = np.array(_py_block(h.tolist(), ctx.tolist(), L, heads, mut))
        assert np.abs(bad - got).max() > 1e-3 * scale, mut


def test_block_through_the_stack_wrapper_against_plain_python_loops():
    # spatial_transformer = proj_in(GroupNorm(x)) -> blocks -> proj_out + x, with the toy block
    # in the middle (GroupNorm with one channel per group would be degenerate: 2 groups of 2)
    h, ctx, blk = _toy_block(seed=22)
    L = _to_lists(blk)
    r = rng(23)
    C = 4
    params = {"gn_g": 1.0 + 0.3 * r.standard_normal(C), "gn_b": 0.2 * r.standard_normal(C),
              "proj_in": {"W": r.standard_normal((C, C)), "b": r.standard_normal(C)},
              "proj_out": {"W": r.standard_normal((C, C)), "b": r.standard_normal(C)}, "blocks": [blk, blk]}
    x = h
    # GroupNorm by loops: 2 groups of 2 adjacent channels, statistics over the sample's tokens
    groups, eps = 2, 1e-6
    xs = x.tolist()
    hn = []
    for b in range(2):
        rows = [[0.0] * C for _ in range(3)]
        for g in range(groups):
            vals = [xs[b][t][c] for t in range(3) for c in (2 * g, 2 * g + 1)]
            mu = sum(vals) / len(vals)
            var = sum((v - mu) ** 2 for v in vals) / len(vals)
            for t in range(3):
                for c in (2 * g, 2 * g + 1):
                    rows[t][c] = (xs[b][t][c] - mu) / math.sqrt(var + eps) * params["gn_g"][c] + params["gn_b"][c]
        hn.append(rows)
    P = {k: {kk: vv.tolist() for kk, vv in params[k].items()} for k in ("proj_in", "proj_out")}
    hh = [_py_proj(rows, P["proj_in"]) for rows in hn]
    for _ in range(2):
        hh = _py_block(hh, ctx.tolist(), L, 2)
    ref = np.array([[[y + xv for y, xv in zip(yr, xr)] for yr, xr in zip(_py_proj(rows, P["proj_out"]), xb)] for rows, xb in zip(hh, xs)])
    import oracle.sdxl_block_oracle as OM
    old = OM.GN_GROUPS
    try:
        OM.GN_GROUPS = groups          # the wrapper takes the module's group count
        got = O.spatial_transformer(x, ctx, params, 2)
    finally:
        OM.GN_GROUPS = old
    assert np.abs(got - ref).max() <= 1e-11 * np.abs(ref).max()
