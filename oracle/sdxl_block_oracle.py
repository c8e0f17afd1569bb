"""CPU oracle for the LoRA-augmented SDXL spatial-transformer path and LoRA patching.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what the
HIP kernels of this repository must compute.  Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import it; the product path never does, and it
imports nothing from the product path.

Every function is the textbook definition written out with numpy, one library
matmul per contraction and no blocking, fusion or re-association beyond what the
definition states.  Floating point is float64 unless `dtype` says otherwise; the
patch functions follow a fixed float32 rounding chain because their result is a
stored float32 weight.

What the paper fixes (arXiv 2407.02031):
  * Section 2, "Low-Rank Adaptation": a patched weight is the base weight plus the
    product of two rank-r matrices.  With weights stored [out, in] this is
    W' = W + scale * B @ A, A [r, in], B [out, r]; the paper's formula is the case
    scale = 1 with the two letters exchanged.
  * Section 4.2, "Efficient LoRA patching": the product is merged into the base
    parameters in place, and taken off again after the request.
  * Section 2, "Diffusion model inference", and Section 3.3: the conditional and
    unconditional latents are denoised as one batch of two with no dependency
    between them.
  * Section 4.3, "Kernel-level optimizations": the base model's transformer blocks
    use attention and a GEGLU feed-forward; GroupNorm precedes them.
The block's internal structure (pre-LayerNorm self-attention, cross-attention to the
text context, GEGLU feed-forward, each with a residual connection, wrapped by
GroupNorm + proj_in and proj_out + input) is the standard SDXL spatial transformer;
the paper prints no shapes or formulas for it, so those parts are pinned by the
brute-force references and properties of tests/test_oracle_pins.py, not by paper values.

  * Section 3.1 (add-on usage table) and Section 4.2: a request carries one or two
    LoRAs, loaded in parallel and each merged into the base weights; several adapters
    on one matrix are the sum of their products, W' = W + sum_i scale_i * B_i @ A_i.
  * Section 2, "Diffusion model inference": the conditionally and unconditionally
    denoised latents of a step are combined by a weighted sum (classifier-free
    guidance); the paper cites the guidance formula eps_u + g * (eps_c - eps_u) and
    prints no weights, so g is an argument.

  * Section 4.2, "Bounded asynchronous LoRA loading": adapters load in the background while
    the base model early-starts unpatched; they are patched at the first step boundary
    after loading completes, and at step k the base model waits for them.

Parity pins: linear / lora_linear / layernorm / groupnorm / attention / gelu / geglu /
lora_patch / multi_lora_linear are pinned by brute-force loops, closed forms and
invariants.  `attn_sublayer`, `ff_sublayer`, `block` and `spatial_transformer` are
pinned against the block's equations written out in plain Python loops (math module
only) at toy size, a reference in which each plausible composition mistake (query or
keys from the un-normalised stream, a missing LayerNorm, gamma and beta exchanged,
sub-layers in another order, a dropped residual, the GEGLU halves exchanged) is shown to
move the result, plus structural identities (identity block, zero adapter, batch
independence, depth composition).  The paper prints no worked numbers for the block, so
none of these is a paper value.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

HEAD_DIM = 64
LN_EPS = 1e-5
GN_EPS = 1e-6
GN_GROUPS = 32


def _as(x, dtype):
    return np.asarray(x, dtype=dtype)


# --------------------------------------------------------------------------- #
# projections
# --------------------------------------------------------------------------- #
def linear(x, W, b=None, dtype=np.float64):
    """y[m, n] = sum_k x[m, k] * W[n, k] + b[n]   (weights stored [out, in])."""
    y = _as(x, dtype) @ _as(W, dtype).T
    if b is not None:
        y = y + _as(b, dtype)
    return y


def lora_linear(x, W, b=None, A=None, B=None, scale=1.0, dtype=np.float64):
    """Unmerged LoRA projection: y = x W^T + b + scale * (x A^T) B^T.

    Section 2, "Low-Rank Adaptation": the adapter adds the rank-r product to the
    weight; applied to an input that is the base output plus the input pushed
    through the down-projection A [r, in] and then the up-projection B [out, r].
    """
    y = linear(x, W, b, dtype)
    if A is not None and B is not None:
        t = _as(x, dtype) @ _as(A, dtype).T          # [M, r]
        y = y + dtype(scale) * (t @ _as(B, dtype).T)
    return y


def merged_weight(W, A, B, scale, dtype=np.float64):
    """W' = W + scale * B @ A  (Section 2, "Low-Rank Adaptation")."""
    return _as(W, dtype) + dtype(scale) * (_as(B, dtype) @ _as(A, dtype))


def proj(x, p: dict, dtype=np.float64):
    """Apply a projection dict {W, b, A, B, scale} as produced by the input generator."""
    return lora_linear(x, p["W"], p.get("b"), p.get("A"), p.get("B"), p.get("scale", 0.0), dtype)


def multi_lora_linear(x, W, b, A_list: Sequence, B_list: Sequence, scales: Sequence[float],
                      seg_offsets: Sequence[int], seg_adapter: Sequence[int], dtype=np.float64):
    """Rows [seg_offsets[i], seg_offsets[i+1]) get adapter seg_adapter[i] (-1: none).

    Each request's rows see their own adapter, i.e. `lora_linear` per row segment.
    """
    x = _as(x, dtype)
    M = x.shape[0]
    N = np.shape(W)[0]
    y = np.empty((M, N), dtype=dtype)
    assert seg_offsets[0] == 0 and seg_offsets[-1] == M
    for i, a in enumerate(seg_adapter):
        lo, hi = int(seg_offsets[i]), int(seg_offsets[i + 1])
        assert lo <= hi
        if a < 0:
            y[lo:hi] = linear(x[lo:hi], W, b, dtype)
        else:
            y[lo:hi] = lora_linear(x[lo:hi], W, b, A_list[a], B_list[a], scales[a], dtype)
    return y


# --------------------------------------------------------------------------- #
# normalisations
# --------------------------------------------------------------------------- #
def layernorm(x, gamma, beta, eps=LN_EPS, dtype=np.float64):
    """Per row: (x - mean) / sqrt(biased_var + eps) * gamma + beta."""
    x = _as(x, dtype)
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + dtype(eps)) * _as(gamma, dtype) + _as(beta, dtype)


def groupnorm(x, gamma, beta, groups=GN_GROUPS, eps=GN_EPS, dtype=np.float64):
    """x [Bn, T, C]; statistics per (sample, group of C/groups adjacent channels) over
    all T tokens and the group's channels; biased variance; per-channel affine."""
    x = _as(x, dtype)
    Bn, T, C = x.shape
    assert C % groups == 0
    xg = x.reshape(Bn, T, groups, C // groups)
    mu = xg.mean(axis=(1, 3), keepdims=True)
    xc = xg - mu
    var = (xc * xc).mean(axis=(1, 3), keepdims=True)
    y = (xc / np.sqrt(var + dtype(eps))).reshape(Bn, T, C)
    return y * _as(gamma, dtype) + _as(beta, dtype)


def silu(z):
    """z * sigmoid(z)."""
    z = np.asarray(z)
    return z / (1.0 + np.exp(-z))


def groupnorm_silu(x, gamma, beta, groups=GN_GROUPS, eps=GN_EPS, dtype=np.float64):
    """GroupNorm followed by SiLU, the pair the base model's ResNet blocks apply and the
    paper fuses into one operator (Section 4.3, "Kernel-level optimizations")."""
    return silu(groupnorm(x, gamma, beta, groups, eps, dtype))


# --------------------------------------------------------------------------- #
# attention
# --------------------------------------------------------------------------- #
def softmax_rows(S):
    """Row-wise softmax with the row maximum subtracted first."""
    Z = np.exp(S - S.max(axis=-1, keepdims=True))
    return Z / Z.sum(axis=-1, keepdims=True)


def attention(q, k, v, heads: int, dtype=np.float64):
    """q [Bn, Tq, C], k and v [Bn, Tk, C], C = heads * d.  Per (sample, head):
    softmax(q k^T / sqrt(d)) v, scores materialised in full, no mask."""
    q, k, v = _as(q, dtype), _as(k, dtype), _as(v, dtype)
    Bn, Tq, C = q.shape
    Tk = k.shape[1]
    d = C // heads
    assert d * heads == C
    out = np.empty((Bn, Tq, C), dtype=dtype)
    inv = dtype(1.0) / np.sqrt(dtype(d))
    for b in range(Bn):
        for h in range(heads):
            sl = slice(h * d, (h + 1) * d)
            S = (q[b, :, sl] @ k[b, :, sl].T) * inv          # [Tq, Tk]
            P = softmax_rows(S)
            out[b, :, sl] = P @ v[b, :, sl]
    return out


# --------------------------------------------------------------------------- #
# feed-forward
# --------------------------------------------------------------------------- #
def gelu(z, dtype=np.float64):
    """Exact GELU: z/2 * (1 + erf(z / sqrt 2))."""
    z = _as(z, dtype)
    return dtype(0.5) * z * (dtype(1.0) + _erf(z / np.sqrt(dtype(2.0))).astype(dtype))


def geglu(u, dtype=np.float64):
    """u [M, 2F] -> u[:, :F] * gelu(u[:, F:]): first half value, second half gate."""
    u = _as(u, dtype)
    F = u.shape[-1] // 2
    return u[..., :F] * gelu(u[..., F:], dtype)


# --------------------------------------------------------------------------- #
# block and stack
# --------------------------------------------------------------------------- #
def attn_sublayer(h, ctx, gamma, beta, pq, pk, pv, po, heads, dtype=np.float64):
    """h [Bn, T, C] -> h + out(attention(q(LN h), k(src), v(src))), src = LN h (self,
    ctx None) or the text context (cross)."""
    h = _as(h, dtype)
    n = layernorm(h, gamma, beta, LN_EPS, dtype)
    src = n if ctx is None else _as(ctx, dtype)
    q = proj(n, pq, dtype)
    k = proj(src, pk, dtype)
    v = proj(src, pv, dtype)
    a = attention(q, k, v, heads, dtype)
    return h + proj(a, po, dtype)


def ff_sublayer(h, gamma, beta, p1, p2, dtype=np.float64):
    """h -> h + ff2(geglu(ff1(LN h)))."""
    h = _as(h, dtype)
    n = layernorm(h, gamma, beta, LN_EPS, dtype)
    return h + proj(geglu(proj(n, p1, dtype), dtype), p2, dtype)


def block(h, ctx, blk: dict, heads: int, dtype=np.float64):
    """One transformer block: self-attention, cross-attention, GEGLU feed-forward."""
    h = attn_sublayer(h, None, blk["ln1_g"], blk["ln1_b"], blk["q1"], blk["k1"], blk["v1"], blk["o1"], heads, dtype)
    h = attn_sublayer(h, ctx, blk["ln2_g"], blk["ln2_b"], blk["q2"], blk["k2"], blk["v2"], blk["o2"], heads, dtype)
    h = ff_sublayer(h, blk["ln3_g"], blk["ln3_b"], blk["ff1"], blk["ff2"], dtype)
    return h


def spatial_transformer(x, ctx, params: dict, heads: int, dtype=np.float64):
    """y = proj_out(blocks(proj_in(GroupNorm(x)))) + x, x [Bn, T, C] token-major."""
    x = _as(x, dtype)
    h = proj(groupnorm(x, params["gn_g"], params["gn_b"], GN_GROUPS, GN_EPS, dtype), params["proj_in"], dtype)
    for blk in params["blocks"]:
        h = block(h, ctx, blk, heads, dtype)
    return proj(h, params["proj_out"], dtype) + x


# --------------------------------------------------------------------------- #
# LoRA patching (float32 result)
# --------------------------------------------------------------------------- #
def lora_patch(W, A, B, scale):
    """In-place-merge semantics (Section 4.2): returns (W', undo).

    W' = fl32(W + fl32(scale * fl32(B @ A))), all in float32; `undo` is the bit
    pattern of W before the merge, which is what taking the adapter off restores.
    """
    W = np.asarray(W, dtype=np.float32)
    delta = (np.asarray(B, np.float32) @ np.asarray(A, np.float32)).astype(np.float32)
    delta = (np.float32(scale) * delta).astype(np.float32)
    return (W + delta).astype(np.float32), W.copy()


def bf16_rne(x):
    """float32 -> nearest bfloat16 (ties to even), returned widened to float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return (u.astype(np.uint32) << 16).view(np.float32).reshape(np.shape(x))


def lora_patch_multi(W, adapters, serving=False):
    """Several adapters merged into one matrix in one pass (Section 4.2; one or two LoRAs
    per request, Section 3.1): the adapters are applied one after the other, each with
    the rounding chain of `lora_patch`,
        W_0 = W,  W_i = fl32(W_{i-1} + fl32(scale_i * fl32(B_i @ A_i))),  W' = W_n,
    so a single pass over W equals n successive single patches bit for bit.  `undo` is
    W's bits before the first adapter.  With serving=True also returns the bfloat16
    copy of W' (round to nearest even) that the bf16 GEMMs read, widened to float32.
    `adapters` is a sequence of (A [r_i, in], B [out, r_i], scale_i).
    """
    W0 = np.asarray(W, dtype=np.float32)
    cur = W0
    for A, B, scale in adapters:
        cur, _ = lora_patch(cur, A, B, scale)
    if serving:
        return cur, W0.copy(), bf16_rne(cur)
    return cur, W0.copy()


def cfg_combine(eps_uncond, eps_cond, guidance, out_bf16=True):
    """Classifier-free-guidance weighted sum of the two denoised latents of a step
    (Section 2, "Diffusion model inference"): eps = eps_u + g * (eps_c - eps_u), formed
    in float32 from the (bfloat16-representable) inputs as
    fl32(eps_u + fl32(g * fl32(eps_c - eps_u))), then rounded to bfloat16 if asked."""
    eu = np.asarray(eps_uncond, dtype=np.float32)
    ec = np.asarray(eps_cond, dtype=np.float32)
    d = (ec - eu).astype(np.float32)
    d = (np.float32(guidance) * d).astype(np.float32)
    out = (eu + d).astype(np.float32)
    return bf16_rne(out) if out_bf16 else out


def controlnet_residual_add(h, residuals, out_bf16=True):
    """Where ControlNet outputs enter the backbone (Section 2, "ControlNet": the outputs are
    incorporated into the skip connections and the middle block, and those of several
    ControlNets are first summed): out = h + (r_1 + r_2 + ... + r_n), the sum formed first,
    left to right, every addition rounded to float32, then bfloat16 (nearest even) if asked.
    With no residual the result is h."""
    hf = np.asarray(h, dtype=np.float32)
    if len(residuals) == 0:
        out = hf.copy()
    else:
        s = np.asarray(residuals[0], dtype=np.float32)
        for r in residuals[1:]:
            s = (s + np.asarray(r, dtype=np.float32)).astype(np.float32)
        out = (hf + s).astype(np.float32)
    return bf16_rne(out) if out_bf16 else out


def bal_timeline(load_done, step_time, n_steps, k, patch_time=0.0):
    """Bounded asynchronous LoRA loading as a timeline (Section 4.2): the adapters finish
    loading `load_done` seconds after the request arrives (the latest of them, since they
    load in parallel); the base model starts at once, unpatched, one step taking `step_time`.
    At the boundary before each step (steps count from 1) the loop patches if the adapters
    are in; at the boundary before step k it waits for them.  Returns (patched_before_step,
    stall_seconds, total_seconds).  Steps run before the patch are the unpatched ones."""
    t = 0.0
    stall = 0.0
    patched_before = None
    for step in range(1, n_steps + 1):
        if patched_before is None:
            if load_done > t and step >= k:          # the bound: hold the base model
                stall += load_done - t
                t = load_done
            if load_done <= t:
                patched_before = step
                t += patch_time
        t += step_time
    return patched_before, stall, t


def lora_unpatch(W_patched, undo):
    """Taking the adapter off restores the saved bits (Section 4.2, patch-off)."""
    del W_patched
    return np.array(undo, dtype=np.float32, copy=True)


def lora_unpatch_by_subtraction(W_patched, A, B, scale):
    """The arithmetic inverse fl32(W' - delta).  NOT what unpatch means: it loses the
    low bits of W wherever |delta| > |W|.  Kept so a test can show that it differs."""
    delta = (np.asarray(B, np.float32) @ np.asarray(A, np.float32)).astype(np.float32)
    delta = (np.float32(scale) * delta).astype(np.float32)
    return (np.asarray(W_patched, np.float32) - delta).astype(np.float32)
