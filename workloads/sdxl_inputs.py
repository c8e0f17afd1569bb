"""Seeded synthetic tensors with the shapes of the SDXL spatial-transformer workloads.

The paper serves SDXL at 1024x1024 with the classifier-free-guidance pair run as
one batch of two latents (Section 2, "Diffusion model inference"; Section 3.3) and
LoRA adapters made of two low-rank matrices per patched weight (Section 2,
"Low-Rank Adaptation").  Trained weights, adapters and prompts are not available,
so every tensor here is drawn from a seeded normal distribution with the shape the
real model has at that position.  Nothing in this module computes any part of the
method: it draws numbers, scales them, and rounds them to the storage type.

Conventions
-----------
* Every array is returned as float32.  For the bf16 workloads the values are
  already rounded to bf16 (round-to-nearest-even), so widening them is exact and
  the same host arrays can be fed to a CPU checker and (as bit patterns, see
  ``bf16_bits``) to the GPU.
* Weights are ``[out, in]`` row-major, LoRA down-projection ``A`` is ``[r, in]``,
  up-projection ``B`` is ``[out, r]``, ``scale = alpha / r``.
* "N(0, s)" always means standard deviation ``s``.
* Draw order is fixed: x, ctx, GroupNorm affine, proj_in, then per block
  (ln1, q1, k1, v1, o1, ln2, q2, k2, v2, o2, ln3, ff1, ff2), each projection as
  (W, bias, A, B), then proj_out.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

HEAD_DIM = 64


# --------------------------------------------------------------------------- #
# storage-type helpers (type conversion only)
# --------------------------------------------------------------------------- #
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) >> 16
    return u.astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 value, returned as float32."""
    return bf16_widen(bf16_bits(x)).reshape(np.shape(x))


# --------------------------------------------------------------------------- #
# workload descriptions
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class StackConfig:
    """One spatial-transformer stack: GroupNorm + proj_in, `depth` blocks, proj_out."""

    name: str
    Bn: int          # samples in the batch (2 = the guidance pair)
    T: int           # latent tokens per sample
    C: int           # channels (= heads * 64)
    heads: int
    depth: int
    r: int           # LoRA rank (0 = no adapter)
    alpha: float     # LoRA alpha; scale = alpha / r
    lora_ff: bool    # adapters on the feed-forward projections as well
    Tc: int = 77     # text tokens
    Dc: int = 2048   # text embedding width
    w_std: float = 0.02
    x_std: float = 1.0
    ctx_std: float = 0.02
    a_std: Optional[float] = None   # default 1 / r
    b_std: float = 0.01

    @property
    def M(self) -> int:
        return self.Bn * self.T

    @property
    def F(self) -> int:
        return 4 * self.C

    @property
    def scale(self) -> float:
        return float(self.alpha) / self.r if self.r else 0.0


TINY = StackConfig("tiny_16x16_c320", Bn=2, T=256, C=320, heads=5, depth=1,
                   r=8, alpha=8.0, lora_ff=False)
SDXL64 = StackConfig("sdxl_64x64_c640_depth2", Bn=2, T=4096, C=640, heads=10, depth=2,
                     r=64, alpha=64.0, lora_ff=True)
SDXL32 = StackConfig("sdxl_32x32_c1280_depth10", Bn=2, T=1024, C=1280, heads=20, depth=10,
                     r=64, alpha=64.0, lora_ff=True)

STACK_CONFIGS: Dict[str, StackConfig] = {c.name: c for c in (TINY, SDXL64, SDXL32)}

# (count, out, in) groups of the fp32 patch sweep
PATCH_SWEEP: Tuple[Tuple[int, int, int], ...] = (
    (140, 1280, 1280),
    (60, 640, 640),
    (70, 1280, 2048),
    (20, 10240, 1280),
    (20, 1280, 5120),
)
PATCH_RANK = 32
PATCH_ALPHA = 32.0


@dataclass(frozen=True)
class MultiLoraConfig:
    name: str = "multi_lora_8req_64x64_c640"
    requests: int = 8
    T: int = 4096
    C: int = 640
    ranks: Tuple[int, ...] = (16, 32, 64, 64)
    # classifier-free-guidance batch order: all unconditional rows, then all conditional
    request_adapter: Tuple[int, ...] = (0, 1, 2, 3, 0, 1, 2, 3)
    std: float = 0.02
    x_std: float = 0.02


MULTI_LORA = MultiLoraConfig()


def with_overrides(cfg: StackConfig, **kw) -> StackConfig:
    return replace(cfg, **kw)


# --------------------------------------------------------------------------- #
# generators
# --------------------------------------------------------------------------- #
def _normal(rng: np.random.Generator, shape, std: float, mean: float = 0.0, bf16: bool = True) -> np.ndarray:
    v = rng.standard_normal(shape, dtype=np.float32)
    v *= np.float32(std)
    if mean:
        v += np.float32(mean)
    return bf16_round(v) if bf16 else v


def make_projection(rng, out_f: int, in_f: int, *, bias: bool, r: int, scale: float,
                    w_std: float, a_std: float, b_std: float, bf16: bool = True) -> dict:
    """One linear layer with an optional rank-r adapter."""
    p = {"W": _normal(rng, (out_f, in_f), w_std, bf16=bf16),
         "b": _normal(rng, (out_f,), w_std, bf16=bf16) if bias else None,
         "A": None, "B": None, "scale": 0.0}
    if r:
        p["A"] = _normal(rng, (r, in_f), a_std, bf16=bf16)
        p["B"] = _normal(rng, (out_f, r), b_std, bf16=bf16)
        p["scale"] = float(scale)
    return p


def _affine(rng, n: int, std: float):
    return _normal(rng, (n,), std, mean=1.0), _normal(rng, (n,), std)


def make_block(rng: np.random.Generator, cfg: StackConfig) -> dict:
    C, F, Dc = cfg.C, cfg.F, cfg.Dc
    a_std = cfg.a_std if cfg.a_std is not None else (1.0 / cfg.r if cfg.r else 0.0)
    kw = dict(w_std=cfg.w_std, a_std=a_std, b_std=cfg.b_std, scale=cfg.scale)
    r_attn = cfg.r
    r_ff = cfg.r if cfg.lora_ff else 0
    blk = {}
    blk["ln1_g"], blk["ln1_b"] = _affine(rng, C, cfg.w_std)
    blk["q1"] = make_projection(rng, C, C, bias=False, r=r_attn, **kw)
    blk["k1"] = make_projection(rng, C, C, bias=False, r=r_attn, **kw)
    blk["v1"] = make_projection(rng, C, C, bias=False, r=r_attn, **kw)
    blk["o1"] = make_projection(rng, C, C, bias=True, r=r_attn, **kw)
    blk["ln2_g"], blk["ln2_b"] = _affine(rng, C, cfg.w_std)
    blk["q2"] = make_projection(rng, C, C, bias=False, r=r_attn, **kw)
    blk["k2"] = make_projection(rng, C, Dc, bias=False, r=r_attn, **kw)
    blk["v2"] = make_projection(rng, C, Dc, bias=False, r=r_attn, **kw)
    blk["o2"] = make_projection(rng, C, C, bias=True, r=r_attn, **kw)
    blk["ln3_g"], blk["ln3_b"] = _affine(rng, C, cfg.w_std)
    blk["ff1"] = make_projection(rng, 2 * F, C, bias=True, r=r_ff, **kw)
    blk["ff2"] = make_projection(rng, C, F, bias=True, r=r_ff, **kw)
    return blk


def make_stack_inputs(cfg: StackConfig, seed: int = 0) -> dict:
    """All tensors of one stack call: latent x, text context, and every parameter."""
    rng = np.random.default_rng(seed)
    out = {"cfg": cfg}
    out["x"] = _normal(rng, (cfg.Bn, cfg.T, cfg.C), cfg.x_std)
    out["ctx"] = _normal(rng, (cfg.Bn, cfg.Tc, cfg.Dc), cfg.ctx_std)
    out["gn_g"], out["gn_b"] = _affine(rng, cfg.C, cfg.w_std)
    nolora = dict(r=0, scale=0.0, w_std=cfg.w_std, a_std=0.0, b_std=0.0)
    out["proj_in"] = make_projection(rng, cfg.C, cfg.C, bias=True, **nolora)
    out["blocks"] = [make_block(rng, cfg) for _ in range(cfg.depth)]
    out["proj_out"] = make_projection(rng, cfg.C, cfg.C, bias=True, **nolora)
    return out


def make_patch_inputs(groups: Sequence[Tuple[int, int, int]] = PATCH_SWEEP, r: int = PATCH_RANK,
                      alpha: float = PATCH_ALPHA, seed: int = 0, std: float = 0.02) -> List[dict]:
    """fp32 weight matrices with one adapter each: W [out,in], A [r,in], B [out,r]."""
    rng = np.random.default_rng(seed)
    mats = []
    for count, out_f, in_f in groups:
        for _ in range(count):
            mats.append({
                "W": _normal(rng, (out_f, in_f), std, bf16=False),
                "A": _normal(rng, (r, in_f), std, bf16=False),
                "B": _normal(rng, (out_f, r), std, bf16=False),
                "scale": float(alpha) / r,
            })
    return mats


def make_multi_lora_inputs(cfg: MultiLoraConfig = MULTI_LORA, seed: int = 0, n_proj: int = 4,
                           bias: bool = False) -> dict:
    """Rows of several requests stacked in one matrix, one adapter per prompt.

    Returns x [requests*T, C], `n_proj` projections (W [C,C], optional bias, and one
    (A_i [r_i,C], B_i [C,r_i], scale_i) per adapter), and the segment table:
    rows [seg_offsets[i], seg_offsets[i+1]) use adapter seg_adapter[i] (-1 = none).
    """
    rng = np.random.default_rng(seed)
    M = cfg.requests * cfg.T
    out = {"cfg": cfg}
    out["x"] = _normal(rng, (M, cfg.C), cfg.x_std)
    projs = []
    for _ in range(n_proj):
        p = {"W": _normal(rng, (cfg.C, cfg.C), cfg.std),
             "b": _normal(rng, (cfg.C,), cfg.std) if bias else None,
             "A": [], "B": [], "scales": []}
        for r in cfg.ranks:
            p["A"].append(_normal(rng, (r, cfg.C), cfg.std))
            p["B"].append(_normal(rng, (cfg.C, r), cfg.std))
            p["scales"].append(1.0)
        projs.append(p)
    out["projs"] = projs
    out["seg_offsets"] = np.arange(cfg.requests + 1, dtype=np.int32) * cfg.T
    out["seg_adapter"] = np.asarray(cfg.request_adapter, dtype=np.int32)
    return out
