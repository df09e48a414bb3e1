"""Seeded synthetic workloads for the verification path.

These stand in for LlamaGen-XL / Anole logits, their VQ codebooks and EAGLE-2
draft trees (experimental setup, Section 5.1 and Appendix B.2 of the paper),
none of which can be loaded here.  Shapes and value distributions follow the
five benchmark configurations; the recipe is:

  codebook   Gaussian entries, optionally L2-normalised per row
  target     logit_scale * N(0,1), rounded to the logit dtype
  draft      (unrounded target) + draft_noise * N(0,1), rounded to the dtype
  token      one draw from softmax(draft) per row, taken as the arg-max of
             draft + Gumbel noise (no softmax is evaluated here)
  uniforms   Philox4x32-10, two per row

Nothing in this module evaluates the method: it only draws inputs, which are
then passed unchanged to the CPU oracle and to the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

from . import philox

BASE_SEED = 241003355


@dataclass(frozen=True)
class Config:
    name: str
    V: int                 # codebook size (vocabulary of image tokens)
    d: int                 # latent width of a code
    cb_dtype: str          # "f32" | "bf16"
    normalise: bool        # L2-normalise codebook rows
    k: int                 # neighbourhood size, self included
    delta: float           # TVD bound
    rows: int              # verifications per step
    steps: int             # steps in the full job
    logit_dtype: str       # "f32" | "bf16"
    logit_scale: float
    draft_noise: float
    index: int = 0


CONFIGS = {
    "tiny": Config("tiny", 1024, 8, "f32", True, 16, 0.1, 64, 1, "f32", 3.0, 1.0, 0),
    "llamagen_step": Config("llamagen_step", 16384, 8, "f32", True, 1000, 0.4, 60, 1, "bf16", 1.2, 0.5, 1),
    "image_batch": Config("image_batch", 16384, 8, "f32", True, 300, 0.2, 960, 256, "bf16", 1.2, 0.5, 2),
    "wide_latent": Config("wide_latent", 8192, 256, "bf16", False, 100, 0.3, 3840, 1, "f32", 1.5, 0.5, 3),
    "stress": Config("stress", 16384, 8, "f32", True, 1000, 0.4, 3840, 576, "bf16", 1.2, 0.5, 4),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_codebook(cfg: Config, seed_offset: int = 0, device: str = "cpu") -> torch.Tensor:
    """[V, d] tensor of the configuration's codebook dtype."""
    g = _gen(BASE_SEED + 1000 * cfg.index + 7 + seed_offset, device)
    cb = torch.randn(cfg.V, cfg.d, generator=g, dtype=torch.float32, device=device)
    if cfg.normalise:
        cb = cb / cb.norm(dim=1, keepdim=True)
    return cb.to(torch_dtype(cfg.cb_dtype)).contiguous()


@dataclass
class Step:
    target_logits: torch.Tensor   # [rows, V] logit dtype
    draft_logits: torch.Tensor    # [rows, V]
    draft_tokens: torch.Tensor    # [rows] int32
    uniforms: torch.Tensor        # [rows, 2] float32


def make_step(cfg: Config, step: int = 0, rows: int | None = None, device: str = "cpu",
              variant: str = "plain") -> Step:
    """One step of synthetic verification input.

    variant "plain"  : the configuration as stated.
    variant "peaked" : target and draft logits multiplied by 5, so a handful
                       of tokens carry most of the mass and the TVD bound cuts
                       the neighbourhood short.
    variant "reject" : acceptance uniforms replaced by 1 - 2**-24, so every row
                       whose acceptance probability is below one is rejected
                       (use together with delta = 0 for a reject-heavy mix).
    """
    n = cfg.rows if rows is None else rows
    g = _gen(BASE_SEED + 1000 * cfg.index + 100003 * step + 11, device)
    scale = cfg.logit_scale * (5.0 if variant == "peaked" else 1.0)
    noise = cfg.draft_noise * (5.0 if variant == "peaked" else 1.0)
    dt = torch_dtype(cfg.logit_dtype)
    t32 = torch.randn(n, cfg.V, generator=g, dtype=torch.float32, device=device) * scale
    g32 = t32 + torch.randn(n, cfg.V, generator=g, dtype=torch.float32, device=device) * noise
    target = t32.to(dt)
    draft = g32.to(dt)
    del t32, g32
    # token ~ softmax(draft): Gumbel-max over the rounded draft logits
    u = torch.rand(n, cfg.V, generator=g, dtype=torch.float32, device=device)
    gumbel = -torch.log(-torch.log(u.clamp_(1e-30, 1.0 - 2.0 ** -24)))
    tokens = (draft.float() + gumbel).argmax(dim=1).to(torch.int32)
    del u, gumbel
    un = philox.uniforms(BASE_SEED + cfg.index, n, stream=0, step=step)
    if variant == "reject":
        un[:, 0] = np.float32(1.0 - 2.0 ** -24)
    uniforms = torch.from_numpy(un).to(device)
    return Step(target.contiguous(), draft.contiguous(), tokens.contiguous(), uniforms.contiguous())


def with_overrides(cfg: Config, **kw) -> Config:
    return replace(cfg, **kw)
