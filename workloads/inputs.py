"""Seeded synthetic inputs for a stage: parameters, activations, upstream grads, ids.

Recipe: one master seed per config; every tensor is drawn from its own child
stream of numpy.random.SeedSequence(seed) (PCG64), children taken in the fixed
order  parameters in flat-layout order, then for each microbatch x (or ids,
then targets), then dY.  Values are drawn in fp32 on the host.  For bf16
configs the working parameters, activations and upstream grads are rounded to
bf16 (round-to-nearest-even, torch's conversion) and handed to both sides as
those rounded values; the fp32 draw of the parameters is the master copy.  fp16 configs
are treated the same with IEEE half.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from .configs import DTYPE_BF16, DTYPE_F16, StageConfig, segments

W_STD = 0.02     # matrices and embedding
DY_STD = 1e-2    # upstream output gradient
PERTURB_STD = 0.02


def round_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest-even bf16 values, returned widened to fp32."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def round_f16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest-even IEEE half values (overflow to inf), returned widened to fp32."""
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


@dataclass
class StageInputs:
    cfg: StageConfig
    master: np.ndarray                 # fp32[P]  unrounded draw
    params: np.ndarray                 # fp32[P]  values the compute uses (bf16-rounded for bf16 configs)
    x: list = field(default_factory=list)        # per microbatch fp32[T,H]   (interior / no embedding)
    ids: list = field(default_factory=list)      # per microbatch int32[mb,S] (has_embed)
    targets: list = field(default_factory=list)  # per microbatch int32[mb,S] (has_head)
    dy: list = field(default_factory=list)       # per microbatch fp32[T,H]   (no head)


def make_inputs(cfg: StageConfig, perturbed: bool = False, num_microbatches: int | None = None,
                dy_scale: float = 1.0) -> StageInputs:
    """Draw every input of one optimizer step of the stage.

    perturbed=True draws biases N(0, 0.02) and gains 1 + N(0, 0.02) instead of the
    benchmark's exact 0 / 1, so that a forgotten bias or gain cannot hide.
    """
    ss = np.random.SeedSequence(cfg.seed)

    def child():
        return np.random.Generator(np.random.PCG64(ss.spawn(1)[0]))

    M = cfg.num_microbatches if num_microbatches is None else num_microbatches
    T, H = cfg.tokens, cfg.hidden
    master = np.empty(cfg.n_params, dtype=np.float32)
    for name, off, rows, cols, kind in segments(cfg):
        g = child()
        n = rows * cols
        if kind == "matrix":
            master[off:off + n] = g.standard_normal(n, dtype=np.float32) * np.float32(W_STD)
        else:
            base = np.float32(1.0 if kind == "gain" else 0.0)
            if perturbed:
                master[off:off + n] = base + g.standard_normal(n, dtype=np.float32) * np.float32(PERTURB_STD)
            else:
                master[off:off + n] = base
    # dy_scale: the loss scale an fp16 run multiplies the upstream gradient by (applied before rounding)
    rnd = round_bf16 if cfg.dtype == DTYPE_BF16 else round_f16 if cfg.dtype == DTYPE_F16 else None
    bf = rnd is not None
    inp = StageInputs(cfg, master, rnd(master) if bf else master.copy())
    for _ in range(M):
        if cfg.has_embed:
            inp.ids.append(child().integers(0, cfg.vocab, size=(cfg.microbatch, cfg.seq), dtype=np.int32))
        else:
            x = child().standard_normal((T, H), dtype=np.float32)
            inp.x.append(rnd(x) if bf else x)
        if cfg.has_head:
            inp.targets.append(child().integers(0, cfg.vocab, size=(cfg.microbatch, cfg.seq), dtype=np.int32))
    if not cfg.has_head:
        for _ in range(M):
            dy = child().standard_normal((T, H), dtype=np.float32) * np.float32(DY_STD) * np.float32(dy_scale)
            inp.dy.append(rnd(dy) if bf else dy)
    return inp
