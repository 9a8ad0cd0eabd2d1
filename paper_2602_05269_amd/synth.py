"""Seeded synthetic inputs for the HGF linear layer.

This module only draws random tensors of the shapes and distributions of the
benchmark configurations.  It holds none of the method's arithmetic (no
quantisation, no packing, no matmul): the CPU oracle and the HIP path both take
what it returns as plain inputs.

Recipe.  Every tensor of projection `proj` in layer `layer` of configuration
`cfg` is drawn from its own generator ``numpy.random.default_rng([seed, t])``
with ``seed = 1000*cfg + 10*layer + proj`` and ``t`` the tensor's index in the
order W, x, A, B, alpha, so a tensor's values do not depend on the sizes of
the others.

  W      fp32 [d_out, d_in]   N(0, 0.02)            latent weights, ternarised downstream
  x      fp16 [M, d_in]       per configuration: N(0,1); N(0,1) with 1% of the
                              channels scaled x20; Student-t nu=4; Student-t nu=3
                              (both clipped to the finite fp16 range)
  A      fp16 [r, d_in]       N(0, 0.02)  (0.01 for configuration 3)
  B      fp16 [d_out, r]      N(0, 0.02)  (0.01 for configuration 3)
  alpha  fp16 [d_out]         N(0, 1)     gate parameter, g = tanh(alpha)
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

_W, _X, _A, _B, _ALPHA = range(5)
FP16_MAX = 65504.0


@dataclass(frozen=True)
class Proj:
    name: str
    d_in: int
    d_out: int


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    n_layers: int
    projections: Tuple[Proj, ...]
    rank: int
    tokens: Tuple[int, ...]          # the M values the configuration is run at
    act: str                         # "normal" | "outlier" | "student_t4" | "student_t3"
    lora_std: float


def _block(d: int, ffn: int, names=("q", "k", "v", "o", "up", "gate", "down")) -> Tuple[Proj, ...]:
    shapes = {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d),
              "up": (d, ffn), "gate": (d, ffn), "down": (ffn, d)}
    return tuple(Proj(n, *shapes[n]) for n in names)


CONFIGS: Dict[int, Config] = {
    0: Config(0, "single-256", 1, (Proj("lin", 256, 256),), 16, (8,), "normal", 0.02),
    1: Config(1, "tinystories-stack-decode", 8, _block(512, 2048), 32, (1,), "normal", 0.02),
    2: Config(2, "1.2B-shape-layer", 1, _block(2048, 8192), 64, (1, 4, 16), "outlier", 0.02),
    3: Config(3, "3B-shape-prefill", 1, _block(3072, 8192), 64, (2048,), "student_t4", 0.01),
    4: Config(4, "7B-shape-batch-sweep", 1, _block(4096, 11008, ("up", "gate", "down")), 128,
              (1, 8, 32, 64), "student_t3", 0.02),
}


def seed_of(cfg: int, layer: int, proj: int) -> int:
    return 1000 * cfg + 10 * layer + proj


def _rng(cfg: int, layer: int, proj: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([seed_of(cfg, layer, proj), tensor])


def draw_activations(kind: str, rng: np.random.Generator, M: int, K: int) -> np.ndarray:
    """fp16 [M, K] activations of the named distribution."""
    if kind == "normal":
        x = rng.standard_normal((M, K))
    elif kind == "outlier":
        n_out = int(np.ceil(0.01 * K))
        chans = rng.choice(K, size=n_out, replace=False)   # fixed per layer: drawn first
        x = rng.standard_normal((M, K))
        x[:, chans] *= 20.0
    elif kind == "student_t4":
        x = rng.standard_t(4.0, size=(M, K))
    elif kind == "student_t3":
        x = rng.standard_t(3.0, size=(M, K))
    else:
        raise ValueError(kind)
    return np.clip(x, -FP16_MAX, FP16_MAX).astype(np.float16)


def make_weights(cfg: int, layer: int, proj: int) -> Dict[str, np.ndarray]:
    """Latent fp32 W and the fp16 correction-path tensors of one projection."""
    c = CONFIGS[cfg]
    p = c.projections[proj]
    W = (0.02 * _rng(cfg, layer, proj, _W).standard_normal((p.d_out, p.d_in), dtype=np.float32))
    A = (c.lora_std * _rng(cfg, layer, proj, _A).standard_normal((c.rank, p.d_in))).astype(np.float16)
    B = (c.lora_std * _rng(cfg, layer, proj, _B).standard_normal((p.d_out, c.rank))).astype(np.float16)
    alpha = _rng(cfg, layer, proj, _ALPHA).standard_normal(p.d_out).astype(np.float16)
    return {"W": W, "A": A, "B": B, "alpha": alpha, "d_in": p.d_in, "d_out": p.d_out,
            "rank": c.rank, "name": p.name}


def make_activations(cfg: int, layer: int, proj: int, M: int) -> np.ndarray:
    c = CONFIGS[cfg]
    p = c.projections[proj]
    return draw_activations(c.act, _rng(cfg, layer, proj, _X), M, p.d_in)


def make_custom(seed: int, M: int, d_in: int, d_out: int, rank: int, act: str = "normal",
                lora_std: float = 0.02, w_std: float = 0.02) -> Dict[str, np.ndarray]:
    """An off-configuration case (ragged shapes, edge cases) with the same recipe."""
    g = lambda t: np.random.default_rng([seed, t])
    W = (w_std * g(_W).standard_normal((d_out, d_in), dtype=np.float32))
    x = draw_activations(act, g(_X), M, d_in)
    A = (lora_std * g(_A).standard_normal((rank, d_in))).astype(np.float16)
    B = (lora_std * g(_B).standard_normal((d_out, rank))).astype(np.float16)
    alpha = g(_ALPHA).standard_normal(d_out).astype(np.float16)
    return {"W": W, "x": x, "A": A, "B": B, "alpha": alpha, "d_in": d_in, "d_out": d_out,
            "rank": rank}


def stack_wiring(cfg: int, chained: bool = True, n_layers: int | None = None):
    """(layer, proj, src_slot, dst_slot) for a configuration run as a list of linears, and
    the dict {slot: layer} of the slots that hold fresh inputs.

    Per block: q, k, v read the block input; o reads v's output; up and gate read o's
    output; down reads up's output.  Every linear writes a slot of its own, so each
    layer's input and output stay available for checking.  A configuration without
    q/k/v/o (up, gate, down only) has up and gate read the block input.

    chained=True : slot 0 holds the only input and each block reads the previous block's
                   `down` output -- a pure chain of linears (no residuals or norms, which
                   are outside the layer), whose values shrink block by block.
    n_layers overrides the configuration's number of blocks (the benchmark repeats a
    one-block configuration over many distinct weight instances).
    chained=False: every block reads a fresh synthetic input slot of its own, so every
                   linear sees activations of a healthy magnitude (used for parity).
    """
    c = CONFIGS[cfg]
    names = [p.name for p in c.projections]
    wiring = []
    inputs = {0: 0}
    block_in = 0
    nxt = 1
    for layer in range(n_layers if n_layers is not None else c.n_layers):
        if layer > 0 and not chained:
            block_in = nxt
            inputs[block_in] = layer
            nxt += 1
        out = {}
        for pi, n in enumerate(names):
            if n in ("q", "k", "v", "lin"):
                src = block_in
            elif n == "o":
                src = out["v"]
            elif n in ("up", "gate"):
                src = out["o"] if "o" in out else block_in
            elif n == "down":
                src = out["up"]
            else:
                raise ValueError(n)
            out[n] = nxt
            wiring.append((layer, pi, src, nxt))
            nxt += 1
        if chained:
            block_in = out.get("down", out[names[-1]])
    return wiring, inputs
