"""Seeded synthetic inputs shaped like the linear layers of image and video DiTs.

The paper evaluates on PixArt-alpha (image) and OpenSORA / STDiT (video) with
their trained weights and prompt sets; none of that is available here, so these
generators stand in for it: only the layer shapes, token counts and the value
structure (Gaussian bulk, a few outlier channels, per-channel spread, GELU-shaped
fc2 inputs, a per-channel balancing mask) are reproduced.

This module holds no arithmetic of the quantized layer itself: it only draws
inputs (numpy, host side).  Both the CPU oracle's tests and the GPU path's tests
and benchmark take their inputs from here.

Stream for a tensor: numpy PCG64 seeded with SeedSequence([SEED, cfg, block, layer, tensor]).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

SEED = 240602540
T_X, T_W, T_BIAS, T_S, T_CHAN, T_PLAN = 0, 1, 2, 3, 4, 99

HIDDEN = 1152
MLP = 4 * HIDDEN
TEXT_DIM = 4096
TEXT_TOKENS = 240          # 2 x 120 caption tokens (CFG pair)
IMAGE_TOKENS = 2 * 4096    # CFG pair of 64 x 64 latent patches
VIDEO_TOKENS = 2 * 16 * 1024  # CFG pair, 16 frames of 32 x 32 patches


def rng(cfg: int, block: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED, cfg, block, layer, tensor])))


@dataclass
class LayerSpec:
    name: str
    M: int
    K: int
    N: int
    w_bits: int = 8
    cfg: int = 0
    block: int = 0
    layer: int = 0
    x_kind: str = "normal"   # normal | outlier30 | gelu | video
    balanced: bool = False   # draw a balancing mask s and chan_mul = 1/s

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K


@dataclass
class LayerData:
    spec: LayerSpec
    x: np.ndarray                 # fp16 [M,K]
    w: np.ndarray                 # fp32 [N,K], before balancing and quantization
    bias: np.ndarray              # fp16 [N]
    s: Optional[np.ndarray] = None         # fp32 [K] balancing mask (weight side), or None
    chan_mul: Optional[np.ndarray] = None  # fp32 [K] = 1/s (activation side), or None
    extra: Dict[str, np.ndarray] = field(default_factory=dict)


def _erf(v: np.ndarray) -> np.ndarray:
    from scipy.special import erf
    return erf(v)


def draw_x(spec: LayerSpec, rows: Optional[int] = None) -> np.ndarray:
    """Activations of one layer as fp16 [M,K] (or only the first `rows` rows' worth of the stream)."""
    M = spec.M if rows is None else rows
    K = spec.K
    g = rng(spec.cfg, spec.block, spec.layer, T_X)
    z = g.standard_normal((M, K), dtype=np.float32)
    gc = rng(spec.cfg, spec.block, spec.layer, T_CHAN)
    if spec.x_kind == "normal":
        pass
    elif spec.x_kind == "outlier30":
        idx = gc.choice(K, 8, replace=False)
        z[:, idx] *= np.float32(30.0)
    elif spec.x_kind == "gelu":
        z = (z * np.float32(0.5) * (np.float32(1.0) + _erf(z / np.float32(np.sqrt(2.0))))).astype(np.float32)
    elif spec.x_kind == "video":
        sigma = np.exp(gc.uniform(np.log(0.1), np.log(10.0), K)).astype(np.float32)
        n_out = int(round(0.01 * K))
        idx = gc.choice(K, n_out, replace=False)
        sigma[idx] *= np.float32(50.0)
        z *= sigma[None, :]
    else:
        raise ValueError(spec.x_kind)
    return z.astype(np.float16)


def draw_layer(spec: LayerSpec) -> LayerData:
    x = draw_x(spec)
    w = rng(spec.cfg, spec.block, spec.layer, T_W).normal(0.0, 0.02, (spec.N, spec.K)).astype(np.float32)
    bias = rng(spec.cfg, spec.block, spec.layer, T_BIAS).normal(0.0, 0.01, spec.N).astype(np.float16)
    s = chan_mul = None
    if spec.balanced:
        s = np.exp(rng(spec.cfg, spec.block, spec.layer, T_S).uniform(np.log(0.25), np.log(4.0), spec.K))
        s = s.astype(np.float32)
        chan_mul = (np.float32(1.0) / s).astype(np.float32)
    return LayerData(spec, x, w, bias, s, chan_mul)


def draw_weights(spec: LayerSpec):
    """(w fp32 [N,K], bias fp16 [N], s or None, chan_mul or None) without the activations."""
    w = rng(spec.cfg, spec.block, spec.layer, T_W).normal(0.0, 0.02, (spec.N, spec.K)).astype(np.float32)
    bias = rng(spec.cfg, spec.block, spec.layer, T_BIAS).normal(0.0, 0.01, spec.N).astype(np.float16)
    s = chan_mul = None
    if spec.balanced:
        s = np.exp(rng(spec.cfg, spec.block, spec.layer, T_S).uniform(np.log(0.25), np.log(4.0), spec.K))
        s = s.astype(np.float32)
        chan_mul = (np.float32(1.0) / s).astype(np.float32)
    return w, bias, s, chan_mul


# ---- the five configurations ---------------------------------------------------

def config1() -> List[LayerSpec]:
    """One W8A8 linear, 256 tokens, hidden 1152, 8 outlier channels x30."""
    return [LayerSpec("linear", 256, HIDDEN, HIDDEN, 8, cfg=1, x_kind="outlier30")]


def config2() -> List[LayerSpec]:
    """W8A8 image-DiT block linears, 8192 tokens, balancing mask s ~ LogUniform(0.25, 4)."""
    M = IMAGE_TOKENS
    return [
        LayerSpec("qkv", M, HIDDEN, 3 * HIDDEN, 8, cfg=2, layer=0, balanced=True),
        LayerSpec("proj", M, HIDDEN, HIDDEN, 8, cfg=2, layer=1, balanced=True),
        LayerSpec("fc1", M, HIDDEN, MLP, 8, cfg=2, layer=2, balanced=True),
        LayerSpec("fc2", M, MLP, HIDDEN, 8, cfg=2, layer=3, x_kind="gelu", balanced=True),
    ]


def config3() -> List[LayerSpec]:
    """Config 1 with 4-bit weights."""
    return [LayerSpec("linear", 256, HIDDEN, HIDDEN, 4, cfg=3, x_kind="outlier30")]


def config4() -> List[LayerSpec]:
    """W8A8 video-DiT linears, 32768 tokens (+ cross-attention kv on 240 text tokens)."""
    M = VIDEO_TOKENS
    return [
        LayerSpec("qkv", M, HIDDEN, 3 * HIDDEN, 8, cfg=4, layer=0, x_kind="video"),
        LayerSpec("proj", M, HIDDEN, HIDDEN, 8, cfg=4, layer=1, x_kind="video"),
        LayerSpec("fc1", M, HIDDEN, MLP, 8, cfg=4, layer=2, x_kind="video"),
        LayerSpec("fc2", M, MLP, HIDDEN, 8, cfg=4, layer=3, x_kind="video"),
        LayerSpec("ca_kv", TEXT_TOKENS, TEXT_DIM, 2 * HIDDEN, 8, cfg=4, layer=4, x_kind="video"),
    ]


CONFIG5_BLOCKS = 28
CONFIG5_STEPS = 20


def config5_plan() -> np.ndarray:
    """Seeded per-layer precision plan of the 28-block video DiT: True = W4A8 (about 30 %)."""
    return rng(5, 0, 0, T_PLAN).random(CONFIG5_BLOCKS * 6) < 0.30


def config5(blocks: int = CONFIG5_BLOCKS) -> List[LayerSpec]:
    """All linears of a video DiT in model order, each with its own weights and precision."""
    M = VIDEO_TOKENS
    plan = config5_plan()
    shapes = [("qkv", M, HIDDEN, 3 * HIDDEN), ("proj", M, HIDDEN, HIDDEN),
              ("ca_q", M, HIDDEN, HIDDEN), ("ca_kv", TEXT_TOKENS, TEXT_DIM, 2 * HIDDEN),
              ("fc1", M, HIDDEN, MLP), ("fc2", M, MLP, HIDDEN)]
    out = []
    for b in range(blocks):
        for li, (name, m, k, n) in enumerate(shapes):
            bits = 4 if plan[b * 6 + li] else 8
            out.append(LayerSpec(name, m, k, n, bits, cfg=5, block=b, layer=li, x_kind="video"))
    return out


def config5_step_scale(t: int) -> float:
    """Activation scale of denoising step t in 1..20."""
    return 0.5 + t / 20.0


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
