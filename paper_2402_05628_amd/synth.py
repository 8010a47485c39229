"""Seeded synthetic workloads: block shapes and random draws only.

This module serves both the HIP path and the CPU oracle with the *same arrays*;
it holds none of the method's arithmetic (no quantizer, no normalisation, no
folding).  Everything is drawn with numpy's counter-based Philox generator, so
a (config, seed) pair names one workload on every machine.

The five workloads stand in for the paper's models (Experimental Setup,
"Models and datasets"): their datasets and checkpoints are not used; only the
shapes and the value distributions the paper describes are (inter-channel
range variation of LayerNorm inputs, "Inter-channel variations in LayerNorm
activations"; power-law post-Softmax values, "Power-law characteristics in
Softmax activations").
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

NORM_LAYERNORM = 0
NORM_RMSNORM = 1
ACT_GELU = 0
ACT_SILU_GATED = 1
MASK_NONE = 0
MASK_CAUSAL = 1


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    name: str
    batch: int          # independent attention groups per head (images, or images x windows)
    seq: int            # tokens per attention group
    D: int              # hidden size
    H: int              # heads
    Dm: int             # MLP width
    bits_w: int
    bits_a: int
    bits_p: int         # softmax (log) bits
    norm: int = NORM_LAYERNORM
    act: int = ACT_GELU
    mask: int = MASK_NONE
    rel_bias: bool = False      # relative-position bias added before softmax
    dual_clip: bool = False     # per-channel clip factors drawn in [0.8, 1.0]
    linear_bias: bool = True
    outlier_mode: str = "lognormal"   # "lognormal" (per-channel input scale) or "gamma" (1% channels)
    eps: float = 1e-6

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def d_head(self) -> int:
        return self.D // self.H

    def with_batch(self, batch: int) -> "BlockConfig":
        return dataclasses.replace(self, batch=batch)


CONFIGS = [
    BlockConfig("vit_s_tiny_w8a8", batch=1, seq=197, D=384, H=6, Dm=1536,
                bits_w=8, bits_a=8, bits_p=8),
    BlockConfig("vit_b_w4a4", batch=64, seq=197, D=768, H=12, Dm=3072,
                bits_w=4, bits_a=4, bits_p=4),
    BlockConfig("swin_b_window_w6a6", batch=32 * 64, seq=49, D=128, H=4, Dm=512,
                bits_w=6, bits_a=6, bits_p=6, rel_bias=True),
    BlockConfig("llama7b_prefill_w4a8", batch=1, seq=2048, D=4096, H=32, Dm=11008,
                bits_w=4, bits_a=8, bits_p=8, norm=NORM_RMSNORM, act=ACT_SILU_GATED,
                mask=MASK_CAUSAL, linear_bias=False, outlier_mode="gamma"),
    BlockConfig("clip_vit_l14_w4a4", batch=128, seq=257, D=1024, H=16, Dm=4096,
                bits_w=4, bits_a=4, bits_p=4, dual_clip=True),
]


def rng_for(cfg_id: int, seed: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=0x5EED0000 + 1000 * seed + cfg_id))


def make_block(cfg: BlockConfig, cfg_id: int = 0, seed: int = 0) -> Dict[str, Optional[np.ndarray]]:
    """Raw (unquantized, unfolded) float32 block parameters and one input batch.

    Weights are stored [out, in] with `in` contiguous.  For the gated MLP the
    first Dm rows of w_fc1 are the gate projection and the next Dm rows the up
    projection.
    """
    g = rng_for(cfg_id, seed)
    T, D, Dm = cfg.tokens, cfg.D, cfg.Dm
    f32 = np.float32

    def normal(shape, std=1.0, mean=0.0):
        return (g.standard_normal(shape, dtype=np.float32) * f32(std) + f32(mean)).astype(f32)

    out: Dict[str, Optional[np.ndarray]] = {}
    x = normal((T, D))
    if cfg.outlier_mode == "lognormal":
        c = np.exp(1.5 * g.standard_normal(D)).astype(f32)
        x *= c[None, :]
    out["x"] = x

    def affine():
        if cfg.outlier_mode == "gamma":
            gam = np.ones(D, dtype=f32)
            n_out = max(1, D // 100)
            idx = g.choice(D, size=n_out, replace=False)
            gam[idx] = g.uniform(50.0, 200.0, size=n_out).astype(f32)
            bet = np.zeros(D, dtype=f32)
        else:
            gam = normal((D,), 0.1, 1.0)
            bet = normal((D,), 0.1, 0.0)
        return gam, bet

    out["ln1_gamma"], out["ln1_beta"] = affine()
    out["ln2_gamma"], out["ln2_beta"] = affine()
    n_fc1 = 2 * Dm if cfg.act == ACT_SILU_GATED else Dm
    for name, (n_out, n_in) in {"qkv": (3 * D, D), "proj": (D, D),
                                "fc1": (n_fc1, D), "fc2": (D, Dm)}.items():
        out["w_" + name] = normal((n_out, n_in), 0.02)
        out["b_" + name] = normal((n_out,), 0.02) if cfg.linear_bias else np.zeros(n_out, dtype=f32)
    out["rel_bias"] = normal((cfg.H, cfg.seq, cfg.seq), 0.5) if cfg.rel_bias else None
    for k in ("ln1", "ln2"):
        if cfg.dual_clip:
            out[k + "_clip_up"] = g.uniform(0.8, 1.0, size=D).astype(f32)
            out[k + "_clip_lo"] = g.uniform(0.8, 1.0, size=D).astype(f32)
        else:
            out[k + "_clip_up"] = None
            out[k + "_clip_lo"] = None
    return out


def make_rows(T: int, D: int, seed: int, outliers: bool = True) -> np.ndarray:
    """[T, D] float32 rows with the per-channel log-normal scale of the LN inputs."""
    g = np.random.Generator(np.random.Philox(key=0xA11CE + seed))
    x = g.standard_normal((T, D), dtype=np.float32)
    if outliers:
        x *= np.exp(1.5 * g.standard_normal(D)).astype(np.float32)[None, :]
    return x


def make_rows_asymmetric(T: int, D: int, seed: int) -> np.ndarray:
    """[T, D] float32 stand-in for a post-LayerNorm activation X' with the structure the per-channel dual clipping is
    designed for: a per-channel scale and offset, and in every channel a few outliers at both extremes whose rate
    and reach differ between the two sides and between channels (some channels left-biased, some right-biased)."""
    g = np.random.Generator(np.random.Philox(key=0xD0A1C + seed))
    f32 = np.float32
    x = g.standard_normal((T, D), dtype=f32)
    x *= np.exp(0.7 * g.standard_normal(D)).astype(f32)[None, :]
    x += (0.5 * g.standard_normal(D)).astype(f32)[None, :]
    for side in (1.0, -1.0):
        rate = g.uniform(0.0, 0.01, size=D)                               # share of tokens that are outliers on this side
        reach = np.exp(g.uniform(np.log(2.0), np.log(12.0), size=D))      # how far beyond the bulk they sit
        hit = g.random((T, D)) < rate[None, :]
        mag = (np.abs(g.standard_normal((T, D))) + 1.0) * reach[None, :]
        x = np.where(hit, x + f32(side) * mag.astype(f32), x)
    return x.astype(f32)


def make_codes(shape, bits: int, seed: int) -> np.ndarray:
    """Uniform random b-bit codes (uint8)."""
    g = np.random.Generator(np.random.Philox(key=0xC0DE5 + seed))
    return g.integers(0, 1 << bits, size=shape, dtype=np.uint8)
