"""Seeded synthetic inputs for the DTS-Gate MoE layer.

This module only draws random arrays and rounds them to the storage type; it
holds none of the method's arithmetic (no softmax, no thresholding, no FFN).
Both the CPU oracle's tests and the HIP path's tests/bench consume exactly the
arrays produced here, so the two sides always see identical bits.

The layer shapes stand in for the paper's workloads (Experiments section:
RoBERTa / GPT / Transformer-MT MoE layers): activations after LayerNorm are
modelled as N(0,1), weights as N(0, 0.02^2), and the gate noise is
Gumbel(0,1) (Stage 2, "Gate with Temperature"), drawn once from the seed and
handed to both sides as an input.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

MASTER_SEED = 20211214


def linear_tau_schedule(n: int, hi: float = 2.0, lo: float = 0.3) -> Tuple[float, ...]:
    """n temperatures from hi down to lo, endpoints included, evenly spaced.

    The paper gives only the endpoints of the anneal (2.0 -> 0.3) and its
    duration, not its shape; a linear ramp is this build's reading.
    """
    if n == 1:
        return (float(hi),)
    return tuple(float(hi - j * (hi - lo) / (n - 1)) for j in range(n))


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                 # tokens
    d: int                 # model width D
    E: int                 # experts N
    F: int                 # expert hidden width
    act: str               # "gelu" | "relu"
    dtype: str             # "f32" | "bf16" (storage type of x, W1, W2, activations)
    taus: Tuple[float, ...]
    threshold: float
    seed: int
    backward: bool = True
    gate_bias_e0: float = 0.0   # bias added to expert 0's logit (load skew)
    bias_std: float = 0.0       # std of b1/b2 (0 = the configs' "biases zero")
    note: str = ""


CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", T=256, d=64, E=4, F=256, act="gelu", dtype="f32",
                        taus=(2.0, 1.0, 0.3), threshold=0.1, seed=MASTER_SEED + 1,
                        backward=False, note="config 1: tiny fp32 forward"),
    "gpt": LayerConfig("gpt", T=8192, d=768, E=16, F=3072, act="gelu", dtype="bf16",
                       taus=linear_tau_schedule(6), threshold=0.05, seed=MASTER_SEED + 2,
                       note="config 2: GPT-style layer, headline metric"),
    "roberta": LayerConfig("roberta", T=16384, d=768, E=32, F=3072, act="gelu", dtype="bf16",
                           taus=(1.0, 0.5, 0.3), threshold=0.03, seed=MASTER_SEED + 3,
                           gate_bias_e0=1.38,
                           note="config 3: RoBERTa-base-shaped, expert 0 ~3x mean load"),
    "mt": LayerConfig("mt", T=8192, d=512, E=64, F=2048, act="relu", dtype="bf16",
                      taus=(0.3,), threshold=0.02, seed=MASTER_SEED + 4,
                      note="config 4: Transformer-MT-shaped, small ragged expert batches"),
    "large": LayerConfig("large", T=32768, d=1024, E=64, F=4096, act="gelu", dtype="bf16",
                         taus=linear_tau_schedule(8), threshold=0.02, seed=MASTER_SEED + 5,
                         note="config 5: large layer, full dense-to-sparse sweep"),
}


def small_variant(cfg: LayerConfig, T: int, d: Optional[int] = None, E: Optional[int] = None,
                  F: Optional[int] = None, **kw) -> LayerConfig:
    """A reduced copy of a config (same distributions), for oracle-sized parity cases."""
    return replace(cfg, name=f"{cfg.name}-small", T=T, d=d or cfg.d, E=E or cfg.E, F=F or cfg.F, **kw)


# ---------------------------------------------------------------------------
# bf16 storage helpers (round-to-nearest-even), pure bit manipulation
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (RNE); returns the uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, np.uint32(0x7FC0), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Value of `a` after rounding to the storage type, returned as float32."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    if dtype == "f32":
        return np.ascontiguousarray(a)
    raise ValueError(f"unknown dtype {dtype!r}")


# ---------------------------------------------------------------------------
# the generator
# ---------------------------------------------------------------------------

@dataclass
class LayerInputs:
    """All arrays one forward+backward pass consumes, as float32 values that are
    exactly representable in the config's storage type."""
    cfg: LayerConfig
    x: np.ndarray        # [T, d]
    Wg: np.ndarray       # [d, E] fp32 always
    bg: Optional[np.ndarray]  # [E] fp32 or None
    noise: np.ndarray    # [T, E] fp32 Gumbel(0,1)
    W1: np.ndarray       # [E, F, d]
    b1: np.ndarray       # [E, F] fp32
    W2: np.ndarray       # [E, d, F]
    b2: np.ndarray       # [E, d] fp32
    dy: np.ndarray       # [T, d] upstream gradient
    extras: dict = field(default_factory=dict)


def make_layer_inputs(cfg: LayerConfig, seed: Optional[int] = None) -> LayerInputs:
    """Draw every array of one layer from one PCG64 stream, in the fixed order
    x, Wg, noise-uniforms, W1, W2, b1, b2, dy."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    T, d, E, F = cfg.T, cfg.d, cfg.E, cfg.F
    x = rng.standard_normal((T, d), dtype=np.float32)
    Wg = (0.02 * rng.standard_normal((d, E))).astype(np.float32)
    # Gumbel(0,1) = -ln(-ln U), U uniform on the open interval (0,1)
    u = rng.random((T, E))
    tiny = np.finfo(np.float64).tiny
    u = np.clip(u, tiny, 1.0 - 2.0 ** -53)
    noise = (-np.log(-np.log(u))).astype(np.float32)
    W1 = (0.02 * rng.standard_normal((E, F, d), dtype=np.float32)).astype(np.float32)
    W2 = (0.02 * rng.standard_normal((E, d, F), dtype=np.float32)).astype(np.float32)
    if cfg.bias_std > 0.0:
        b1 = (cfg.bias_std * rng.standard_normal((E, F))).astype(np.float32)
        b2 = (cfg.bias_std * rng.standard_normal((E, d))).astype(np.float32)
    else:
        b1 = np.zeros((E, F), np.float32)
        b2 = np.zeros((E, d), np.float32)
    dy = rng.standard_normal((T, d), dtype=np.float32)
    bg = None
    if cfg.gate_bias_e0 != 0.0:
        bg = np.zeros((E,), np.float32)
        bg[0] = np.float32(cfg.gate_bias_e0)
    return LayerInputs(
        cfg=cfg,
        x=round_to_storage(x, cfg.dtype), Wg=Wg, bg=bg, noise=noise,
        W1=round_to_storage(W1, cfg.dtype), b1=b1,
        W2=round_to_storage(W2, cfg.dtype), b2=b2,
        dy=round_to_storage(dy, cfg.dtype),
    )
