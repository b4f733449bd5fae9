"""Seeded synthetic layers shaped like the paper's workloads.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no Hessian, no grid, no rounding to codes, no
scores).  Both the test oracle and the HIP path are fed from here, so neither
has to import the other.

The paper calibrates on real activations of Gemma / PaLM2 layers (Section 4,
"Training": 1280 sequences of 2048 tokens).  Those are not available, so each
configuration below is a synthetic stand-in with the same shapes and the kind
of structure that matters for the method: a few very large input channels,
heavy tails, or widely spread per-channel scales.

All arrays are host numpy arrays.  Layouts:
  X   [n][d_in]      activations, float32 values (already rounded to bf16
                     precision when ``x_dtype == "bf16"``)
  Wt  [d_out][d_in]  the layer weight, transposed so that one output column of
                     the paper's W is one contiguous row
"""
from __future__ import annotations

import dataclasses

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    d_in: int
    d_out: int
    n: int
    bits: int
    group: int          # group size along d_in; == d_in means per-channel
    T: int              # greedy CD iterations
    x_dtype: str        # "f32" or "bf16"
    x_kind: str         # recipe for X, see make_x
    init: str           # "rtn" or "owc"
    seed: int = 0


# The five workloads, in the order they are listed for this build.
CONFIGS = {
    "tiny": LayerConfig("tiny", 128, 64, 512, 4, 128, 128, "f32", "normal", "rtn"),
    "attn_proj": LayerConfig("attn_proj", 2048, 2048, 16384, 3, 2048, 2048, "bf16", "outlier8x20", "rtn"),
    "mlp_up": LayerConfig("mlp_up", 2048, 16384, 16384, 2, 128, 4096, "bf16", "student_t4", "rtn"),
    "mlp_down": LayerConfig("mlp_down", 16384, 2048, 32768, 4, 16384, 16384, "bf16", "outlier0.1pct_x50", "rtn"),
    "large": LayerConfig("large", 8192, 32768, 32768, 3, 8192, 8192, "bf16", "lognormal_scales", "owc"),
}
CONFIG_ORDER = ["tiny", "attn_proj", "mlp_up", "mlp_down", "large"]


def _rng(seed: int, stream: int) -> np.random.Generator:
    # stream 0 = X, 1 = W, 2 = channel choice / channel scales, 3 = random codes, 4 = random partitions
    return np.random.default_rng([seed, stream])


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x_bf16_valued: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x_bf16_valued, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def make_x(kind: str, n: int, d_in: int, seed: int = 0, x_dtype: str = "bf16") -> np.ndarray:
    """Activations X [n][d_in] as float32 (bf16-rounded if x_dtype == 'bf16')."""
    rx = _rng(seed, 0)
    rc = _rng(seed, 2)
    if kind == "normal":
        x = rx.standard_normal((n, d_in), dtype=np.float32)
    elif kind == "outlier8x20":
        x = rx.standard_normal((n, d_in), dtype=np.float32)
        ch = rc.choice(d_in, size=min(8, d_in), replace=False)
        x[:, ch] *= np.float32(20.0)
    elif kind == "outlier0.1pct_x50":
        x = rx.standard_normal((n, d_in), dtype=np.float32)
        k = max(1, int(round(0.001 * d_in)))
        ch = rc.choice(d_in, size=k, replace=False)
        x[:, ch] *= np.float32(50.0)
    elif kind == "student_t4":
        x = rx.standard_t(4.0, size=(n, d_in)).astype(np.float32)
    elif kind == "lognormal_scales":
        x = rx.standard_normal((n, d_in), dtype=np.float32)
        s = np.exp(rc.standard_normal(d_in)).astype(np.float32)
        x *= s[None, :]
    else:
        raise ValueError(f"unknown X recipe {kind!r}")
    if x_dtype == "bf16":
        x = round_to_bf16(x)
    elif x_dtype != "f32":
        raise ValueError(x_dtype)
    return x


def make_wt(d_out: int, d_in: int, seed: int = 0) -> np.ndarray:
    """Weights ~ N(0, 1/d_in), float32, laid out [d_out][d_in]."""
    w = _rng(seed, 1).standard_normal((d_out, d_in), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(d_in))
    return w


def make_random_codes(d_out: int, d_in: int, bits: int, seed: int = 0) -> np.ndarray:
    """Uniform random codes: a free choice of the algorithm's 'initial estimate'
    input that keeps almost every iteration committing a move (stress mode)."""
    return _rng(seed, 3).integers(0, 1 << bits, size=(d_out, d_in), dtype=np.uint8)


def make_partitions(T: int, d_in: int, seed: int = 0) -> np.ndarray:
    """T independent uniform random permutations of 0..d_in-1 (int32 [T][d_in]): the random
    partitions a block coordinate descent draws, one per iteration; consecutive entries of a row
    form a block.  Drawn here so that every implementation is handed the same ones."""
    rng = _rng(seed, 4)
    out = np.empty((T, d_in), np.int32)
    for t in range(T):
        out[t] = rng.permutation(d_in)
    return out


def make_layer(cfg: LayerConfig, d_out: int | None = None, n: int | None = None):
    """Returns (X, Wt) for a configuration; d_out / n can be cut down for
    column-subset or short-calibration test cases (rows of Wt are independent
    problems, so the first d_out rows are the same problems as in the full layer)."""
    x = make_x(cfg.x_kind, n or cfg.n, cfg.d_in, cfg.seed, cfg.x_dtype)
    # the generator fills row-major from one stream, so asking for fewer rows
    # yields exactly the leading rows of the full matrix
    wt = make_wt(d_out or cfg.d_out, cfg.d_in, cfg.seed)
    return x, wt
