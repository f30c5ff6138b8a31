"""Seeded synthetic stand-ins for VGGT-1B linear-layer inputs.

The paper measures on VGGT-1B activations over CO3Dv2 frames; neither the
checkpoint nor the dataset is available here, so these draws take only what
the paper describes of them (Sec. 3.2, Observation 1 and Fig. "motivation"):
1374 tokens per frame of which the first five (camera + register tokens) are
much larger than patch tokens, a few outlier channels, and heavy tails.

Every random stream is keyed by (layer seed, stream id, frame index) so any
frame, or any subset of rows, can be regenerated without drawing the rest.

Values are handed out as exact bit patterns: bf16 tensors are uint16 arrays of
bf16 bits (fp32 rounded to nearest even), fp32 tensors are float32 arrays.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Iterable, List, Sequence

import numpy as np

TOKENS_PER_FRAME = 1374   # 1369 patch tokens + 5 special tokens
SPECIAL_TOKENS = 5        # rows 0..4 of every frame

# stream ids (second word of the seed sequence)
_S_WEIGHT, _S_BIAS, _S_SIGNS, _S_CHAN, _S_ACT, _S_CAL, _S_WROWS = range(7)


@dataclass(frozen=True)
class LayerSpec:
    config: int            # 1..5, index into the benchmark's configs (1-based)
    name: str              # "tiny", "qkv", "proj", "fc1", "fc2"
    M: int                 # tokens
    K: int                 # input features (Hadamard size)
    N: int                 # output features
    rows_per_frame: int    # 1374 except for the tiny config (one "frame" of M rows)
    x_dtype: str           # "bf16" or "f32"
    df: float              # Student-t degrees of freedom of the body; 0 => Gaussian
    chan_frac: float       # fraction of outlier channels (at least chan_min)
    chan_min: int
    chan_mult: float       # outlier channel multiplier
    special_mult: float    # multiplier of the first five rows of each frame
    w_std: float           # weight std (the configs' "N(0, 0.02)" read as std)
    w_row_frac: float      # fraction of output channels scaled up
    w_row_mult: float
    has_bias: bool
    seed: int

    @property
    def frames(self) -> int:
        return (self.M + self.rows_per_frame - 1) // self.rows_per_frame

    @property
    def n_outlier_channels(self) -> int:
        return max(self.chan_min, int(round(self.chan_frac * self.K)))


_SHAPES = {"qkv": (1024, 3072), "proj": (1024, 1024), "fc1": (1024, 4096), "fc2": (4096, 1024)}
_LAYER_ID = {"qkv": 0, "proj": 1, "fc1": 2, "fc2": 3}


def layer_spec(config: int, name: str = "") -> LayerSpec:
    """Recipe of one linear layer of the benchmark's configs[config-1]."""
    if config == 1:
        return LayerSpec(1, "tiny", 64, 128, 128, 64, "f32", 0.0, 0.0, 2, 50.0, 20.0,
                         0.02, 0.0, 1.0, False, 0)
    if config == 2:
        name = name or "qkv"
        if name != "qkv":
            raise ValueError("config 2 is the qkv layer")
        K, N = _SHAPES[name]
        return LayerSpec(2, name, TOKENS_PER_FRAME, K, N, TOKENS_PER_FRAME, "bf16", 3.0, 0.01, 1,
                         50.0, 20.0, 0.02, 0.0, 1.0, True, 2000)
    if config in (3, 4):
        frames = 8 if config == 3 else 24
        allowed = ("fc1", "fc2") if config == 3 else ("qkv", "proj", "fc1", "fc2")
        if name not in allowed:
            raise ValueError(f"config {config} has layers {allowed}")
        K, N = _SHAPES[name]
        return LayerSpec(config, name, frames * TOKENS_PER_FRAME, K, N, TOKENS_PER_FRAME, "bf16", 3.0,
                         0.01, 1, 50.0, 20.0, 0.02, 0.0, 1.0, True, config * 1000 + _LAYER_ID[name])
    if config == 5:
        if name not in ("fc1", "fc2"):
            raise ValueError("config 5 has layers fc1, fc2")
        K, N = _SHAPES[name]
        return LayerSpec(5, name, 100 * TOKENS_PER_FRAME, K, N, TOKENS_PER_FRAME, "bf16", 2.5,
                         0.02, 1, 100.0, 50.0, 0.02, 0.005, 10.0, True, 5000 + _LAYER_ID[name])
    raise ValueError("config must be 1..5")


def config_layers(config: int) -> List[str]:
    return {1: ["tiny"], 2: ["qkv"], 3: ["fc1", "fc2"], 4: ["qkv", "proj", "fc1", "fc2"],
            5: ["fc1", "fc2"]}[config]


# ---------------------------------------------------------------- dtype packing
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(spec: LayerSpec, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([spec.seed, stream, index])))


def _pack(x32: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(x32) if dtype == "bf16" else np.ascontiguousarray(x32, dtype=np.float32)


# ---------------------------------------------------------------- tensors
def outlier_channels(spec: LayerSpec) -> np.ndarray:
    """Sorted indices of the outlier input channels of this layer (fixed per layer)."""
    n = spec.n_outlier_channels
    return np.sort(_rng(spec, _S_CHAN).choice(spec.K, size=n, replace=False))


def make_weights(spec: LayerSpec) -> np.ndarray:
    """W [N, K]: N(0, w_std); a fraction of output channels (rows) scaled by w_row_mult."""
    w = _rng(spec, _S_WEIGHT).standard_normal((spec.N, spec.K), dtype=np.float32) * np.float32(spec.w_std)
    n_rows = int(round(spec.w_row_frac * spec.N))
    if n_rows > 0:
        rows = _rng(spec, _S_WROWS).choice(spec.N, size=n_rows, replace=False)
        w[rows, :] *= np.float32(spec.w_row_mult)
    return _pack(w, "bf16" if spec.x_dtype == "bf16" else "f32")


def make_bias(spec: LayerSpec):
    """bias [N] as bf16 bits, or None for layers without bias."""
    if not spec.has_bias:
        return None
    b = _rng(spec, _S_BIAS).standard_normal(spec.N, dtype=np.float32) * np.float32(spec.w_std)
    return f32_to_bf16_bits(b)


def make_signs(spec: LayerSpec) -> np.ndarray:
    """Random +/-1 vector (int8, length K) of the randomised Hadamard rotation."""
    return (_rng(spec, _S_SIGNS).integers(0, 2, size=spec.K, dtype=np.int8) * 2 - 1).astype(np.int8)


def _frame_f32(spec: LayerSpec, stream: int, frame: int, rows: int) -> np.ndarray:
    g = _rng(spec, stream, frame)
    if spec.df > 0:
        x = g.standard_t(spec.df, size=(rows, spec.K)).astype(np.float32)
    else:
        x = g.standard_normal((rows, spec.K), dtype=np.float32)
    x[:, outlier_channels(spec)] *= np.float32(spec.chan_mult)
    x[:SPECIAL_TOKENS, :] *= np.float32(spec.special_mult)
    return x


def _frame_rows(spec: LayerSpec, frame: int) -> int:
    return min(spec.rows_per_frame, spec.M - frame * spec.rows_per_frame)


def make_activation_frames(spec: LayerSpec, frames: Iterable[int] = None, workers: int = 8) -> np.ndarray:
    """Rows of X for the given frames (default: all), concatenated in the given order."""
    frames = list(range(spec.frames)) if frames is None else list(frames)
    if not frames:
        return _pack(np.zeros((0, spec.K), np.float32), spec.x_dtype)

    def one(f):
        return _pack(_frame_f32(spec, _S_ACT, f, _frame_rows(spec, f)), spec.x_dtype)

    if len(frames) == 1 or workers <= 1:
        parts = [one(f) for f in frames]
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            parts = list(ex.map(one, frames))
    return np.concatenate(parts, axis=0)


def make_activation_rows(spec: LayerSpec, rows: Sequence[int]) -> np.ndarray:
    """Selected global rows of X (regenerates only the frames they fall in)."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((rows.size, spec.K), dtype=np.uint16 if spec.x_dtype == "bf16" else np.float32)
    fr = rows // spec.rows_per_frame
    for f in np.unique(fr):
        sel = np.nonzero(fr == f)[0]
        frame = make_activation_frames(spec, [int(f)])
        out[sel] = frame[rows[sel] - int(f) * spec.rows_per_frame]
    return out


def make_calibration(spec: LayerSpec) -> np.ndarray:
    """Calibration activation from which the smoothing factor's activation statistic is taken.

    Config 1 calibrates on X itself; the others on a separate one-frame draw with the
    same outlier channels (a stand-in for a statically calibrated factor).
    """
    if spec.config == 1:
        return make_activation_frames(spec)
    return _pack(_frame_f32(spec, _S_CAL, 0, spec.rows_per_frame), spec.x_dtype)
