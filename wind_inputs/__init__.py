"""Seeded synthetic inputs for the WIND greedy-decoding hot path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and benchmark.  It
holds no arithmetic of the decoding method: it only draws random tensors of the right shapes,
rounds them to bf16-representable values where a configuration stores bf16, and looks up two
per-configuration scalars (blank-logit bias, prediction-projection gain) from a table that a
committed calibration script wrote by running the oracle.

The paper evaluates on LibriSpeech with trained Parakeet RNN-T checkpoints (Experiments section,
Tables 1, 2 and 5).  Neither audio nor checkpoints are available, so every tensor here is a
synthetic stand-in shaped like those workloads: encoder frames ~ N(0,1), weights ~ N(0,1/fan_in),
BPE-sized vocabularies, and a blank bias tuned so that most joiner evaluations return blank, which
is the property the method exploits (Introduction; Method, remark after Algorithm 2).
"""
from __future__ import annotations

import dataclasses
import json
import os
from typing import Dict, Optional, Tuple

import numpy as np

_CALIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "calibration.json")


@dataclasses.dataclass(frozen=True)
class WindConfig:
    """Shape of one workload.  Symbols follow the usual RNN-T notation."""

    name: str
    seed: int
    B: int            # utterances in the batch
    len_lo: int       # lengths are integer-uniform on [len_lo, len_hi]
    len_hi: int
    D: int            # encoder output dimension
    E: int            # embedding dimension of the prediction network
    L: int            # stacked LSTM layers
    Hp: int           # LSTM hidden size
    Hj: int           # joint hidden size
    V: int            # non-blank labels; blank id = V, start-of-sequence id = V
    dtype: str        # "f32" or "bf16": storage type of the weight matrices and of enc_out
    windows: Tuple[int, ...]
    S: int            # max symbols emitted on one frame
    blank_rate: float  # target fraction of sequential joiner evaluations that return blank

    def replace(self, **kw) -> "WindConfig":
        return dataclasses.replace(self, **kw)


# Index i is benchmark configs[i].
CONFIGS: Dict[str, WindConfig] = {
    c.name: c
    for c in [
        WindConfig("tiny", 0, 1, 64, 64, 64, 64, 1, 64, 64, 32, "f32", (4,), 5, 0.80),
        WindConfig("greedy_b1", 1, 1, 1000, 1000, 1024, 640, 1, 640, 640, 1024, "bf16",
                   (1, 2, 4, 8, 16), 10, 0.85),
        WindConfig("batch32", 2, 32, 200, 1500, 1024, 640, 1, 640, 640, 1024, "bf16", (8,), 10, 0.85),
        WindConfig("largevocab_b128", 3, 128, 500, 2000, 1024, 640, 2, 640, 1024, 8192, "bf16",
                   (4, 8, 16), 10, 0.85),
        WindConfig("lowblank_b256", 4, 256, 100, 1000, 512, 640, 1, 640, 640, 4096, "bf16",
                   (16,), 3, 0.50),
    ]
}
CONFIG_ORDER = ("tiny", "greedy_b1", "batch32", "largevocab_b128", "lowblank_b256")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def load_calibration() -> dict:
    if not os.path.exists(_CALIB_PATH):
        return {}
    with open(_CALIB_PATH) as f:
        return json.load(f)


def make_weights(cfg: WindConfig, blank_bias: Optional[float] = None,
                 pred_gain: Optional[float] = None) -> Dict[str, np.ndarray]:
    """Random-init model.  Draw order: emb, per layer (w_ih, w_hh, b_ih, b_hh), w_enc, b_enc,
    w_pred, b_pred, w_out, b_out.  Every entry ~ N(0, 1/fan_in); the embedding has fan_in 1.

    `pred_gain` multiplies w_pred and b_pred (before bf16 rounding); `blank_bias` is added to
    b_out[V].  When None they come from calibration.json (0 and 1 if the config is absent).
    """
    calib = load_calibration().get(cfg.name, {})
    if blank_bias is None:
        blank_bias = float(calib.get("blank_bias", 0.0))
    if pred_gain is None:
        pred_gain = float(calib.get("pred_gain", 1.0))
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 1]))

    def normal(shape, fan_in):
        return (rng.standard_normal(shape, dtype=np.float32) / np.float32(np.sqrt(fan_in)))

    w: Dict[str, np.ndarray] = {}
    w["emb"] = normal((cfg.V + 1, cfg.E), 1)
    for l in range(cfg.L):
        in_l = cfg.E if l == 0 else cfg.Hp
        w[f"w_ih{l}"] = normal((4 * cfg.Hp, in_l), in_l)
        w[f"w_hh{l}"] = normal((4 * cfg.Hp, cfg.Hp), cfg.Hp)
        w[f"b_ih{l}"] = normal((4 * cfg.Hp,), in_l)
        w[f"b_hh{l}"] = normal((4 * cfg.Hp,), cfg.Hp)
    w["w_enc"] = normal((cfg.Hj, cfg.D), cfg.D)
    w["b_enc"] = normal((cfg.Hj,), cfg.D)
    w["w_pred"] = normal((cfg.Hj, cfg.Hp), cfg.Hp) * np.float32(pred_gain)
    w["b_pred"] = normal((cfg.Hj,), cfg.Hp) * np.float32(pred_gain)
    w["w_out"] = normal((cfg.V + 1, cfg.Hj), cfg.Hj)
    w["b_out"] = normal((cfg.V + 1,), cfg.Hj)
    w["b_out"][cfg.V] += np.float32(blank_bias)
    if cfg.dtype == "bf16":
        # weight matrices are stored in bf16 by the device path; biases stay fp32
        for k in list(w):
            if k.startswith(("emb", "w_")):
                w[k] = round_to_bf16(w[k])
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in w.items()}


def sharpened(weights: Dict[str, np.ndarray], gain: float = 8.0) -> Dict[str, np.ndarray]:
    """The same model with its output layer (w_out, b_out) multiplied by `gain`: every argmax, hence
    every greedy result, is unchanged, but the soft-max becomes peaked like a trained model's (a
    random output layer gives nearly flat probabilities, under which a search over probabilities
    never prefers "blank on every frame of the window").  A power of two keeps bf16 values bf16."""
    w = dict(weights)
    w["w_out"] = np.ascontiguousarray(weights["w_out"] * np.float32(gain))
    w["b_out"] = np.ascontiguousarray(weights["b_out"] * np.float32(gain))
    return w


def make_batch(cfg: WindConfig) -> Tuple[np.ndarray, np.ndarray]:
    """Encoder outputs enc_out[B, T, D] ~ N(0,1) and lengths[B]; T = max(lengths).

    Frames at or beyond an utterance's length hold ordinary random values; tests that want
    poison there overwrite them."""
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 2, cfg.B, cfg.len_lo, cfg.len_hi]))
    lengths = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    T = int(lengths.max()) if cfg.B > 0 else 0
    enc = rng.standard_normal((cfg.B, T, cfg.D), dtype=np.float32)
    if cfg.dtype == "bf16":
        enc = round_to_bf16(enc)
    return enc, lengths


def scaled(cfg: WindConfig, B: int, len_lo: int, len_hi: int) -> WindConfig:
    """Same model (same weight seed), smaller batch: used where the oracle must finish in seconds."""
    return cfg.replace(B=B, len_lo=len_lo, len_hi=len_hi)
