"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: only shapes, seeds, random draws, rounding of
the *inputs* to the storage type, and the choice of sampled rows.

Shapes follow the paper: 384x224 frames through a 16x tokenizer give a 24x14
latent grid, T = 336 tokens per frame (Sec. 5, Implementation Details); the
310M model has 16 heads of width 64 (Appendix, model-size table); evaluation
uses 16 frames and the context window is 32 frames (Sec. 5, Limitations);
speculative chunks of N = 2..4 frames (Tab. 2).  Values are iid N(0,1), a
stand-in for the projected activations of a trained model, which are not
available.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 2506013800

# name -> B, H, D, T, kv_frames, q_frames, F (capacity, frames), dtype
CONFIGS = {
    "c1_tiny_fp32":     dict(B=1, H=2,  D=64, T=16,  kv_frames=4,  q_frames=4,  F=4,  dtype="fp32", seed=BASE_SEED + 1),
    "c2_train":         dict(B=4, H=16, D=64, T=336, kv_frames=16, q_frames=16, F=16, dtype="bf16", seed=BASE_SEED + 2),
    "c3_decode":        dict(B=1, H=16, D=64, T=336, kv_frames=33, q_frames=1,  F=40, dtype="bf16", seed=BASE_SEED + 3),
    "c4_spec_k2":       dict(B=1, H=16, D=64, T=336, kv_frames=34, q_frames=2,  F=40, dtype="bf16", seed=BASE_SEED + 14),
    "c4_spec_k4":       dict(B=1, H=16, D=64, T=336, kv_frames=36, q_frames=4,  F=40, dtype="bf16", seed=BASE_SEED + 4),
    "c4_spec_k8":       dict(B=1, H=16, D=64, T=336, kv_frames=40, q_frames=8,  F=40, dtype="bf16", seed=BASE_SEED + 24),
    "c5a_long_train":   dict(B=2, H=16, D=64, T=576, kv_frames=64, q_frames=64, F=64, dtype="bf16", seed=BASE_SEED + 5),
    "c5b_batch_decode": dict(B=8, H=16, D=64, T=576, kv_frames=64, q_frames=1,  F=64, dtype="bf16", seed=BASE_SEED + 15),
}

# The paper's other model sizes (Appendix, model-size table: 130M has 12 heads, 774M has 24, width 64)
# and its third speculative chunk length (Tab. 2: N = 3).  Parity cases, not bench lines.
EXTRA_CONFIGS = {
    "x_train_h12":  dict(B=2, H=12, D=64, T=336, kv_frames=16, q_frames=16, F=16, dtype="bf16", seed=BASE_SEED + 31),
    "x_train_h24":  dict(B=1, H=24, D=64, T=336, kv_frames=16, q_frames=16, F=16, dtype="bf16", seed=BASE_SEED + 32),
    "x_decode_h12": dict(B=1, H=12, D=64, T=336, kv_frames=33, q_frames=1,  F=40, dtype="bf16", seed=BASE_SEED + 33),
    "x_decode_h24": dict(B=1, H=24, D=64, T=336, kv_frames=33, q_frames=1,  F=40, dtype="bf16", seed=BASE_SEED + 34),
    "x_spec_k3":    dict(B=1, H=16, D=64, T=336, kv_frames=35, q_frames=3,  F=40, dtype="bf16", seed=BASE_SEED + 35),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


def randn(shape, seed: int, dtype: str = "bf16", std: float = 1.0) -> np.ndarray:
    """iid N(0, std^2) as fp32, rounded to bf16-representable values when dtype == 'bf16'."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if dtype == "bf16":
        x = round_to_bf16(x)
    elif dtype != "fp32":
        raise ValueError("dtype must be 'bf16' or 'fp32'")
    return x


def make_qkv(B, H, D, T, kv_frames, q_frames, F=None, dtype="bf16", seed=BASE_SEED, **_):
    """Q [B,H,q_frames*T,D] and K, V [B,H,F*T,D] (all F frames filled; only the
    first kv_frames are meant to be read)."""
    F = kv_frames if F is None else F
    q = randn((B, H, q_frames * T, D), seed * 10 + 1, dtype)
    k = randn((B, H, F * T, D), seed * 10 + 2, dtype)
    v = randn((B, H, F * T, D), seed * 10 + 3, dtype)
    return q, k, v


def make_config(name: str):
    cfg = dict(CONFIGS[name] if name in CONFIGS else EXTRA_CONFIGS[name])
    q, k, v = make_qkv(**cfg)
    return cfg, q, k, v


def sample_rows(T: int, q_frames: int, per_frame: int, seed: int) -> np.ndarray:
    """Query rows for sampled checks: the first and last row of every query
    frame plus ``per_frame`` seeded random rows in each frame, sorted, unique."""
    rng = np.random.default_rng(seed)
    rows = []
    for f in range(q_frames):
        rows += [f * T, f * T + T - 1]
        rows += list(f * T + rng.integers(0, T, size=per_frame))
    return np.unique(np.asarray(rows, dtype=np.int64))
