"""Seeded synthetic inputs shaped like LLaMA activations.

This module holds no arithmetic of the quantization method: it only draws
random fp16 tensors with the outlier structure the paper describes for LLM
activations (a few persistent outlier channels, and "pivot" tokens with massive
activations -- Sec. 1 / Sec. 2.2), so that the CPU oracle and the HIP library
can be fed byte-identical inputs.  numpy only; no GPU, no library import.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 241009426
X_ABS_CLAMP = 30000.0     # keeps |x| and the fp16 intermediates finite


def _rng(config_index: int, tensor_index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config_index + tensor_index))


def near_identity(rng: np.random.Generator, d: int, sigma: float, batch: Optional[int] = None) -> np.ndarray:
    """I + sigma * N(0, 1) as fp16: well conditioned, like a trained transform."""
    shape = (d, d) if batch is None else (batch, d, d)
    m = rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)
    m += np.eye(d, dtype=np.float32)
    return m.astype(np.float16)


def activations(rng: np.random.Generator, T: int, n: int, *, outlier_channels=None,
                outlier_frac: float = 0.0, outlier_lo: float = 20.0, outlier_hi: float = 100.0,
                outlier_gain: Optional[float] = None, massive_tokens=(), massive_gain: float = 500.0,
                chunk_rows: int = 1024) -> np.ndarray:
    """[T, n] fp16 ~ N(0,1), selected channels amplified, selected tokens x massive_gain."""
    if outlier_channels is None:
        k = int(round(outlier_frac * n))
        outlier_channels = np.sort(rng.choice(n, size=k, replace=False)) if k else np.zeros(0, dtype=np.int64)
    outlier_channels = np.asarray(outlier_channels, dtype=np.int64)
    if outlier_gain is not None:
        gains = np.full(outlier_channels.shape, outlier_gain, dtype=np.float32)
    else:
        gains = rng.uniform(outlier_lo, outlier_hi, size=outlier_channels.shape).astype(np.float32)
    col_gain = np.ones(n, dtype=np.float32)
    col_gain[outlier_channels] = gains
    massive = np.zeros(T, dtype=bool)
    for t in massive_tokens:
        if 0 <= t < T:
            massive[t] = True
    out = np.empty((T, n), dtype=np.float16)
    for r0 in range(0, T, chunk_rows):
        r1 = min(T, r0 + chunk_rows)
        blk = rng.standard_normal((r1 - r0, n), dtype=np.float32)
        blk *= col_gain[None, :]
        blk[massive[r0:r1]] *= np.float32(massive_gain)
        np.clip(blk, -X_ABS_CLAMP, X_ABS_CLAMP, out=blk)
        out[r0:r1] = blk.astype(np.float16)
    return out


def sigmoid_clip(rng: np.random.Generator, T: int, lo: float = 1.5, hi: float = 3.0) -> np.ndarray:
    """Per-token clipping ratio: the logistic function of a ~ U(lo, hi), fp32."""
    a = rng.uniform(lo, hi, size=T)
    return (1.0 / (1.0 + np.exp(-a))).astype(np.float32)


@dataclass
class ActCase:
    name: str
    T: int
    n1: int
    n2: int
    x: np.ndarray          # fp16 [T, n]
    P1: np.ndarray         # fp16 [n1, n1]
    P2: np.ndarray         # fp16 [n2, n2]
    clip: np.ndarray       # fp32 [1] or [T]
    clip_mode: int         # 0 scalar, 1 per token

    @property
    def n(self) -> int:
        return self.n1 * self.n2


@dataclass
class KVCase:
    name: str
    T: int
    H: int
    D: int
    k: np.ndarray          # fp16 [T, H, D]
    v: np.ndarray
    P: np.ndarray          # fp16 [H, D, D]
    clip: float


def tiny(T: int = 16) -> ActCase:
    """Config "Tiny": T=16, n=256 (16 x 16), 4 fixed outlier channels x50, clip 1."""
    r = _rng(0, 0)
    x = activations(r, T, 256, outlier_channels=[3, 77, 130, 201], outlier_gain=50.0)
    P1 = near_identity(_rng(0, 1), 16, 0.1)
    P2 = near_identity(_rng(0, 2), 16, 0.1)
    return ActCase("tiny", T, 16, 16, x, P1, P2, np.array([1.0], dtype=np.float32), 0)


def llama_like(name: str, config_index: int, T: int, n1: int, n2: int, *, massive_every: int = 0,
               sigma: float = 0.05, per_token_clip: bool = True) -> ActCase:
    """LLaMA-shaped case: 1 % outlier channels x U(20,100); token 0 (and the first
    token of every `massive_every`-long sequence) x500; P = I + sigma N(0,1)."""
    n = n1 * n2
    massive = [0] if massive_every <= 0 else list(range(0, T, massive_every))
    x = activations(_rng(config_index, 0), T, n, outlier_frac=0.01, massive_tokens=massive)
    P1 = near_identity(_rng(config_index, 1), n1, sigma)
    P2 = near_identity(_rng(config_index, 2), n2, sigma)
    if per_token_clip:
        clip, mode = sigmoid_clip(_rng(config_index, 3), T), 1
    else:
        clip, mode = np.array([1.0], dtype=np.float32), 0
    return ActCase(name, T, n1, n2, x, P1, P2, clip, mode)


def prefill_7b(T: int = 2048) -> ActCase:
    """LLaMA-2-7B prefill shape: T=2048, n=4096 (64 x 64)."""
    return llama_like("prefill_7b", 1, T, 64, 64)


def decode_7b(T: int = 64, wide: bool = False) -> ActCase:
    """Decode shapes: T=64 at n=4096 (64 x 64) or n=11008 (86 x 128)."""
    return llama_like("decode_11008" if wide else "decode_4096", 2 if not wide else 3, T,
                      86 if wide else 64, 128 if wide else 64)


def prefill_70b(T: int = 16384, wide: bool = False) -> ActCase:
    """LLaMA-3-70B prefill shapes: n=8192 (64 x 128) or n=28672 (112 x 256)."""
    return llama_like("prefill_70b_28672" if wide else "prefill_70b_8192", 5 if wide else 4, T,
                      112 if wide else 64, 256 if wide else 128, massive_every=2048)


def kv_cache(T: int = 32768, H: int = 8, D: int = 128) -> KVCase:
    """KV-cache case: K, V ~ N(0,1) with 2 outlier dims per head x30, P_h = I + 0.05 N."""
    def one(tensor_index):
        r = _rng(6, tensor_index)
        a = np.empty((T, H, D), dtype=np.float16)
        dims = np.stack([r.choice(D, size=2, replace=False) for _ in range(H)])
        for r0 in range(0, T, 4096):
            r1 = min(T, r0 + 4096)
            blk = r.standard_normal((r1 - r0, H, D), dtype=np.float32)
            for h in range(H):
                blk[:, h, dims[h]] *= np.float32(30.0)
            a[r0:r1] = blk.astype(np.float16)
        return a
    P = near_identity(_rng(6, 2), D, 0.05, batch=H)
    return KVCase("kv_cache", T, H, D, one(0), one(1), P, 0.95)


def generic(seed: int, T: int, n1: int, n2: int, *, sigma: float = 0.05, clip_mode: int = 1,
            outlier_frac: float = 0.01, massive_tokens=(0,)) -> ActCase:
    """Free-form case for shape sweeps in the tests."""
    r = np.random.Generator(np.random.PCG64(BASE_SEED + 7919 * seed))
    x = activations(r, T, n1 * n2, outlier_frac=outlier_frac, massive_tokens=massive_tokens)
    P1 = near_identity(r, n1, sigma)
    P2 = near_identity(r, n2, sigma)
    clip = sigmoid_clip(r, T) if clip_mode == 1 else np.array([0.9], dtype=np.float32)
    return ActCase(f"generic_{n1}x{n2}_T{T}", T, n1, n2, x, P1, P2, clip, clip_mode)


def weights(config_index: int, m: int, n: int, *, sigma: float = 0.02, heavy_frac: float = 0.002) -> np.ndarray:
    """[m, n] fp16 weight matrix of a linear layer: N(0, sigma^2) with a few heavier input channels (x8)."""
    r = _rng(config_index, 7)
    w = r.standard_normal((m, n), dtype=np.float32) * np.float32(sigma)
    k = max(1, int(round(heavy_frac * n)))
    w[:, r.choice(n, size=k, replace=False)] *= np.float32(8.0)
    return w.astype(np.float16)


def weight_clip(config_index: int, m: int) -> np.ndarray:
    """Per-output-channel weight clipping ratios in (0.85, 1) (fp32 [m])."""
    return _rng(config_index, 8).uniform(0.85, 1.0, size=m).astype(np.float32)
