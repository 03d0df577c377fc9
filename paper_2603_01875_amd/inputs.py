"""Seeded synthetic inputs shaped like LLM distillation batches.

Holds no arithmetic of the distillation loss itself: it only draws hidden
states, output heads and token masks, and rounds them to the storage dtype.
Both the CPU oracle's tests and the GPU path are fed from here so that they
see bit-identical arrays.

The paper trains Qwen3 students (vocabulary 151936, Sec. 1 footnote and
Sec. 3.2) on sequences of up to 4096 tokens (Table 3 caption).  No dataset,
tokenizer or trained weight is available, so these stand-ins reproduce the
shapes, the value scales (unit-RMS final hidden states, N(0, 0.02^2) heads as
at LLM initialisation, wider teacher heads for sharper teachers) and the mask
structure (padding tails, random drops).
"""
from __future__ import annotations

import dataclasses
import numpy as np

FKL, RKL, JSD, TVD, SKEW_FKL, SKEW_RKL, AKL = 0, 1, 2, 3, 4, 5, 6   # divergence ids (as in the C header)
BF16, F32 = 0, 1                 # storage dtypes


@dataclasses.dataclass
class KDConfig:
    name: str
    batch: int
    seq: int
    H_t: int
    H_s: int
    V: int
    dtype: int
    w_t_std: float
    w_s_std: float
    rms_norm: bool
    kind: int
    tau: float
    beta: float
    mask: str                    # "ones" | "tail25" | "bernoulli10"
    seed: int

    @property
    def T(self):
        return self.batch * self.seq


def workload(name: str) -> KDConfig:
    """The five benchmark workloads (index = position in the benchmark list;
    seed = 18750 + index)."""
    table = {
        "tiny_fkl_f32": KDConfig("tiny_fkl_f32", 2, 64, 256, 128, 4096, F32, 0.02, 0.02,
                                 False, FKL, 1.0, 0.5, "ones", 18750),
        "fkl_bf16": KDConfig("fkl_bf16", 4, 1024, 4096, 1024, 151936, BF16, 0.02, 0.02,
                             True, FKL, 1.0, 0.5, "tail25", 18751),
        "rkl_bf16": KDConfig("rkl_bf16", 4, 1024, 4096, 1024, 151936, BF16, 0.04, 0.02,
                             True, RKL, 1.0, 0.5, "tail25", 18752),
        "jsd_bf16": KDConfig("jsd_bf16", 4, 1024, 4096, 1024, 151936, BF16, 0.04, 0.02,
                             True, JSD, 1.0, 0.5, "tail25", 18752),
        "large_teacher": KDConfig("large_teacher", 2, 4096, 8192, 2048, 128256, BF16, 0.02, 0.02,
                                  True, FKL, 2.0, 0.5, "bernoulli10", 18753),
        "long_peaked": KDConfig("long_peaked", 1, 32768, 5120, 4096, 151936, BF16, 0.1, 0.02,
                                True, JSD, 1.0, 0.1, "ones", 18754),
    }
    return dataclasses.replace(table[name])


WORKLOADS = ("tiny_fkl_f32", "fkl_bf16", "rkl_bf16", "jsd_bf16", "large_teacher", "long_peaked")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """fp32 values of uint16 bf16 bit patterns."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _hidden(rng, T, H, rms_norm, dtype):
    h = rng.standard_normal((T, H), dtype=np.float32)
    if rms_norm:
        h /= np.sqrt(np.mean(h.astype(np.float32) ** 2, axis=1, keepdims=True, dtype=np.float32))
    return round_to_bf16(h) if dtype == BF16 else h


def _head(rng, V, H, std, dtype):
    W = rng.standard_normal((V, H), dtype=np.float32)
    W *= np.float32(std)
    return round_to_bf16(W) if dtype == BF16 else W


def _mask(rng, cfg: KDConfig):
    T = cfg.T
    if cfg.mask == "ones":
        return np.ones(T, dtype=np.uint8)
    if cfg.mask == "tail25":
        m = np.ones((cfg.batch, cfg.seq), dtype=np.uint8)
        tails = rng.integers(0, cfg.seq // 4 + 1, size=cfg.batch)
        for b, k in enumerate(tails):
            if k:
                m[b, cfg.seq - int(k):] = 0
        return m.reshape(T)
    if cfg.mask == "bernoulli10":
        return (rng.random(T) >= 0.1).astype(np.uint8)
    raise ValueError(cfg.mask)


def generate(cfg: KDConfig):
    """Draw h_t, h_s, W_t, W_s, mask (in that order) from default_rng(cfg.seed).

    Heads are drawn in [V, H] storage order (one row per vocabulary entry).
    Arrays are fp32 holding values exactly representable in cfg.dtype.
    """
    rng = np.random.default_rng(cfg.seed)
    h_t = _hidden(rng, cfg.T, cfg.H_t, cfg.rms_norm, cfg.dtype)
    h_s = _hidden(rng, cfg.T, cfg.H_s, cfg.rms_norm, cfg.dtype)
    W_t = _head(rng, cfg.V, cfg.H_t, cfg.w_t_std, cfg.dtype)
    W_s = _head(rng, cfg.V, cfg.H_s, cfg.w_s_std, cfg.dtype)
    mask = _mask(rng, cfg)
    return dict(h_t=h_t, h_s=h_s, W_t=W_t, W_s=W_s, mask=mask)


def scaled(cfg: KDConfig, **kw) -> KDConfig:
    """Same recipe at other sizes (for parity cases the oracle finishes quickly)."""
    return dataclasses.replace(cfg, **kw)


def to_device(x: np.ndarray, dtype: int, device="cuda"):
    """Upload an array made by `generate` as a torch tensor of the storage dtype (bit-exact)."""
    import torch
    if dtype == BF16:
        bits = bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
