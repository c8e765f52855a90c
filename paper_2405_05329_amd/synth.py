"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds no arithmetic of the method: it only draws N(0,1) numbers and rounds them to
bf16.  The paper ran real prompts through pretrained LLaMA-7B / Falcon-7B (Sec. 5);
attention cost depends on shapes only, so seeded Gaussians of those shapes stand in.
"""
from __future__ import annotations

import math

import numpy as np

# (n_q_heads, n_kv_heads, head_dim, context_len, boundaries)
CONFIGS = {
    "tiny": dict(cfg_id=1, H=2, Hkv=2, d=64, C=256, boundaries=[0, 160, 256]),
    "llama7b_4k_equal": dict(cfg_id=2, H=32, Hkv=32, d=128, C=4096,
                             boundaries=[0, 1024, 2048, 3072, 4096]),
    "llama7b_16k_balanced": dict(cfg_id=3, H=32, Hkv=32, d=128, C=16384,
                                 boundaries=[0, 5824, 8192, 10048, 11584, 12928, 14208, 15296, 16384]),
    "falcon7b_8k_balanced": dict(cfg_id=4, H=71, Hkv=1, d=64, C=8192,
                                 boundaries=[0, 4096, 5824, 7104, 8192]),
    "llama7b_32k_balanced": dict(cfg_id=5, H=32, Hkv=32, d=128, C=32768,
                                 boundaries=[0, 11584, 16384, 20096, 23168, 25920, 28352, 30656, 32768]),
    # grouped-query and multi-query variants of the Llama-7B shape (Sec. 5, the GQA8 / MQA rows of the
    # model table), on the 16k balanced boundaries
    "llama7b_gqa8_16k_balanced": dict(cfg_id=6, H=32, Hkv=8, d=128, C=16384,
                                      boundaries=[0, 5824, 8192, 10048, 11584, 12928, 14208, 15296, 16384]),
    "llama7b_mqa_16k_balanced": dict(cfg_id=7, H=32, Hkv=1, d=128, C=16384,
                                     boundaries=[0, 5824, 8192, 10048, 11584, 12928, 14208, 15296, 16384]),
}
ROPE_BASE = 10000.0


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, cfg_id: int, tensor_id: int, shape, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns of N(0, std^2) draws from the stream keyed by (seed, cfg_id, tensor_id)."""
    rng = np.random.default_rng([seed, cfg_id, tensor_id])
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x = x * np.float32(std)
    return f32_to_bf16_bits(x)


def make_qkv(seed: int, cfg_id: int, C: int, H: int, Hkv: int, d: int, q_gain: float = 1.0):
    """Un-rotated Q [C,H,d], K [C,Hkv,d], V [C,Hkv,d] as bf16 bit patterns (uint16)."""
    q = normal_bf16(seed, cfg_id, 0, (C, H, d), std=q_gain)
    k = normal_bf16(seed, cfg_id, 1, (C, Hkv, d))
    v = normal_bf16(seed, cfg_id, 2, (C, Hkv, d))
    return q, k, v


def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)


# Decoder-layer shapes (hidden, ffn) that go with the attention shapes above; the weights of the
# pretrained models are not available, so Gaussians of the usual initialisation width stand in.
LAYER_SHAPES = {
    "llama7b": dict(hidden=4096, ffn=11008, H=32, Hkv=32, d=128, weight_std=0.02),
}
RMS_EPS = 1e-6


def make_layer_weights(seed: int, cfg_id: int, hidden: int, ffn: int, H: int, Hkv: int, d: int,
                       weight_std: float):
    """bf16 bit patterns of one layer's parameters: norm gains ~ 1 + N(0, 0.1^2), matrices
    ~ N(0, weight_std^2), stored [out_features, in_features]; wqkv = query rows, key rows, value rows."""
    def mat(tid, rows, cols):
        return normal_bf16(seed, cfg_id, tid, (rows, cols), std=weight_std)
    def gain(tid):
        rng = np.random.default_rng([seed, cfg_id, tid])
        return f32_to_bf16_bits(1.0 + 0.1 * rng.standard_normal(size=hidden, dtype=np.float32))
    return {
        "norm1": gain(10), "norm2": gain(11),
        "wqkv": mat(12, (H + 2 * Hkv) * d, hidden),
        "wo": mat(13, hidden, H * d),
        "w_gate": mat(14, ffn, hidden), "w_up": mat(15, ffn, hidden),
        "w_down": mat(16, hidden, ffn),
    }
