"""Seeded generators for the five synthetic workloads and the paper's two random benchmark families.

Every tensor is drawn in fp64 with numpy's PCG64 and rounded once (round-to-nearest-even) to fp16.
Each (tensor, batch, head) has its own random stream keyed by (seed, tensor id, batch, head), so a
single head of a large workload can be produced without generating the rest, and the oracle side and
the GPU side of a test always see the same bits.

Second parameter of a normal distribution is always the standard deviation.

The Qwen2-shaped and Stable-Video-Diffusion-shaped workloads are stand-ins for real model activations
(which need trained weights): only the tensor shapes and the qualitative structure the paper describes
(sequence-dimension bias, outlier channels, query/key resonance along the head dimension; paper
section 3.3.2) are reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import math

import numpy as np

_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_AUX = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    d: int
    causal: bool
    seed: int
    kind: str

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def group(self) -> int:
        return self.Hq // self.Hkv

    @property
    def flops(self) -> float:
        """Counted FLOPs: 4*B*Hq*N^2*d, halved when causal."""
        f = 4.0 * self.B * self.Hq * float(self.N) ** 2 * self.d
        return f / 2 if self.causal else f

    def with_n(self, n: int) -> "Workload":
        return replace(self, N=n)


WORKLOADS = {
    # 1: benign, constant key bias
    "tiny_bias4": Workload("tiny_bias4", 1, 1, 1, 256, 64, False, 0, "tiny"),
    # 2: large sequence-dimension bias, unscaled QK^T averages 128*8*80 = 81920 > 65504
    "overflow_bias": Workload("overflow_bias", 1, 8, 8, 4096, 128, False, 1, "overflow"),
    # 3: Qwen2-7B-shaped GQA prefill with outlier channels (throughput target workload)
    "qwen2_gqa_n8192": Workload("qwen2_gqa_n8192", 1, 28, 4, 8192, 128, True, 2, "qwen"),
    # 4: Stable-Video-Diffusion-shaped spatial attention with Q/K resonance
    "svd_resonance": Workload("svd_resonance", 14, 5, 5, 9216, 64, False, 3, "svd"),
    # 5: long-context Qwen2-shaped prefill with per-block key bias
    "qwen2_long_n32768": Workload("qwen2_long_n32768", 2, 28, 4, 32768, 128, True, 4, "long"),
}
_ORDER = ["tiny_bias4", "overflow_bias", "qwen2_gqa_n8192", "svd_resonance", "qwen2_long_n32768"]


def workload(key) -> Workload:
    """Look a workload up by name or by 1-based index."""
    if isinstance(key, int):
        return WORKLOADS[_ORDER[key - 1]]
    return WORKLOADS[key]


def _rng(w: Workload, tensor: int, b: int, h: int) -> np.random.Generator:
    return np.random.default_rng([w.seed, tensor, b, h])


def _to_f16(x: np.ndarray) -> np.ndarray:
    return x.astype(np.float16)


def _outlier_channels(w: Workload, b: int, hk: int) -> np.ndarray:
    return _rng(w, _TENSOR_AUX, b, hk).choice(w.d, 4, replace=False)


_SVD_FREQ = 4.0
_SVD_AMP = 30.0


def _svd_phase_q(w: Workload, b: int, h: int) -> float:
    return float(_rng(w, _TENSOR_AUX, b, h).uniform(0.0, 2.0 * math.pi))


def gen_q_head(w: Workload, b: int, h: int) -> np.ndarray:
    """Queries of one (batch, query head): fp16 [N, d]."""
    g = _rng(w, _TENSOR_Q, b, h)
    x = g.standard_normal((w.N, w.d))
    if w.kind == "overflow":
        x += 8.0
    elif w.kind == "qwen":
        ch = _outlier_channels(w, b, h // w.group)
        x[:, ch] *= 20.0
    elif w.kind == "svd":
        c = np.arange(w.d)
        x += _SVD_AMP * np.sin(2.0 * math.pi * _SVD_FREQ * c / w.d + _svd_phase_q(w, b, h))[None, :]
    return _to_f16(x)


def gen_kv_head(w: Workload, b: int, hk: int):
    """Keys and values of one (batch, KV head): two fp16 [N, d] arrays."""
    gk = _rng(w, _TENSOR_K, b, hk)
    k = gk.standard_normal((w.N, w.d))
    if w.kind == "tiny":
        k += 4.0
    elif w.kind == "overflow":
        k = 80.0 + 2.0 * k
    elif w.kind == "qwen":
        ch = _outlier_channels(w, b, hk)
        k[:, ch] += 60.0
    elif w.kind == "svd":
        c = np.arange(w.d)
        phase = _svd_phase_q(w, b, hk) + (math.pi if hk % 2 else 0.0)
        k += _SVD_AMP * np.sin(2.0 * math.pi * _SVD_FREQ * c / w.d + phase)[None, :]
    elif w.kind == "long":
        nblk = (w.N + 1023) // 1024
        bias = gk.uniform(20.0, 60.0, nblk)
        k += np.repeat(bias, 1024)[: w.N, None]
    v = _rng(w, _TENSOR_V, b, hk).standard_normal((w.N, w.d))
    return _to_f16(k), _to_f16(v)


def gen_full(w: Workload):
    """All of Q [B,Hq,N,d], K and V [B,Hkv,N,d] as fp16."""
    q = np.empty((w.B, w.Hq, w.N, w.d), np.float16)
    k = np.empty((w.B, w.Hkv, w.N, w.d), np.float16)
    v = np.empty((w.B, w.Hkv, w.N, w.d), np.float16)
    for b in range(w.B):
        for h in range(w.Hq):
            q[b, h] = gen_q_head(w, b, h)
        for hk in range(w.Hkv):
            k[b, hk], v[b, hk] = gen_kv_head(w, b, hk)
    return q, k, v


def gen_uniform_benchmark(x0: float, am: float, seed: int, shape=(1, 16, 1280, 128)):
    """Q, K, V ~ U(x0 - am, x0 + am) (paper Eq. 17), fp16, shape (B, heads, S, D)."""
    g = np.random.default_rng([seed, 17])
    return tuple(_to_f16(g.uniform(x0 - am, x0 + am, shape)) for _ in range(3))


def gen_hybrid_benchmark(x0: float, am: float, seed: int, p: float = 0.001, shape=(1, 16, 1280, 128)):
    """Q, K, V ~ N(x0, 1) + N(0, am) * Bernoulli(p) (paper Eq. 18; am is a standard deviation)."""
    g = np.random.default_rng([seed, 18])
    out = []
    for _ in range(3):
        x = x0 + g.standard_normal(shape)
        x += am * g.standard_normal(shape) * (g.random(shape) < p)
        out.append(_to_f16(x))
    return tuple(out)
