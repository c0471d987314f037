"""Seeded synthetic inputs for the L4Q layer.

This module draws random tensors and rounds them to the storage type.  It holds
none of the method's arithmetic (no merge, no quantizer, no initialisation of
scale/zero): both the CPU checker and the HIP path receive the arrays made here.

Shapes follow the layer notation of the paper's problem statement (Sec. 2.1,
Sec. 3.2): tokens T, in-features i, out-features o, LoRA rank r, group size g.
Value distributions: X ~ N(0,1); W0 ~ N(0, 0.02) with an optional independent
Bernoulli(1e-3) set of entries multiplied by 20 (stand-in for LLM weight
outliers, Sec. 3.3); A ~ U(-1/sqrt(i), +1/sqrt(i)) (Kaiming-uniform as used for
LoRA's A, Sec. 4.1); B ~ N(0, 1e-3) (non-zero so that dA is exercised);
dY ~ N(0, 1e-2).  The second argument of N(.,.) is a standard deviation.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

DTYPE_F32 = 0
DTYPE_BF16 = 1


@dataclass(frozen=True)
class LayerSpec:
    name: str
    tokens: int
    in_features: int
    out_features: int
    rank: int
    alpha: float
    bits: int
    group_size: int
    dtype: int = DTYPE_BF16
    outliers: bool = True

    @property
    def groups(self) -> int:
        return self.in_features // self.group_size

    def gemm_flops(self) -> float:
        """Algorithmic FLOPs of one fwd+bwd: three GEMMs plus merge, dA, dB."""
        t, i, o, r = self.tokens, self.in_features, self.out_features, self.rank
        return 6.0 * t * o * i + 6.0 * o * i * r

    def with_(self, **kw) -> "LayerSpec":
        return replace(self, **kw)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), keep float32 storage."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bfloat16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("values are not bfloat16-representable")
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits16: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (bits16.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def make_layer_inputs(spec: LayerSpec, seed: int = 0) -> Dict[str, np.ndarray]:
    """Return X [T,i], W0 [o,i], A [r,i], B [o,r], dY [T,o] as float32 arrays.

    In bf16 mode every value is rounded once to bfloat16 here, before either
    side sees it; the arrays stay float32 so they widen exactly to float64.
    """
    t, i, o, r = spec.tokens, spec.in_features, spec.out_features, spec.rank
    x = _rng(seed, 1).standard_normal((t, i), dtype=np.float32)
    w0 = _rng(seed, 2).standard_normal((o, i), dtype=np.float32) * np.float32(0.02)
    if spec.outliers:
        hit = _rng(seed, 3).random((o, i), dtype=np.float32) < np.float32(1e-3)
        w0[hit] *= np.float32(20.0)
    bound = np.float32(1.0 / np.sqrt(float(i)))
    a = (_rng(seed, 4).random((r, i), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)) * bound
    b = _rng(seed, 5).standard_normal((o, r), dtype=np.float32) * np.float32(1e-3)
    dy = _rng(seed, 6).standard_normal((t, o), dtype=np.float32) * np.float32(1e-2)
    out = {"X": x, "W0": w0, "A": a, "B": b, "dY": dy}
    if spec.dtype == DTYPE_BF16:
        out = {k: round_to_bf16(v) for k, v in out.items()}
    return out


# ---- the named workloads (shapes of LLaMA-7B / Mistral-7B linear layers) ----

def config1() -> List[LayerSpec]:
    return [LayerSpec("c1_fp32_256x256", 64, 256, 256, 8, 16.0, 4, 64, DTYPE_F32, outliers=False)]


def config2() -> List[LayerSpec]:
    return [LayerSpec("llama7b_attn_4096x4096", 4096, 4096, 4096, 16, 32.0, 4, 128)]


def config3() -> List[LayerSpec]:
    return [
        LayerSpec("llama7b_mlp_up_11008x4096", 4096, 4096, 11008, 16, 32.0, 4, 128),
        LayerSpec("llama7b_mlp_down_4096x11008", 4096, 11008, 4096, 16, 32.0, 4, 128),
    ]


def config4() -> List[LayerSpec]:
    base = [s.with_(bits=3, name=s.name + "_3bit") for s in config3()]
    sweep = [config3()[0].with_(bits=3, group_size=g, name=f"llama7b_mlp_up_3bit_g{g}") for g in (64, 256)]
    return base + sweep


def config5() -> List[LayerSpec]:
    t = 8192
    mk = lambda n, o, i: LayerSpec(f"mistral7b_{n}_{o}x{i}", t, i, o, 16, 32.0, 4, 128)
    return [mk("q", 4096, 4096), mk("k", 1024, 4096), mk("v", 1024, 4096), mk("o", 4096, 4096),
            mk("gate", 14336, 4096), mk("up", 14336, 4096), mk("down", 4096, 14336)]


CONFIGS = {"c1": config1, "c2": config2, "c3": config3, "c4": config4, "c5": config5}
