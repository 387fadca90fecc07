"""Seeded synthetic inputs for the H-BitLinear workloads.

This module only draws random tensors with the shapes and outlier structure of
the five benchmark configurations (activations with a few large "outlier"
channels, Gaussian latent weights).  It contains none of the method's
arithmetic: no Hadamard transform, no quantizer, no GEMM.  Both the HIP path
and the CPU oracle are fed from here by the tests and the benchmark; neither
of them imports the other.

bf16 tensors are carried on the host as ``uint16`` bit patterns (numpy has no
bf16 type); ``f32_to_bf16_bits`` rounds to nearest-even, ``bf16_bits_to_f32``
is exact.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np

F32 = 0   # dtype tags shared with the C ABI (HBL_F32 / HBL_BF16)
BF16 = 1


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round an fp32 array to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


@dataclass(frozen=True)
class Site:
    """One linear projection of a benchmark configuration.

    T tokens, K in-features (= Hadamard size when ``hadamard``), N out-features.
    ``x_kind``: 'gauss' = N(0,1); 'swiglu' = SiLU(a)*b with a,b ~ N(0,1).
    ``outlier_channels`` fixed channel list, else ceil(outlier_frac*K) channels
    taken from a seeded permutation; those channels are multiplied by
    ``outlier_scale``.  ``groups`` = number of equal row-groups of W that carry
    their own absmean scale (3 for a fused QKV, 2 for up|gate, else 1).
    """
    name: str
    T: int
    K: int
    N: int
    hadamard: bool = True
    bits: Tuple[int, ...] = (4,)
    x_dtype: int = BF16
    x_kind: str = "gauss"
    outlier_frac: float = 0.0
    outlier_scale: float = 1.0
    outlier_channels: Tuple[int, ...] = ()
    groups: int = 1
    w_std: float = 0.02
    seed: int = 0
    x_stream: int = 0
    w_stream: int = 1000

    @property
    def gemm_ops(self) -> int:
        return 2 * self.T * self.K * self.N


def outlier_channels(site: Site) -> np.ndarray:
    if site.outlier_channels:
        return np.asarray(site.outlier_channels, dtype=np.int64)
    n = int(math.ceil(site.outlier_frac * site.K - 1e-9)) if site.outlier_frac > 0 else 0
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    perm = _rng(site.seed, 7_000 + site.x_stream).permutation(site.K)
    return np.sort(perm[:n]).astype(np.int64)


def make_x_f32(site: Site, rows: slice | None = None) -> np.ndarray:
    """Activations [T,K] as fp32 before any bf16 rounding (whole tensor is drawn, then sliced)."""
    g = _rng(site.seed, site.x_stream)
    if site.x_kind == "gauss":
        x = g.standard_normal((site.T, site.K), dtype=np.float32)
    elif site.x_kind == "swiglu":
        a = g.standard_normal((site.T, site.K), dtype=np.float32)
        b = g.standard_normal((site.T, site.K), dtype=np.float32)
        x = (a / (1.0 + np.exp(-a))) * b
        x = x.astype(np.float32)
    else:
        raise ValueError(site.x_kind)
    ch = outlier_channels(site)
    if ch.size:
        x[:, ch] *= np.float32(site.outlier_scale)
    if rows is not None:
        x = x[rows]
    return np.ascontiguousarray(x, dtype=np.float32)


def make_x(site: Site) -> np.ndarray:
    """Activations in the site's storage dtype: fp32 array, or uint16 bf16 bit patterns."""
    x = make_x_f32(site)
    if site.x_dtype == BF16:
        return f32_to_bf16_bits(x)
    return x


def make_w(site: Site) -> np.ndarray:
    """Latent (unquantized) weights [N,K] fp32 ~ N(0, w_std^2)."""
    g = _rng(site.seed, site.w_stream)
    w = g.standard_normal((site.N, site.K), dtype=np.float32)
    w *= np.float32(site.w_std)
    return w


# ---------------------------------------------------------------------------
# The five benchmark configurations
# ---------------------------------------------------------------------------

def config_sites(cfg: int, batch: int = 64, layer: int = 0) -> List[Site]:
    """Sites of configuration ``cfg`` (1..5).  For cfg 5, ``batch`` tokens and
    an independent weight draw per ``layer``."""
    if cfg == 1:
        return [Site("tiny", 16, 256, 256, x_dtype=F32, outlier_channels=(3, 97),
                     outlier_scale=20.0, seed=0)]
    if cfg == 2:
        return [Site("wo_1p3b", 2048, 2048, 2048, bits=(4, 8), outlier_frac=0.01,
                     outlier_scale=30.0, seed=1)]
    if cfg == 3:
        return [Site("wdown_3b", 4096, 8192, 3072, x_kind="swiglu", outlier_frac=0.005,
                     outlier_scale=50.0, seed=2)]
    if cfg == 4:
        return [
            Site("wo_7b", 8192, 4096, 4096, outlier_frac=0.01, outlier_scale=50.0, seed=3,
                 x_stream=0, w_stream=1000),
            Site("wdown_7b", 8192, 16384, 4096, outlier_frac=0.01, outlier_scale=50.0, seed=3,
                 x_stream=1, w_stream=1001),
        ]
    if cfg == 5:
        common = dict(outlier_frac=0.01, outlier_scale=30.0, seed=4)
        ws = 1000 + 16 * layer
        return [
            Site("dec_qkv", batch, 4096, 3 * 4096, hadamard=False, groups=3, x_stream=0,
                 w_stream=ws + 0, **common),
            Site("dec_wo", batch, 4096, 4096, hadamard=True, x_stream=1, w_stream=ws + 1, **common),
            Site("dec_upgate", batch, 4096, 2 * 16384, hadamard=False, groups=2, x_stream=2,
                 w_stream=ws + 2, **common),
            Site("dec_wdown", batch, 16384, 4096, hadamard=True, x_stream=3, w_stream=ws + 3, **common),
        ]
    raise ValueError(f"unknown config {cfg}")


def config4_wdown_swiglu() -> Site:
    """Parity-only variant of the configuration-4 W_down site: the same shape, weights and outlier channels,
    with the input drawn as a gated-activation output, SiLU(a)*b, instead of a Gaussian (the configuration's
    wording allows both readings: "as in config 3" names the SwiGLU draw, its parenthesis the Gaussian one)."""
    return replace(config_sites(4)[1], name="wdown_7b_swiglu", x_kind="swiglu", x_stream=2)


def shrink(site: Site, T: int | None = None, K: int | None = None, N: int | None = None) -> Site:
    """Same recipe at a smaller shape (parity cases the oracle finishes in seconds)."""
    return replace(site, T=T or site.T, K=K or site.K, N=N or site.N)
