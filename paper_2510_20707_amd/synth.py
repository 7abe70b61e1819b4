"""Seeded synthetic KV caches shaped like the paper's workloads.

This module only draws random inputs.  It contains none of the method's
arithmetic (no scores, no softmax, no normalisation of keys for scoring) and is
the one piece of code that both the CPU oracle's tests and the HIP path's tests
use, so that both sides see bit-identical inputs.

The caches stand in for the model caches the paper measures on (Qwen2-VL /
LLaVA-OneVision / Llama-3 prefill caches); the value structure follows the
paper's redundancy analysis (Sec. 1 and Fig. 1-2: keys of vision-language
heads have mean pairwise cosine around 0.6-0.8, text-only models 0.2-0.4, and
heads differ widely).

All values are drawn in float32 on the host and, for bf16 workloads, rounded
once to bf16 (round to nearest even).  `Unit.K/V` and `Layer.Q` hold float32
arrays whose values are exactly representable in the workload's dtype, so a
float64 upcast on the CPU and a bf16 upload to the GPU describe the same
numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "round_to_bf16_bits", "bf16_bits_to_f32",
    "make_layer", "layer_arrays",
]


@dataclass(frozen=True)
class Workload:
    """Shape and value recipe of one synthetic cache."""
    name: str
    cfg_id: int                 # enters the RNG key
    dtype: str                  # "f32" or "bf16"
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int                # N, window included
    window: int                 # W
    budget: int                 # B per head, window included
    pool: str = "max"
    pool_kernel: int = 7
    budget_mode: str = "fixed"  # or "adaptive"
    budget_floor: int = 0
    keys: str = "iid"           # iid | image | text_offset | video
    text_prefix: int = 0        # image/video: tokens [0, text_prefix) are text
    text_suffix_start: int = 0  # image/video: tokens [text_suffix_start, N) are text
    sigma: Tuple[float, float] = (0.3, 0.3)   # visual noise, drawn U[lo, hi] per head
    text_offset: float = 0.0    # length of the shared mean offset of text keys
    n_frames: int = 0
    frame_tokens: int = 0
    softmax_scale: float = 1.0  # queries already carry 1/sqrt(D)
    eps: float = 1e-6

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_units(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # tiny single layer, fp32
    "c1": Workload("c1", 1, "f32", 1, 1, 4, 2, 64, 512, 8, 64, keys="iid"),
    # Qwen2-VL-7B-shaped single layer
    "c2": Workload("c2", 2, "bf16", 1, 1, 28, 4, 128, 4096, 32, 64, keys="image",
                   text_prefix=64, text_suffix_start=3648, sigma=(0.3, 0.3), text_offset=7.4),
    # Qwen2-VL-7B-shaped full cache, one high-resolution image
    "c3": Workload("c3", 3, "bf16", 28, 1, 28, 4, 128, 8192, 32, 64, keys="image",
                   text_prefix=64, text_suffix_start=7616, sigma=(0.1, 0.8), text_offset=7.4),
    # Llama-3-8B-shaped text-only cache
    "c4": Workload("c4", 4, "bf16", 32, 1, 32, 8, 128, 16384, 32, 256, keys="text_offset",
                   text_offset=0.5),
    # long video, head-adaptive budgets
    "c5": Workload("c5", 5, "bf16", 28, 4, 28, 4, 128, 32768, 32, 128, keys="video",
                   budget_mode="adaptive", budget_floor=32,
                   text_prefix=64, text_suffix_start=32704, sigma=(0.3, 0.3), text_offset=7.4,
                   n_frames=64, frame_tokens=510),
}

_VIS_OFFSET = 8.0       # length of the shared offset of visual keys
_N_CENTROIDS = 64
_SUBSPACE = 16
_DRIFT = 0.1


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _quantise(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(round_to_bf16_bits(x))
    return np.ascontiguousarray(x, dtype=np.float32)


def _rng(seed: int, wl: Workload, layer: int, b: int, head: int, stream: int):
    return np.random.default_rng([seed, wl.cfg_id, layer, b, head, stream])


def _unit_vector(rng, d: int) -> np.ndarray:
    v = rng.standard_normal(d)
    return (v / np.sqrt((v * v).sum())).astype(np.float32)


def _keys(wl: Workload, seed: int, layer: int, b: int, h: int) -> np.ndarray:
    n, d = wl.seq_len, wl.head_dim
    rs = _rng(seed, wl, layer, b, h, 0)      # head structure
    rz = _rng(seed, wl, layer, b, h, 1)      # per-token noise
    z = rz.standard_normal((n, d), dtype=np.float32)
    if wl.keys == "iid":
        return z
    mu = _unit_vector(rs, d)
    if wl.keys == "text_offset":
        return z + np.float32(wl.text_offset) * mu
    # image / video: text spans around a block of clustered visual keys
    lo, hi = wl.sigma
    sigma = np.float32(lo if lo == hi else rs.uniform(lo, hi))
    basis, _ = np.linalg.qr(rs.standard_normal((d, _SUBSPACE)))
    cent = (rs.standard_normal((_N_CENTROIDS, _SUBSPACE)) @ basis.T).astype(np.float32)  # [64, d]
    k = np.empty((n, d), dtype=np.float32)
    p0, p1 = wl.text_prefix, wl.text_suffix_start
    text = np.float32(wl.text_offset) * mu
    k[:p0] = z[:p0] + text
    k[p1:] = z[p1:] + text
    vis = np.float32(_VIS_OFFSET) * mu
    if wl.keys == "image":
        which = rs.integers(0, _N_CENTROIDS, size=p1 - p0)
        k[p0:p1] = vis + cent[which] + sigma * z[p0:p1]
    elif wl.keys == "video":
        assert p1 - p0 == wl.n_frames * wl.frame_tokens
        for f in range(wl.n_frames):
            if f > 0:
                cent = cent + np.float32(_DRIFT) * rs.standard_normal(cent.shape, dtype=np.float32)
            a = p0 + f * wl.frame_tokens
            which = rs.integers(0, _N_CENTROIDS, size=wl.frame_tokens)
            k[a:a + wl.frame_tokens] = vis + cent[which] + sigma * z[a:a + wl.frame_tokens]
    else:
        raise ValueError(wl.keys)
    return k


@dataclass
class Layer:
    """One layer of a synthetic cache, values exactly representable in wl.dtype."""
    K: np.ndarray    # [batch, n_kv_heads, N, D] float32
    V: np.ndarray    # [batch, n_kv_heads, N, D] float32
    Q: np.ndarray    # [batch, n_q_heads, W, D] float32 (observation-window queries)


def make_layer(wl: Workload, layer: int, seed: int = 0) -> Layer:
    bt, hkv, hq, n, d, w = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.seq_len, wl.head_dim, wl.window
    K = np.empty((bt, hkv, n, d), dtype=np.float32)
    V = np.empty((bt, hkv, n, d), dtype=np.float32)
    Q = np.empty((bt, hq, w, d), dtype=np.float32)
    inv = np.float32(1.0 / np.sqrt(d))
    for b in range(bt):
        for h in range(hkv):
            K[b, h] = _quantise(_keys(wl, seed, layer, b, h), wl.dtype)
            V[b, h] = _quantise(_rng(seed, wl, layer, b, h, 2).standard_normal((n, d), dtype=np.float32), wl.dtype)
        for q in range(hq):
            Q[b, q] = _quantise(_rng(seed, wl, layer, b, q, 3).standard_normal((w, d), dtype=np.float32) * inv, wl.dtype)
    return Layer(K, V, Q)


def layer_arrays(wl: Workload, lay: Layer):
    """Arrays ready for upload: float32 as is, bf16 as uint16 bit patterns."""
    if wl.dtype == "bf16":
        return round_to_bf16_bits(lay.K), round_to_bf16_bits(lay.V), round_to_bf16_bits(lay.Q)
    return lay.K, lay.V, lay.Q


def window_lse(wl: Workload, lay: Layer, causal: bool = True) -> np.ndarray:
    """Stand-in for a by-product of the prefill attention kernel, an optional INPUT of the compression
    step: for every window query row the natural logarithm of sum_i exp(softmax_scale * q.k_i) over
    the keys the row attends to (0..Nc+w with the causal window, else all N), float32 [batch, Hq, W].
    Computed in float64 from the layer's values; tests pin it against a library log-sum-exp."""
    n, w, g = wl.seq_len, wl.window, wl.group
    out = np.empty((wl.batch, wl.n_q_heads, w), dtype=np.float32)
    vis = np.arange(n)[None, :] <= ((n - w + np.arange(w)) if causal else np.full(w, n - 1))[:, None]
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            s = wl.softmax_scale * (lay.Q[b, h].astype(np.float64) @ lay.K[b, h // g].astype(np.float64).T)
            s = np.where(vis, s, -np.inf)
            m = s.max(axis=1)
            out[b, h] = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    return out
