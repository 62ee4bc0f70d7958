"""Seeded dense inputs: features, labels, train mask, Glorot weights."""
from __future__ import annotations

import numpy as np


def features(n: int, d: int, seed: int, gen: str = "numpy") -> np.ndarray:
    """``[n, d]`` float32 standard-normal features.  ``gen="counter"``: the parallel
    counter-based stream of the large workloads (a config's ``gen`` key)."""
    if gen == "counter":
        from .graphs import normal_counter
        return normal_counter(n, d, seed)
    rng = np.random.default_rng([seed, 0xBB67AE85])
    return rng.standard_normal((n, d), dtype=np.float32)


def labels_and_mask(n: int, n_classes: int, train_frac: float, seed: int):
    """Uniform int32 labels in ``[0, n_classes)`` and a uint8 Bernoulli train mask."""
    rng = np.random.default_rng([seed, 0x3C6EF372])
    y = rng.integers(0, n_classes, size=n, dtype=np.int32)
    m = (rng.random(n) < train_frac).astype(np.uint8)
    if n > 0 and m.sum() == 0:
        m[0] = 1
    return y, m


def glorot_weights(dims, seed: int, *, sage: bool, bias_scale: float = 0.0):
    """Per-layer weights drawn ``U(-a, a)``, ``a = sqrt(6 / (d_in + d_out))``.

    Returns a list with one dict per layer: ``W`` ``[d_in, d_out]``, ``Ws`` (same shape,
    only when ``sage``) and ``b`` ``[d_out]`` (zeros unless ``bias_scale`` > 0, which tests
    use so that a bias mistake cannot hide).
    """
    rng = np.random.default_rng([seed, 0xA54FF53A])
    out = []
    for l in range(len(dims) - 1):
        din, dout = int(dims[l]), int(dims[l + 1])
        a = np.sqrt(6.0 / (din + dout))
        layer = {"W": rng.uniform(-a, a, size=(din, dout)).astype(np.float32)}
        layer["Ws"] = rng.uniform(-a, a, size=(din, dout)).astype(np.float32) if sage else None
        layer["b"] = (bias_scale * rng.standard_normal(dout)).astype(np.float32)
        out.append(layer)
    return out


def attention_vectors(weights, seed: int, scale: float = 0.5):
    """Adds the two attention vectors of a graph-attention layer (``a_src``, ``a_dst``, each
    ``[d_out]``, ``N(0, scale^2 / d_out)`` so that scores stay O(1)) to every layer dict."""
    rng = np.random.default_rng([seed, 0x6A7])
    for layer in weights:
        dout = layer["W"].shape[1]
        layer["a_src"] = (rng.standard_normal(dout) * scale / np.sqrt(dout)).astype(np.float32)
        layer["a_dst"] = (rng.standard_normal(dout) * scale / np.sqrt(dout)).astype(np.float32)
    return weights


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)
