"""Seeded tensor generators.

Every tensor is a pure function of (master seed, config id, layer index, role),
drawn with numpy's counter-based Philox generator on the CPU in fp32, so both
the CPU oracle and the GPU library are fed identical bits.

The pruned tensors stand in for the ADMM-pruned checkpoints of the paper
(Section 3): the pruning step there is a Euclidean projection onto a
cardinality constraint, i.e. the k largest-magnitude weights survive and the
rest are *exactly* zero.  The same projection is applied here to iid He-normal
weights, which makes the surviving positions uniformly random (unstructured).
"""
from __future__ import annotations

import hashlib
import numpy as np

MASTER_SEED = 190500571

_ROLES = ("x", "w", "b", "r", "misc")


def rng_for(config: str, layer: int, role: str, master: int = MASTER_SEED) -> np.random.Generator:
    """Philox generator keyed by a hash of (master, config, layer, role)."""
    if role not in _ROLES:
        raise ValueError(f"unknown role {role!r}")
    h = hashlib.blake2b(f"{master}/{config}/{layer}/{role}".encode(), digest_size=16).digest()
    key = [int.from_bytes(h[:8], "little"), int.from_bytes(h[8:], "little")]
    return np.random.Generator(np.random.Philox(key=key))


def conv_out_size(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def activation(shape, config: str, layer: int, relu: bool, role: str = "x",
               dtype=np.float32) -> np.ndarray:
    """N(0,1) tensor, optionally passed through max(.,0) (a post-ReLU feature map)."""
    g = rng_for(config, layer, role)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if relu:
        x = np.maximum(x, np.float32(0.0))
    return np.ascontiguousarray(x.astype(dtype))


def bias_vector(cout: int, config: str, layer: int, sigma: float = 0.01) -> np.ndarray:
    g = rng_for(config, layer, "b")
    return (g.standard_normal(size=(cout,), dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def keep_count(total: int, sparsity: float) -> int:
    """Number of surviving weights: round-half-even of (1 - s) * total."""
    v = (1.0 - float(sparsity)) * total
    return int(np.clip(np.round(v), 0, total))  # np.round is half-to-even


def pruned_weights(cout: int, cin: int, kh: int, kw: int, sparsity: float, config: str,
                   layer: int, mask: str = "magnitude", row_skew: float = 0.0) -> np.ndarray:
    """He-normal [cout][cin][kh][kw] fp32 tensor pruned per layer (not per row).

    mask="magnitude": keep the `keep_count` largest |w| (ties -> lower flat index).
    mask="random":    keep a seeded uniformly random subset of exactly that size.
    row_skew > 0 scales row r's magnitudes by exp(row_skew * z_r) before the
    magnitude ranking only (values themselves are untouched), which skews the
    per-row nonzero counts the way real pruned layers are skewed.
    Pruned entries are written as +0.0f.
    """
    g = rng_for(config, layer, "w")
    fan_in = cin * kh * kw
    sigma = np.float32(np.sqrt(2.0 / fan_in))
    w = g.standard_normal(size=(cout, cin, kh, kw), dtype=np.float32) * sigma
    total = w.size
    k = keep_count(total, sparsity)
    if k == total:
        return np.ascontiguousarray(w)
    flat = w.reshape(-1)
    keep = np.zeros(total, dtype=bool)
    if k > 0:
        if mask == "magnitude":
            score = np.abs(flat).astype(np.float64)
            if row_skew != 0.0:
                z = rng_for(config, layer, "misc").standard_normal(size=(cout,))
                score = (score.reshape(cout, -1) * np.exp(row_skew * z)[:, None]).reshape(-1)
            order = np.argsort(-score, kind="stable")
            keep[order[:k]] = True
        elif mask == "random":
            order = rng_for(config, layer, "misc").permutation(total)
            keep[order[:k]] = True
        else:
            raise ValueError(mask)
    out = np.where(keep, flat, np.float32(0.0)).astype(np.float32)
    return np.ascontiguousarray(out.reshape(cout, cin, kh, kw))


def embed_filter(w: np.ndarray, k: int) -> np.ndarray:
    """Centres a [cout][cin][kh][kw] filter bank (kh, kw odd, <= k) in a zero [cout][cin][k][k]
    one.  With padding (k-1)/2 the square bank computes what the rectangular one computes with
    padding ((kh-1)/2, (kw-1)/2): the added taps are exact zeros, which a compact format does
    not store.  This is how 1x7 / 7x1 filters are handed to an interface with one padding."""
    cout, cin, kh, kw = w.shape
    if kh > k or kw > k or (k - kh) % 2 or (k - kw) % 2:
        raise ValueError("cannot centre a %dx%d filter in %dx%d" % (kh, kw, k, k))
    out = np.zeros((cout, cin, k, k), dtype=w.dtype)
    r0, c0 = (k - kh) // 2, (k - kw) // 2
    out[:, :, r0:r0 + kh, c0:c0 + kw] = w
    return np.ascontiguousarray(out)
