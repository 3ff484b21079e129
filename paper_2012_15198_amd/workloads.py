"""Seeded synthetic inputs for the segment-wise gossip mixing path.

This module only *describes and generates inputs*: worker matrices, gradients,
segment offsets, layer sizes and column samples.  It holds none of the method's
arithmetic (no topology draw, no averaging) and imports neither the HIP binding
nor the CPU oracle, so both sides can be fed from it.

The five workloads stand in for the paper's ResNet-on-ImageNet runs (Section 4.1,
Table 1): only the *shapes* are taken from there -- 25,557,032 and 11,689,512 are
the flat parameter counts of ResNet-50 / ResNet-18, 161 is the number of
ResNet-50 parameter tensors ("Model segment: segmenting blocks and FC layer").
Values are Gaussian with the stated standard deviation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration (shapes only, no data)."""
    name: str
    W: int                 # simulated workers = rows of the parameter matrix
    P: int                 # parameters per worker = used columns
    S: int                 # segments per worker vector
    rounds: int            # gossip rounds
    seed: int              # seed for data *and* topology
    sigma: float           # std-dev of the parameter values
    G: int = 1             # group size for the hierarchical mode (1 = flat gossip)
    layers: int = 0        # >0: segments aligned to this many ragged layer tensors
    grad_sigma: float = 0.0  # >0: synthetic gradients for the fused SGD step
    lr: float = 0.0
    mu: float = 0.0
    wd: float = 0.0
    kind: str = "gossip"   # gossip | hier | fused+pushsum

    @property
    def L(self) -> int:
        """Number of gossiping rows (group leaders in hierarchical mode)."""
        return self.W // self.G


WORKLOADS = {
    "C1": Workload("C1", W=8, P=1_000_000, S=4, rounds=10, seed=1, sigma=1.0),
    "C2": Workload("C2", W=32, P=25_557_032, S=8, rounds=50, seed=2, sigma=0.05),
    "C3": Workload("C3", W=64, P=11_689_512, S=16, rounds=20, seed=3, sigma=0.05,
                   G=8, kind="hier"),
    "C4": Workload("C4", W=128, P=25_557_032, S=8, rounds=20, seed=4, sigma=0.05,
                   grad_sigma=1e-2, lr=0.1, mu=0.9, wd=1e-4, kind="fused+pushsum"),
    "C5": Workload("C5", W=256, P=25_557_032, S=32, rounds=10, seed=5, sigma=0.05,
                   G=8, layers=161, kind="hier"),
}


# --------------------------------------------------------------------------- #
# segment layout (an *input* of the path: offsets are handed to both sides)
# --------------------------------------------------------------------------- #
def equal_seg_off(P: int, S: int) -> np.ndarray:
    """S "equal" contiguous segments: boundary s at floor(s*P/S); sizes differ by <= 1."""
    if S < 1 or P < S:
        raise ValueError("need 1 <= S <= P")
    return np.array([(s * P) // S for s in range(S + 1)], dtype=np.int64)


def layer_sizes(P: int, n_layers: int, seed: int,
                lo: float = 64.0, hi: float = 2.4e6) -> np.ndarray:
    """n_layers ragged tensor sizes, log-uniform in [lo, hi], rescaled to sum to P.

    Each size is floor(scale * raw) but at least 1; what is left over after the
    floor goes to the largest layer.
    """
    rng = np.random.default_rng(seed)
    u = rng.random(n_layers)
    raw = np.exp(math.log(lo) + u * math.log(hi / lo))
    scaled = np.maximum(np.floor(raw * (P / raw.sum())), 1.0).astype(np.int64)
    scaled[int(np.argmax(scaled))] += P - int(scaled.sum())
    if scaled.min() < 1 or int(scaled.sum()) != P:
        raise ValueError("layer sizes could not be rescaled to P")
    return scaled


def layer_aligned_seg_off(sizes: np.ndarray, S: int) -> np.ndarray:
    """S contiguous groups of whole layers; boundary k sits on the layer edge
    nearest to k*P/S, and every segment keeps at least one layer."""
    edges = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = len(sizes)
    if not 1 <= S <= n:
        raise ValueError("need 1 <= S <= number of layers")
    P = int(edges[-1])
    cut = [0]
    for k in range(1, S):
        target = k * P / S
        j = int(np.argmin(np.abs(edges - target)))
        j = max(j, cut[-1] + 1)          # at least one layer in segment k-1
        j = min(j, n - (S - k))          # leave one layer for each later segment
        cut.append(j)
    cut.append(n)
    return edges[np.array(cut)].astype(np.int64)


def seg_off_for(wl: Workload) -> np.ndarray:
    if wl.layers:
        return layer_aligned_seg_off(layer_sizes(wl.P, wl.layers, wl.seed), wl.S)
    return equal_seg_off(wl.P, wl.S)


# --------------------------------------------------------------------------- #
# values
# --------------------------------------------------------------------------- #
def gen_matrix(W: int, P: int, sigma: float, seed: int, ld: Optional[int] = None,
               stream: int = 0) -> np.ndarray:
    """float32 [W][ld] with columns [0,P) ~ N(0, sigma) and the padding set to a
    sentinel (so a kernel that touches padding is caught). `stream` separates the
    parameter, gradient and momentum draws of one seed."""
    ld = P if ld is None else ld
    rng = np.random.default_rng([seed, stream])
    out = np.full((W, ld), 12345.0, dtype=np.float32)
    for i in range(W):
        out[i, :P] = rng.standard_normal(P, dtype=np.float32) * np.float32(sigma)
    return out


def gen_matrix_device(W: int, P: int, sigma: float, seed: int, ld: Optional[int] = None,
                      stream: int = 0, device: str = "cuda:0", out=None):
    """Same shape/distribution as gen_matrix, drawn on the device by torch's
    generator (for the full-size workloads, where host generation is too slow).
    The values differ from gen_matrix's; parity at full size downloads what it needs.
    `out`: a [W][ld] device tensor to fill instead of a new one; float32 rows are drawn
    in place, 16-bit rows are drawn in float32 and rounded to nearest even row by row."""
    import torch
    ld = P if ld is None else ld
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream)
    if out is None:
        out = torch.empty((W, ld), dtype=torch.float32, device=device)
    assert tuple(out.shape) == (W, ld)
    row = None if out.dtype == torch.float32 else torch.empty(P, dtype=torch.float32, device=device)
    for i in range(W):
        if row is None:
            out[i, :P].normal_(0.0, sigma, generator=g)
        else:
            out[i, :P].copy_(row.normal_(0.0, sigma, generator=g))
    if ld > P:
        out[:, P:] = 12345.0
    return out


def edge_values(n: int, seed: int) -> np.ndarray:
    """n float32 values that stress rounding: signed zeros, subnormals, values
    whose sum is subnormal / overflows / cancels, plus ordinary normals."""
    rng = np.random.default_rng([seed, 99])
    specials = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754942e-38, -1.1754942e-38,
                         1.1754944e-38, 3.0e-39, -7.0e-42, 3.4028235e38, -3.4028235e38,
                         1.7014118e38, 1.0, -1.0, 1.0000001, 0.99999994, 16777216.0,
                         16777217.0, 3.0, 5e-324, np.inf, -np.inf], dtype=np.float32)
    pick = rng.integers(0, len(specials), size=n)
    out = specials[pick]
    plain = rng.random(n) < 0.5
    out = np.where(plain, rng.standard_normal(n).astype(np.float32), out)
    return out.astype(np.float32)


# --------------------------------------------------------------------------- #
# column sampling for full-size parity (mixing is independent per column)
# --------------------------------------------------------------------------- #
def sample_columns(P: int, seg_off: np.ndarray, seed: int, n_random: int = 20000,
                   halo: int = 64, ends: int = 4096) -> np.ndarray:
    """Sorted unique column ids: everything within `halo` of a segment boundary,
    the first and last `ends` columns, and n_random seeded uniform draws."""
    rng = np.random.default_rng([seed, 7])
    parts = [np.arange(0, min(ends, P)), np.arange(max(0, P - ends), P),
             rng.integers(0, P, size=n_random)]
    for b in np.asarray(seg_off, dtype=np.int64):
        parts.append(np.arange(max(0, b - halo), min(P, b + halo)))
    return np.unique(np.concatenate(parts)).astype(np.int64)


def sub_seg_off(cols: np.ndarray, seg_off: np.ndarray) -> np.ndarray:
    """Segment offsets of the sub-matrix made of the sorted columns `cols`:
    entry s = number of sampled columns that lie before seg_off[s]."""
    return np.searchsorted(cols, np.asarray(seg_off, dtype=np.int64), side="left").astype(np.int64)
