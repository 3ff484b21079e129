"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch

from paper_2012_15198_amd import cxmix as cx

DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def same_bits(a, b):
    """Bit equality, except that any NaN matches any NaN (payloads are not specified)."""
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return bool(((bits(a) == bits(b)) | (np.isnan(a) & np.isnan(b))).all())


class Tuning:
    """Context manager: set the library's launch parameters, restore defaults after."""

    def __init__(self, slices=-1, waves=-1, nt=-1, depth=-1, lockstep=-1, force_walk=-1, cluster=-1,
                 xcd_aware=-1, ordered=-1, wgs_per_cu=-1):
        self.v = (slices, waves, nt, depth, lockstep, force_walk, cluster, xcd_aware, ordered, wgs_per_cu)

    def __enter__(self):
        for k, v in enumerate(self.v):
            cx.cx_set_tuning(k, v)

    def __exit__(self, *exc):
        for k in range(10):
            cx.cx_set_tuning(k, -1)


ALL_TUNINGS = [(-1, -1, -1, -1), (1, 1, 0, 2), (2, 2, 1, 4), (4, 8, 0, 2), (1, 4, 1, 8), (2, 3, 0, 8),
               (4, 4, 1, 4), (1, 2, 1, 4), (2, 5, 0, 2), (1, 2, 1, 4, 1), (4, 4, 1, 2, 1), (2, 8, 0, 4, 1),
               (1, 1, 1, 8, 1),
               # out-of-place launches: (slices, waves, nt, -, -, force_walk, cluster, xcd_aware)
               (1, 4, 1, -1, -1, 0, 1, 0), (2, 2, 0, -1, -1, 0, 7, 1), (4, 8, 1, -1, -1, 0, 64, 1),
               (4, 1, 1, 2, 0, 1, -1, -1), (2, 4, 1, 4, 1, 1, -1, -1),
               (1, 4, 1, -1, -1, 0, 3, 1, 0), (2, 2, 1, -1, -1, 0, -1, 0, 0), (1, 2, 1, -1, -1, 0, 2, 1, 1),
               # in-place launches with a cap on resident workgroups per CU (last value)
               (1, 2, 1, 2, 1, 1, -1, -1, -1, 8), (2, 4, 1, 4, 0, 1, -1, -1, -1, 2), (4, 8, 0, 2, 1, 1, -1, -1, -1, 0),
               (1, 3, 1, 4, 1, 1, -1, -1, -1, 16)]


def fused_scales(x, v, g, lr, mu, wd, seg_off, peers):
    """Magnitudes the 1e-6 relative bound of the fused step is taken against.  The fp32 path
    rounds six times on the way to x' (wd*x, +g, mu*v, +, lr*v', x-); each rounding is
    relative to an intermediate no larger than M = |x| + lr*(mu*|v| + |g| + wd*|x|), so the
    error of x' is a few 2^-24 of max(M_own, M_partner), however small x' itself is.  For v'
    the same holds with N = mu*|v| + |g| + wd*|x|."""
    x, v, g = (np.abs(a.astype(np.float64)) for a in (x, v, g))
    n = mu * v + g + wd * x
    m = x + lr * n
    mp = m.copy()
    for s in range(len(seg_off) - 1):
        c0, c1 = seg_off[s], seg_off[s + 1]
        mp[:, c0:c1] = np.maximum(m[:, c0:c1], m[peers[s], c0:c1])
    return mp, n
