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
                 xcd_aware=-1, ordered=-1, wgs_per_cu=-1, lds_mean=-1):
        self.v = (slices, waves, nt, depth, lockstep, force_walk, cluster, xcd_aware, ordered, wgs_per_cu, lds_mean)

    def __enter__(self):
        for k, v in enumerate(self.v):
            cx.cx_set_tuning(k, v)

    def __exit__(self, *exc):
        for k in range(11):
            cx.cx_set_tuning(k, -1)


ALL_TUNINGS = [(-1, -1, -1, -1), (1, 1, 0, 2), (2, 2, 1, 4), (4, 8, 0, 2), (1, 4, 1, 8), (2, 3, 0, 8),
               (4, 4, 1, 4), (1, 2, 1, 4), (2, 5, 0, 2), (1, 2, 1, 4, 1), (4, 4, 1, 2, 1), (2, 8, 0, 4, 1),
               (1, 1, 1, 8, 1),
               # out-of-place launches: (slices, waves, nt, -, -, force_walk, cluster, xcd_aware)
               (1, 4, 1, -1, -1, 0, 1, 0), (2, 2, 0, -1, -1, 0, 7, 1), (4, 8, 1, -1, -1, 0, 64, 1),
               (4, 1, 1, 2, 0, 1, -1, -1), (2, 4, 1, 4, 1, 1, -1, -1),
               (1, 4, 1, -1, -1, 0, 3, 1, 0), (2, 2, 1, -1, -1, 0, -1, 0, 0), (1, 2, 1, -1, -1, 0, 2, 1, 1),
               # rows in cycle order forced on (small matrices run without the order table by default)
               (-1, -1, -1, -1, -1, -1, -1, -1, 1), (-1, -1, -1, -1, -1, 0, 1, 1, 1), (2, 8, 0, -1, -1, 0, 5, 0, 1),
               # in-place launches with a cap on resident workgroups per CU (last value)
               (1, 2, 1, 2, 1, 1, -1, -1, -1, 8), (2, 4, 1, 4, 0, 1, -1, -1, -1, 2), (4, 8, 0, 2, 1, 1, -1, -1, -1, 0),
               (1, 3, 1, 4, 1, 1, -1, -1, -1, 16),
               # the hierarchical mean staged through LDS (groups of 8, out of place, rows in cycle order)
               (-1, -1, -1, -1, -1, -1, -1, -1, 1, -1, 1), (-1, -1, 0, -1, -1, 0, 2, 1, 1, 2, 1)]


REL = 1e-6
TINY = 2.0 ** -150          # half the smallest fp32 subnormal: the floor of any fp32 rounding error


def once(ref64):
    """The fp64 reference rounded once to fp32 (nearest even): what the optimizer entry points
    must return bit for bit, since they carry their whole chain in fp64 registers."""
    with np.errstate(over="ignore"):
        return np.asarray(ref64, dtype=np.float64).astype(np.float32)


def within_rel(got, ref64, rel=REL):
    """The benchmark's bar as it is stated: |got - ref| <= 1e-6 * |ref| element by element (an
    absolute floor only where fp32 itself cannot resolve the reference: below its subnormal
    spacing, and an overflow to infinity where the reference exceeds the fp32 range)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref64, dtype=np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        ok = np.abs(got - ref) <= np.maximum(rel * np.abs(ref), TINY)
        ok |= np.isnan(got) & np.isnan(ref)
        ok |= np.isinf(got) & (np.abs(ref) >= 3.4028235677973366e38) & (np.sign(got) == np.sign(ref))
    return bool(ok.all())


def worst_rel(got, ref64, floor=1e-30):
    """Largest |got - ref| / |ref| over the elements with |ref| above `floor` (reported by the tests)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref64, dtype=np.float64)
    m = np.isfinite(ref) & (np.abs(ref) > floor)
    return float((np.abs(got[m] - ref[m]) / np.abs(ref[m])).max()) if m.any() else 0.0
