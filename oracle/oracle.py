"""ctypes front end of the plain-C CPU oracle (oracle/cx_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It imports nothing from the HIP package.  All functions take
and return NumPy arrays; outputs are fresh arrays (inputs are never modified).
Matrices are float32 [W][ld] with columns [0,P) in use; `peers[s][i]` is the row
that row i receives segment s from (Algorithm 1 of the paper).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cx_oracle.c")
_LIB = os.path.join(_HERE, "libcx_oracle.so")
_lib = None

__all__ = ["build_oracle", "mix64", "key", "draw", "uniform", "fair_draw", "topology",
           "gossip_mix", "hier_mix_f64", "hier_mix_f32", "sgd_fused_mix_f64",
           "sgd_fused_mix_f32", "pushsum_mix_f64", "pushsum_mix_f32",
           "hier_sgd_fused_mix_f64", "hier_sgd_fused_mix_f32", "gossip_mix_bf16", "f32_to_bf16",
           "bf16_to_f32", "gossip_mix_f16", "f32_to_f16", "f16_to_f32", "hier_mix16_f64", "hier_mix16_f32",
           "f64_to_bf16", "f64_to_f16", "sgd_fused_mix16_f64", "sgd_fused_mix16",
           "hier_sgd_fused_mix16_f64", "hier_sgd_fused_mix16", "narrow16", "hier_mix16",
           "pushsum_mix16", "pushsum_mix16_f64"]


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math).  CX_ORACLE_LIB names a build
    to load instead (the sanitizer test points it at an instrumented one)."""
    if os.environ.get("CX_ORACLE_LIB"):
        return os.environ["CX_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
                               "-fexcess-precision=standard", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        u64, i32, i64, f32 = ctypes.c_uint64, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        vp = ctypes.c_void_p
        lib.oracle_mix64.restype = u64
        lib.oracle_mix64.argtypes = [u64]
        lib.oracle_key.restype = u64
        lib.oracle_key.argtypes = [u64, i32, i32]
        lib.oracle_draw.restype = u64
        lib.oracle_draw.argtypes = [u64, ctypes.c_uint32]
        lib.oracle_uniform.restype = ctypes.c_uint32
        lib.oracle_uniform.argtypes = [u64, ctypes.c_uint32]
        lib.oracle_fair_draw.argtypes = [u64, i32, vp]
        lib.oracle_topology.argtypes = [u64, i32, i32, i32, i32, i32, vp]
        lib.oracle_gossip_mix.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp]
        lib.oracle_gossip_mix_bf16.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp]
        lib.oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f32_to_bf16.argtypes = [f32]
        lib.oracle_bf16_to_f32.restype = f32
        lib.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.oracle_gossip_mix_f16.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp]
        lib.oracle_f32_to_f16.restype = ctypes.c_uint16
        lib.oracle_f32_to_f16.argtypes = [f32]
        lib.oracle_f16_to_f32.restype = f32
        lib.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.oracle_hier_mix_f64.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_hier_mix16_f64.argtypes = [i32, vp, vp, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_hier_mix16_f32.argtypes = [i32, vp, vp, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_hier_mix_f32.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_sgd_fused_mix_f64.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32,
                                                 i64, i32, i64, i32, vp, vp]
        lib.oracle_sgd_fused_mix_f32.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32,
                                                 i64, i32, i64, i32, vp, vp]
        for fn in (lib.oracle_hier_sgd_fused_mix_f64, lib.oracle_hier_sgd_fused_mix_f32):
            fn.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, i32, vp, vp]
        for fn in (lib.oracle_f64_to_bf16, lib.oracle_f64_to_f16):
            fn.restype = ctypes.c_uint16
            fn.argtypes = [ctypes.c_double]
        for fn in (lib.oracle_sgd_fused_mix16_f64, lib.oracle_sgd_fused_mix16):
            fn.argtypes = [i32, vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, vp, vp]
        for fn in (lib.oracle_hier_sgd_fused_mix16_f64, lib.oracle_hier_sgd_fused_mix16):
            fn.argtypes = [i32, vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_narrow16_array.restype = None
        lib.oracle_narrow16_array.argtypes = [i32, vp, vp, i64]
        lib.oracle_hier_mix16.argtypes = [i32, vp, vp, i64, i32, i64, i32, i32, vp, vp]
        lib.oracle_pushsum_mix_f64.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32]
        lib.oracle_pushsum_mix_f32.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32]
        lib.oracle_pushsum_mix16.argtypes = [i32, vp, vp, vp, vp, vp, i64, i32, i64, i32]
        lib.oracle_pushsum_mix16_f64.argtypes = [i32, vp, vp, vp, vp, vp, i64, i32, i64, i32]
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _mat(x, dtype=np.float32):
    x = np.ascontiguousarray(x, dtype=dtype)
    if x.ndim != 2:
        raise ValueError("expected a [W][ld] matrix")
    return x


def _seg(seg_off, P):
    so = np.ascontiguousarray(seg_off, dtype=np.int64)
    if so.ndim != 1 or len(so) < 2 or so[0] != 0 or so[-1] != P or np.any(np.diff(so) < 0):
        raise ValueError("seg_off must run non-decreasing from 0 to P")
    return so


def _peers(peers, S, n):
    p = np.ascontiguousarray(peers, dtype=np.int32).reshape(S, n)
    if p.min() < 0 or p.max() >= n:
        raise ValueError("peer index out of range")
    return p


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


# ------------------------------------------------------------------ topology
def mix64(z: int) -> int:
    return int(_L().oracle_mix64(z & (2**64 - 1)))


def key(seed: int, rnd: int, seg: int) -> int:
    return int(_L().oracle_key(seed & (2**64 - 1), rnd, seg))


def draw(k: int, idx: int) -> int:
    return int(_L().oracle_draw(k, idx))


def uniform(v: int, m: int) -> int:
    return int(_L().oracle_uniform(v, m))


def fair_draw(k: int, n: int) -> np.ndarray:
    d = np.full(n, -1, dtype=np.int32)
    _check(_L().oracle_fair_draw(k, n, _p(d)), "oracle_fair_draw")
    return d


def topology(seed: int, n: int, S: int, round0: int, R: int, mode: int = 0) -> np.ndarray:
    """int32 [R][S][n] peer tables (mode 0: fair random, 1: directed exponential, 2: random
    without fair selection; +16: one table for all segments of a round)."""
    out = np.full((R, S, n), -1, dtype=np.int32)
    _check(_L().oracle_topology(seed & (2**64 - 1), n, S, round0, R, mode, _p(out)),
           "oracle_topology")
    return out


# ----------------------------------------------------------------------- mix
def gossip_mix(x, P, seg_off, peers, out=None) -> np.ndarray:
    """`out` (optional, float32, same shape, not overlapping x) receives the result; its
    padding columns are left as they are.  Without it a copy of x is made first."""
    x = _mat(x)
    W, ld = x.shape
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(peers, S, W)
    if out is None:
        out = x.copy()
    elif (out.dtype != np.float32 or out.shape != x.shape or not out.flags.c_contiguous
          or np.shares_memory(out, x)):
        raise ValueError("out must be a separate contiguous float32 array of x's shape")
    _check(_L().oracle_gossip_mix(_p(x), _p(out), ld, W, P, S, _p(so), _p(pe)), "gossip_mix")
    return out


def _hier(fn, odtype, x, P, G, seg_off, leader_peers):
    x = _mat(x)
    W, ld = x.shape
    if G < 1 or W % G:
        raise ValueError("G must divide W")
    L = W // G
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(leader_peers, S, L) if L > 1 else None
    out = x.astype(odtype)
    _check(fn(_p(x), _p(out), ld, W, P, G, S, _p(so), _p(pe)), "hier_mix")
    return out


def hier_mix_f64(x, P, G, seg_off, leader_peers) -> np.ndarray:
    return _hier(_L().oracle_hier_mix_f64, np.float64, x, P, G, seg_off, leader_peers)


def hier_mix_f32(x, P, G, seg_off, leader_peers) -> np.ndarray:
    return _hier(_L().oracle_hier_mix_f32, np.float32, x, P, G, seg_off, leader_peers)


def _fused(fn, odtype, x, v, g, lr, mu, wd, P, seg_off, peers):
    x, v, g = _mat(x), _mat(v), _mat(g)
    if not (x.shape == v.shape == g.shape):
        raise ValueError("x, v, g must have one shape")
    W, ld = x.shape
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(peers, S, W)
    xo, vo = x.astype(odtype), v.astype(odtype)
    _check(fn(_p(x), _p(v), _p(g), _p(xo), _p(vo), lr, mu, wd, ld, W, P, S, _p(so), _p(pe)),
           "sgd_fused_mix")
    return xo, vo


def sgd_fused_mix_f64(x, v, g, lr, mu, wd, P, seg_off, peers):
    return _fused(_L().oracle_sgd_fused_mix_f64, np.float64, x, v, g, lr, mu, wd, P, seg_off, peers)


def sgd_fused_mix_f32(x, v, g, lr, mu, wd, P, seg_off, peers):
    return _fused(_L().oracle_sgd_fused_mix_f32, np.float32, x, v, g, lr, mu, wd, P, seg_off, peers)


def _push(fn, odtype, x, w, P, hop, want_z):
    x = _mat(x)
    W, ld = x.shape
    w = np.ascontiguousarray(w, dtype=np.float32).reshape(W)
    if not 1 <= hop < W:
        raise ValueError("hop must be in [1, W)")
    xo, wo = x.astype(odtype), w.astype(odtype)
    zo = x.astype(odtype) if want_z else None
    _check(fn(_p(x), _p(w), _p(xo), _p(wo), _p(zo), ld, W, P, hop), "pushsum_mix")
    return xo, wo, zo


def pushsum_mix_f64(x, w, P, hop, want_z=True):
    return _push(_L().oracle_pushsum_mix_f64, np.float64, x, w, P, hop, want_z)


def pushsum_mix_f32(x, w, P, hop, want_z=True):
    return _push(_L().oracle_pushsum_mix_f32, np.float32, x, w, P, hop, want_z)


def _hier_fused(fn, odtype, x, v, g, lr, mu, wd, P, G, seg_off, leader_peers):
    x, v, g = _mat(x), _mat(v), _mat(g)
    W, ld = x.shape
    if G < 1 or W % G:
        raise ValueError("G must divide W")
    L = W // G
    if g.shape != x.shape or v.shape != (L, ld):
        raise ValueError("g must be [W][ld] and v [W/G][ld]")
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(leader_peers, S, L) if L > 1 else None
    xo, vo = x.astype(odtype), v.astype(odtype)
    _check(fn(_p(x), _p(v), _p(g), _p(xo), _p(vo), lr, mu, wd, ld, W, P, G, S, _p(so), _p(pe)),
           "hier_sgd_fused_mix")
    return xo, vo


def hier_sgd_fused_mix_f64(x, v, g, lr, mu, wd, P, G, seg_off, leader_peers):
    """Section 3.3 with gradients: x [W][ld] (leader rows read), v [W/G][ld], g [W][ld]."""
    return _hier_fused(_L().oracle_hier_sgd_fused_mix_f64, np.float64, x, v, g, lr, mu, wd, P, G,
                       seg_off, leader_peers)


def hier_sgd_fused_mix_f32(x, v, g, lr, mu, wd, P, G, seg_off, leader_peers):
    return _hier_fused(_L().oracle_hier_sgd_fused_mix_f32, np.float32, x, v, g, lr, mu, wd, P, G,
                       seg_off, leader_peers)


def f32_to_bf16(a) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of float32 values, round-to-nearest-even."""
    a = np.asarray(a, dtype=np.float32)
    fn = _L().oracle_f32_to_bf16
    return np.array([fn(float(v)) for v in a.ravel()], dtype=np.uint16).reshape(a.shape)


def bf16_to_f32(h) -> np.ndarray:
    h = np.asarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)


def _mix16(fn, name, x, P, seg_off, peers):
    x = _mat(x, dtype=np.uint16)
    W, ld = x.shape
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(peers, S, W)
    out = x.copy()
    _check(fn(_p(x), _p(out), ld, W, P, S, _p(so), _p(pe)), name)
    return out


def gossip_mix_bf16(x, P, seg_off, peers) -> np.ndarray:
    """x: uint16 [W][ld] of bfloat16 bit patterns; returns the mixed patterns."""
    return _mix16(_L().oracle_gossip_mix_bf16, "gossip_mix_bf16", x, P, seg_off, peers)


def f32_to_f16(a) -> np.ndarray:
    """IEEE binary16 bit patterns (uint16) of float32 values, round-to-nearest-even."""
    a = np.asarray(a, dtype=np.float32)
    fn = _L().oracle_f32_to_f16
    return np.array([fn(float(v)) for v in a.ravel()], dtype=np.uint16).reshape(a.shape)


def f16_to_f32(h) -> np.ndarray:
    h = np.asarray(h, dtype=np.uint16)
    fn = _L().oracle_f16_to_f32
    return np.array([fn(int(v)) for v in h.ravel()], dtype=np.float32).reshape(h.shape)


def gossip_mix_f16(x, P, seg_off, peers) -> np.ndarray:
    """x: uint16 [W][ld] of binary16 bit patterns; returns the mixed patterns."""
    return _mix16(_L().oracle_gossip_mix_f16, "gossip_mix_f16", x, P, seg_off, peers)


_FMT = {"bf16": 0, "f16": 1}


def _hier16(fn, fmt, x, out, P, G, seg_off, leader_peers):
    W, ld = x.shape
    if G < 1 or W % G:
        raise ValueError("G must divide W")
    L = W // G
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(leader_peers, S, L) if L > 1 else None
    _check(fn(_FMT[fmt], _p(x), _p(out), ld, W, P, G, S, _p(so), _p(pe)), "hier_mix16")
    return out


def hier_mix16_f64(fmt, x, P, G, seg_off, leader_peers) -> np.ndarray:
    """Hierarchical step on 16-bit rows ("bf16" or "f16" bit patterns), exact widening, double
    arithmetic, NOT rounded back: float64 [W][ld]."""
    x = _mat(x, dtype=np.uint16)
    widened = bf16_to_f32(x) if fmt == "bf16" else f16_to_f32(x)
    return _hier16(_L().oracle_hier_mix16_f64, fmt, x, widened.astype(np.float64), P, G, seg_off, leader_peers)


def hier_mix16_f32(fmt, x, P, G, seg_off, leader_peers) -> np.ndarray:
    """The same in fp32 with the fixed pairwise-tree order and one rounding to the 16-bit
    format: uint16 [W][ld]."""
    x = _mat(x, dtype=np.uint16)
    return _hier16(_L().oracle_hier_mix16_f32, fmt, x, x.copy(), P, G, seg_off, leader_peers)


# ------------------------------------------------- optimizer steps on 16-bit rows
def f64_to_bf16(a) -> np.ndarray:
    """bfloat16 bit patterns of doubles, ONE rounding to nearest even straight from the double."""
    a = np.asarray(a, dtype=np.float64)
    fn = _L().oracle_f64_to_bf16
    return np.array([fn(float(v)) for v in a.ravel()], dtype=np.uint16).reshape(a.shape)


def f64_to_f16(a) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    fn = _L().oracle_f64_to_f16
    return np.array([fn(float(v)) for v in a.ravel()], dtype=np.uint16).reshape(a.shape)


def _fused16(fn, reference, fmt, x, v, g, lr, mu, wd, P, seg_off, peers, G=None):
    x, g, v = _mat(x, dtype=np.uint16), _mat(g, dtype=np.uint16), _mat(v)
    W, ld = x.shape
    n = W if G is None else W // G
    if G is not None and (G < 1 or W % G):
        raise ValueError("G must divide W")
    if g.shape != x.shape or v.shape != (n, ld):
        raise ValueError("x, g: uint16 [W][ld]; v: float32 [W or W/G][ld]")
    so = _seg(seg_off, P)
    S = len(so) - 1
    pe = _peers(peers, S, n) if n > 1 else None
    widened = bf16_to_f32(x) if fmt == "bf16" else f16_to_f32(x)
    xo = widened.astype(np.float64) if reference else x.copy()
    vo = v.astype(np.float64) if reference else v.copy()
    args = [_FMT[fmt], _p(x), _p(v), _p(g), _p(xo), _p(vo), lr, mu, wd, ld, W, P]
    args += [S, _p(so), _p(pe)] if G is None else [G, S, _p(so), _p(pe)]
    _check(fn(*args), "sgd_fused_mix16")
    return xo, vo


def sgd_fused_mix16_f64(fmt, x, v, g, lr, mu, wd, P, seg_off, peers):
    """Momentum-SGD + mix on 16-bit parameter and gradient rows ("bf16" / "f16" bit patterns) with
    fp32 momentum, in double, NOT rounded back: (float64 x', float64 v')."""
    return _fused16(_L().oracle_sgd_fused_mix16_f64, True, fmt, x, v, g, lr, mu, wd, P, seg_off, peers)


def sgd_fused_mix16(fmt, x, v, g, lr, mu, wd, P, seg_off, peers):
    """The same with x' rounded once to the 16-bit format and v' once to fp32: (uint16, float32)."""
    return _fused16(_L().oracle_sgd_fused_mix16, False, fmt, x, v, g, lr, mu, wd, P, seg_off, peers)


def hier_sgd_fused_mix16_f64(fmt, x, v, g, lr, mu, wd, P, G, seg_off, leader_peers):
    return _fused16(_L().oracle_hier_sgd_fused_mix16_f64, True, fmt, x, v, g, lr, mu, wd, P, seg_off, leader_peers, G)


def hier_sgd_fused_mix16(fmt, x, v, g, lr, mu, wd, P, G, seg_off, leader_peers):
    return _fused16(_L().oracle_hier_sgd_fused_mix16, False, fmt, x, v, g, lr, mu, wd, P, seg_off, leader_peers, G)


def narrow16(fmt, a) -> np.ndarray:
    """Doubles -> 16-bit patterns ("bf16" / "f16"), each rounded once; the array form of f64_to_bf16 / f64_to_f16."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty(a.shape, dtype=np.uint16)
    _L().oracle_narrow16_array(_FMT[fmt], _p(a), _p(out), a.size)
    return out


def hier_mix16(fmt, x, P, G, seg_off, leader_peers) -> np.ndarray:
    """The hierarchical step on 16-bit rows in double with ONE rounding to the 16-bit format: uint16 [W][ld]."""
    x = _mat(x, dtype=np.uint16)
    return _hier16(_L().oracle_hier_mix16, fmt, x, x.copy(), P, G, seg_off, leader_peers)


def _push16(fn, odtype, fmt, x, w, P, hop, want_z):
    x = _mat(x, dtype=np.uint16)
    W, ld = x.shape
    w = np.ascontiguousarray(w, dtype=np.float32).reshape(W)
    if not 1 <= hop < W:
        raise ValueError("hop must be in [1, W)")
    xo = x.copy() if odtype == np.uint16 else np.zeros(x.shape, dtype=np.float64)
    wo = w.astype(np.float32 if odtype == np.uint16 else np.float64)
    zo = xo.copy() if want_z else None
    _check(fn(_FMT[fmt], _p(x), _p(w), _p(xo), _p(wo), _p(zo), ld, W, P, hop), "pushsum_mix16")
    return xo, wo, zo


def pushsum_mix16(fmt, x, w, P, hop, want_z=True):
    """Push-sum round on 16-bit rows ("bf16" / "f16" bit patterns, uint16 [W][ld]), fp32 weights:
    (x' patterns, w' float32, z patterns or None).  Padding columns of x' and z keep x's."""
    return _push16(_L().oracle_pushsum_mix16, np.uint16, fmt, x, w, P, hop, want_z)


def pushsum_mix16_f64(fmt, x, w, P, hop, want_z=True):
    """The same round in double arithmetic, unrounded (float64 arrays; padding columns zero)."""
    return _push16(_L().oracle_pushsum_mix16_f64, np.float64, fmt, x, w, P, hop, want_z)

