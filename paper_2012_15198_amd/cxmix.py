"""Thin ctypes binding of the C-ABI library (include/cx_mix.h).

Argument marshalling only: every step of the path runs inside libcxmix.so.  The
functions carry the names of the C entry points.  Device buffers are torch tensors
(torch provides device memory and streams, nothing else); host tables are NumPy
arrays.  There is no CPU fallback: if the library has not been built, importing
the symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcxmix.so")

CX_MAX_ROWS = 1024
CX_OK = 0
STATUS = {0: "CX_OK", -1: "CX_ERR_NULL", -2: "CX_ERR_SHAPE", -3: "CX_ERR_SEGMENTS",
          -4: "CX_ERR_PEERS", -5: "CX_ERR_ALIGN", -6: "CX_ERR_ALIAS", -7: "CX_ERR_HIP",
          -8: "CX_ERR_UNSUPPORTED", -9: "CX_ERR_MEMORY"}
CX_TOPO_FAIR, CX_TOPO_DIRECTED_EXP, CX_TOPO_UNFAIR, CX_TOPO_SAME_ALL_SEGMENTS = 0, 1, 2, 16
TUNE_SLICES, TUNE_WAVES, TUNE_NONTEMPORAL, TUNE_DEPTH = 0, 1, 2, 3
TUNE_LOCKSTEP, TUNE_FORCE_WALK, TUNE_CLUSTER, TUNE_XCD_AWARE, TUNE_ORDERED, TUNE_WGS_PER_CU = 4, 5, 6, 7, 8, 9
TUNE_LDS_MEAN = 10

EXPORTS = ["cx_status_string", "cx_abi_version", "cx_topology_gen", "cx_check_segments",
           "cx_check_peers", "cx_gossip_mix", "cx_hier_mix", "cx_pushsum_mix",
           "cx_sgd_fused_mix", "cx_hier_sgd_fused_mix", "cx_gossip_mix_noalloc", "cx_gossip_mix_bf16", "cx_gossip_mix_f16", "cx_hier_mix_bf16", "cx_hier_mix_f16",
           "cx_sgd_fused_mix_bf16", "cx_sgd_fused_mix_f16", "cx_hier_sgd_fused_mix_bf16", "cx_hier_sgd_fused_mix_f16",
           "cx_pushsum_mix_bf16", "cx_pushsum_mix_f16",
           "cx_hbm_alloc", "cx_hbm_free", "cx_copy_baseline", "cx_set_tuning",
           "cx_get_tuning"]


class CxError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {STATUS.get(status, status)}")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it was not built (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2012_15198_amd.build` (hipcc, gfx950)")
    # torch first: its wheel carries its own HIP runtime, and the library must bind to the SAME runtime
    # instance that owns the tensors and streams it is handed (loaded the other way round, the two end
    # up on different instances and every launch on a torch stream fails with CX_ERR_HIP)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, u32, u64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64
    f32, vp = ctypes.c_float, ctypes.c_void_p
    L.cx_status_string.restype = ctypes.c_char_p
    L.cx_status_string.argtypes = [ctypes.c_int]
    L.cx_abi_version.restype = ctypes.c_int
    L.cx_abi_version.argtypes = []
    L.cx_topology_gen.argtypes = [u64, i32, i32, i32, i32, i32, vp]
    L.cx_check_segments.argtypes = [vp, i32, i64]
    L.cx_check_peers.argtypes = [vp, i32, i32, i32]
    L.cx_gossip_mix.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp, u32, vp]
    L.cx_gossip_mix_noalloc.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp, u32, vp]
    L.cx_gossip_mix_bf16.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp, u32, vp]
    L.cx_gossip_mix_f16.argtypes = [vp, vp, i64, i32, i64, i32, vp, vp, u32, vp]
    L.cx_hier_mix_bf16.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp, u32, vp]
    L.cx_hier_mix_f16.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp, u32, vp]
    L.cx_hier_mix.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp, u32, vp]
    L.cx_pushsum_mix.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32, u32, vp]
    L.cx_sgd_fused_mix.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32,
                                   vp, vp, u32, vp]
    L.cx_hier_sgd_fused_mix.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, i32,
                                        vp, vp, u32, vp]
    for name in ("cx_sgd_fused_mix_bf16", "cx_sgd_fused_mix_f16"):
        getattr(L, name).argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, vp, vp, u32, vp]
    for name in ("cx_hier_sgd_fused_mix_bf16", "cx_hier_sgd_fused_mix_f16"):
        getattr(L, name).argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, i64, i32, i64, i32, i32, vp, vp, u32, vp]
    for name in ("cx_pushsum_mix_bf16", "cx_pushsum_mix_f16"):
        getattr(L, name).argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32, u32, vp]
    L.cx_hbm_alloc.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(i64), i32, u32]
    L.cx_hbm_free.argtypes = [vp]
    L.cx_copy_baseline.argtypes = [vp, vp, i64, vp]
    L.cx_set_tuning.argtypes = [i32, i32]
    L.cx_get_tuning.argtypes = [i32]
    for name in EXPORTS:
        if name != "cx_status_string":
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _ok(fn: str, status: int) -> None:
    if status != CX_OK:
        raise CxError(fn, status)


def _dptr(t) -> Optional[int]:
    """Raw address of a torch tensor (device or host) or None."""
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _shape(x, elem_size=4):
    """(rows, ld) of the matrix that fixes a call's geometry."""
    _matrix("x_in", x, None, None, elem_size)
    return x.shape[0], x.stride(0)


def _matrix(name, t, rows, ld, elem_size):
    """The C ABI sees one ld and raw addresses, so a tensor of another shape, stride or element
    size would send the kernels past its allocation: refuse it here."""
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name}: expected a row-major [rows][ld] tensor (use a view of the padded matrix)")
    if t.element_size() != elem_size or (elem_size == 4 and not t.is_floating_point()):
        raise ValueError(f"{name}: expected {'float32' if elem_size == 4 else '16-bit'} elements, got {t.dtype}")
    if rows is not None and t.shape[0] != rows:
        raise ValueError(f"{name}: expected {rows} rows, got {t.shape[0]}")
    if ld is not None and t.shape[0] > 1 and t.stride(0) != ld:
        raise ValueError(f"{name}: row stride {t.stride(0)} differs from x_in's {ld}")
    if ld is not None and t.shape[1] > ld:
        raise ValueError(f"{name}: rows longer than the leading dimension")


def _vector(name, t, n, elem_size, integer=False):
    if t.dim() != 1 or (t.numel() > 1 and t.stride(0) != 1) or t.numel() < n:
        raise ValueError(f"{name}: expected a contiguous vector of at least {n} elements")
    if t.element_size() != elem_size or t.is_floating_point() == integer:
        raise ValueError(f"{name}: unexpected element type {t.dtype}")


def _tables(x_in, P, seg_off_dev, peers_dev, n):
    """S, after checking the device tables' types and sizes (their CONTENT is checked on the host
    mirrors by cx_check_segments / cx_check_peers)."""
    if seg_off_dev.dim() != 1 or seg_off_dev.numel() < 2:
        raise ValueError("seg_off_dev: expected int64 [S+1]")
    S = seg_off_dev.numel() - 1
    _vector("seg_off_dev", seg_off_dev, S + 1, 8, integer=True)
    if peers_dev is not None:
        if not peers_dev.is_contiguous() or peers_dev.numel() != S * n:
            raise ValueError(f"peers_dev: expected a contiguous int32 [S={S}][n={n}] table")
        _vector("peers_dev", peers_dev.reshape(-1), S * n, 4, integer=True)
    if P < 1 or P > x_in.shape[1]:
        raise ValueError("P must lie in [1, row length]")
    return S


def _same_device(*tensors):
    """Last check before the call: every buffer lives on one GPU."""
    first = tensors[0]
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("expected device tensors (the mixing calls take device pointers)")
        if t.device != first.device:
            raise ValueError(f"buffers on different devices: {t.device} and {first.device}")


# ----------------------------------------------------------------------------- host calls
def cx_status_string(status: int) -> str:
    return lib().cx_status_string(status).decode()


def cx_abi_version() -> int:
    return lib().cx_abi_version()


def cx_topology_gen(seed: int, n: int, S: int, round0: int, R: int, mode: int = 0,
                    out: Optional[np.ndarray] = None) -> np.ndarray:
    """int32 [R][S][n] peer tables on the host (see include/cx_mix.h)."""
    if out is None:
        out = np.empty((max(R, 0), max(S, 0), max(n, 0)), dtype=np.int32)
    _ok("cx_topology_gen", lib().cx_topology_gen(seed & (2**64 - 1), n, S, round0, R, mode,
                                                 out.ctypes.data))
    return out


def cx_check_segments(seg_off_host: np.ndarray, P: int) -> None:
    so = np.ascontiguousarray(seg_off_host, dtype=np.int64)
    _ok("cx_check_segments", lib().cx_check_segments(so.ctypes.data, len(so) - 1, P))


def cx_check_peers(peers_host: np.ndarray, mode: int = CX_TOPO_FAIR) -> None:
    """Raises unless one round's [S][n] table is what `mode` promises (see include/cx_mix.h):
    a fixed-point-free permutation per segment, or, for CX_TOPO_UNFAIR, entries in range that never
    name their own row (then mix out of place)."""
    p = np.ascontiguousarray(peers_host, dtype=np.int32)
    if p.ndim != 2:
        raise ValueError("expected one round's [S][n] table")
    _ok("cx_check_peers", lib().cx_check_peers(p.ctypes.data, p.shape[0], p.shape[1], mode))


def cx_set_tuning(key: int, value: int) -> None:
    _ok("cx_set_tuning", lib().cx_set_tuning(key, value))


def cx_get_tuning(key: int) -> int:
    return lib().cx_get_tuning(key)


# --------------------------------------------------------------------------- device calls
def cx_gossip_mix(x_in, x_out, P: int, seg_off_dev, peers_dev, flags: int = 0, stream=None):
    W, ld = _shape(x_in)
    _matrix("x_out", x_out, W, ld, 4)
    S = _tables(x_in, P, seg_off_dev, peers_dev, W)
    _same_device(x_in, x_out, seg_off_dev, peers_dev)
    _ok("cx_gossip_mix", lib().cx_gossip_mix(_dptr(x_in), _dptr(x_out), ld, W, P, S,
                                             _dptr(seg_off_dev), _dptr(peers_dev), flags,
                                             _stream(stream)))


def cx_gossip_mix_noalloc(x_in, x_out, P: int, seg_off_dev, peers_dev, flags: int = 0, stream=None):
    """cx_gossip_mix with its scratch in a static device array (out of place only)."""
    W, ld = _shape(x_in)
    _matrix("x_out", x_out, W, ld, 4)
    S = _tables(x_in, P, seg_off_dev, peers_dev, W)
    _same_device(x_in, x_out, seg_off_dev, peers_dev)
    _ok("cx_gossip_mix_noalloc", lib().cx_gossip_mix_noalloc(_dptr(x_in), _dptr(x_out), ld, W, P, S,
                                                             _dptr(seg_off_dev), _dptr(peers_dev), flags,
                                                             _stream(stream)))


def _mix16(name, x_in, x_out, P, seg_off_dev, peers_dev, flags, stream):
    W, ld = _shape(x_in, 2)
    _matrix("x_out", x_out, W, ld, 2)
    S = _tables(x_in, P, seg_off_dev, peers_dev, W)
    _same_device(x_in, x_out, seg_off_dev, peers_dev)
    _ok(name, getattr(lib(), name)(_dptr(x_in), _dptr(x_out), ld, W, P, S, _dptr(seg_off_dev),
                                   _dptr(peers_dev), flags, _stream(stream)))


def cx_gossip_mix_bf16(x_in, x_out, P: int, seg_off_dev, peers_dev, flags: int = 0, stream=None):
    """x: torch.bfloat16 (or int16 bit patterns) [W][ld]."""
    _mix16("cx_gossip_mix_bf16", x_in, x_out, P, seg_off_dev, peers_dev, flags, stream)


def cx_gossip_mix_f16(x_in, x_out, P: int, seg_off_dev, peers_dev, flags: int = 0, stream=None):
    """x: torch.float16 (or int16 bit patterns) [W][ld]."""
    _mix16("cx_gossip_mix_f16", x_in, x_out, P, seg_off_dev, peers_dev, flags, stream)


def _leaders(W, G):
    if G < 1 or W % G:
        raise ValueError("G must divide the number of rows")
    return W // G


def _hier16(name, x_in, x_out, P, G, seg_off_dev, leader_peers_dev, flags, stream):
    W, ld = _shape(x_in, 2)
    _matrix("x_out", x_out, W, ld, 2)
    S = _tables(x_in, P, seg_off_dev, leader_peers_dev, _leaders(W, G))
    _same_device(x_in, x_out, seg_off_dev, leader_peers_dev)
    _ok(name, getattr(lib(), name)(_dptr(x_in), _dptr(x_out), ld, W, P, G, S, _dptr(seg_off_dev),
                                   _dptr(leader_peers_dev), flags, _stream(stream)))


def cx_hier_mix_bf16(x_in, x_out, P: int, G: int, seg_off_dev, leader_peers_dev, flags: int = 0, stream=None):
    """x: torch.bfloat16 (or int16 bit patterns) [W][ld]."""
    _hier16("cx_hier_mix_bf16", x_in, x_out, P, G, seg_off_dev, leader_peers_dev, flags, stream)


def cx_hier_mix_f16(x_in, x_out, P: int, G: int, seg_off_dev, leader_peers_dev, flags: int = 0, stream=None):
    """x: torch.float16 (or int16 bit patterns) [W][ld]."""
    _hier16("cx_hier_mix_f16", x_in, x_out, P, G, seg_off_dev, leader_peers_dev, flags, stream)


def cx_hier_mix(x_in, x_out, P: int, G: int, seg_off_dev, leader_peers_dev, flags: int = 0,
                stream=None):
    W, ld = _shape(x_in)
    _matrix("x_out", x_out, W, ld, 4)
    S = _tables(x_in, P, seg_off_dev, leader_peers_dev, _leaders(W, G))
    _same_device(x_in, x_out, seg_off_dev, leader_peers_dev)
    _ok("cx_hier_mix", lib().cx_hier_mix(_dptr(x_in), _dptr(x_out), ld, W, P, G, S,
                                         _dptr(seg_off_dev), _dptr(leader_peers_dev), flags,
                                         _stream(stream)))


def cx_pushsum_mix(x_in, x_out, w_in, w_out, z_out, P: int, hop: int, flags: int = 0,
                   stream=None):
    W, ld = _shape(x_in)
    _matrix("x_out", x_out, W, ld, 4)
    if z_out is not None:
        _matrix("z_out", z_out, W, ld, 4)
    _vector("w_in", w_in, W, 4)
    _vector("w_out", w_out, W, 4)
    if P < 1 or P > x_in.shape[1]:
        raise ValueError("P must lie in [1, row length]")
    _same_device(x_in, x_out, w_in, w_out, z_out)
    _ok("cx_pushsum_mix", lib().cx_pushsum_mix(_dptr(x_in), _dptr(x_out), _dptr(w_in),
                                               _dptr(w_out), _dptr(z_out), ld, W, P, hop, flags,
                                               _stream(stream)))


def _pushsum16(name, x_in, x_out, w_in, w_out, z_out, P, hop, flags, stream):
    W, ld = _shape(x_in, 2)
    _matrix("x_out", x_out, W, ld, 2)
    if z_out is not None:
        _matrix("z_out", z_out, W, ld, 2)
    _vector("w_in", w_in, W, 4)
    _vector("w_out", w_out, W, 4)
    if P < 1 or P > x_in.shape[1]:
        raise ValueError("P must lie in [1, row length]")
    _same_device(x_in, x_out, w_in, w_out, z_out)
    _ok(name, getattr(lib(), name)(_dptr(x_in), _dptr(x_out), _dptr(w_in), _dptr(w_out), _dptr(z_out), ld, W, P, hop,
                                   flags, _stream(stream)))


def cx_pushsum_mix_bf16(x_in, x_out, w_in, w_out, z_out, P: int, hop: int, flags: int = 0, stream=None):
    """x, z: torch.bfloat16 (or int16 bit patterns) [W][ld]; w: float32 [W]."""
    _pushsum16("cx_pushsum_mix_bf16", x_in, x_out, w_in, w_out, z_out, P, hop, flags, stream)


def cx_pushsum_mix_f16(x_in, x_out, w_in, w_out, z_out, P: int, hop: int, flags: int = 0, stream=None):
    """x, z: torch.float16 (or int16 bit patterns) [W][ld]; w: float32 [W]."""
    _pushsum16("cx_pushsum_mix_f16", x_in, x_out, w_in, w_out, z_out, P, hop, flags, stream)


def cx_sgd_fused_mix(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int,
                     seg_off_dev, peers_dev, flags: int = 0, stream=None):
    W, ld = _shape(x_in)
    for name, t in (("x_out", x_out), ("v_in", v_in), ("v_out", v_out), ("g", g)):
        _matrix(name, t, W, ld, 4)
    S = _tables(x_in, P, seg_off_dev, peers_dev, W)
    _same_device(x_in, x_out, v_in, v_out, g, seg_off_dev, peers_dev)
    _ok("cx_sgd_fused_mix", lib().cx_sgd_fused_mix(_dptr(x_in), _dptr(x_out), _dptr(v_in),
                                                   _dptr(v_out), _dptr(g), lr, mu, wd, ld, W, P,
                                                   S, _dptr(seg_off_dev), _dptr(peers_dev), flags,
                                                   _stream(stream)))


def cx_hier_sgd_fused_mix(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int,
                          G: int, seg_off_dev, leader_peers_dev, flags: int = 0, stream=None):
    """x, g: [W][ld]; v: [W/G][ld] with the same ld (see include/cx_mix.h)."""
    W, ld = _shape(x_in)
    L = _leaders(W, G)
    for name, t, rows in (("x_out", x_out, W), ("g", g, W), ("v_in", v_in, L), ("v_out", v_out, L)):
        _matrix(name, t, rows, ld, 4)
    S = _tables(x_in, P, seg_off_dev, leader_peers_dev, L)
    _same_device(x_in, x_out, v_in, v_out, g, seg_off_dev, leader_peers_dev)
    _ok("cx_hier_sgd_fused_mix", lib().cx_hier_sgd_fused_mix(
        _dptr(x_in), _dptr(x_out), _dptr(v_in), _dptr(v_out), _dptr(g), lr, mu, wd, ld, W, P, G, S,
        _dptr(seg_off_dev), _dptr(leader_peers_dev), flags, _stream(stream)))


def _fused16(name, x_in, x_out, v_in, v_out, g, lr, mu, wd, P, seg_off_dev, peers_dev, flags, stream):
    W, ld = _shape(x_in, 2)
    for nm, t, size in (("x_out", x_out, 2), ("g", g, 2), ("v_in", v_in, 4), ("v_out", v_out, 4)):
        _matrix(nm, t, W, ld, size)
    S = _tables(x_in, P, seg_off_dev, peers_dev, W)
    _same_device(x_in, x_out, v_in, v_out, g, seg_off_dev, peers_dev)
    _ok(name, getattr(lib(), name)(_dptr(x_in), _dptr(x_out), _dptr(v_in), _dptr(v_out), _dptr(g), lr, mu, wd,
                                   ld, W, P, S, _dptr(seg_off_dev), _dptr(peers_dev), flags, _stream(stream)))


def cx_sgd_fused_mix_bf16(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int,
                          seg_off_dev, peers_dev, flags: int = 0, stream=None):
    """x, g: torch.bfloat16 (or int16 bit patterns) [W][ld]; v: float32 [W][ld], same ld."""
    _fused16("cx_sgd_fused_mix_bf16", x_in, x_out, v_in, v_out, g, lr, mu, wd, P, seg_off_dev, peers_dev, flags, stream)


def cx_sgd_fused_mix_f16(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int,
                         seg_off_dev, peers_dev, flags: int = 0, stream=None):
    """x, g: torch.float16 (or int16 bit patterns) [W][ld]; v: float32 [W][ld], same ld."""
    _fused16("cx_sgd_fused_mix_f16", x_in, x_out, v_in, v_out, g, lr, mu, wd, P, seg_off_dev, peers_dev, flags, stream)


def _hier_fused16(name, x_in, x_out, v_in, v_out, g, lr, mu, wd, P, G, seg_off_dev, leader_peers_dev, flags, stream):
    W, ld = _shape(x_in, 2)
    L = _leaders(W, G)
    for nm, t, rows, size in (("x_out", x_out, W, 2), ("g", g, W, 2), ("v_in", v_in, L, 4), ("v_out", v_out, L, 4)):
        _matrix(nm, t, rows, ld, size)
    S = _tables(x_in, P, seg_off_dev, leader_peers_dev, L)
    _same_device(x_in, x_out, v_in, v_out, g, seg_off_dev, leader_peers_dev)
    _ok(name, getattr(lib(), name)(_dptr(x_in), _dptr(x_out), _dptr(v_in), _dptr(v_out), _dptr(g), lr, mu, wd,
                                   ld, W, P, G, S, _dptr(seg_off_dev), _dptr(leader_peers_dev), flags,
                                   _stream(stream)))


def cx_hier_sgd_fused_mix_bf16(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int, G: int,
                               seg_off_dev, leader_peers_dev, flags: int = 0, stream=None):
    """x, g: bfloat16 [W][ld]; v: float32 [W/G][ld], same ld."""
    _hier_fused16("cx_hier_sgd_fused_mix_bf16", x_in, x_out, v_in, v_out, g, lr, mu, wd, P, G, seg_off_dev,
                  leader_peers_dev, flags, stream)


def cx_hier_sgd_fused_mix_f16(x_in, x_out, v_in, v_out, g, lr: float, mu: float, wd: float, P: int, G: int,
                              seg_off_dev, leader_peers_dev, flags: int = 0, stream=None):
    """x, g: float16 [W][ld]; v: float32 [W/G][ld], same ld."""
    _hier_fused16("cx_hier_sgd_fused_mix_f16", x_in, x_out, v_in, v_out, g, lr, mu, wd, P, G, seg_off_dev,
                  leader_peers_dev, flags, stream)


def cx_hbm_alloc(sizes, flags: int = 0):
    """Device addresses (ints) of len(sizes) blocks placed together; release each with cx_hbm_free."""
    n = len(sizes)
    ptrs = (ctypes.c_void_p * max(n, 1))()
    nbytes = (ctypes.c_int64 * max(n, 1))(*[int(b) for b in sizes])
    _ok("cx_hbm_alloc", lib().cx_hbm_alloc(ptrs, nbytes, n, flags))
    return [int(p) for p in ptrs[:n]]


def cx_hbm_free(ptr: int) -> None:
    _ok("cx_hbm_free", lib().cx_hbm_free(ctypes.c_void_p(ptr)))


class _HbmBlock:
    """Owner of one block of cx_hbm_alloc: torch views it through the array interface and keeps this
    object alive as long as a tensor (or a view of one) uses the memory; then the block is released."""

    def __init__(self, ptr, shape, typestr):
        self.ptr = ptr
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (ptr, False),
                                         "version": 2, "strides": None}

    def __del__(self):
        try:
            lib().cx_hbm_free(ctypes.c_void_p(self.ptr))
        except Exception:            # interpreter shutdown: the process gives the memory back
            pass


def hbm_empty(shapes, dtypes=None, device="cuda:0"):
    """Uninitialised torch tensors of the given shapes in memory from ONE cx_hbm_alloc call, so that every
    tensor is spread over the device's physical memory.  `dtypes`: one torch dtype for all (default
    float32) or one per shape; each block is handed to torch as integers of the element size and
    reinterpreted, which covers float32, float16, bfloat16 and the integer types."""
    import torch
    shapes = [tuple(int(d) for d in sh) for sh in shapes]
    if dtypes is None or isinstance(dtypes, torch.dtype):
        dtypes = [dtypes or torch.float32] * len(shapes)
    sizes = [torch.empty((), dtype=dt).element_size() for dt in dtypes]
    carrier = {4: (torch.int32, "<i4"), 2: (torch.int16, "<i2"), 1: (torch.uint8, "|u1"), 8: (torch.int64, "<i8")}
    with torch.cuda.device(device):
        ptrs = cx_hbm_alloc([int(np.prod(sh, dtype=np.int64)) * sz for sh, sz in zip(shapes, sizes)])
    out = []
    for ptr, sh, dt, sz in zip(ptrs, shapes, dtypes, sizes):
        t = torch.as_tensor(_HbmBlock(ptr, sh, carrier[sz][1]), device=device)
        if t.data_ptr() != ptr or t.dtype != carrier[sz][0]:
            raise RuntimeError("torch copied the block instead of viewing it")
        out.append(t.view(dt))
    return out


def cx_copy_baseline(src, dst, stream=None):
    if src.element_size() != 4 or dst.element_size() != 4 or dst.numel() < src.numel():
        raise ValueError("expected float32 buffers, dst at least as long as src")
    if not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("expected contiguous buffers")
    _same_device(src, dst)
    _ok("cx_copy_baseline", lib().cx_copy_baseline(_dptr(src), _dptr(dst), src.numel(),
                                                   _stream(stream)))
