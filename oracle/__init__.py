"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE, not the product).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It compiles ``fsa_oracle.cpp`` with g++ on first use (or via ``build()``) and exposes thin
numpy wrappers with the oracle's own names.  Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fsa_oracle.cpp")
_HDR = os.path.join(_HERE, "fsa_oracle.h")
_LIB = os.path.join(_HERE, "libfsa_oracle.so")

X_F32, X_BF16, X_F64 = 0, 1, 2
I32, I64 = 0, 1

_lib: Optional[ctypes.CDLL] = None


def build(force: bool = True) -> str:
    """Compile the oracle into ``libfsa_oracle.so`` next to its source."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", tmp, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
        os.replace(tmp, _LIB)
    return _LIB


def _vp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, u32, u64 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                  ctypes.c_uint32, ctypes.c_uint64)
        L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_philox4x32_10.restype = None
        L.orc_draw.argtypes = [u64, u32, u32, u32, u32]
        L.orc_draw.restype = u32
        L.orc_floyd_select.argtypes = [i64, i32, vp, vp]
        L.orc_floyd_select.restype = i32
        L.orc_sample_row.argtypes = [vp, ctypes.c_int, vp, i64, u32, i32, u64, vp, vp]
        L.orc_sample_row.restype = i32
        L.orc_sample_mean_fwd.argtypes = [vp, ctypes.c_int, vp, i64, vp, ctypes.c_int, i64,
                                          vp, i64, vp, ctypes.c_int, u64, vp, vp, vp, vp]
        L.orc_sample_mean_fwd.restype = ctypes.c_int
        L.orc_mean_replay_fwd.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp, i64, i32, i32, vp, vp]
        L.orc_mean_replay_fwd.restype = ctypes.c_int
        L.orc_mean_bwd.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, vp, i64]
        L.orc_mean_bwd.restype = ctypes.c_int
        L.orc_sample_wmean_fwd.argtypes = [vp, ctypes.c_int, vp, vp, i64, vp, ctypes.c_int, i64,
                                           vp, i64, vp, ctypes.c_int, u64, vp, vp, vp, vp, vp, vp]
        L.orc_sample_wmean_fwd.restype = ctypes.c_int
        L.orc_wmean_replay_fwd.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp, vp, vp, i64, i32, i32, vp, vp]
        L.orc_wmean_replay_fwd.restype = ctypes.c_int
        L.orc_wmean_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i64, vp, i64]
        L.orc_wmean_bwd.restype = ctypes.c_int
        L.orc_sample_mean3_fwd.argtypes = [vp, ctypes.c_int, vp, i64, vp, ctypes.c_int, i64, vp, i64, vp, u64,
                                           vp, vp, vp, vp, vp, vp, vp, vp]
        L.orc_sample_mean3_fwd.restype = ctypes.c_int
        L.orc_mean3_replay_fwd.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp, vp, i64, i32, i32, i32,
                                           vp, vp, vp, vp, vp]
        L.orc_mean3_replay_fwd.restype = ctypes.c_int
        L.orc_mean3_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, vp, i64]
        L.orc_mean3_bwd.restype = ctypes.c_int
        L.orc_round_to_bf16.argtypes = [vp, i64, vp]
        L.orc_round_to_bf16.restype = None
        L.orc_round_to_f32.argtypes = [vp, i64, vp]
        L.orc_round_to_f32.restype = None
        _lib = L
    return _lib


# ---- typed-array helpers ---------------------------------------------------------------

def _indptr_type(indptr: np.ndarray) -> int:
    if indptr.dtype == np.int32:
        return I32
    if indptr.dtype == np.int64:
        return I64
    raise TypeError("indptr must be int32 or int64")


def _x_type(x: np.ndarray, bf16: bool) -> int:
    if bf16:
        if x.dtype != np.uint16:
            raise TypeError("bf16 features are passed as their uint16 bit patterns")
        return X_BF16
    if x.dtype == np.float32:
        return X_F32
    if x.dtype == np.float64:
        return X_F64
    raise TypeError("x must be float32, float64 or uint16 (bf16 bits)")


def _c(a: np.ndarray, dtype=None) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


# ---- wrappers ---------------------------------------------------------------------------

def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_vp(c), _vp(k), _vp(o))
    return tuple(int(v) for v in o)


def draw(seed: int, node: int, hop: int, step: int, n: int) -> int:
    return int(lib().orc_draw(seed, node, hop, step, n))


def floyd_select(deg: int, k: int, t: Sequence[int]) -> np.ndarray:
    tt = np.asarray(t, dtype=np.uint32)
    if tt.size < k:
        tt = np.concatenate([tt, np.zeros(k - tt.size, dtype=np.uint32)])
    pos = np.full(max(k, 1), -1, dtype=np.int64)
    cnt = lib().orc_floyd_select(deg, k, _vp(tt), _vp(pos))
    return pos[:cnt].copy()


def sample_row(indptr: np.ndarray, indices: np.ndarray, node: int, hop: int, k: int,
               seed: int) -> Tuple[np.ndarray, np.ndarray, int]:
    indptr = _c(indptr)
    indices = _c(indices, np.int32)
    pos = np.full(k, -1, dtype=np.int64)
    ids = np.full(k, -1, dtype=np.int32)
    cnt = lib().orc_sample_row(_vp(indptr), _indptr_type(indptr), _vp(indices), node, hop, k,
                               seed, _vp(pos), _vp(ids))
    return pos, ids, int(cnt)


def sample_mean_fwd(indptr, indices, x, seeds, fanouts, seed, *, bf16=False,
                    want_h1=True, want_ids=True):
    """Returns (out, out_h1 | None, ids1 | None, ids2 | None), means in float64."""
    indptr = _c(indptr)
    indices = _c(indices, np.int32)
    x = _c(x)
    seeds = _c(seeds, np.int32)
    fan = np.asarray(list(fanouts), dtype=np.int32)
    hops = int(fan.size)
    N = indptr.shape[0] - 1
    D = x.shape[1]
    B = seeds.shape[0]
    k1 = int(fan[0])
    k2 = int(fan[1]) if hops == 2 else 0
    out = np.zeros((B, D), dtype=np.float64)
    out_h1 = np.zeros((B, k1, D), dtype=np.float64) if (hops == 2 and want_h1) else None
    ids1 = np.full((B, k1), -7, dtype=np.int32) if want_ids else None
    ids2 = np.full((B, k1, k2), -7, dtype=np.int32) if (want_ids and hops == 2) else None
    rc = lib().orc_sample_mean_fwd(_vp(indptr), _indptr_type(indptr), _vp(indices), N,
                                   _vp(x), _x_type(x, bf16), D, _vp(seeds), B, _vp(fan), hops,
                                   seed, _vp(out), _vp(out_h1), _vp(ids1), _vp(ids2))
    if rc != 0:
        raise ValueError("orc_sample_mean_fwd failed with %d" % rc)
    return out, out_h1, ids1, ids2


def mean_replay_fwd(x, ids1, ids2=None, *, bf16=False, want_h1=True):
    x = _c(x)
    ids1 = _c(ids1, np.int32)
    B, k1 = ids1.shape
    D = x.shape[1]
    k2 = 0
    if ids2 is not None:
        ids2 = _c(ids2, np.int32)
        k2 = ids2.shape[2]
    out = np.zeros((B, D), dtype=np.float64)
    out_h1 = np.zeros((B, k1, D), dtype=np.float64) if (ids2 is not None and want_h1) else None
    rc = lib().orc_mean_replay_fwd(_vp(x), _x_type(x, bf16), D, x.shape[0], _vp(ids1), _vp(ids2),
                                   B, k1, k2, _vp(out), _vp(out_h1))
    if rc != 0:
        raise ValueError("orc_mean_replay_fwd failed with %d" % rc)
    return out, out_h1


def mean_bwd(grad_out, ids1, ids2=None, grad_h1=None, *, num_nodes: int, grad_x=None):
    grad_out = _c(grad_out, np.float64)
    ids1 = _c(ids1, np.int32)
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    k2 = 0
    if ids2 is not None:
        ids2 = _c(ids2, np.int32)
        k2 = ids2.shape[2]
    if grad_h1 is not None:
        grad_h1 = _c(grad_h1, np.float64)
    if grad_x is None:
        grad_x = np.zeros((num_nodes, D), dtype=np.float64)
    rc = lib().orc_mean_bwd(_vp(grad_out), _vp(grad_h1), _vp(ids1), _vp(ids2), B, k1, k2, D,
                            _vp(grad_x), num_nodes)
    if rc != 0:
        raise ValueError("orc_mean_bwd failed with %d" % rc)
    return grad_x


def sample_mean3_fwd(indptr, indices, x, seeds, fanouts, seed, *, bf16=False, want_h2=True):
    """Three hops.  Returns a dict: out, out_h1, out_h2 | None, out_m1 (float64), ids1, ids2, ids3, cnt2."""
    indptr = _c(indptr)
    indices = _c(indices, np.int32)
    x = _c(x)
    seeds = _c(seeds, np.int32)
    fan = np.asarray(list(fanouts), dtype=np.int32)
    if fan.size != 3:
        raise ValueError("three fanouts expected")
    k1, k2, k3 = (int(v) for v in fan)
    N, D, B = indptr.shape[0] - 1, x.shape[1], seeds.shape[0]
    r = {"out": np.zeros((B, D)), "out_h1": np.zeros((B, k1, D)),
         "out_h2": np.zeros((B, k1, k2, D)) if want_h2 else None, "out_m1": np.zeros((B, D)),
         "ids1": np.full((B, k1), -7, dtype=np.int32), "ids2": np.full((B, k1, k2), -7, dtype=np.int32),
         "ids3": np.full((B, k1, k2, k3), -7, dtype=np.int32), "cnt2": np.full((B, k1), -7, dtype=np.int32)}
    rc = lib().orc_sample_mean3_fwd(_vp(indptr), _indptr_type(indptr), _vp(indices), N, _vp(x), _x_type(x, bf16), D,
                                    _vp(seeds), B, _vp(fan), seed, _vp(r["out"]), _vp(r["out_h1"]), _vp(r["out_h2"]),
                                    _vp(r["out_m1"]), _vp(r["ids1"]), _vp(r["ids2"]), _vp(r["ids3"]), _vp(r["cnt2"]))
    if rc != 0:
        raise ValueError("orc_sample_mean3_fwd failed with %d" % rc)
    return r


def mean3_replay_fwd(x, ids1, ids2, ids3, *, bf16=False, want_h2=True):
    x = _c(x)
    ids1, ids2, ids3 = _c(ids1, np.int32), _c(ids2, np.int32), _c(ids3, np.int32)
    B, k1, k2, k3 = ids3.shape
    D = x.shape[1]
    r = {"out": np.zeros((B, D)), "out_h1": np.zeros((B, k1, D)),
         "out_h2": np.zeros((B, k1, k2, D)) if want_h2 else None, "out_m1": np.zeros((B, D)),
         "cnt2": np.full((B, k1), -7, dtype=np.int32)}
    rc = lib().orc_mean3_replay_fwd(_vp(x), _x_type(x, bf16), D, x.shape[0], _vp(ids1), _vp(ids2), _vp(ids3),
                                    B, k1, k2, k3, _vp(r["out"]), _vp(r["out_h1"]), _vp(r["out_h2"]),
                                    _vp(r["out_m1"]), _vp(r["cnt2"]))
    if rc != 0:
        raise ValueError("orc_mean3_replay_fwd failed with %d" % rc)
    return r


def mean3_bwd(grad_out, ids1, ids2, ids3, *, grad_h1=None, grad_h2=None, grad_m1=None, num_nodes: int):
    grad_out = _c(grad_out, np.float64)
    ids1, ids2, ids3 = _c(ids1, np.int32), _c(ids2, np.int32), _c(ids3, np.int32)
    B, k1, k2, k3 = ids3.shape
    D = grad_out.shape[1]
    opt = [None if g is None else _c(g, np.float64) for g in (grad_h1, grad_h2, grad_m1)]
    grad_x = np.zeros((num_nodes, D), dtype=np.float64)
    rc = lib().orc_mean3_bwd(_vp(grad_out), _vp(opt[0]), _vp(opt[1]), _vp(opt[2]), _vp(ids1), _vp(ids2), _vp(ids3),
                             B, k1, k2, k3, D, _vp(grad_x), num_nodes)
    if rc != 0:
        raise ValueError("orc_mean3_bwd failed with %d" % rc)
    return grad_x


def sample_wmean_fwd(indptr, indices, edge_weight, x, seeds, fanouts, seed, *, bf16=False):
    """Weighted variant.  Returns (out, out_h1 | None, ids1, ids2 | None, w1, w2 | None)."""
    indptr = _c(indptr)
    indices = _c(indices, np.int32)
    edge_weight = _c(edge_weight, np.float32)
    x = _c(x)
    seeds = _c(seeds, np.int32)
    fan = np.asarray(list(fanouts), dtype=np.int32)
    hops = int(fan.size)
    N, D, B = indptr.shape[0] - 1, x.shape[1], seeds.shape[0]
    k1 = int(fan[0])
    k2 = int(fan[1]) if hops == 2 else 0
    out = np.zeros((B, D), dtype=np.float64)
    out_h1 = np.zeros((B, k1, D), dtype=np.float64) if hops == 2 else None
    ids1 = np.full((B, k1), -7, dtype=np.int32)
    ids2 = np.full((B, k1, k2), -7, dtype=np.int32) if hops == 2 else None
    w1 = np.full((B, k1), -7, dtype=np.float32)
    w2 = np.full((B, k1, k2), -7, dtype=np.float32) if hops == 2 else None
    rc = lib().orc_sample_wmean_fwd(_vp(indptr), _indptr_type(indptr), _vp(indices), _vp(edge_weight), N,
                                    _vp(x), _x_type(x, bf16), D, _vp(seeds), B, _vp(fan), hops, seed,
                                    _vp(out), _vp(out_h1), _vp(ids1), _vp(ids2), _vp(w1), _vp(w2))
    if rc != 0:
        raise ValueError("orc_sample_wmean_fwd failed with %d" % rc)
    return out, out_h1, ids1, ids2, w1, w2


def wmean_replay_fwd(x, ids1, w1, ids2=None, w2=None, *, bf16=False):
    x = _c(x)
    ids1 = _c(ids1, np.int32)
    w1 = _c(w1, np.float32)
    B, k1 = ids1.shape
    D = x.shape[1]
    k2 = 0
    if ids2 is not None:
        ids2 = _c(ids2, np.int32)
        w2 = _c(w2, np.float32)
        k2 = ids2.shape[2]
    out = np.zeros((B, D), dtype=np.float64)
    out_h1 = np.zeros((B, k1, D), dtype=np.float64) if ids2 is not None else None
    rc = lib().orc_wmean_replay_fwd(_vp(x), _x_type(x, bf16), D, x.shape[0], _vp(ids1), _vp(ids2), _vp(w1),
                                    _vp(w2), B, k1, k2, _vp(out), _vp(out_h1))
    if rc != 0:
        raise ValueError("orc_wmean_replay_fwd failed with %d" % rc)
    return out, out_h1


def wmean_bwd(grad_out, ids1, w1, ids2=None, w2=None, grad_h1=None, *, num_nodes: int):
    grad_out = _c(grad_out, np.float64)
    ids1 = _c(ids1, np.int32)
    w1 = _c(w1, np.float32)
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    k2 = 0
    if ids2 is not None:
        ids2 = _c(ids2, np.int32)
        w2 = _c(w2, np.float32)
        k2 = ids2.shape[2]
    if grad_h1 is not None:
        grad_h1 = _c(grad_h1, np.float64)
    grad_x = np.zeros((num_nodes, D), dtype=np.float64)
    rc = lib().orc_wmean_bwd(_vp(grad_out), _vp(grad_h1), _vp(ids1), _vp(ids2), _vp(w1), _vp(w2), B, k1, k2, D,
                             _vp(grad_x), num_nodes)
    if rc != 0:
        raise ValueError("orc_wmean_bwd failed with %d" % rc)
    return grad_x


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    a = _c(a, np.float64)
    o = np.zeros(a.shape, dtype=np.uint16)
    lib().orc_round_to_bf16(_vp(a), a.size, _vp(o))
    return o


def round_to_f32(a: np.ndarray) -> np.ndarray:
    a = _c(a, np.float64)
    o = np.zeros(a.shape, dtype=np.float32)
    lib().orc_round_to_f32(_vp(a), a.size, _vp(o))
    return o


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    w = bits.astype(np.uint32) << np.uint32(16)
    return w.view(np.float32).astype(np.float64)
