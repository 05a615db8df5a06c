"""Thin ctypes binding of the C-ABI HIP library (include/fsa.h), same names as the C entry
points.  Argument marshalling only: every step of the path runs inside the library's
kernels.  PyTorch is used for device memory and the current stream, nothing else.

The library must have been built (``python -m paper_2511_13645_amd.build`` or
``__graft_entry__.build()``); there is no CPU fallback -- a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfsa_hip.so")

FSA_F32, FSA_BF16, FSA_F16 = 0, 1, 2
FSA_I32, FSA_I64 = 0, 1
FSA_OK = 0
FSA_KMAX = 64
FSA_SCRATCH_FLOATS = 8 * 1024 * 1024

EXPORTS = ("fsa_sample_mean_fwd", "fsa_mean_replay_fwd", "fsa_mean_bwd", "fsa_mean_bwd_lp", "fsa_status_string",
           "fsa_sample_mean_layerwise_fwd", "fsa_sample_mean3_fwd", "fsa_mean3_replay_fwd", "fsa_mean3_bwd",
           "fsa_mean3_bwd_noalloc", "fsa_mean_bwd_ws", "fsa_mean_bwd_workspace_bytes",
           "fsa_sample_wmean_fwd", "fsa_wmean_replay_fwd", "fsa_wmean_bwd")

_lib: Optional[ctypes.CDLL] = None


class FsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


def lib() -> ctypes.CDLL:
    """Load the HIP library; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library missing: %s (build it with __graft_entry__.build())" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
        L.fsa_sample_mean_fwd.argtypes = [vp, ci, vp, i64, vp, ci, i64, vp, i64, vp, ci, u64,
                                          vp, vp, vp, vp, vp]
        L.fsa_sample_mean_fwd.restype = ci
        L.fsa_mean_replay_fwd.argtypes = [vp, ci, i64, i64, vp, vp, i64, i32, i32, vp, vp, vp]
        L.fsa_mean_replay_fwd.restype = ci
        L.fsa_mean_bwd.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, vp, i64, vp]
        L.fsa_mean_bwd.restype = ci
        L.fsa_mean_bwd_ws.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, vp, i64, vp, i64, vp]
        L.fsa_mean_bwd_ws.restype = ci
        L.fsa_mean_bwd_workspace_bytes.argtypes = [i64, i32, i32, i64]
        L.fsa_mean_bwd_workspace_bytes.restype = i64
        L.fsa_mean_bwd_lp.argtypes = [vp, vp, ci, vp, vp, i64, i32, i32, i64, vp, ci, i64, vp]
        L.fsa_mean_bwd_lp.restype = ci
        L.fsa_sample_wmean_fwd.argtypes = [vp, ci, vp, vp, i64, vp, ci, i64, vp, i64, vp, ci, u64,
                                           vp, vp, vp, vp, vp, vp, vp]
        L.fsa_sample_wmean_fwd.restype = ci
        L.fsa_wmean_replay_fwd.argtypes = [vp, ci, i64, i64, vp, vp, vp, vp, i64, i32, i32, vp, vp, vp]
        L.fsa_wmean_replay_fwd.restype = ci
        L.fsa_wmean_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i64, vp, i64, vp]
        L.fsa_wmean_bwd.restype = ci
        L.fsa_sample_mean_layerwise_fwd.argtypes = [vp, ci, vp, i64, vp, ci, i64, vp, i64, vp, u64,
                                                    vp, vp, vp, vp, vp, vp]
        L.fsa_sample_mean_layerwise_fwd.restype = ci
        L.fsa_sample_mean3_fwd.argtypes = [vp, ci, vp, i64, vp, ci, i64, vp, i64, vp, u64,
                                           vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fsa_sample_mean3_fwd.restype = ci
        L.fsa_mean3_replay_fwd.argtypes = [vp, ci, i64, i64, vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.fsa_mean3_replay_fwd.restype = ci
        L.fsa_mean3_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, vp, i64, vp, vp]
        L.fsa_mean3_bwd.restype = ci
        L.fsa_mean3_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, vp, i64, vp]
        L.fsa_mean3_bwd_noalloc.restype = ci
        L.fsa_status_string.argtypes = [ci]
        L.fsa_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fsa_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _x_dtype(x: torch.Tensor) -> int:
    if x.dtype == torch.float32:
        return FSA_F32
    if x.dtype == torch.bfloat16:
        return FSA_BF16
    if x.dtype == torch.float16:
        return FSA_F16
    raise TypeError("expected float32, bfloat16 or float16, got %s" % x.dtype)


def _indptr_type(indptr: torch.Tensor) -> int:
    if indptr.dtype == torch.int32:
        return FSA_I32
    if indptr.dtype == torch.int64:
        return FSA_I64
    raise TypeError("indptr must be int32 or int64, got %s" % indptr.dtype)


def _need(t: torch.Tensor, name: str, dtype=None) -> None:
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))


def _shape(t: Optional[torch.Tensor], name: str, shape) -> None:
    if t is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must be %s, got %s" % (name, tuple(shape), tuple(t.shape)))


def _same_device(ref: torch.Tensor, *named) -> None:
    for t, name in named:
        if t is not None and t.device != ref.device:
            raise ValueError("%s lives on %s, expected %s" % (name, t.device, ref.device))


def _stream(stream: Optional[torch.cuda.Stream], like: torch.Tensor) -> int:
    """The stream to launch on: the caller's, else the current stream of the device that holds `like`."""
    s = torch.cuda.current_stream(like.device) if stream is None else stream
    return s.cuda_stream


def fsa_sample_mean_fwd(indptr: torch.Tensor, indices: torch.Tensor, x: torch.Tensor,
                        seeds: torch.Tensor, fanouts: Sequence[int], seed: int, *,
                        out: Optional[torch.Tensor] = None, out_h1: Optional[torch.Tensor] = None,
                        out_ids1: Optional[torch.Tensor] = None, out_ids2: Optional[torch.Tensor] = None,
                        emit_h1: bool = True, emit_ids: bool = True,
                        stream: Optional[torch.cuda.Stream] = None
                        ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor], Optional[torch.Tensor]]:
    """Fused sample + mean forward.  Output tensors are allocated here (torch) unless given.
    Returns (out, out_h1, ids1, ids2); entries not asked for are None."""
    _need(indptr, "indptr"); _need(indices, "indices", torch.int32); _need(x, "x")
    _need(seeds, "seeds", torch.int32)
    fan = [int(k) for k in fanouts]
    hops = len(fan)
    B, (N, D) = seeds.shape[0], x.shape
    if indptr.shape[0] != N + 1:
        raise ValueError("indptr must have num_nodes+1 entries")
    dev = x.device
    k1 = fan[0] if hops >= 1 else 0
    k2 = fan[1] if hops >= 2 else 0
    if out is None:
        out = torch.empty((B, D), dtype=x.dtype, device=dev)
    if hops == 2 and emit_h1 and out_h1 is None:
        out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev)
    if emit_ids and out_ids1 is None:
        out_ids1 = torch.empty((B, k1), dtype=torch.int32, device=dev)
    if emit_ids and hops == 2 and out_ids2 is None:
        out_ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=dev)
    for t, n, dt, shp in ((out, "out", x.dtype, (B, D)), (out_h1, "out_h1", x.dtype, (B, k1, D)),
                          (out_ids1, "out_ids1", torch.int32, (B, k1)), (out_ids2, "out_ids2", torch.int32, (B, k1, k2))):
        if t is not None:
            _need(t, n, dt)
            _shape(t, n, shp)
    _same_device(x, (indptr, "indptr"), (indices, "indices"), (seeds, "seeds"), (out, "out"), (out_h1, "out_h1"),
                 (out_ids1, "out_ids1"), (out_ids2, "out_ids2"))
    fan_host = (ctypes.c_int32 * max(1, hops))(*fan)
    rc = lib().fsa_sample_mean_fwd(_ptr(indptr), _indptr_type(indptr), _ptr(indices), N,
                                   _ptr(x), _x_dtype(x), D, _ptr(seeds), B,
                                   ctypes.cast(fan_host, ctypes.c_void_p), hops, seed & (2**64 - 1),
                                   _ptr(out), _ptr(out_h1), _ptr(out_ids1), _ptr(out_ids2), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_sample_mean_fwd")
    return out, out_h1, out_ids1, out_ids2


def fsa_mean_replay_fwd(x: torch.Tensor, ids1: torch.Tensor, ids2: Optional[torch.Tensor] = None, *,
                        out: Optional[torch.Tensor] = None, out_h1: Optional[torch.Tensor] = None,
                        emit_h1: bool = True, stream: Optional[torch.cuda.Stream] = None
                        ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """Mean over saved IDs (no sampling).  Returns (out, out_h1)."""
    _need(x, "x"); _need(ids1, "ids1", torch.int32)
    B, k1 = ids1.shape
    N, D = x.shape
    k2 = 0
    if ids2 is not None:
        _need(ids2, "ids2", torch.int32)
        if ids2.shape[0] != B or ids2.shape[1] != k1:
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
    if out is None:
        out = torch.empty((B, D), dtype=x.dtype, device=x.device)
    if ids2 is not None and emit_h1 and out_h1 is None:
        out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=x.device)
    for t, n, shp in ((out, "out", (B, D)), (out_h1, "out_h1", (B, k1, D))):
        if t is not None:
            _need(t, n, x.dtype)
            _shape(t, n, shp)
    _same_device(x, (ids1, "ids1"), (ids2, "ids2"), (out, "out"), (out_h1, "out_h1"))
    rc = lib().fsa_mean_replay_fwd(_ptr(x), _x_dtype(x), D, N, _ptr(ids1), _ptr(ids2), B, k1, k2,
                                   _ptr(out), _ptr(out_h1), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean_replay_fwd")
    return out, out_h1


def fsa_mean_bwd(grad_out: torch.Tensor, ids1: torch.Tensor, ids2: Optional[torch.Tensor] = None,
                 grad_h1: Optional[torch.Tensor] = None, *, grad_x: torch.Tensor,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Scatter-add the mean's gradient into grad_x [N,D] fp32 (accumulated, not zeroed)."""
    _need(grad_out, "grad_out", torch.float32); _need(ids1, "ids1", torch.int32)
    _need(grad_x, "grad_x", torch.float32)
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    N = grad_x.shape[0]
    if grad_x.shape[1] != D or grad_out.shape[0] != B:
        raise ValueError("shape mismatch between grad_out, ids1 and grad_x")
    k2 = 0
    if ids2 is not None:
        _need(ids2, "ids2", torch.int32)
        if ids2.dim() != 3 or tuple(ids2.shape[:2]) != (B, k1):
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
    if grad_h1 is not None:
        _need(grad_h1, "grad_h1", torch.float32)
        _shape(grad_h1, "grad_h1", (B, k1, D))
    _same_device(grad_x, (grad_out, "grad_out"), (grad_h1, "grad_h1"), (ids1, "ids1"), (ids2, "ids2"))
    rc = lib().fsa_mean_bwd(_ptr(grad_out), _ptr(grad_h1), _ptr(ids1), _ptr(ids2), B, k1, k2, D,
                            _ptr(grad_x), N, _stream(stream, grad_x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean_bwd")
    return grad_x


def fsa_mean_bwd_workspace_bytes(B: int, k1: int, k2: int, D: int) -> int:
    """Workspace bytes fsa_mean_bwd_ws can use for this shape (0: it always takes the atomic route)."""
    return int(lib().fsa_mean_bwd_workspace_bytes(B, k1, k2, D))


def fsa_mean_bwd_ws(grad_out: torch.Tensor, ids1: torch.Tensor, ids2: Optional[torch.Tensor] = None,
                    grad_h1: Optional[torch.Tensor] = None, *, grad_x: torch.Tensor,
                    workspace: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """fsa_mean_bwd with a caller workspace (any contiguous GPU tensor; torch allocations are
    256-byte aligned): wide-row 2-hop calls then update every destination row once, without atomics."""
    _need(grad_out, "grad_out", torch.float32); _need(ids1, "ids1", torch.int32)
    _need(grad_x, "grad_x", torch.float32)
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    N = grad_x.shape[0]
    if grad_x.shape[1] != D or grad_out.shape[0] != B:
        raise ValueError("shape mismatch between grad_out, ids1 and grad_x")
    k2 = 0
    if ids2 is not None:
        _need(ids2, "ids2", torch.int32)
        if ids2.dim() != 3 or tuple(ids2.shape[:2]) != (B, k1):
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
    if grad_h1 is not None:
        _need(grad_h1, "grad_h1", torch.float32)
        _shape(grad_h1, "grad_h1", (B, k1, D))
    ws_bytes = 0
    if workspace is not None:
        _need(workspace, "workspace")
        ws_bytes = workspace.numel() * workspace.element_size()
    _same_device(grad_x, (grad_out, "grad_out"), (grad_h1, "grad_h1"), (ids1, "ids1"), (ids2, "ids2"), (workspace, "workspace"))
    rc = lib().fsa_mean_bwd_ws(_ptr(grad_out), _ptr(grad_h1), _ptr(ids1), _ptr(ids2), B, k1, k2, D,
                               _ptr(grad_x), N, _ptr(workspace), ws_bytes, _stream(stream, grad_x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean_bwd_ws")
    return grad_x


def fsa_mean_bwd_lp(grad_out: torch.Tensor, ids1: torch.Tensor, ids2: Optional[torch.Tensor] = None,
                    grad_h1: Optional[torch.Tensor] = None, *, grad_x: torch.Tensor,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Reduced-precision backward: grad_out / grad_h1 in fp32, bf16 or fp16; grad_x [N,D] either an
    fp32 master gradient or a 16-bit table added to with packed atomics (accumulated, not zeroed)."""
    _need(grad_out, "grad_out"); _need(ids1, "ids1", torch.int32); _need(grad_x, "grad_x")
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    N = grad_x.shape[0]
    if grad_x.shape[1] != D or grad_out.shape[0] != B:
        raise ValueError("shape mismatch between grad_out, ids1 and grad_x")
    k2 = 0
    if ids2 is not None:
        _need(ids2, "ids2", torch.int32)
        if ids2.dim() != 3 or tuple(ids2.shape[:2]) != (B, k1):
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
    if grad_h1 is not None:
        _need(grad_h1, "grad_h1", grad_out.dtype)
        _shape(grad_h1, "grad_h1", (B, k1, D))
    _same_device(grad_x, (grad_out, "grad_out"), (grad_h1, "grad_h1"), (ids1, "ids1"), (ids2, "ids2"))
    rc = lib().fsa_mean_bwd_lp(_ptr(grad_out), _ptr(grad_h1), _x_dtype(grad_out), _ptr(ids1), _ptr(ids2),
                               B, k1, k2, D, _ptr(grad_x), _x_dtype(grad_x), N, _stream(stream, grad_x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean_bwd_lp")
    return grad_x


def fsa_sample_mean_layerwise_fwd(indptr: torch.Tensor, indices: torch.Tensor, x: torch.Tensor, seeds: torch.Tensor,
                                  fanouts: Sequence[int], seed: int, *, emit_h1: bool = True, emit_ids: bool = True,
                                  stream: Optional[torch.cuda.Stream] = None):
    """Two-hop forward that also returns the plain hop-1 mean: (out, out_h1 | None, out_m1, ids1 | None, ids2 | None)."""
    _need(indptr, "indptr"); _need(indices, "indices", torch.int32); _need(x, "x"); _need(seeds, "seeds", torch.int32)
    fan = [int(k) for k in fanouts]
    if len(fan) != 2:
        raise ValueError("two fanouts expected")
    k1, k2 = fan
    B, (N, D), dev = seeds.shape[0], x.shape, x.device
    if indptr.shape[0] != N + 1:
        raise ValueError("indptr must have num_nodes+1 entries")
    _same_device(x, (indptr, "indptr"), (indices, "indices"), (seeds, "seeds"))
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_m1 = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev) if emit_h1 else None
    ids1 = torch.empty((B, k1), dtype=torch.int32, device=dev) if emit_ids else None
    ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=dev) if emit_ids else None
    fan_host = (ctypes.c_int32 * 2)(*fan)
    rc = lib().fsa_sample_mean_layerwise_fwd(_ptr(indptr), _indptr_type(indptr), _ptr(indices), N, _ptr(x), _x_dtype(x), D,
                                             _ptr(seeds), B, ctypes.cast(fan_host, ctypes.c_void_p), int(seed) & (2**64 - 1),
                                             _ptr(out), _ptr(out_h1), _ptr(out_m1), _ptr(ids1), _ptr(ids2), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_sample_mean_layerwise_fwd")
    return out, out_h1, out_m1, ids1, ids2


def fsa_sample_mean3_fwd(indptr: torch.Tensor, indices: torch.Tensor, x: torch.Tensor, seeds: torch.Tensor,
                         fanouts: Sequence[int], seed: int, *, emit_h2: bool = False, emit_ids: bool = True,
                         stream: Optional[torch.cuda.Stream] = None) -> dict:
    """Three-hop forward.  Returns a dict: out, out_h1, out_h2 | None, out_m1, ids1, ids2 | None, ids3 | None, cnt2."""
    _need(indptr, "indptr"); _need(indices, "indices", torch.int32); _need(x, "x"); _need(seeds, "seeds", torch.int32)
    fan = [int(k) for k in fanouts]
    if len(fan) != 3:
        raise ValueError("three fanouts expected")
    k1, k2, k3 = fan
    B, (N, D), dev = seeds.shape[0], x.shape, x.device
    if indptr.shape[0] != N + 1:
        raise ValueError("indptr must have num_nodes+1 entries")
    _same_device(x, (indptr, "indptr"), (indices, "indices"), (seeds, "seeds"))
    r = {"out": torch.empty((B, D), dtype=x.dtype, device=dev),
         "out_h1": torch.empty((B, k1, D), dtype=x.dtype, device=dev),
         "out_h2": torch.empty((B, k1, k2, D), dtype=x.dtype, device=dev) if emit_h2 else None,
         "out_m1": torch.empty((B, D), dtype=x.dtype, device=dev),
         "ids1": torch.empty((B, k1), dtype=torch.int32, device=dev),
         "ids2": torch.empty((B, k1, k2), dtype=torch.int32, device=dev) if emit_ids else None,
         "ids3": torch.empty((B, k1, k2, k3), dtype=torch.int32, device=dev) if emit_ids else None,
         "cnt2": torch.empty((B, k1), dtype=torch.int32, device=dev)}
    fan_host = (ctypes.c_int32 * 3)(*fan)
    rc = lib().fsa_sample_mean3_fwd(_ptr(indptr), _indptr_type(indptr), _ptr(indices), N, _ptr(x), _x_dtype(x), D,
                                    _ptr(seeds), B, ctypes.cast(fan_host, ctypes.c_void_p), int(seed) & (2**64 - 1),
                                    _ptr(r["out"]), _ptr(r["out_h1"]), _ptr(r["out_h2"]), _ptr(r["out_m1"]),
                                    _ptr(r["ids1"]), _ptr(r["ids2"]), _ptr(r["ids3"]), _ptr(r["cnt2"]), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_sample_mean3_fwd")
    return r


def fsa_mean3_replay_fwd(x: torch.Tensor, ids1: torch.Tensor, ids2: torch.Tensor, ids3: torch.Tensor, *,
                         emit_h2: bool = False, emit_m1: bool = True,
                         stream: Optional[torch.cuda.Stream] = None) -> dict:
    _need(x, "x"); _need(ids1, "ids1", torch.int32); _need(ids2, "ids2", torch.int32); _need(ids3, "ids3", torch.int32)
    B, k1, k2, k3 = ids3.shape
    if tuple(ids1.shape) != (B, k1) or tuple(ids2.shape) != (B, k1, k2):
        raise ValueError("ids1 / ids2 / ids3 shapes do not nest")
    N, D = x.shape
    dev = x.device
    _same_device(x, (ids1, "ids1"), (ids2, "ids2"), (ids3, "ids3"))
    r = {"out": torch.empty((B, D), dtype=x.dtype, device=dev),
         "out_h1": torch.empty((B, k1, D), dtype=x.dtype, device=dev),
         "out_h2": torch.empty((B, k1, k2, D), dtype=x.dtype, device=dev) if emit_h2 else None,
         "out_m1": torch.empty((B, D), dtype=x.dtype, device=dev) if emit_m1 else None,
         "cnt2": torch.empty((B, k1), dtype=torch.int32, device=dev)}
    rc = lib().fsa_mean3_replay_fwd(_ptr(x), _x_dtype(x), D, N, _ptr(ids1), _ptr(ids2), _ptr(ids3), B, k1, k2, k3,
                                    _ptr(r["out"]), _ptr(r["out_h1"]), _ptr(r["out_h2"]), _ptr(r["out_m1"]),
                                    _ptr(r["cnt2"]), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean3_replay_fwd")
    return r


def fsa_mean3_bwd(grad_out: torch.Tensor, ids1: torch.Tensor, ids2: torch.Tensor, ids3: torch.Tensor, *,
                  grad_h1: Optional[torch.Tensor] = None, grad_h2: Optional[torch.Tensor] = None,
                  grad_m1: Optional[torch.Tensor] = None, grad_x: torch.Tensor,
                  work: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                  noalloc: bool = False) -> torch.Tensor:
    """Scatter-add the three-hop mean's gradient into grad_x [N,D] fp32 (accumulated, not zeroed).
    noalloc=True calls fsa_mean3_bwd_noalloc: no workspace, the library's fixed scratch array."""
    _need(grad_out, "grad_out", torch.float32); _need(grad_x, "grad_x", torch.float32)
    _need(ids1, "ids1", torch.int32); _need(ids2, "ids2", torch.int32); _need(ids3, "ids3", torch.int32)
    B, k1, k2, k3 = ids3.shape
    D = grad_out.shape[1]
    _shape(ids1, "ids1", (B, k1)); _shape(ids2, "ids2", (B, k1, k2))
    _shape(grad_out, "grad_out", (B, D))
    if grad_x.dim() != 2 or grad_x.shape[1] != D:
        raise ValueError("grad_x must be [N,%d]" % D)
    _same_device(grad_x, (grad_out, "grad_out"), (grad_h1, "grad_h1"), (grad_h2, "grad_h2"), (grad_m1, "grad_m1"),
                 (ids1, "ids1"), (ids2, "ids2"), (ids3, "ids3"), (work, "work"))
    for g, name, shape in ((grad_h1, "grad_h1", (B, k1, D)), (grad_h2, "grad_h2", (B, k1, k2, D)), (grad_m1, "grad_m1", (B, D))):
        if g is not None:
            _need(g, name, torch.float32)
            if tuple(g.shape) != shape:
                raise ValueError("%s must be %s" % (name, shape))
    if noalloc:
        rc = lib().fsa_mean3_bwd_noalloc(_ptr(grad_out), _ptr(grad_h1), _ptr(grad_h2), _ptr(grad_m1), _ptr(ids1), _ptr(ids2),
                                         _ptr(ids3), B, k1, k2, k3, D, _ptr(grad_x), grad_x.shape[0], _stream(stream, grad_x))
        if rc != FSA_OK:
            raise FsaError(rc, "fsa_mean3_bwd_noalloc")
        return grad_x
    if work is None:
        work = torch.empty((B, k1, D), dtype=torch.float32, device=grad_x.device)
    elif work.numel() < B * k1 * D or work.dtype != torch.float32 or not work.is_cuda or not work.is_contiguous():
        raise ValueError("work must be a contiguous GPU tensor that holds B*k1*D floats")
    rc = lib().fsa_mean3_bwd(_ptr(grad_out), _ptr(grad_h1), _ptr(grad_h2), _ptr(grad_m1), _ptr(ids1), _ptr(ids2), _ptr(ids3),
                             B, k1, k2, k3, D, _ptr(grad_x), grad_x.shape[0], _ptr(work), _stream(stream, grad_x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_mean3_bwd")
    return grad_x


def fsa_sample_wmean_fwd(indptr: torch.Tensor, indices: torch.Tensor, edge_weight: torch.Tensor, x: torch.Tensor,
                         seeds: torch.Tensor, fanouts: Sequence[int], seed: int, *,
                         emit_h1: bool = True, emit_ids: bool = True,
                         stream: Optional[torch.cuda.Stream] = None):
    """Weighted fused sample + mean.  Returns (out, out_h1, ids1, ids2, w1, w2); IDs and weights
    are emitted together (emit_ids), entries not asked for are None."""
    _need(indptr, "indptr"); _need(indices, "indices", torch.int32); _need(x, "x")
    _need(seeds, "seeds", torch.int32); _need(edge_weight, "edge_weight", torch.float32)
    if edge_weight.shape[0] != indices.shape[0]:
        raise ValueError("edge_weight must have one entry per CSR entry")
    fan = [int(k) for k in fanouts]
    hops = len(fan)
    B, (N, D) = seeds.shape[0], x.shape
    dev = x.device
    if indptr.shape[0] != N + 1:
        raise ValueError("indptr must have num_nodes+1 entries")
    _same_device(x, (indptr, "indptr"), (indices, "indices"), (edge_weight, "edge_weight"), (seeds, "seeds"))
    k1 = fan[0] if hops >= 1 else 0
    k2 = fan[1] if hops >= 2 else 0
    out = torch.empty((B, D), dtype=x.dtype, device=dev)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=dev) if (hops == 2 and emit_h1) else None
    ids1 = torch.empty((B, k1), dtype=torch.int32, device=dev) if emit_ids else None
    w1 = torch.empty((B, k1), dtype=torch.float32, device=dev) if emit_ids else None
    ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=dev) if (emit_ids and hops == 2) else None
    w2 = torch.empty((B, k1, k2), dtype=torch.float32, device=dev) if (emit_ids and hops == 2) else None
    fan_host = (ctypes.c_int32 * max(1, hops))(*fan)
    rc = lib().fsa_sample_wmean_fwd(_ptr(indptr), _indptr_type(indptr), _ptr(indices), _ptr(edge_weight), N,
                                    _ptr(x), _x_dtype(x), D, _ptr(seeds), B,
                                    ctypes.cast(fan_host, ctypes.c_void_p), hops, seed & (2**64 - 1),
                                    _ptr(out), _ptr(out_h1), _ptr(ids1), _ptr(ids2), _ptr(w1), _ptr(w2),
                                    _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_sample_wmean_fwd")
    return out, out_h1, ids1, ids2, w1, w2


def fsa_wmean_replay_fwd(x: torch.Tensor, ids1: torch.Tensor, w1: torch.Tensor,
                         ids2: Optional[torch.Tensor] = None, w2: Optional[torch.Tensor] = None, *,
                         emit_h1: bool = True, stream: Optional[torch.cuda.Stream] = None):
    """Weighted mean over saved IDs and weights.  Returns (out, out_h1)."""
    _need(x, "x"); _need(ids1, "ids1", torch.int32); _need(w1, "w1", torch.float32)
    B, k1 = ids1.shape
    N, D = x.shape
    _shape(w1, "w1", (B, k1))
    k2 = 0
    if ids2 is not None:
        if w2 is None:
            raise ValueError("ids2 needs w2")
        _need(ids2, "ids2", torch.int32); _need(w2, "w2", torch.float32)
        if ids2.dim() != 3 or tuple(ids2.shape[:2]) != (B, k1):
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
        _shape(w2, "w2", (B, k1, k2))
    _same_device(x, (ids1, "ids1"), (w1, "w1"), (ids2, "ids2"), (w2, "w2"))
    out = torch.empty((B, D), dtype=x.dtype, device=x.device)
    out_h1 = torch.empty((B, k1, D), dtype=x.dtype, device=x.device) if (ids2 is not None and emit_h1) else None
    rc = lib().fsa_wmean_replay_fwd(_ptr(x), _x_dtype(x), D, N, _ptr(ids1), _ptr(ids2), _ptr(w1), _ptr(w2),
                                    B, k1, k2, _ptr(out), _ptr(out_h1), _stream(stream, x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_wmean_replay_fwd")
    return out, out_h1


def fsa_wmean_bwd(grad_out: torch.Tensor, ids1: torch.Tensor, w1: torch.Tensor,
                  ids2: Optional[torch.Tensor] = None, w2: Optional[torch.Tensor] = None,
                  grad_h1: Optional[torch.Tensor] = None, *, grad_x: torch.Tensor,
                  stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Weighted backward: scatter-add into grad_x [N,D] fp32 (accumulated, not zeroed)."""
    _need(grad_out, "grad_out", torch.float32); _need(ids1, "ids1", torch.int32); _need(w1, "w1", torch.float32)
    _need(grad_x, "grad_x", torch.float32)
    B, k1 = ids1.shape
    D = grad_out.shape[1]
    _shape(grad_out, "grad_out", (B, D)); _shape(w1, "w1", (B, k1))
    if grad_x.dim() != 2 or grad_x.shape[1] != D:
        raise ValueError("grad_x must be [N,%d]" % D)
    k2 = 0
    if ids2 is not None:
        if w2 is None:
            raise ValueError("ids2 needs w2")
        _need(ids2, "ids2", torch.int32); _need(w2, "w2", torch.float32)
        if ids2.dim() != 3 or tuple(ids2.shape[:2]) != (B, k1):
            raise ValueError("ids2 must be [B,k1,k2]")
        k2 = ids2.shape[2]
        _shape(w2, "w2", (B, k1, k2))
    if grad_h1 is not None:
        _need(grad_h1, "grad_h1", torch.float32)
        _shape(grad_h1, "grad_h1", (B, k1, D))
    _same_device(grad_x, (grad_out, "grad_out"), (grad_h1, "grad_h1"), (ids1, "ids1"), (ids2, "ids2"), (w1, "w1"), (w2, "w2"))
    rc = lib().fsa_wmean_bwd(_ptr(grad_out), _ptr(grad_h1), _ptr(ids1), _ptr(ids2), _ptr(w1), _ptr(w2),
                             B, k1, k2, D, _ptr(grad_x), grad_x.shape[0], _stream(stream, grad_x))
    if rc != FSA_OK:
        raise FsaError(rc, "fsa_wmean_bwd")
    return grad_x
