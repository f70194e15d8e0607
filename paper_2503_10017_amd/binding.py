"""ctypes binding of libfnn.so: argument marshalling only.

Every function here has the name and meaning of the C entry point it wraps (see
include/fnn.h, include/fnn_measure.h).  torch supplies device memory and the current stream; all arithmetic of
the matching path runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Union

import torch

FNN_F32, FNN_F16, FNN_BF16 = 0, 1, 2
FNN_MAX_D = 32
FNN_MAX_BATCH = 64

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libfnn.so")
_lib = None


class FnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({fnn_status_string(status)})")


class _Map(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("n", ctypes.c_int64), ("d", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("row_stride", ctypes.c_int64)]


class _Opts(ctypes.Structure):
    _fields_ = [("compute", ctypes.c_int32), ("max_iter", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 5)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load lib/libfnn.so (built by ``paper_2503_10017_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2503_10017_amd.build` "
                           "(there is no fallback implementation)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.fnn_status_string.restype = ctypes.c_char_p
    lib.fnn_status_string.argtypes = [i32]
    lib.fnn_workspace_bytes.restype = sz
    lib.fnn_workspace_bytes.argtypes = [i32, i64, i64, i32, i64, i32]
    lib.fnn_workspace_bytes_opts.restype = sz
    lib.fnn_workspace_bytes_opts.argtypes = [i32, i64, i64, i32, i64, vp]
    lib.fnn_nearest.restype = i32
    lib.fnn_nearest.argtypes = [i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fnn_reciprocal.restype = i32
    lib.fnn_reciprocal.argtypes = [i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fnn_reciprocal_static.restype = i32
    lib.fnn_reciprocal_static.argtypes = [i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.fnn_mutual_dense.restype = i32
    lib.fnn_mutual_dense.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fnn_blocked_workspace_bytes.restype = sz
    lib.fnn_blocked_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32]
    lib.fnn_nearest_blocked.restype = i32
    lib.fnn_nearest_blocked.argtypes = [vp, vp, i64, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.fnn_pairs_to_pixels.restype = i32
    lib.fnn_pairs_to_pixels.argtypes = [i32, vp, vp, i64, i64, i32, i64, i32, vp, vp, ctypes.c_float, ctypes.c_float,
                                        vp, vp, vp]
    lib.fnn_trace_begin.restype = i32
    lib.fnn_trace_begin.argtypes = [i32]
    lib.fnn_trace_end.restype = i32
    lib.fnn_trace_end.argtypes = [i32, vp, vp, vp, vp]
    lib.fnn_trace_kind_name.restype = ctypes.c_char_p
    lib.fnn_trace_kind_name.argtypes = [i32]
    lib.fnn_measure_ceiling.restype = i32
    lib.fnn_measure_ceiling.argtypes = [i32, i32, vp, sz, vp, vp]
    _lib = lib
    return lib


def fnn_status_string(status: int) -> str:
    return load_library().fnn_status_string(int(status)).decode()


_DTYPES = {torch.float32: FNN_F32, torch.float16: FNN_F16, torch.bfloat16: FNN_BF16}
_COMPUTE = {"f32": FNN_F32, "fp32": FNN_F32, "f16": FNN_F16, "fp16": FNN_F16, "bf16": FNN_BF16,
            FNN_F32: FNN_F32, FNN_F16: FNN_F16, FNN_BF16: FNN_BF16}

MapsLike = Union[torch.Tensor, Sequence[torch.Tensor]]


def _as_pairs(maps: MapsLike):
    """[n][d] tensor, [batch][n][d] tensor or a sequence of [n][d] tensors -> list of 2-D views."""
    if isinstance(maps, torch.Tensor):
        if maps.dim() == 2:
            return [maps]
        if maps.dim() == 3:
            return [maps[b] for b in range(maps.shape[0])]
        raise ValueError("a map is [n][d] or [batch][n][d]")
    return list(maps)


def _map_array(views):
    arr = (_Map * len(views))()
    for b, t in enumerate(views):
        if t.dim() != 2 or not t.is_cuda:
            raise ValueError("maps must be 2-D device tensors")
        if t.dtype not in _DTYPES:
            raise ValueError(f"unsupported map dtype {t.dtype}")
        if t.shape[1] > 1 and t.stride(1) != 1:
            raise ValueError("channels of a map must be contiguous")
        arr[b].data = t.data_ptr()
        arr[b].n = t.shape[0]
        arr[b].d = t.shape[1]
        arr[b].dtype = _DTYPES[t.dtype]
        arr[b].row_stride = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return arr


FNN_FLAG_NORMALIZE = 1
FNN_FLAG_HALF_ACCUMULATE = 2
FNN_FLAG_L2 = 4
FNN_FLAG_SPLIT = 8


def _opts(compute, max_iter=0, normalize=False, half_accumulate=False, l2=False, split=False):
    o = _Opts()
    o.compute = _COMPUTE[compute]
    o.max_iter = int(max_iter)
    o.flags = ((FNN_FLAG_NORMALIZE if normalize else 0) | (FNN_FLAG_HALF_ACCUMULATE if half_accumulate else 0) |
               (FNN_FLAG_L2 if l2 else 0) | (FNN_FLAG_SPLIT if split else 0))
    return o


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream, device):
    if stream is None:
        stream = torch.cuda.current_stream(device)
    return ctypes.c_void_p(stream.cuda_stream)


def fnn_workspace_bytes(batch: int, n: int, m: int, d: int, n_queries: int, compute) -> int:
    return int(load_library().fnn_workspace_bytes(batch, n, m, d, n_queries, _COMPUTE[compute]))


def fnn_workspace_bytes_opts(batch: int, n: int, m: int, d: int, n_queries: int, compute, max_iter: int = 0,
                             normalize: bool = False, l2: bool = False, split: bool = False) -> int:
    """Workspace for a call made with these options (0 when shape or options are invalid)."""
    o = _opts(compute, max_iter, normalize, l2=l2, split=split)
    return int(load_library().fnn_workspace_bytes_opts(batch, n, m, d, n_queries, ctypes.byref(o)))


def _workspace(workspace, need, device):
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def fnn_nearest(src: MapsLike, tgt: MapsLike, q_idx: Optional[torch.Tensor] = None,
                nq: Optional[int] = None, nq_active: Optional[torch.Tensor] = None, compute="f16",
                out_idx: Optional[torch.Tensor] = None, out_score: Optional[torch.Tensor] = None,
                want_score: bool = True, normalize: bool = False, l2: bool = False, split: bool = False,
                workspace: Optional[torch.Tensor] = None, stream=None):
    """One-directional search; returns (out_idx int32[batch][nq], out_score float32[batch][nq] or None).
    ``l2`` sets FNN_FLAG_L2 (scores are then -1/2 of the squared distance), ``split`` FNN_FLAG_SPLIT
    (two-term fp16 representation of fp32 descriptors, compute "f16" only)."""
    lib = load_library()
    sv, tv = _as_pairs(src), _as_pairs(tgt)
    batch = len(sv)
    device = sv[0].device
    if nq is None:
        nq = q_idx.shape[-1] if q_idx is not None else sv[0].shape[0]
    if out_idx is None:
        out_idx = torch.empty((batch, nq), dtype=torch.int32, device=device)
    if out_score is None and want_score:
        out_score = torch.empty((batch, nq), dtype=torch.float32, device=device)
    o = _opts(compute, normalize=normalize, l2=l2, split=split)
    need = fnn_workspace_bytes_opts(batch, sv[0].shape[0], tv[0].shape[0], sv[0].shape[1], nq, compute, l2=l2, split=split)
    workspace = _workspace(workspace, need, device)
    sa, ta = _map_array(sv), _map_array(tv)
    st = lib.fnn_nearest(batch, ctypes.cast(sa, ctypes.c_void_p), _ptr(q_idx), nq, _ptr(nq_active),
                         ctypes.cast(ta, ctypes.c_void_p), ctypes.byref(o), _ptr(out_idx), _ptr(out_score),
                         _ptr(workspace), workspace.numel(), _stream_ptr(stream, device))
    if st != 0:
        raise FnnError(st, "fnn_nearest")
    return out_idx, out_score


def fnn_reciprocal(d1: MapsLike, d2: MapsLike, seeds: torch.Tensor, max_iter: int = 10, compute="f16",
                   out: Optional[dict] = None, normalize: bool = False, l2: bool = False, split: bool = False,
                   workspace: Optional[torch.Tensor] = None, stream=None):
    """The FastNN iteration; returns a dict of device tensors
    seed_i, seed_j, seed_iter [batch][n_seeds], pairs [batch][n_seeds][2], n_pairs [batch]."""
    lib = load_library()
    v1, v2 = _as_pairs(d1), _as_pairs(d2)
    batch = len(v1)
    device = v1[0].device
    n_seeds = seeds.shape[-1]
    if out is None:
        out = {
            "seed_i": torch.empty((batch, n_seeds), dtype=torch.int32, device=device),
            "seed_j": torch.empty((batch, n_seeds), dtype=torch.int32, device=device),
            "seed_iter": torch.empty((batch, n_seeds), dtype=torch.int32, device=device),
            "pairs": torch.empty((batch, n_seeds, 2), dtype=torch.int32, device=device),
            "n_pairs": torch.empty((batch,), dtype=torch.int32, device=device),
        }
    o = _opts(compute, max_iter, normalize, l2=l2, split=split)
    need = fnn_workspace_bytes_opts(batch, v1[0].shape[0], v2[0].shape[0], v1[0].shape[1], n_seeds, compute, l2=l2, split=split)
    workspace = _workspace(workspace, need, device)
    a1, a2 = _map_array(v1), _map_array(v2)
    st = lib.fnn_reciprocal(batch, ctypes.cast(a1, ctypes.c_void_p), ctypes.cast(a2, ctypes.c_void_p),
                            _ptr(seeds), n_seeds, ctypes.byref(o),
                            _ptr(out["seed_i"]), _ptr(out["seed_j"]), _ptr(out["seed_iter"]),
                            _ptr(out["pairs"]), _ptr(out["n_pairs"]),
                            _ptr(workspace), workspace.numel(), _stream_ptr(stream, device))
    if st != 0:
        raise FnnError(st, "fnn_reciprocal")
    return out


FNN_STATIC_SCRATCH_BYTES = 48 << 20


def fnn_reciprocal_static(d1: MapsLike, d2: MapsLike, seeds: torch.Tensor, out: dict, max_iter: int = 10, compute="f16",
                          normalize: bool = False, l2: bool = False, split: bool = False, stream=None):
    """fnn_reciprocal on the library's own scratch array: no workspace, and this wrapper allocates
    nothing either -- ``out`` (the dict of tensors fnn_reciprocal returns) must be passed in."""
    lib = load_library()
    v1, v2 = _as_pairs(d1), _as_pairs(d2)
    batch = len(v1)
    o = _opts(compute, max_iter, normalize, l2=l2, split=split)
    a1, a2 = _map_array(v1), _map_array(v2)
    st = lib.fnn_reciprocal_static(batch, ctypes.cast(a1, ctypes.c_void_p), ctypes.cast(a2, ctypes.c_void_p),
                                   _ptr(seeds), seeds.shape[-1], ctypes.byref(o),
                                   _ptr(out["seed_i"]), _ptr(out["seed_j"]), _ptr(out["seed_iter"]),
                                   _ptr(out["pairs"]), _ptr(out["n_pairs"]), _stream_ptr(stream, v1[0].device))
    if st != 0:
        raise FnnError(st, "fnn_reciprocal_static")
    return out


def fnn_mutual_dense(d1: MapsLike, d2: MapsLike, compute="f16", out: Optional[dict] = None,
                     normalize: bool = False, l2: bool = False, split: bool = False, workspace: Optional[torch.Tensor] = None,
                     stream=None):
    """All-pairs mutual nearest neighbours; returns a dict of device tensors
    nn12, s12 [batch][n], nn21, s21 [batch][m], pairs [batch][min(n,m)][2], n_pairs [batch]."""
    lib = load_library()
    v1, v2 = _as_pairs(d1), _as_pairs(d2)
    batch = len(v1)
    device = v1[0].device
    n, m = v1[0].shape[0], v2[0].shape[0]
    if out is None:
        out = {
            "nn12": torch.empty((batch, n), dtype=torch.int32, device=device),
            "s12": torch.empty((batch, n), dtype=torch.float32, device=device),
            "nn21": torch.empty((batch, m), dtype=torch.int32, device=device),
            "s21": torch.empty((batch, m), dtype=torch.float32, device=device),
            "pairs": torch.empty((batch, min(n, m), 2), dtype=torch.int32, device=device),
            "n_pairs": torch.empty((batch,), dtype=torch.int32, device=device),
        }
    o = _opts(compute, normalize=normalize, l2=l2, split=split)
    need = fnn_workspace_bytes_opts(batch, n, m, v1[0].shape[1], 0, compute, l2=l2, split=split)
    workspace = _workspace(workspace, need, device)
    a1, a2 = _map_array(v1), _map_array(v2)
    st = lib.fnn_mutual_dense(batch, ctypes.cast(a1, ctypes.c_void_p), ctypes.cast(a2, ctypes.c_void_p),
                              ctypes.byref(o), _ptr(out["nn12"]), _ptr(out.get("s12")), _ptr(out["nn21"]),
                              _ptr(out.get("s21")), _ptr(out["pairs"]), _ptr(out["n_pairs"]),
                              _ptr(workspace), workspace.numel(), _stream_ptr(stream, device))
    if st != 0:
        raise FnnError(st, "fnn_mutual_dense")
    return out


def fnn_nearest_blocked(src: torch.Tensor, tgt: torch.Tensor, block_rows: int, block_cols: int = 0,
                        q_idx: Optional[torch.Tensor] = None, compute="f16", normalize: bool = False,
                        half_accumulate: bool = False, workspace: Optional[torch.Tensor] = None, stream=None):
    """The paper's blocked schedules (block_cols == 0: single loop, else double loop) on one pair;
    returns (out_idx int32[nq], out_score float32[nq])."""
    lib = load_library()
    device = src.device
    nq = q_idx.shape[-1] if q_idx is not None else src.shape[0]
    out_idx = torch.empty((nq,), dtype=torch.int32, device=device)
    out_score = torch.empty((nq,), dtype=torch.float32, device=device)
    need = int(lib.fnn_blocked_workspace_bytes(src.shape[0], tgt.shape[0], src.shape[1], block_rows, block_cols,
                                               _COMPUTE[compute]))
    workspace = _workspace(workspace, need, device)
    o = _opts(compute, normalize=normalize, half_accumulate=half_accumulate)
    sa, ta = _map_array([src]), _map_array([tgt])
    st = lib.fnn_nearest_blocked(ctypes.cast(sa, ctypes.c_void_p), _ptr(q_idx), nq, ctypes.cast(ta, ctypes.c_void_p),
                                 ctypes.byref(o), block_rows, block_cols, _ptr(out_idx), _ptr(out_score),
                                 _ptr(workspace), workspace.numel(), _stream_ptr(stream, device))
    if st != 0:
        raise FnnError(st, "fnn_nearest_blocked")
    return out_idx, out_score


def fnn_pairs_to_pixels(pairs: torch.Tensor, n_pairs: torch.Tensor, n: int, width1: int, m: int, width2: int,
                        conf1: Optional[torch.Tensor] = None, conf2: Optional[torch.Tensor] = None,
                        min_conf1: float = 0.0, min_conf2: float = 0.0, stream=None):
    """Matches as pixel coordinates with an optional confidence filter; ``pairs`` int32[batch][max_pairs][2].
    Returns (out_xy int32[batch][max_pairs][4], out_count int32[batch])."""
    lib = load_library()
    batch, max_pairs = pairs.shape[0], pairs.shape[1]
    device = pairs.device
    out_xy = torch.empty((batch, max_pairs, 4), dtype=torch.int32, device=device)
    out_count = torch.empty((batch,), dtype=torch.int32, device=device)
    st = lib.fnn_pairs_to_pixels(batch, _ptr(pairs), _ptr(n_pairs), max_pairs, n, width1, m, width2, _ptr(conf1),
                                 _ptr(conf2), float(min_conf1), float(min_conf2), _ptr(out_xy), _ptr(out_count),
                                 _stream_ptr(stream, device))
    if st != 0:
        raise FnnError(st, "fnn_pairs_to_pixels")
    return out_xy, out_count


def fnn_trace_begin(max_kernels: int = 4096) -> None:
    st = load_library().fnn_trace_begin(int(max_kernels))
    if st != 0:
        raise FnnError(st, "fnn_trace_begin")


def fnn_trace_end(capacity: int = 4096, details: bool = False):
    """Returns a list of (kernel name, milliseconds) in launch order and closes the trace; with
    ``details`` the entries are (kernel name, milliseconds, detail) -- see include/fnn_measure.h."""
    lib = load_library()
    kinds = (ctypes.c_int32 * capacity)()
    ms = (ctypes.c_float * capacity)()
    det = (ctypes.c_int32 * capacity)()
    n = ctypes.c_int32(0)
    st = lib.fnn_trace_end(capacity, kinds, ms, det, ctypes.byref(n))
    if st != 0:
        raise FnnError(st, "fnn_trace_end")
    count = min(int(n.value), capacity)
    if details:
        return [(lib.fnn_trace_kind_name(kinds[i]).decode(), float(ms[i]), int(det[i])) for i in range(count)]
    return [(lib.fnn_trace_kind_name(kinds[i]).decode(), float(ms[i])) for i in range(count)]


def fnn_measure_ceiling(mix: int, blocks_per_wave: int = 65536, scratch: Optional[torch.Tensor] = None, stream=None) -> float:
    """Nanoseconds per 32x32 score block and SIMD for the bare instruction mix ``mix`` (see fnn_measure.h); waits for the result."""
    lib = load_library()
    if scratch is None:
        scratch = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    ns = ctypes.c_float(0.0)
    st = lib.fnn_measure_ceiling(mix, blocks_per_wave, _ptr(scratch), scratch.numel() * scratch.element_size(),
                                 ctypes.byref(ns), _stream_ptr(stream, scratch.device))
    if st != 0:
        raise FnnError(st, "fnn_measure_ceiling")
    return float(ns.value)
