"""CPU oracle for fast reciprocal nearest-neighbour matching -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It shares no code with the HIP library and never imports it.

What each function follows:

* ``nearest``       -- the per-pixel reading of the paper's Algorithm 1 (section 3.4.3):
                       brute force over all candidates, strict improvement, lowest index
                       on ties, score = dot product in fp32 (C, ``fnn_oracle.c``).
* ``mutual_dense``  -- the "traditional mutual nearest neighbour" definition the paper
                       contrasts FastNN with (section 3.2.5, "Problem Context"): a pair
                       (i, j) is kept when j is i's best candidate and i is j's.
* ``normalize``     -- the producer step in front of the search: the matching head's maps
                       (section 3.2.4) L2-normalised per pixel, in fp32.
* ``nearest_l2``    -- the same search with dist_func = squared Euclidean distance (the other
                       reading of the undefined dist_func; differs on maps that are not unit-norm).
* ``nearest_split`` -- the same search on the two-term fp16 representation of fp32 descriptors
                       (hi*hi + hi*lo + lo*hi, fp32 sums): the precise end of HybridCast's
                       trade-off (section 3.4.4).
* ``pairs_to_pixels`` -- the step after the path: matches as (w, h) pixel coordinates (section 3.1),
                       thinned by the confidence maps of section 3.2.3.
* ``nearest_half_accumulate`` -- the "naive FP16 only" negative control of section 3.4.4.
* ``reciprocal``    -- the FastNN iteration (section 3.2.5, "FastNN Algorithm", steps 1-4),
                       step by step: U^0 = seeds, V^0 = NN_2(U^0); each iteration
                       U^{t+1} = NN_1(V^t), matches M_t are the seeds with
                       U^{t+1} = U^t, converged seeds leave, M is the union of the M_t.

Readings where the paper is silent: dist_func is the
negated dot product; ties go to the lowest index; a seed n with U^{t+1}[n] == U^t[n]
contributes the pair (U^t[n], V^t[n]); the loop stops only when every seed has converged
or after ``max_iter`` iterations; unconverged seeds are reported with iter = -1 and are
not in M; M is returned as a sorted set.

Pins: see tests/test_oracle_*.py (numpy/scipy library routines on exactly representable
inputs, closed forms, a hand-worked score-matrix example, exhaustive enumeration on tiny
inputs, invariants).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            path = _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_nearest.restype = None
        lib.oracle_nearest.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ]
        lib.oracle_nearest_l2.restype = None
        lib.oracle_nearest_l2.argtypes = lib.oracle_nearest.argtypes
        lib.oracle_normalize.restype = None
        lib.oracle_normalize.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p]
        lib.oracle_threads.restype = ctypes.c_int32
        lib.oracle_threads.argtypes = []
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads ``nearest`` runs on."""
    return int(_load().oracle_threads())


def round_fp16(x: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE binary16 (round to nearest even) -> fp32."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 (round to nearest even; finite inputs) -> fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    u = (u & np.uint64(0xFFFF0000)).astype(np.uint32)
    return u.view(np.float32).reshape(np.shape(x))


def normalize(x: np.ndarray) -> np.ndarray:
    """Every row divided by its Euclidean norm, in fp32 as the library's normalise option defines it."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty_like(x)
    _load().oracle_normalize(x.ctypes.data, x.shape[0], x.shape[1], y.ctypes.data)
    return y


def nearest(a: np.ndarray, b: np.ndarray):
    """For every row of ``a``: lowest index of the row of ``b`` with the largest dot product.

    Returns (idx int32[K], best float32[K], second float32[K]); ``best - second`` is the
    top-1/top-2 gap (0 on a tie).
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.ndim == 2 and b.ndim == 2 and a.shape[1] == b.shape[1]
    k, d = a.shape
    m = b.shape[0]
    idx = np.empty(k, dtype=np.int32)
    best = np.empty(k, dtype=np.float32)
    second = np.empty(k, dtype=np.float32)
    _load().oracle_nearest(a.ctypes.data, k, b.ctypes.data, m, d,
                           idx.ctypes.data, best.ctypes.data, second.ctypes.data)
    return idx, best, second


def nearest_l2(a: np.ndarray, b: np.ndarray):
    """For every row of ``a``: lowest index of the row of ``b`` at the smallest squared Euclidean distance.

    Returns (idx int32[K], best float32[K], second float32[K]): the smallest and second smallest
    squared distance; ``second - best`` is the gap (0 on a tie).
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.ndim == 2 and b.ndim == 2 and a.shape[1] == b.shape[1]
    k, d = a.shape
    m = b.shape[0]
    idx = np.empty(k, dtype=np.int32)
    best = np.empty(k, dtype=np.float32)
    second = np.empty(k, dtype=np.float32)
    _load().oracle_nearest_l2(a.ctypes.data, k, b.ctypes.data, m, d,
                              idx.ctypes.data, best.ctypes.data, second.ctypes.data)
    return idx, best, second


def split_fp16(x: np.ndarray):
    """x as the unevaluated sum of two binary16 numbers: hi = fp16(x), lo = fp16(x - hi), the
    difference taken in fp32 (it is exact there).  Returns (hi, lo) as float32 arrays."""
    x = np.asarray(x, dtype=np.float32)
    hi = round_fp16(x)
    lo = round_fp16(x - hi)
    return hi, lo


def nearest_split(a: np.ndarray, b: np.ndarray):
    """``nearest`` for the two-term fp16 representation of fp32 descriptors (the extension of the
    paper's HybridCast, section 3.4.4, that keeps fp32-grade scores on 16-bit matrix hardware):

        score(a, b) = sum_k a_hi[k] b_hi[k] + sum_k a_hi[k] b_lo[k] + sum_k a_lo[k] b_hi[k]

    every product exact (two 11-bit significands), accumulated in fp32 in the order written, k
    ascending within each sum; the lo*lo term (below 2^-22 of the score) is dropped by definition.
    Returns (idx, best, second) like ``nearest``.
    """
    a_hi, a_lo = split_fp16(a)
    b_hi, b_lo = split_fp16(b)
    wide_a = np.concatenate([a_hi, a_hi, a_lo], axis=1)
    wide_b = np.concatenate([b_hi, b_lo, b_hi], axis=1)
    return nearest(wide_a, wide_b)


def _search(a, b, metric):
    """(idx, best, second) with "larger is better" scores: the dot product (plain, or of the two-term
    fp16 representation), or minus the squared distance."""
    if metric == "dot":
        return nearest(a, b)
    if metric == "split":
        return nearest_split(a, b)
    if metric == "l2":
        idx, best, second = nearest_l2(a, b)
        return idx, -best, -second
    raise ValueError(f"unknown metric {metric!r}")


def nearest_half_accumulate(a: np.ndarray, b: np.ndarray):
    """The "naive FP16 only" control of the paper's HybridCast section (3.4.4): inputs rounded to
    fp16, every product rounded to fp16, the sum accumulated in fp16 (k ascending, multiply and
    add rounded separately); the selection (lowest index of the largest score) as in ``nearest``.

    numpy's float16 arithmetic rounds each operation once to binary16, which is what is meant.
    Returns (idx int32[K], best float32[K]).  O(K*M) memory: small inputs only.
    """
    a16 = np.asarray(a, dtype=np.float32).astype(np.float16)
    b16 = np.asarray(b, dtype=np.float32).astype(np.float16)
    acc = np.zeros((a16.shape[0], b16.shape[0]), dtype=np.float16)
    for k in range(a16.shape[1]):
        prod = a16[:, k][:, None] * b16[:, k][None, :]          # float16 * float16 -> float16
        acc = acc + prod                                          # float16 + float16 -> float16
    scores = acc.astype(np.float32)
    idx = np.argmax(scores, axis=1).astype(np.int32)              # first maximum = lowest index
    return idx, scores[np.arange(scores.shape[0]), idx]


def pairs_to_pixels(pairs: np.ndarray, width1: int, width2: int, n: int, m: int, conf1=None, conf2=None,
                    min_conf1: float = 0.0, min_conf2: float = 0.0) -> np.ndarray:
    """The matches (flat pixel ids) as the paper's problem statement writes them (section 3.1):
    i = (w_i, h_i), j = (w_j, h_j), keeping only matches whose confidences (section 3.2.3's maps
    c1, c2, when given) reach the thresholds.  One match at a time, in order; int32[P'][4]."""
    rows = []
    for i, j in np.asarray(pairs).reshape(-1, 2).tolist():
        if not (0 <= i < n and 0 <= j < m):
            continue
        if conf1 is not None and not (np.float32(conf1[i]) >= np.float32(min_conf1)):
            continue
        if conf2 is not None and not (np.float32(conf2[j]) >= np.float32(min_conf2)):
            continue
        rows.append((i % width1, i // width1, j % width2, j // width2))
    return np.asarray(rows, dtype=np.int32).reshape(-1, 4)


def mutual_dense(d1: np.ndarray, d2: np.ndarray, metric: str = "dot"):
    """All-pairs mutual nearest neighbours (``metric`` "dot": scores are dot products; "split": dot products of the two-term fp16 representation; "l2": scores
    are minus the squared distance).

    Returns a dict with nn12/s12/gap12 (best candidate in d2 for every row of d1),
    nn21/s21/gap21 (the other direction) and ``pairs`` int32[P][2], the (i, nn12[i]) with
    nn21[nn12[i]] == i, ascending in i.
    """
    nn12, s12, r12 = _search(d1, d2, metric)
    nn21, s21, r21 = _search(d2, d1, metric)
    i = np.arange(d1.shape[0], dtype=np.int32)
    keep = (nn12 >= 0)
    keep[keep] = nn21[nn12[keep]] == i[keep]
    pairs = np.stack([i[keep], nn12[keep]], axis=1).astype(np.int32)
    return {
        "nn12": nn12, "s12": s12, "gap12": s12 - r12,
        "nn21": nn21, "s21": s21, "gap21": s21 - r21,
        "pairs": pairs,
    }


def reciprocal(d1: np.ndarray, d2: np.ndarray, seeds: np.ndarray, max_iter: int, metric: str = "dot"):
    """The FastNN iteration from the given seed pixels of image 1 (``metric`` as in ``mutual_dense``).

    Returns a dict:
      seed_i, seed_j, seed_iter  int32[n_seeds]  per seed: the pair it converged to and the
                                 iteration t at which U^{t+1} == U^t held; iter == -1 for a
                                 seed still moving after ``max_iter`` iterations, with
                                 (seed_i, seed_j) its last state (U^{T-1}, V^{T-1})
      pairs     int32[P][2]      M = union of the M_t, as a set sorted by (i, j)
      min_gap   float32[n_seeds] smallest top-1/top-2 gap over every search the seed took
                                 part in (tells which seeds a rounding difference may move)
      active    list[int]        number of queries in each search, in order
    """
    d1 = np.ascontiguousarray(d1, dtype=np.float32)
    d2 = np.ascontiguousarray(d2, dtype=np.float32)
    seeds = np.asarray(seeds, dtype=np.int32)
    n = seeds.shape[0]
    u = seeds.copy()                                   # U^t
    v = np.full(n, -1, dtype=np.int32)                 # V^t
    seed_iter = np.full(n, -1, dtype=np.int32)
    min_gap = np.full(n, np.inf, dtype=np.float32)
    searches = []

    act = np.arange(n)
    if n:
        # step 1: V^0 = NN_2(U^0)
        v[act], best, second = _search(d1[u[act]], d2, metric)
        min_gap[act] = np.minimum(min_gap[act], best - second)
        searches.append(int(act.size))
    for t in range(max_iter):
        if act.size == 0:
            break
        # step 2: U^{t+1} = NN_1(V^t)
        u_next, best, second = _search(d2[v[act]], d1, metric)
        min_gap[act] = np.minimum(min_gap[act], best - second)
        searches.append(int(act.size))
        conv = u_next == u[act]
        seed_iter[act[conv]] = t                       # M_t: (U^t[n], V^t[n]) for these n
        moved = ~conv
        u_next = u_next[moved]
        act = act[moved]                               # converged seeds leave
        if act.size == 0 or t == max_iter - 1:
            break
        u[act] = u_next
        v[act], best, second = _search(d1[u[act]], d2, metric)   # V^{t+1} = NN_2(U^{t+1})
        min_gap[act] = np.minimum(min_gap[act], best - second)
        searches.append(int(act.size))

    done = seed_iter >= 0
    if done.any():
        pairs = np.unique(np.stack([u[done], v[done]], axis=1), axis=0).astype(np.int32)
    else:
        pairs = np.zeros((0, 2), dtype=np.int32)
    return {"seed_i": u, "seed_j": v, "seed_iter": seed_iter, "pairs": pairs,
            "min_gap": min_gap, "active": searches}
