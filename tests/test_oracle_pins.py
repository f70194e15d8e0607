"""Pins for the CPU oracle: it is checked against things other than itself.

* library routines on inputs where they must agree exactly (numpy float64 matmul +
  first-argmax on exactly representable data; scipy's k-d tree on unit vectors, where the
  largest dot product is the smallest Euclidean distance),
* closed forms (identical maps, a permuted copy, all-equal descriptors),
* a score matrix worked by hand (tests/golden/handworked_walk.json),
* exhaustive enumeration on tiny inputs (functional-graph formulation of the iteration),
* invariants of reciprocal matching.
"""
import json
import os

import numpy as np
import pytest
from scipy.spatial import cKDTree

import oracle
import synth_inputs as synth


# ----------------------------------------------------------------------------- helpers
def first_argmax_f64(a, b):
    """Row-wise first argmax, best and runner-up of a @ b.T in float64 (numpy library calls)."""
    s = a.astype(np.float64) @ b.astype(np.float64).T
    idx = np.argmax(s, axis=1)                     # numpy returns the first maximum
    best = s[np.arange(s.shape[0]), idx]
    s2 = s.copy()
    s2[np.arange(s.shape[0]), idx] = -np.inf
    second = s2.max(axis=1) if s.shape[1] > 1 else np.full(s.shape[0], -np.inf)
    return idx.astype(np.int32), best, second


def unit_rows(rng, n, d):
    x = rng.standard_normal((n, d))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(np.float32)


# ------------------------------------------------------------------- nearest: library pins
@pytest.mark.parametrize("seed,k,m,d", [(0, 97, 301, 24), (1, 64, 64, 1), (2, 5, 1000, 2), (3, 300, 33, 32)])
def test_nearest_matches_numpy_on_exact_inputs(seed, k, m, d):
    rng = np.random.default_rng(seed)
    a = rng.integers(-8, 9, size=(k, d)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(m, d)).astype(np.float32) / 8
    idx, best, second = oracle.nearest(a, b)
    ridx, rbest, rsecond = first_argmax_f64(a, b)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(best.astype(np.float64), rbest)      # exact arithmetic: same bits
    assert np.array_equal(second.astype(np.float64), rsecond)


def test_nearest_cfg1_full_matches_numpy():
    a, b = synth.config_pair(1)
    idx, best, second = oracle.nearest(a, b)
    ridx, rbest, rsecond = first_argmax_f64(a, b)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(best.astype(np.float64), rbest)
    assert np.array_equal(second.astype(np.float64), rsecond)
    # ties really occur on this workload, so the tie-break is exercised
    assert (best == second).sum() > 10


def test_nearest_matches_kdtree_on_unit_vectors():
    rng = np.random.default_rng(7)
    a = unit_rows(rng, 500, 24)
    b = unit_rows(rng, 4000, 24)
    idx, best, second = oracle.nearest(a, b)
    _, tidx = cKDTree(b.astype(np.float64)).query(a.astype(np.float64), k=1)
    clear = (best - second) > 1e-5
    assert clear.sum() > 450
    assert np.array_equal(idx[clear], tidx[clear].astype(np.int32))
    # the score is the cosine: 1 - |a-b|^2 / 2 for unit vectors
    dist2 = ((a.astype(np.float64) - b[idx].astype(np.float64)) ** 2).sum(axis=1)
    assert np.allclose(best, 1.0 - dist2 / 2.0, atol=2e-6)


def test_nearest_is_not_symmetric_in_its_operands():
    # a transposed-operand mistake must show: search b from a and a from b differ
    rng = np.random.default_rng(11)
    a = unit_rows(rng, 40, 8)
    b = unit_rows(rng, 50, 8)
    i_ab, _, _ = oracle.nearest(a, b)
    i_ba, _, _ = oracle.nearest(b, a)
    assert i_ab.shape == (40,) and i_ba.shape == (50,)
    assert i_ab.max() < 50 and i_ba.max() < 40
    s = a.astype(np.float64) @ b.astype(np.float64).T
    assert np.array_equal(i_ab, np.argmax(s, axis=1))
    assert np.array_equal(i_ba, np.argmax(s, axis=0))


# ------------------------------------------------------------------ nearest: closed forms
def test_identical_unit_maps_match_themselves():
    rng = np.random.default_rng(3)
    a = unit_rows(rng, 700, 24)
    idx, best, _ = oracle.nearest(a, a)
    assert np.array_equal(idx, np.arange(700))
    assert np.allclose(best, 1.0, atol=1e-6)


def test_permuted_copy_is_recovered():
    rng = np.random.default_rng(4)
    a = unit_rows(rng, 513, 24)
    perm = rng.permutation(513)
    b = np.empty_like(a)
    b[perm] = a                                   # b[perm[i]] = a[i]
    idx, _, _ = oracle.nearest(a, b)
    assert np.array_equal(idx, perm)
    out = oracle.mutual_dense(a, b)
    assert np.array_equal(out["pairs"], np.stack([np.arange(513), perm], axis=1))


def test_all_equal_descriptors_go_to_index_zero():
    a = np.full((9, 5), 0.5, dtype=np.float32)
    b = np.full((17, 5), 0.25, dtype=np.float32)
    idx, best, second = oracle.nearest(a, b)
    assert np.array_equal(idx, np.zeros(9, dtype=np.int32))
    assert np.array_equal(best, second)            # a tie has gap zero
    assert np.allclose(best, 5 * 0.125)


def test_lowest_index_wins_among_duplicates():
    rng = np.random.default_rng(5)
    b = unit_rows(rng, 50, 6)
    b[31] = b[12]
    b[44] = b[12]
    a = b[[12, 31, 44]].copy()
    idx, _, _ = oracle.nearest(a, b)
    assert np.array_equal(idx, [12, 12, 12])


def test_negative_scores_and_single_candidate():
    a = np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float32)
    b = np.array([[-1.0, -2.0]], dtype=np.float32)
    idx, best, second = oracle.nearest(a, b)
    assert np.array_equal(idx, [0, 0])
    assert np.array_equal(best, [-1.0, -2.0])
    assert np.all(np.isneginf(second))
    b2 = np.array([[-1.0, -2.0], [-3.0, -1.0]], dtype=np.float32)
    idx, best, second = oracle.nearest(a, b2)
    assert np.array_equal(idx, [0, 1])
    assert np.array_equal(best, [-1.0, -1.0])
    assert np.array_equal(second, [-3.0, -2.0])


def test_empty_inputs():
    a = np.zeros((0, 4), dtype=np.float32)
    b = np.ones((3, 4), dtype=np.float32)
    idx, best, _ = oracle.nearest(a, b)
    assert idx.shape == (0,) and best.shape == (0,)
    idx, best, _ = oracle.nearest(b, a)
    assert np.array_equal(idx, [-1, -1, -1]) and np.all(np.isneginf(best))


# ------------------------------------------------------------------------- rounding helpers
def test_rounding_helpers_match_library_casts():
    import torch
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32),
                        (rng.standard_normal(5000) * 1e-3).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 3.0e-5], dtype=np.float32)])
    t = torch.from_numpy(x)
    assert np.array_equal(oracle.round_bf16(x), t.to(torch.bfloat16).to(torch.float32).numpy())
    assert np.array_equal(oracle.round_fp16(x), t.to(torch.float16).to(torch.float32).numpy())


# --------------------------------------------------------------------- hand-worked example
def _load_walk(golden_dir):
    with open(os.path.join(golden_dir, "handworked_walk.json")) as f:
        g = json.load(f)
    d1 = np.asarray(g["scores"], dtype=np.float32)
    d2 = np.eye(d1.shape[1], dtype=np.float32)
    return g, d1, d2


def test_handworked_dense(golden_dir):
    g, d1, d2 = _load_walk(golden_dir)
    out = oracle.mutual_dense(d1, d2)
    assert out["nn12"].tolist() == g["nn12"]
    assert out["nn21"].tolist() == g["nn21"]
    assert out["s12"].tolist() == g["s12"]
    assert out["s21"].tolist() == g["s21"]
    assert (out["s12"] - out["gap12"]).tolist() == g["second12"]
    assert (out["s21"] - out["gap21"]).tolist() == g["second21"]
    assert out["pairs"].tolist() == g["mutual_pairs"]


def test_handworked_walks(golden_dir):
    g, d1, d2 = _load_walk(golden_dir)
    seeds = np.asarray(g["seeds"], dtype=np.int32)
    for case in g["cases"]:
        out = oracle.reciprocal(d1, d2, seeds, case["max_iter"])
        assert out["seed_i"].tolist() == case["seed_i"], case["max_iter"]
        assert out["seed_j"].tolist() == case["seed_j"], case["max_iter"]
        assert out["seed_iter"].tolist() == case["seed_iter"], case["max_iter"]
        assert out["pairs"].tolist() == case["pairs"], case["max_iter"]
        assert out["active"] == case["active"], case["max_iter"]


def test_handworked_subset_and_repeated_seeds(golden_dir):
    g, d1, d2 = _load_walk(golden_dir)
    out = oracle.reciprocal(d1, d2, np.array([5, 5, 0], dtype=np.int32), 3)
    assert out["seed_i"].tolist() == [1, 1, 1]
    assert out["seed_j"].tolist() == [1, 1, 1]
    assert out["seed_iter"].tolist() == [2, 2, 1]
    assert out["pairs"].tolist() == [[1, 1]]       # M is a set
    out = oracle.reciprocal(d1, d2, np.zeros(0, dtype=np.int32), 3)
    assert out["pairs"].shape == (0, 2) and out["active"] == []
    out = oracle.reciprocal(d1, d2, np.array([5], dtype=np.int32), 0)
    assert out["seed_iter"].tolist() == [-1] and out["seed_i"].tolist() == [5] and out["seed_j"].tolist() == [5]


# ----------------------------------------------------------- dense mutual: exhaustive check
@pytest.mark.parametrize("seed,n,m,d", [(0, 12, 12, 1), (1, 48, 35, 2), (2, 192, 192, 24), (3, 100, 260, 24)])
def test_mutual_dense_matches_enumeration(seed, n, m, d):
    rng = np.random.default_rng(seed)
    a = rng.integers(-8, 9, size=(n, d)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(m, d)).astype(np.float32) / 8
    out = oracle.mutual_dense(a, b)
    s = a.astype(np.float64) @ b.astype(np.float64).T
    row = np.argmax(s, axis=1)
    col = np.argmax(s, axis=0)
    want = [[i, int(row[i])] for i in range(n) if col[row[i]] == i]
    assert out["pairs"].tolist() == want
    assert np.array_equal(out["nn12"], row) and np.array_equal(out["nn21"], col)


# ------------------------------------------------ reciprocal: functional-graph enumeration
def _walk_by_function_powers(a, b, seeds, max_iter):
    """Independent formulation on exactly representable inputs.

    f = NN_1 o NN_2 maps pixels of image 1 to pixels of image 1.  A seed converges at the
    first t with f^{t+1}(seed) == f^t(seed); its pair is (f^t(seed), NN_2(f^t(seed))).
    Computed for ALL pixels at once by composing index arrays -- no active set, no
    per-seed bookkeeping.
    """
    s = a.astype(np.float64) @ b.astype(np.float64).T
    nn2 = np.argmax(s, axis=1)
    nn1 = np.argmax(s, axis=0)
    f = nn1[nn2]
    n = a.shape[0]
    power = np.arange(n)                       # f^t
    first_t = np.full(n, -1)
    at = np.arange(n)
    for t in range(max_iter):
        nxt = f[power]                         # f^{t+1}
        newly = (nxt == power) & (first_t < 0)
        first_t[newly] = t
        at[newly] = power[newly]
        power = nxt
    # seeds that never converged: state after max_iter-1 moves
    if max_iter > 0:
        last = np.arange(n)
        for _ in range(max_iter - 1):
            last = f[last]
    else:
        last = np.arange(n)
    at = np.where(first_t >= 0, at, last)
    return at[seeds], nn2[at[seeds]], first_t[seeds]


@pytest.mark.parametrize("seed,w,h,d,max_iter", [(0, 16, 12, 24, 10), (1, 16, 12, 2, 10), (2, 8, 6, 1, 4),
                                                  (3, 16, 12, 3, 1), (4, 12, 9, 4, 2), (5, 16, 12, 24, 3)])
def test_reciprocal_matches_function_powers(seed, w, h, d, max_iter):
    a, b = synth.exact_pair(seed, w, h, d)
    seeds = np.arange(w * h, dtype=np.int32)
    out = oracle.reciprocal(a, b, seeds, max_iter)
    wi, wj, wt = _walk_by_function_powers(a, b, seeds, max_iter)
    assert np.array_equal(out["seed_iter"], wt)
    assert np.array_equal(out["seed_i"], wi)
    assert np.array_equal(out["seed_j"], wj)
    done = wt >= 0
    want = sorted(set(zip(wi[done].tolist(), wj[done].tolist())))
    assert out["pairs"].tolist() == [list(p) for p in want]


# ------------------------------------------------------------------ reciprocal: invariants
def _check_invariants(a, b, seeds, max_iter, dense=None):
    out = oracle.reciprocal(a, b, seeds, max_iter)
    pairs = out["pairs"]
    # (i) every returned pair is mutually nearest
    if len(pairs):
        j_of_i, _, _ = oracle.nearest(a[pairs[:, 0]], b)
        i_of_j, _, _ = oracle.nearest(b[pairs[:, 1]], a)
        assert np.array_equal(j_of_i, pairs[:, 1])
        assert np.array_equal(i_of_j, pairs[:, 0])
    # (ii) fixed point: restarting from the matched pixels converges at once to the same set
    again = oracle.reciprocal(a, b, pairs[:, 0].copy(), max_iter=1)
    assert np.all(again["seed_iter"] == 0)
    assert np.array_equal(again["pairs"], pairs)
    # (iii) subset of the all-pairs mutual nearest neighbours
    if dense is None:
        dense = oracle.mutual_dense(a, b)
    dense_set = set(map(tuple, dense["pairs"].tolist()))
    assert set(map(tuple, pairs.tolist())) <= dense_set
    # sorted set, no duplicates
    assert np.array_equal(pairs, np.unique(pairs, axis=0))
    # per-seed outputs agree with the pair list
    done = out["seed_iter"] >= 0
    assert set(zip(out["seed_i"][done].tolist(), out["seed_j"][done].tolist())) == set(map(tuple, pairs.tolist()))
    # number of searches is bounded by 2 * max_iter and never grows
    assert len(out["active"]) <= 2 * max_iter
    assert all(x >= y for x, y in zip(out["active"], out["active"][1:]))
    return out, dense


def test_reciprocal_invariants_cfg1():
    a, b = synth.config_pair(1)
    seeds = synth.grid_seeds(64, 48, 8)
    assert seeds.shape == (48,)
    _check_invariants(a, b, seeds, 10)


def test_reciprocal_invariants_gaussian():
    a, b, _ = synth.warped_pair(42, 96, 64, 24)
    seeds = synth.grid_seeds(96, 64, 4)
    out, _ = _check_invariants(a, b, seeds, 10)
    assert (out["seed_iter"] >= 0).mean() > 0.9


def test_all_pixel_seeds_recover_every_mutual_pair():
    # a mutual pair (i*, j*) is found at t = 0 by its own seed i*, so with every pixel a
    # seed the result equals the all-pairs mutual nearest neighbours exactly
    a, b = synth.config_pair(1)
    seeds = np.arange(a.shape[0], dtype=np.int32)
    out, dense = _check_invariants(a, b, seeds, 10)
    assert np.array_equal(out["pairs"], dense["pairs"])


def test_scores_never_decrease_along_a_walk():
    # with lowest-index tie-breaking each hop strictly improves the score or keeps it and
    # lowers an index, so walks cannot cycle; check the score part on a random case
    a, b, _ = synth.warped_pair(9, 64, 48, 24)
    seeds = synth.grid_seeds(64, 48, 4)
    s = a.astype(np.float64) @ b.astype(np.float64).T
    prev = oracle.reciprocal(a, b, seeds, 0)
    score_prev = s[prev["seed_i"], prev["seed_j"]]
    for t in range(1, 6):
        cur = oracle.reciprocal(a, b, seeds, t)
        score = s[cur["seed_i"], cur["seed_j"]]
        assert np.all(score >= score_prev - 1e-6)
        score_prev = score


# ------------------------------------------------------------------- generator properties
def test_generator_shapes_and_determinism():
    a, b = synth.config_pair(1)
    assert a.shape == (3072, 24) and a.dtype == np.float32
    assert set(np.unique(a * 8).tolist()) <= set(range(-8, 9))
    a2, b2 = synth.config_pair(1)
    assert np.array_equal(a, a2) and np.array_equal(b, b2)
    m1, m2, hmat = synth.warped_pair(5, 64, 48, 24)
    assert np.allclose(np.linalg.norm(m1, axis=1), 1, atol=1e-6)
    assert np.allclose(np.linalg.norm(m2, axis=1), 1, atol=1e-6)
    # the homography moves each corner by at most 15 % of the image size
    c = np.array([[0, 0, 1], [63, 0, 1], [63, 47, 1], [0, 47, 1]], dtype=np.float64).T
    w = hmat @ c
    w = (w[:2] / w[2]).T
    assert np.all(np.abs(w[:, 0] - c[0]) <= 0.15 * 64 + 1e-9)
    assert np.all(np.abs(w[:, 1] - c[1]) <= 0.15 * 48 + 1e-9)
    assert synth.grid_seeds(512, 384, 8).shape == (3072,)
    assert synth.grid_seeds(512, 384, 8)[65] == 8 * 512 + 8


# ------------------------------------------------------------------------------ normalise
def test_normalize_closed_forms_and_invariants():
    x = np.array([[3.0, 4.0], [0.0, 0.0], [-5.0, 12.0], [1.0, 0.0]], dtype=np.float32)
    y = oracle.normalize(x)
    assert np.array_equal(y[0], np.array([3.0, 4.0], dtype=np.float32) / np.float32(5.0))
    assert np.array_equal(y[1], [0.0, 0.0])                       # an all-zero descriptor stays zero
    assert np.array_equal(y[2], np.array([-5.0, 12.0], dtype=np.float32) / np.float32(13.0))
    assert np.array_equal(y[3], [1.0, 0.0])
    rng = np.random.default_rng(12)
    z = (rng.standard_normal((2000, 24)) * rng.uniform(0.01, 50.0, size=(2000, 1))).astype(np.float32)
    yz = oracle.normalize(z)
    z64 = z.astype(np.float64)
    want = z64 / np.linalg.norm(z64, axis=1, keepdims=True)
    assert np.max(np.abs(yz - want)) < 3e-7                       # a few fp32 roundings at most
    assert np.allclose(np.linalg.norm(yz.astype(np.float64), axis=1), 1.0, atol=3e-7)
    # scaling by a power of two commutes with every rounding: bit-identical result
    assert np.array_equal(oracle.normalize(z * np.float32(8.0)), yz)
    assert np.array_equal(oracle.normalize(z * np.float32(0.25)), yz)
    # the sign pattern and the ordering of channels survive
    assert np.array_equal(np.sign(yz), np.sign(z))
    assert np.array_equal(np.argmax(np.abs(yz), axis=1), np.argmax(np.abs(z), axis=1))


# ----------------------------------------------------------- fp16-accumulation control
def test_half_accumulate_equals_fp32_when_everything_is_exact():
    # entries k/8, |sum| <= 24: every partial sum is a multiple of 1/64 below 32, exact in fp16
    a, b = synth.exact_pair(3, 24, 20, 24)
    idx, best = oracle.nearest_half_accumulate(a, b)
    ridx, rbest, _ = oracle.nearest(a, b)
    assert np.array_equal(idx, ridx) and np.array_equal(best, rbest)


def test_half_accumulate_worked_flip():
    # fp16 has steps of 2 between 2048 and 4096.  Query (32, 1, 1):
    #   candidate 0 = (64, 1, 1): exact 2050; in fp16 2048 + 1 -> 2048 (tie to even), + 1 -> 2048
    #   candidate 1 = (64, 1.5, 0): exact 2049.5; in fp16 2048 + 1.5 = 2049.5 -> 2050, + 0 -> 2050
    # so fp32 accumulation prefers candidate 0 and fp16 accumulation prefers candidate 1
    a = np.array([[32.0, 1.0, 1.0]], dtype=np.float32)
    b = np.array([[64.0, 1.0, 1.0], [64.0, 1.5, 0.0]], dtype=np.float32)
    idx, best = oracle.nearest_half_accumulate(a, b)
    assert idx.tolist() == [1] and best.tolist() == [2050.0]
    ridx, rbest, rsecond = oracle.nearest(a, b)
    assert ridx.tolist() == [0] and rbest.tolist() == [2050.0] and rsecond.tolist() == [2049.5]


# --------------------------------------------------------- squared-distance dist_func: pins
def test_nearest_l2_matches_kdtree_on_exact_inputs():
    # scipy's k-d tree is an independent algorithm; on multiples of 1/8 every distance is exact
    # in fp32 and in float64, so the distances must agree bit for bit and the index wherever the
    # nearest candidate is unique
    rng = np.random.default_rng(21)
    a = rng.integers(-8, 9, size=(211, 6)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(997, 6)).astype(np.float32) / 8
    idx, best, second = oracle.nearest_l2(a, b)
    dist, tidx = cKDTree(b.astype(np.float64)).query(a.astype(np.float64), k=2)
    # the tree reports distances, the oracle their squares: both exact, so the correctly rounded
    # float64 square roots must coincide
    assert np.array_equal(np.sqrt(best.astype(np.float64)), dist[:, 0])
    assert np.array_equal(np.sqrt(second.astype(np.float64)), dist[:, 1])
    unique = second > best
    assert unique.sum() > 50 and (~unique).sum() > 5
    assert np.array_equal(idx[unique], tidx[unique, 0])
    # among equals the lowest index: no earlier candidate is as close
    for q in np.nonzero(~unique)[0]:
        d2 = ((b.astype(np.float64) - a[q].astype(np.float64)) ** 2).sum(axis=1)
        assert idx[q] == int(np.nonzero(d2 == d2.min())[0][0])


def test_nearest_l2_on_unit_vectors_is_the_dot_product_search():
    # |a - b|^2 = 2 - 2<a, b> for unit vectors: same neighbours, distances from the scores
    rng = np.random.default_rng(22)
    a, b = unit_rows(rng, 300, 24), unit_rows(rng, 2000, 24)
    li, lbest, lsecond = oracle.nearest_l2(a, b)
    di, dbest, dsecond = oracle.nearest(a, b)
    clear = (dbest - dsecond) > 1e-5
    assert clear.mean() > 0.95
    assert np.array_equal(li[clear], di[clear])
    assert np.allclose(lbest, 2.0 - 2.0 * dbest, atol=2e-6)


def test_nearest_l2_differs_from_the_dot_product_where_it_must():
    # worked by hand: the query is the origin, so every dot product is 0 (tie -> index 0), while
    # the distances are 9, 4, 4, 16 -> index 1 (the first of the two at distance 4)
    a = np.zeros((1, 2), dtype=np.float32)
    b = np.array([[3, 0], [0, 2], [2, 0], [0, -4]], dtype=np.float32)
    assert oracle.nearest(a, b)[0].tolist() == [0]
    idx, best, second = oracle.nearest_l2(a, b)
    assert idx.tolist() == [1] and best.tolist() == [4.0] and second.tolist() == [4.0]
    # a long candidate wins the dot product but not the distance
    a = np.array([[1, 0]], dtype=np.float32)
    b = np.array([[1, 0.5], [8, 0]], dtype=np.float32)
    assert oracle.nearest(a, b)[0].tolist() == [1]
    idx, best, second = oracle.nearest_l2(a, b)
    assert idx.tolist() == [0] and best.tolist() == [0.25] and second.tolist() == [49.0]


def test_nearest_l2_is_translation_invariant_and_symmetric_in_value():
    rng = np.random.default_rng(23)
    a = rng.integers(-8, 9, size=(64, 5)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(200, 5)).astype(np.float32) / 8
    shift = rng.integers(-8, 9, size=(1, 5)).astype(np.float32) / 4
    i0, b0, s0 = oracle.nearest_l2(a, b)
    i1, b1, s1 = oracle.nearest_l2(a + shift, b + shift)          # still exact: small dyadic numbers
    assert np.array_equal(i0, i1) and np.array_equal(b0, b1) and np.array_equal(s0, s1)
    # d(a, b) = d(b, a): the distance of a's neighbour is what b's search sees for that pair
    j0, c0, _ = oracle.nearest_l2(b, a)
    for q in range(a.shape[0]):
        assert c0[i0[q]] <= b0[q]                                  # b's own best is at least as close
    # empty candidate set
    idx, best, second = oracle.nearest_l2(a, np.zeros((0, 5), dtype=np.float32))
    assert (idx == -1).all() and np.isinf(best).all() and np.isinf(second).all()


def test_l2_matching_on_unit_maps_equals_dot_matching():
    # the whole iteration and the dense filter only see the ranking, which is the same
    d1, d2 = synth.warped_pair(31, 24, 16, 8)[:2]
    seeds = synth.grid_seeds(24, 16, 4)
    rd = oracle.reciprocal(d1, d2, seeds, 10, metric="dot")
    rl = oracle.reciprocal(d1, d2, seeds, 10, metric="l2")
    clear = rd["min_gap"] > 1e-5
    assert clear.mean() > 0.9
    for key in ("seed_i", "seed_j", "seed_iter"):
        assert np.array_equal(rd[key][clear], rl[key][clear])
    md, ml = oracle.mutual_dense(d1, d2), oracle.mutual_dense(d1, d2, metric="l2")
    ok = (md["gap12"] > 1e-5)
    assert np.array_equal(md["nn12"][ok], ml["nn12"][ok])
    assert np.allclose(ml["s12"], -(2.0 - 2.0 * md["s12"]), atol=2e-6)


def test_l2_reciprocal_invariants_on_raw_maps():
    # un-normalised maps: pairs are mutually nearest in distance and a fixed point of one more step
    rng = np.random.default_rng(32)
    d1 = rng.standard_normal((24 * 16, 8)).astype(np.float32)
    d2 = (d1[rng.permutation(d1.shape[0])] + 0.1 * rng.standard_normal(d1.shape)).astype(np.float32)
    seeds = synth.grid_seeds(24, 16, 2)
    r = oracle.reciprocal(d1, d2, seeds, 10, metric="l2")
    dense = oracle.mutual_dense(d1, d2, metric="l2")
    dense_pairs = {tuple(p) for p in dense["pairs"].tolist()}
    assert len(r["pairs"]) > 10
    for i, j in r["pairs"].tolist():
        assert (i, j) in dense_pairs
        assert oracle.nearest_l2(d1[i:i + 1], d2)[0][0] == j and oracle.nearest_l2(d2[j:j + 1], d1)[0][0] == i
    # and it is not the dot-product answer: the maps are far from unit norm
    assert not np.array_equal(dense["nn12"], oracle.mutual_dense(d1, d2)["nn12"])


# ------------------------------------------------------ matches as pixel coordinates: pins
def test_pairs_to_pixels_worked_example():
    # images of width 5 (3 rows) and width 4 (2 rows); worked by hand:
    #   pixel 7 of image 1 = (w 2, h 1), 14 = (4, 2), 0 = (0, 0); pixel 6 of image 2 = (2, 1), 3 = (3, 0), 7 = (3, 1)
    pairs = np.array([[0, 3], [7, 6], [14, 7]], dtype=np.int32)
    xy = oracle.pairs_to_pixels(pairs, 5, 4, 15, 8)
    assert xy.tolist() == [[0, 0, 3, 0], [2, 1, 2, 1], [4, 2, 3, 1]]
    conf1 = np.array([0.9] * 7 + [0.2] + [0.9] * 7, dtype=np.float32)       # pixel 7 is unsure
    conf2 = np.array([0.5] * 8, dtype=np.float32)
    assert oracle.pairs_to_pixels(pairs, 5, 4, 15, 8, conf1, conf2, 0.3, 0.5).tolist() == [[0, 0, 3, 0], [4, 2, 3, 1]]
    assert oracle.pairs_to_pixels(pairs, 5, 4, 15, 8, conf1, conf2, 0.3, 0.6).shape == (0, 4)
    # ">=": a confidence equal to the threshold stays; NaN never does; ids outside the image are dropped
    conf2[3] = np.nan
    assert oracle.pairs_to_pixels(pairs, 5, 4, 15, 8, None, conf2, 0.0, 0.5).tolist() == [[2, 1, 2, 1], [4, 2, 3, 1]]
    assert oracle.pairs_to_pixels(np.array([[15, 0], [-1, 2], [3, 8]]), 5, 4, 15, 8).shape == (0, 4)


def test_pairs_to_pixels_round_trip_and_monotone_filter():
    rng = np.random.default_rng(41)
    w1, h1, w2, h2 = 37, 11, 23, 29
    pairs = np.stack([rng.integers(0, w1 * h1, 500), rng.integers(0, w2 * h2, 500)], axis=1).astype(np.int32)
    xy = oracle.pairs_to_pixels(pairs, w1, w2, w1 * h1, w2 * h2)
    assert xy.shape == (500, 4)
    assert np.array_equal(xy[:, 1] * w1 + xy[:, 0], pairs[:, 0]) and np.array_equal(xy[:, 3] * w2 + xy[:, 2], pairs[:, 1])
    assert (xy[:, 0] < w1).all() and (xy[:, 1] < h1).all() and (xy[:, 2] < w2).all() and (xy[:, 3] < h2).all()
    conf1, conf2 = rng.random(w1 * h1).astype(np.float32), rng.random(w2 * h2).astype(np.float32)
    counts = [oracle.pairs_to_pixels(pairs, w1, w2, w1 * h1, w2 * h2, conf1, conf2, t, t).shape[0] for t in (0.0, 0.3, 0.6, 1.1)]
    assert counts[0] == 500 and counts[-1] == 0 and counts == sorted(counts, reverse=True)
    # the survivors are a subsequence of the unfiltered list (order kept)
    kept = oracle.pairs_to_pixels(pairs, w1, w2, w1 * h1, w2 * h2, conf1, conf2, 0.3, 0.3).tolist()
    it = iter(xy.tolist())
    assert all(any(row == other for other in it) for row in kept)


# ---------------------------------------------------- two-term fp16 representation ("split")
def test_split_fp16_reconstructs_fp32_values():
    rng = np.random.default_rng(70)
    x = np.concatenate([rng.standard_normal(5000), rng.standard_normal(5000) * 1e-3, [0.0, 1.0, -2.5, 65504.0]]).astype(np.float32)
    hi, lo = oracle.split_fp16(x)
    # both halves are binary16 numbers
    assert np.array_equal(hi.astype(np.float16).astype(np.float32), hi)
    assert np.array_equal(lo.astype(np.float16).astype(np.float32), lo)
    # hi is the nearest binary16 number; what is left after lo is below 2^-22 |x| (or below the
    # binary16 subnormal spacing 2^-24, whichever is larger)
    assert np.all(np.abs(x - hi) <= np.abs(x) * 2.0 ** -11 + 2.0 ** -25)
    err = np.abs(x.astype(np.float64) - hi.astype(np.float64) - lo.astype(np.float64))
    assert np.all(err <= np.maximum(np.abs(x) * 2.0 ** -22, 2.0 ** -25))
    # an fp16-representable value has no second term
    exact = (rng.integers(-2048, 2049, size=1000) / 256).astype(np.float32)
    hi, lo = oracle.split_fp16(exact)
    assert np.array_equal(hi, exact) and not lo.any()


def test_nearest_split_scores_are_fp32_grade():
    rng = np.random.default_rng(71)
    a, b = unit_rows(rng, 300, 24), unit_rows(rng, 2000, 24)
    idx, best, second = oracle.nearest_split(a, b)
    ref_idx, ref_best, ref_second = first_argmax_f64(a, b)          # exact scores of the fp32 inputs
    # dropped lo*lo term and representation error: < 4 * 2^-22 * sum|a_k b_k| <= 1e-6 for unit rows;
    # fp32 accumulation of 72 terms adds a few 2^-24.  A dropped cross term would show as ~1e-4.
    assert np.abs(best - ref_best).max() < 1.5e-6
    clear = (ref_best - ref_second) > 1e-5
    assert clear.mean() > 0.99
    assert np.array_equal(idx[clear], ref_idx[clear])
    # plain fp16 rounding of the same inputs is two orders of magnitude coarser
    _, half_best, _ = oracle.nearest(oracle.round_fp16(a), oracle.round_fp16(b))
    assert np.abs(half_best - ref_best).max() > 5e-5


def test_nearest_split_equals_nearest_on_fp16_representable_maps():
    rng = np.random.default_rng(72)
    a = (rng.integers(-8, 9, size=(100, 24)) / 8).astype(np.float32)
    b = (rng.integers(-8, 9, size=(700, 24)) / 8).astype(np.float32)
    for got, want in zip(oracle.nearest_split(a, b), oracle.nearest(a, b)):
        assert np.array_equal(got, want)


def test_nearest_split_worked_example():
    # binary16 has 10 fraction bits, so 1 + 2^-12 and 1 + 2^-13 both round to 1:
    #   a  = (1 + 2^-12, 1)        hi = (1, 1), lo = (2^-12, 0)
    #   b0 = (0, 1 + 2^-13)        hi = (0, 1), lo = (0, 2^-13)     exact score 1 + 2^-13
    #   b1 = (1, 0)                hi = (1, 0), lo = (0, 0)         exact score 1 + 2^-12  <- the winner
    # split scores: b0: hi.hi = 1, hi.lo = 2^-13, lo.hi = 0;  b1: hi.hi = 1, hi.lo = 0, lo.hi = 2^-12.
    a = np.array([[1.0 + 2.0 ** -12, 1.0]], dtype=np.float32)
    b = np.array([[0.0, 1.0 + 2.0 ** -13], [1.0, 0.0]], dtype=np.float32)
    idx, best, second = oracle.nearest_split(a, b)
    assert idx[0] == 1 and best[0] == np.float32(1.0 + 2.0 ** -12) and second[0] == np.float32(1.0 + 2.0 ** -13)
    # rounded to fp16 the two candidates tie at 1 and the lower index wins: the wrong one
    hidx, hbest, hsecond = oracle.nearest(oracle.round_fp16(a), oracle.round_fp16(b))
    assert hidx[0] == 0 and hbest[0] == 1.0 and hsecond[0] == 1.0


def test_split_matching_equals_fp32_matching_where_gaps_are_clear():
    rng = np.random.default_rng(73)
    a, b = unit_rows(rng, 1200, 24), unit_rows(rng, 1200, 24)
    ds = oracle.mutual_dense(a, b, metric="split")
    dd = oracle.mutual_dense(a, b)
    clear12, clear21 = dd["gap12"] > 1e-5, dd["gap21"] > 1e-5
    assert np.array_equal(ds["nn12"][clear12], dd["nn12"][clear12])
    assert np.array_equal(ds["nn21"][clear21], dd["nn21"][clear21])
    assert np.abs(ds["s12"] - dd["s12"]).max() < 2e-6
