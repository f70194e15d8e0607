"""GPU parity of FNN_FLAG_SPLIT (fp32 descriptors held as two fp16 numbers, three matrix products)
against the oracle, through the C ABI.

Tolerances.  On fp16-representable maps (entries k/8) the second term is zero and every sum is exact:
bit-exact against the plain oracle.  On Gaussian unit maps the library and ``oracle.nearest_split``
form the same 3*d exact products and differ only in the order of the fp32 additions (72 terms for
d = 24, partial sums below 1 in magnitude: a few 2^-24 each), so: indices equal wherever the oracle's
gap exceeds 2e-5, scores within 4e-6 (the bar used for every "same inputs, other summation order"
comparison in this suite).  Against the plain fp32 oracle on the caller's unrounded maps the dropped
lo*lo term and the representation error add < 1e-6: indices equal where the gap exceeds 2e-5 as well.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import (GAP_ROUNDED, SCORE_TOL_ROUNDED, check_nearest_against, check_reciprocal_exact, dev, exact_maps,
                         host, unit_maps)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,m,d", [(1000, 3001, 24), (77, 4100, 12), (300, 300, 5), (64, 999, 28), (130, 2000, 32),
                                   (257, 1025, 10), (96, 640, 16), (500, 777, 20), (33, 100, 1)])
def test_nearest_split_exact_maps_bit_exact(n, m, d):
    a, b = exact_maps(200 + d, n, m, d)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute="f16", split=True)
    torch.cuda.synchronize()
    ri, rbest, _ = oracle.nearest(a, b)
    assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rbest)
    si, sbest, _ = oracle.nearest_split(a, b)
    assert np.array_equal(ri, si) and np.array_equal(rbest, sbest)


def test_worked_example_where_fp16_rounding_picks_the_wrong_candidate():
    # 1 + 2^-12 and 1 + 2^-13 both round to 1 in fp16; the true scores are 1 + 2^-13 (candidate 0)
    # and 1 + 2^-12 (candidate 1)
    a = np.array([[1.0 + 2.0 ** -12, 1.0]], dtype=np.float32)
    b = np.array([[0.0, 1.0 + 2.0 ** -13], [1.0, 0.0]], dtype=np.float32)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute="f16", split=True)
    hi, hs = fnn.fnn_nearest(dev(a), dev(b), compute="f16")
    torch.cuda.synchronize()
    assert int(gi[0, 0]) == 1 and float(gs[0, 0]) == float(np.float32(1.0 + 2.0 ** -12))
    assert int(hi[0, 0]) == 0 and float(hs[0, 0]) == 1.0
    ri, rbest, _ = oracle.nearest_split(a, b)
    assert ri[0] == 1 and rbest[0] == host(gs)[0, 0]


@pytest.mark.parametrize("d", [24, 16, 32, 11])
def test_nearest_split_gaussian_maps(d):
    a, b = unit_maps(300 + d, 3000, 20000, d)
    rng = np.random.default_rng(d)
    q = rng.integers(0, a.shape[0], size=1500).astype(np.int32)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), q_idx=dev(q)[None], compute="f16", split=True)
    torch.cuda.synchronize()
    gi, gs = host(gi)[0], host(gs)[0]
    ri, rbest, rsecond = oracle.nearest_split(a[q], b)
    clear = check_nearest_against(gi, gs, ri, rbest, rsecond, GAP_ROUNDED, SCORE_TOL_ROUNDED, "two-term oracle")
    assert clear.mean() > 0.99
    fi, fbest, fsecond = oracle.nearest(a[q], b)                       # fp32 products of the unrounded maps
    check_nearest_against(gi, gs, fi, fbest, fsecond, GAP_ROUNDED, SCORE_TOL_ROUNDED, "fp32 oracle")
    # the plain fp16 path on the same maps is two orders of magnitude further from the fp32 scores
    _, hs = fnn.fnn_nearest(dev(a), dev(b), q_idx=dev(q)[None], compute="f16")
    assert np.abs(host(hs)[0] - fbest).max() > 20 * np.abs(gs - fbest).max()


def test_storage_formats_strides_and_normalisation():
    a, b = unit_maps(41, 500, 3000, 24)
    ri, rbest, rsecond = oracle.nearest_split(a, b)
    # rows 40 elements apart (the generic prepare kernel)
    wide = np.zeros((3000, 40), dtype=np.float32)
    wide[:, :24] = b
    gi, gs = fnn.fnn_nearest(dev(a), dev(wide)[:, :24], compute="f16", split=True)
    torch.cuda.synchronize()
    check_nearest_against(host(gi)[0], host(gs)[0], ri, rbest, rsecond, GAP_ROUNDED, SCORE_TOL_ROUNDED, "strided")
    # fp16-stored maps have no second term: the answer is the plain fp16 one, bit for bit
    hi, hs = fnn.fnn_nearest(dev(a).half(), dev(b).half(), compute="f16", split=True)
    pi, ps = fnn.fnn_nearest(dev(a).half(), dev(b).half(), compute="f16")
    torch.cuda.synchronize()
    oi, obest, osecond = oracle.nearest(oracle.round_fp16(a), oracle.round_fp16(b))
    check_nearest_against(host(hi)[0], host(hs)[0], oi, obest, osecond, GAP_ROUNDED, SCORE_TOL_ROUNDED, "fp16 storage")
    clear = (obest - osecond) > GAP_ROUNDED
    assert np.array_equal(host(hi)[0][clear], host(pi)[0][clear])
    # raw head outputs: normalised first, then split
    raw = (a * np.linspace(0.5, 7.0, a.shape[0], dtype=np.float32)[:, None]).astype(np.float32)
    rawb = (b * np.linspace(9.0, 0.3, b.shape[0], dtype=np.float32)[:, None]).astype(np.float32)
    gi, gs = fnn.fnn_nearest(dev(raw), dev(rawb), compute="f16", split=True, normalize=True)
    torch.cuda.synchronize()
    ni, nbest, nsecond = oracle.nearest_split(oracle.normalize(raw), oracle.normalize(rawb))
    check_nearest_against(host(gi)[0], host(gs)[0], ni, nbest, nsecond, GAP_ROUNDED, SCORE_TOL_ROUNDED, "normalised")


def test_reciprocal_and_dense_split_exact_maps():
    w, h, d = 40, 28, 24
    d1, d2 = synth.exact_pair(78, w, h, d)
    seeds = synth.grid_seeds(w, h, 4)
    out = fnn.fnn_reciprocal(dev(d1), dev(d2), dev(seeds)[None], max_iter=10, compute="f16", split=True)
    torch.cuda.synchronize()
    check_reciprocal_exact({k: host(v) for k, v in out.items()}, 0, oracle.reciprocal(d1, d2, seeds, 10, metric="split"))
    dense = fnn.fnn_mutual_dense(dev(d1), dev(d2), compute="f16", split=True)
    torch.cuda.synchronize()
    rd = oracle.mutual_dense(d1, d2, metric="split")
    n_pairs = int(host(dense["n_pairs"])[0])
    for k in ("nn12", "nn21", "s12", "s21"):
        assert np.array_equal(host(dense[k])[0], rd[k]), k
    assert np.array_equal(host(dense["pairs"])[0, :n_pairs], rd["pairs"])


def test_dense_and_reciprocal_split_gaussian_pair():
    # two pairs, ragged sizes spanning several super-blocks of the dense kernel
    pairs = [unit_maps(500 + p, 4500, 5001, 24) for p in range(2)]
    out = fnn.fnn_mutual_dense([dev(p[0]) for p in pairs], [dev(p[1]) for p in pairs], compute="f16", split=True)
    torch.cuda.synchronize()
    got = {k: host(v) for k, v in out.items()}
    for p, (d1, d2) in enumerate(pairs):
        rd = oracle.mutual_dense(d1, d2, metric="split")
        c12, c21 = rd["gap12"] > GAP_ROUNDED, rd["gap21"] > GAP_ROUNDED
        assert c12.mean() > 0.99 and c21.mean() > 0.99
        assert np.array_equal(got["nn12"][p][c12], rd["nn12"][c12]) and np.array_equal(got["nn21"][p][c21], rd["nn21"][c21])
        assert np.abs(got["s12"][p] - rd["s12"]).max() <= SCORE_TOL_ROUNDED
        assert np.abs(got["s21"][p] - rd["s21"]).max() <= SCORE_TOL_ROUNDED
        # the filter is integer logic on the library's own tables
        nn12, nn21 = got["nn12"][p], got["nn21"][p]
        i = np.arange(d1.shape[0])
        keep = nn21[nn12] == i
        n_pairs = int(got["n_pairs"][p])
        assert n_pairs == int(keep.sum())
        assert np.array_equal(got["pairs"][p, :n_pairs], np.stack([i[keep], nn12[keep]], axis=1))
    seeds = np.arange(0, 4500, 7, dtype=np.int32)
    rec = fnn.fnn_reciprocal([dev(p[0]) for p in pairs], [dev(p[1]) for p in pairs], dev(np.stack([seeds, seeds])),
                             max_iter=10, compute="f16", split=True)
    torch.cuda.synchronize()
    rec = {k: host(v) for k, v in rec.items()}
    for p, (d1, d2) in enumerate(pairs):
        ref = oracle.reciprocal(d1, d2, seeds, 10, metric="split")
        pinned = ref["min_gap"] > GAP_ROUNDED
        assert pinned.mean() > 0.98
        for key in ("seed_i", "seed_j", "seed_iter"):
            assert np.array_equal(rec[key][p][pinned], ref[key][pinned]), key
