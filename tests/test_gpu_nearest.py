"""fnn_nearest on the GPU against the CPU oracle (element by element)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import DEV, check_nearest_gaussian, dev, exact_maps, host, unit_maps

pytestmark = pytest.mark.gpu

COMPUTES = ["f16", "bf16", "f32"]


@pytest.mark.parametrize("compute", COMPUTES)
@pytest.mark.parametrize("k,m,d", [(1, 1, 1), (1, 70, 24), (5, 40, 24), (63, 31, 24), (64, 32, 16), (65, 33, 8),
                                   (127, 129, 17), (128, 128, 32), (129, 1000, 24), (200, 4097, 3),
                                   (3072, 3072, 24), (1000, 20011, 24)])
def test_exact_inputs_bit_exact(compute, k, m, d):
    a, b = exact_maps(1000 * k + m + d, k, m, d)
    ri, rb, _ = oracle.nearest(a, b)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute=compute)
    torch.cuda.synchronize()
    assert np.array_equal(host(gi)[0], ri)
    assert np.array_equal(host(gs)[0], rb)


@pytest.mark.parametrize("compute", COMPUTES)
@pytest.mark.parametrize("k,m,d", [(300, 5000, 24), (1000, 40000, 24), (77, 3333, 32), (500, 9000, 12)])
def test_gaussian_inputs(compute, k, m, d):
    a, b = unit_maps(7 * k + m, k, m, d)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute=compute)
    torch.cuda.synchronize()
    clear = check_nearest_gaussian(a, b, compute, host(gi)[0], host(gs)[0], f"{compute} {k}x{m}x{d}")
    assert clear.mean() > 0.9


@pytest.mark.parametrize("compute", ["f16", "f32"])
def test_query_list_active_count_and_batch(compute):
    batch, n, m, d, nq = 3, 700, 2100, 24, 333
    rng = np.random.default_rng(5)
    srcs, tgts = [], []
    for b in range(batch):
        a, t = exact_maps(50 + b, n, m, d)
        srcs.append(a)
        tgts.append(t)
    q = rng.integers(0, n, size=(batch, nq)).astype(np.int32)
    active = np.array([333, 0, 97], dtype=np.int32)
    out_idx = torch.full((batch, nq), -7, dtype=torch.int32, device=DEV)
    out_score = torch.full((batch, nq), -7.0, dtype=torch.float32, device=DEV)
    fnn.fnn_nearest([dev(x) for x in srcs], [dev(x) for x in tgts], q_idx=dev(q), nq_active=dev(active),
                    compute=compute, out_idx=out_idx, out_score=out_score)
    torch.cuda.synchronize()
    gi, gs = host(out_idx), host(out_score)
    for b in range(batch):
        k = int(active[b])
        ri, rb, _ = oracle.nearest(srcs[b][q[b, :k]], tgts[b])
        assert np.array_equal(gi[b, :k], ri)
        assert np.array_equal(gs[b, :k], rb)
        assert np.all(gi[b, k:] == -7) and np.all(gs[b, k:] == -7.0)     # untouched


def test_storage_formats_and_row_stride():
    # fp16 / bf16 storage, rows 40 elements apart; exactly representable values
    n, m, d = 257, 1111, 24
    a, b = exact_maps(9, n, m, d)
    ri, rb, _ = oracle.nearest(a, b)
    for dtype in (torch.float16, torch.bfloat16, torch.float32):
        wide_a = torch.zeros((n, 40), dtype=dtype, device=DEV)
        wide_b = torch.zeros((m, 40), dtype=dtype, device=DEV)
        wide_a[:, :d] = dev(a).to(dtype)
        wide_b[:, :d] = dev(b).to(dtype)
        wide_a[:, d:] = 3.0                          # junk beyond d must be ignored
        for compute in COMPUTES:
            gi, gs = fnn.fnn_nearest(wide_a[:, :d], wide_b[:, :d], compute=compute)
            torch.cuda.synchronize()
            assert np.array_equal(host(gi)[0], ri), (dtype, compute)
            assert np.array_equal(host(gs)[0], rb), (dtype, compute)


def test_empty_candidates_and_queries():
    a, b = exact_maps(3, 10, 10, 24)
    gi, gs = fnn.fnn_nearest(dev(a), torch.zeros((0, 24), device=DEV), compute="f16")
    torch.cuda.synchronize()
    assert np.all(host(gi) == -1) and np.all(np.isneginf(host(gs)))
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), nq=0, compute="f16")
    assert gi.shape == (1, 0)


def test_negative_scores_and_ties_to_lowest_index():
    # all scores negative; many exact ties
    a = -np.abs(exact_maps(4, 50, 1, 24)[0]) - 0.125
    b = np.repeat(np.abs(exact_maps(5, 7, 1, 24)[0]) + 0.125, 40, axis=0)    # each candidate 40 times
    ri, rb, rs = oracle.nearest(a, b)
    assert np.all(rb < 0) and np.all(rb == rs)
    for compute in COMPUTES:
        gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute=compute)
        torch.cuda.synchronize()
        assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rb)
    assert np.all(ri % 40 == 0)


def test_subnormal_descriptor_values_are_kept():
    # entries k * 2^-20, |k| < 64: subnormal as fp16 (below 2^-14), ordinary as bf16 and fp32.  Products
    # k1 k2 2^-40 and their sums are exact in fp32, so a matrix unit that flushed small inputs to
    # zero would return all-zero scores and index 0 instead of the oracle's answer.
    rng = np.random.default_rng(21)
    a = (rng.integers(-63, 64, size=(70, 24)) * 2.0 ** -20).astype(np.float32)
    b = (rng.integers(-63, 64, size=(900, 24)) * 2.0 ** -20).astype(np.float32)
    ri, rb, _ = oracle.nearest(a, b)
    assert rb.max() < 2.0 ** -23 and rb.min() > 0 and len(set(ri.tolist())) > 20
    for compute in COMPUTES:
        gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute=compute)
        torch.cuda.synchronize()
        assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rb), compute
    # small queries against ordinary candidates (scores around 2^-17)
    b2 = exact_maps(22, 1, 900, 24)[1]
    ri, rb, _ = oracle.nearest(a, b2)
    gi, gs = fnn.fnn_nearest(dev(a), dev(b2), compute="f16")
    di = fnn.fnn_mutual_dense(dev(a), dev(b2), compute="f16")
    torch.cuda.synchronize()
    assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rb)
    assert np.array_equal(host(di["nn12"])[0], ri) and np.array_equal(host(di["s12"])[0], rb)


def test_repeated_calls_are_deterministic():
    a, b = unit_maps(11, 2000, 30000, 24)
    ta, tb = dev(a), dev(b)
    first = [host(x) for x in fnn.fnn_nearest(ta, tb, compute="f16")]
    for _ in range(3):
        again = [host(x) for x in fnn.fnn_nearest(ta, tb, compute="f16")]
        assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])


def test_more_queries_than_resident_units_and_side_stream():
    # every pixel a query (rows groups outnumber the waves of the grid, so waves loop over units),
    # issued on a non-default stream
    a, b = exact_maps(21, 20000, 3000, 24)
    ri, rb, _ = oracle.nearest(a, b)
    stream = torch.cuda.Stream()
    ta, tb = dev(a), dev(b)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        gi, gs = fnn.fnn_nearest(ta, tb, compute="bf16", stream=stream)
    stream.synchronize()
    assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rb)


def test_maximum_batch_of_small_pairs():
    batch = 64
    maps = [exact_maps(500 + b, 130, 70, 24) for b in range(batch)]
    gi, gs = fnn.fnn_nearest([dev(m[0]) for m in maps], [dev(m[1]) for m in maps], compute="f16")
    torch.cuda.synchronize()
    gi, gs = host(gi), host(gs)
    for b in range(batch):
        ri, rb, _ = oracle.nearest(*maps[b])
        assert np.array_equal(gi[b], ri) and np.array_equal(gs[b], rb)
    with pytest.raises(fnn.FnnError):
        fnn.fnn_nearest([dev(m[0]) for m in maps] + [dev(maps[0][0])], [dev(m[1]) for m in maps] + [dev(maps[0][1])])


@pytest.mark.parametrize("compute", COMPUTES)
def test_fused_normalisation(compute):
    # raw (un-normalised) head outputs: the prepare pass normalises, casts and pads in one go;
    # the oracle normalises in fp32 the same way, then rounds like the compute format
    from gpu_helpers import GAP_ROUNDED, ROUNDERS, SCORE_TOL_ROUNDED, check_nearest_against
    rng = np.random.default_rng(77)
    a = (rng.standard_normal((700, 24)) * rng.uniform(0.05, 20.0, size=(700, 1))).astype(np.float32)
    b = (rng.standard_normal((9000, 24)) * rng.uniform(0.05, 20.0, size=(9000, 1))).astype(np.float32)
    a[13] = 0.0                                            # an all-zero descriptor stays zero
    gi, gs = fnn.fnn_nearest(dev(a), dev(b), compute=compute, normalize=True)
    torch.cuda.synchronize()
    rnd = ROUNDERS[compute]
    ri, rb, rs = oracle.nearest(rnd(oracle.normalize(a)), rnd(oracle.normalize(b)))
    clear = check_nearest_against(host(gi)[0], host(gs)[0], ri, rb, rs, GAP_ROUNDED, SCORE_TOL_ROUNDED, compute)
    assert clear.mean() > 0.95
    assert host(gs)[0][13] == 0.0
    # strided fp16 storage goes through the generic prepare path
    wide = torch.zeros((9000, 40), dtype=torch.float16, device=dev(b).device)
    wide[:, :24] = dev(b).to(torch.float16)
    b16 = host(wide[:, :24].float())
    gi, gs = fnn.fnn_nearest(dev(a), wide[:, :24], compute=compute, normalize=True)
    torch.cuda.synchronize()
    ri, rb, rs = oracle.nearest(rnd(oracle.normalize(a)), rnd(oracle.normalize(b16)))
    check_nearest_against(host(gi)[0], host(gs)[0], ri, rb, rs, GAP_ROUNDED, SCORE_TOL_ROUNDED, compute + " strided")
