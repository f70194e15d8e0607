"""The first forward and the first backward search of fnn_reciprocal on 24-channel maps with a 16-bit
compute format, at least 1536 seeds and chunks of at least 32 candidate tiles per workgroup (many pairs, or
large maps) run in a kernel of their own: candidate tiles are staged through
LDS once per workgroup, and fp32 maps are read where the caller holds them (rounded on the way, the
prepared copy written as a by-product, no prepare pass).  Exactly representable maps: everything must
match the oracle bit for bit, whichever path a call takes, and the trace says which one it took."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import check_reciprocal_exact, dev, host

pytestmark = pytest.mark.gpu

STAGED = 103   # trace detail of the LDS-staged first-search kernel (100 + groups of query blocks per wave)


def traced_reciprocal(t1, t2, seeds, compute):
    fnn.fnn_trace_begin(128)
    try:
        out = fnn.fnn_reciprocal(t1, t2, seeds, max_iter=10, compute=compute)
        torch.cuda.synchronize()
    finally:
        trace = fnn.fnn_trace_end(128, details=True)
    searches = [detail for name, _, detail in trace if name == "search_kernel"]
    prep_ms = [ms for name, ms, _ in trace if name == "prep_kernel"]
    return {k: host(v) for k, v in out.items()}, searches, prep_ms


def exact(rng, rows, stride=24):
    wide = np.zeros((rows, stride), dtype=np.float32)
    wide[:, :24] = rng.integers(-8, 9, size=(rows, 24)).astype(np.float32) / 8
    wide[:, 24:] = 5.0   # junk between the rows must be ignored
    return wide


@pytest.mark.parametrize("compute", ["f16", "bf16"])
@pytest.mark.parametrize("n,m,n_seeds,batch,stride", [
    (5000, 7013, 1600, 64, 24),    # partial tiles on both sides; 5 row groups: the second quad has three idle waves
    (4096, 4128, 3072, 64, 28),    # rows 28 floats apart
    (9001, 9333, 1536, 64, 24),    # exactly one quad
])
def test_fp32_maps_are_searched_where_they_are(compute, n, m, n_seeds, batch, stride):
    rng = np.random.default_rng(n + m)
    a = [exact(rng, n, stride) for _ in range(batch)]
    b = [exact(rng, m, stride) for _ in range(batch)]
    seeds = rng.integers(0, n, size=(batch, n_seeds)).astype(np.int32)
    t1 = [dev(x)[:, :24] for x in a]
    t2 = [dev(x)[:, :24] for x in b]
    got, searches, _ = traced_reciprocal(t1, t2, dev(seeds), compute)
    assert searches[:2] == [STAGED, STAGED] and STAGED not in searches[2:]
    for p in range(batch):
        check_reciprocal_exact(got, p, oracle.reciprocal(a[p][:, :24], b[p][:, :24], seeds[p], 10))


def test_prepared_maps_take_the_staged_kernel_too_and_small_calls_do_not():
    rng = np.random.default_rng(77)
    n, m, batch = 4096, 6400, 64
    a = np.stack([exact(rng, n) for _ in range(batch)])
    b = np.stack([exact(rng, m) for _ in range(batch)])
    seeds = rng.integers(0, n, size=(batch, 2000)).astype(np.int32)
    ref = [oracle.reciprocal(a[p], b[p], seeds[p], 10) for p in range(batch)]

    def check(got):
        for p in (0, 31, 63):
            check_reciprocal_exact(got, p, ref[p])

    # stored in the compute format: read in place, no copy, staged first searches
    got, searches, _ = traced_reciprocal(dev(a).half(), dev(b).half(), dev(seeds), "f16")
    assert searches[:2] == [STAGED, STAGED]
    check(got)
    # fp16 storage with padded rows: prepare pass, then the staged kernel on the prepared copy
    wide_a = torch.zeros((batch, n, 40), dtype=torch.float16, device="cuda:0")
    wide_b = torch.zeros((batch, m, 40), dtype=torch.float16, device="cuda:0")
    wide_a[:, :, :24], wide_b[:, :, :24] = dev(a).half(), dev(b).half()
    got, searches, _ = traced_reciprocal(wide_a[:, :, :24], wide_b[:, :, :24], dev(seeds), "f16")
    assert searches[:2] == [STAGED, STAGED]
    check(got)
    # fewer seeds than one quad of row groups: the ordinary search kernel
    few = np.ascontiguousarray(seeds[:, :1535])
    got, searches, _ = traced_reciprocal(dev(a), dev(b), dev(few), "f16")
    assert STAGED not in searches
    check_reciprocal_exact(got, 5, oracle.reciprocal(a[5], b[5], few[5], 10))
    # one pair alone: so many workgroups per pair that a chunk would be a few tiles: the ordinary kernels
    got, searches, _ = traced_reciprocal(dev(a[7]), dev(b[7]), dev(seeds[7:8]), "f16")
    assert STAGED not in searches
    check_reciprocal_exact(got, 0, ref[7])
    # fp32 products: the ordinary kernels
    got, searches, _ = traced_reciprocal(dev(a), dev(b), dev(seeds), "f32")
    assert STAGED not in searches
    check(got)


def test_misaligned_fp32_rows_fall_back_to_the_prepare_pass():
    rng = np.random.default_rng(78)
    n, m, batch = 4096, 4096, 64
    a = np.stack([exact(rng, n, 25) for _ in range(batch)])     # rows 25 floats apart: no 16-byte alignment
    b = np.stack([exact(rng, m, 25) for _ in range(batch)])
    seeds = rng.integers(0, n, size=(batch, 1600)).astype(np.int32)
    got, searches, prep_ms = traced_reciprocal(dev(a)[:, :, :24], dev(b)[:, :, :24], dev(seeds), "f16")
    assert searches[:2] == [STAGED, STAGED]           # the staged kernel, on the copy the prepare pass made
    for p in (0, 63):
        check_reciprocal_exact(got, p, oracle.reciprocal(a[p][:, :24], b[p][:, :24], seeds[p], 10))


def test_single_large_pair_is_staged():
    """One pair is staged when its maps are large enough for long chunks (1024x768: 24576 tiles)."""
    rng = np.random.default_rng(79)
    n = 1024 * 768
    a, b = exact(rng, n), exact(rng, n)
    seeds = rng.integers(0, n, size=(1, 1536)).astype(np.int32)
    got, searches, _ = traced_reciprocal(dev(a), dev(b), dev(seeds), "bf16")
    assert searches[:2] == [STAGED, STAGED]
    check_reciprocal_exact(got, 0, oracle.reciprocal(a, b, seeds[0], 10))


def traced_nearest(t1, t2, compute, q_idx=None):
    fnn.fnn_trace_begin(16)
    try:
        idx, score = fnn.fnn_nearest(t1, t2, q_idx=q_idx, compute=compute)
        torch.cuda.synchronize()
    finally:
        trace = fnn.fnn_trace_end(16, details=True)
    return host(idx), host(score), [d for name, _, d in trace if name == "search_kernel"], [ms for name, ms, _ in trace if name == "prep_kernel"]


@pytest.mark.parametrize("compute", ["f16", "bf16"])
def test_nearest_takes_the_staged_kernel_when_every_query_is_live(compute):
    """fnn_nearest with enough queries: fp32 maps are searched where they are (staged kernel, no prepare
    pass over the maps), with and without a query list; maps in another storage format are prepared
    first and then take the same kernel; few queries, or a live count on the device, keep the
    ordinary one.  Exact inputs: indices and scores equal the oracle's bit for bit every time."""
    rng = np.random.default_rng(5)
    n, m, batch = 4100, 6401, 64
    a = [exact(rng, n, 28) for _ in range(batch)]
    b = [exact(rng, m, 28) for _ in range(batch)]
    t1 = [dev(x)[:, :24] for x in a]
    t2 = [dev(x)[:, :24] for x in b]
    ref_all = [oracle.nearest(a[p][:, :24], b[p][:, :24]) for p in (0, 40, 63)]

    idx, score, searches, prep_ms = traced_nearest(t1, t2, compute)            # every pixel of image 1 is a query
    assert searches == [STAGED]
    for k, p in enumerate((0, 40, 63)):
        assert np.array_equal(idx[p], ref_all[k][0]) and np.array_equal(score[p], ref_all[k][1])

    q = rng.integers(0, n, size=(batch, 1700)).astype(np.int32)
    idx, score, searches, _ = traced_nearest(t1, t2, compute, dev(q))
    assert searches == [STAGED]
    for k, p in enumerate((0, 40, 63)):
        assert np.array_equal(idx[p], ref_all[k][0][q[p]]) and np.array_equal(score[p], ref_all[k][1][q[p]])

    tdt = torch.float16 if compute == "f16" else torch.bfloat16
    idx, score, searches, _ = traced_nearest([x.to(tdt) for x in t1], [x.to(tdt) for x in t2], compute, dev(q))   # strided 16-bit rows: prepared first
    assert searches == [STAGED]
    for k, p in enumerate((0, 40, 63)):
        assert np.array_equal(idx[p], ref_all[k][0][q[p]]) and np.array_equal(score[p], ref_all[k][1][q[p]])

    idx, score, searches, _ = traced_nearest(t1, t2, compute, dev(q[:, :1000]))    # too few queries for a quad of row groups
    assert STAGED not in searches
    for k, p in enumerate((0, 40, 63)):
        assert np.array_equal(idx[p], ref_all[k][0][q[p, :1000]])
