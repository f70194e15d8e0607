"""A candidate map whose prepared copy is larger than 2^31 bytes: byte offsets must be 64-bit everywhere.

46 000 017 candidates x 24 channels (fp16 storage, 48 bytes per prepared pixel).  Entries are k/8,
so every score is exact and the comparison with the oracle is bit for bit.  The candidates below
the 2^31-byte mark only use |k| <= 4, the ones above it the full range |k| <= 8: the nearest
neighbours therefore lie above the mark, where a truncated offset would read the wrong pixel.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import dev, host

pytestmark = pytest.mark.gpu


def test_nearest_beyond_two_gib_of_candidates():
    m, d, k = 46_000_017, 24, 96
    strong_from = 44_800_000                                          # 44.8e6 * 48 B > 2^31 B
    assert strong_from * 48 > 2 ** 31
    rng = np.random.default_rng(2024)
    lut = (np.arange(-8, 9) / 8).astype(np.float16)
    code = np.empty((m, d), dtype=np.uint8)                           # index into lut
    step = 4_000_000
    for start in range(0, m, step):                                   # in slices: bounded temporaries
        stop = min(start + step, m)
        weak = rng.integers(4, 13, size=(stop - start, d), dtype=np.uint8)      # |k| <= 4
        full = rng.integers(0, 17, size=(stop - start, d), dtype=np.uint8)
        rows = np.arange(start, stop)[:, None]
        code[start:stop] = np.where(rows >= strong_from, full, weak)
    b16 = lut[code]
    a = rng.integers(-8, 9, size=(k, d)).astype(np.float32) / 8
    tb = torch.from_numpy(b16).to("cuda:0")
    gi, gs = fnn.fnn_nearest(dev(a), tb, compute="f16")
    torch.cuda.synchronize()
    gi, gs = host(gi)[0], host(gs)[0]
    del tb
    torch.cuda.empty_cache()
    ri, rbest, _ = oracle.nearest(a, lut.astype(np.float32)[code])
    assert (ri >= strong_from).mean() > 0.9                           # the case is exercised
    assert np.array_equal(gi, ri)
    assert np.array_equal(gs, rbest)


def test_dense_with_more_bucket_units_than_fit_in_lds():
    # 2.2 million query pixels make more than 16384 runs of 128 queries: the second pass of the dense mode
    # then buckets with direct global atomics instead of its LDS histograms.  Few candidates keep it cheap.
    n, m, d = 2_200_003, 100, 8
    rng = np.random.default_rng(77)
    a = rng.integers(-8, 9, size=(n, d)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(m, d)).astype(np.float32) / 8
    assert (n + 4095) // 4096 * 32 > 16384
    out = fnn.fnn_mutual_dense(dev(a), dev(b), compute="f16")
    torch.cuda.synchronize()
    ref = oracle.mutual_dense(a, b)
    assert np.array_equal(host(out["nn12"])[0], ref["nn12"]) and np.array_equal(host(out["s12"])[0], ref["s12"])
    assert np.array_equal(host(out["nn21"])[0], ref["nn21"]) and np.array_equal(host(out["s21"])[0], ref["s21"])
    k = int(host(out["n_pairs"])[0])
    assert np.array_equal(host(out["pairs"])[0, :k], ref["pairs"])
