"""GPU parity of fnn_pairs_to_pixels (matches as pixel coordinates, confidence filter): integer work, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import dev, host

pytestmark = pytest.mark.gpu


def check(pairs, n_pairs, w1, n, w2, m, conf1=None, conf2=None, t1=0.0, t2=0.0):
    xy, count = fnn.fnn_pairs_to_pixels(dev(pairs), dev(n_pairs), n, w1, m, w2,
                                        None if conf1 is None else dev(conf1), None if conf2 is None else dev(conf2), t1, t2)
    torch.cuda.synchronize()
    xy, count = host(xy), host(count)
    for b in range(pairs.shape[0]):
        want = oracle.pairs_to_pixels(pairs[b, :max(0, min(int(n_pairs[b]), pairs.shape[1]))], w1, w2, n, m,
                                      None if conf1 is None else conf1[b], None if conf2 is None else conf2[b], t1, t2)
        assert count[b] == want.shape[0]
        assert np.array_equal(xy[b, :count[b]], want)
        assert np.all(xy[b, count[b]:] == -1)
    return count


def test_random_pairs_with_and_without_filter():
    rng = np.random.default_rng(3)
    w1, h1, w2, h2 = 61, 45, 64, 48                       # the two images differ in size
    n, m = w1 * h1, w2 * h2
    batch, max_pairs = 3, 5000                            # several chunks of 1024 and a ragged tail
    pairs = np.stack([rng.integers(0, n, (batch, max_pairs)), rng.integers(0, m, (batch, max_pairs))], axis=2).astype(np.int32)
    n_pairs = np.array([max_pairs, 1025, 0], dtype=np.int32)
    assert check(pairs, n_pairs, w1, n, w2, m).tolist() == [5000, 1025, 0]
    conf1 = rng.random((batch, n)).astype(np.float32)
    conf2 = rng.random((batch, m)).astype(np.float32)
    conf2[0, :50] = np.nan
    counts = check(pairs, n_pairs, w1, n, w2, m, conf1, conf2, 0.25, 0.5)
    assert 0 < counts[0] < 5000 and 0 < counts[1] < 1025 and counts[2] == 0
    check(pairs, n_pairs, w1, n, w2, m, conf1, None, 0.9, 0.0)
    check(pairs, n_pairs, w1, n, w2, m, None, conf2, 0.0, 2.0)        # nothing survives
    # counts beyond the buffer and negative counts are clamped; ids outside the images are dropped
    pairs[1, 3] = (n, 0)
    pairs[1, 4] = (0, -1)
    check(pairs, np.array([max_pairs + 7, 10, -5], dtype=np.int32), w1, n, w2, m)


def test_on_the_outputs_of_the_matching_calls():
    w, h = 64, 48
    d1, d2 = synth.config_pair(1)
    seeds = synth.grid_seeds(w, h, 8)
    out = fnn.fnn_reciprocal(dev(d1), dev(d2), dev(seeds)[None], max_iter=10, compute="f16")
    xy, count = fnn.fnn_pairs_to_pixels(out["pairs"], out["n_pairs"], w * h, w, w * h, w)
    torch.cuda.synchronize()
    ref = oracle.reciprocal(d1, d2, seeds, 10)
    want = oracle.pairs_to_pixels(ref["pairs"], w, w, w * h, w * h)
    assert int(host(count)[0]) == want.shape[0] and np.array_equal(host(xy)[0, :want.shape[0]], want)
    dense = fnn.fnn_mutual_dense(dev(d1), dev(d2), compute="f16")
    conf = np.random.default_rng(5).random((1, w * h)).astype(np.float32)
    xy, count = fnn.fnn_pairs_to_pixels(dense["pairs"], dense["n_pairs"], w * h, w, w * h, w, dev(conf), dev(conf), 0.5, 0.5)
    torch.cuda.synchronize()
    want = oracle.pairs_to_pixels(oracle.mutual_dense(d1, d2)["pairs"], w, w, w * h, w * h, conf[0], conf[0], 0.5, 0.5)
    assert int(host(count)[0]) == want.shape[0] and np.array_equal(host(xy)[0, :want.shape[0]], want)
