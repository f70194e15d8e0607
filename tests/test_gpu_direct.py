"""Maps that already have the layout the kernels read (stored in the compute format, rows packed, whole
32-pixel tiles, pairs stacked in one array) are used in place instead of being copied by the prepare
pass.  The answers must not depend on which way a map took: every case here is compared with the oracle
bit for bit (entries k/8) and with the same data handed over in a layout that has to be copied."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import check_reciprocal_exact, dev, host

pytestmark = pytest.mark.gpu

TORCH = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}


@pytest.mark.parametrize("compute,d", [("f16", 24), ("bf16", 24), ("f32", 24), ("f16", 16), ("f16", 32), ("f32", 8)])
def test_nearest_on_maps_used_in_place(compute, d):
    batch, n, m = 3, 64 * 3, 32 * 41                                       # whole tiles
    rng = np.random.default_rng(d)
    a = rng.integers(-8, 9, size=(batch, n, d)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(batch, m, d)).astype(np.float32) / 8
    ta, tb = dev(a).to(TORCH[compute]), dev(b).to(TORCH[compute])          # stacked, packed, compute format: in place
    gi, gs = fnn.fnn_nearest(ta, tb, compute=compute)
    # the same values in layouts that must be copied: fp32 storage / separately allocated pairs / padded rows
    unstacked = [tb[p].clone() for p in range(batch)]                      # separately allocated pairs
    wide = dev(np.pad(a, ((0, 0), (0, 0), (0, 8)))).to(TORCH[compute])[:, :, :d]   # rows d + 8 apart
    ci, cs = fnn.fnn_nearest([wide[p] for p in range(batch)], unstacked, compute=compute)
    torch.cuda.synchronize()
    assert np.array_equal(host(gi), host(ci)) and np.array_equal(host(gs), host(cs))
    for p in range(batch):
        ri, rbest, _ = oracle.nearest(a[p], b[p])
        assert np.array_equal(host(gi)[p], ri) and np.array_equal(host(gs)[p], rbest)


def test_only_whole_tiles_and_packed_rows_are_used_in_place():
    # 100 rows are not whole tiles, and a strided view is not packed: both are copied, answers unchanged
    rng = np.random.default_rng(5)
    a = rng.integers(-8, 9, size=(100, 24)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(320, 40)).astype(np.float32) / 8
    tb = dev(b).half()[:, :24]                                            # row stride 40
    gi, gs = fnn.fnn_nearest(dev(a).half(), tb, compute="f16")
    torch.cuda.synchronize()
    ri, rbest, _ = oracle.nearest(a, b[:, :24])
    assert np.array_equal(host(gi)[0], ri) and np.array_equal(host(gs)[0], rbest)


@pytest.mark.parametrize("compute", ["f16", "bf16"])
def test_reciprocal_on_maps_used_in_place(compute):
    w, h, d, batch = 64, 48, 24, 2
    pairs = [synth.exact_pair(300 + p, w, h, d) for p in range(batch)]
    seeds = np.stack([synth.grid_seeds(w, h, 4)] * batch)
    t1 = dev(np.stack([p[0] for p in pairs])).to(TORCH[compute])
    t2 = dev(np.stack([p[1] for p in pairs])).to(TORCH[compute])
    out = fnn.fnn_reciprocal(t1, t2, dev(seeds), max_iter=10, compute=compute)
    torch.cuda.synchronize()
    got = {k: host(v) for k, v in out.items()}
    for p in range(batch):
        check_reciprocal_exact(got, p, oracle.reciprocal(pairs[p][0], pairs[p][1], seeds[p], 10))
    # one side in place, the other copied (fp32 storage)
    out2 = fnn.fnn_reciprocal(t1, dev(np.stack([p[1] for p in pairs])), dev(seeds), max_iter=10, compute=compute)
    torch.cuda.synchronize()
    for k in got:
        assert np.array_equal(host(out2[k]), got[k]), k
    # the caller's maps are read, never written
    assert torch.equal(t1, dev(np.stack([p[0] for p in pairs])).to(TORCH[compute]))


def test_unequally_spaced_batch_is_copied():
    # pairs 0, 1, 2 of the second image at offsets 0, 1, 3 (in maps): not one strided array
    rng = np.random.default_rng(9)
    a = rng.integers(-8, 9, size=(3, 64, 24)).astype(np.float32) / 8
    b = rng.integers(-8, 9, size=(4, 320, 24)).astype(np.float32) / 8
    tb = dev(b).half()
    gi, gs = fnn.fnn_nearest(dev(a).half(), [tb[0], tb[1], tb[3]], compute="f16")
    torch.cuda.synchronize()
    for p, src in enumerate((0, 1, 3)):
        ri, rbest, _ = oracle.nearest(a[p], b[src])
        assert np.array_equal(host(gi)[p], ri) and np.array_equal(host(gs)[p], rbest)
    # descending addresses: also copied
    gi, gs = fnn.fnn_nearest(dev(a).half()[:2], [tb[2], tb[0]], compute="f16")
    torch.cuda.synchronize()
    for p, src in enumerate((2, 0)):
        ri, rbest, _ = oracle.nearest(a[p], b[src])
        assert np.array_equal(host(gi)[p], ri) and np.array_equal(host(gs)[p], rbest)
    # equally spaced with a gap (every other map of the stack): used in place
    gi, gs = fnn.fnn_nearest(dev(a).half()[:2], [tb[1], tb[3]], compute="f16")
    torch.cuda.synchronize()
    for p, src in enumerate((1, 3)):
        ri, rbest, _ = oracle.nearest(a[p], b[src])
        assert np.array_equal(host(gi)[p], ri) and np.array_equal(host(gs)[p], rbest)
