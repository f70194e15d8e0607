"""The paper's blocked schedules (Algorithms 1 and 2 with a materialised score block) must
return exactly what the fused search returns."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import check_nearest_gaussian, dev, exact_maps, host, unit_maps

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("compute", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("k,m,d,rows,cols", [(1, 1, 1, 1, 0), (70, 333, 24, 32, 0), (300, 1000, 24, 128, 0), (300, 1000, 24, 128, 256),
                                               (257, 4100, 24, 100, 1000), (1000, 3072, 8, 512, 32), (513, 700, 32, 1024, 0)])
def test_exact_inputs_bit_exact(compute, k, m, d, rows, cols):
    a, b = exact_maps(k + 7 * m + rows + cols, k, m, d)
    ri, rb, _ = oracle.nearest(a, b)
    gi, gs = fnn.fnn_nearest_blocked(dev(a), dev(b), rows, cols, compute=compute)
    torch.cuda.synchronize()
    assert np.array_equal(host(gi), ri)
    assert np.array_equal(host(gs), rb)


def test_query_list_and_agreement_with_the_fused_search():
    a, b = unit_maps(3, 5000, 20000, 24)
    rng = np.random.default_rng(4)
    q = rng.integers(0, 5000, size=777).astype(np.int32)
    fused_i, fused_s = fnn.fnn_nearest(dev(a), dev(b), q_idx=dev(q)[None], compute="f16")
    for rows, cols in ((256, 0), (256, 2048)):
        gi, gs = fnn.fnn_nearest_blocked(dev(a), dev(b), rows, cols, q_idx=dev(q), compute="f16")
        torch.cuda.synchronize()
        check_nearest_gaussian(a[q], b, "f16", host(gi), host(gs), f"blocked {rows}x{cols}")
        assert np.array_equal(host(gi), host(fused_i)[0])          # same arithmetic, other schedule
        assert np.array_equal(host(gs), host(fused_s)[0])


def test_half_accumulate_control_matches_its_oracle():
    # bit-exact: IEEE binary16 multiply and add on both sides
    a, b = unit_maps(9, 300, 5000, 24)
    for rows, cols in ((128, 0), (128, 1024)):
        gi, gs = fnn.fnn_nearest_blocked(dev(a), dev(b), rows, cols, compute="f16", half_accumulate=True)
        torch.cuda.synchronize()
        ri, rb = oracle.nearest_half_accumulate(a, b)
        assert np.array_equal(host(gi), ri)
        assert np.array_equal(host(gs), rb)
    a2 = np.array([[32.0, 1.0, 1.0]], dtype=np.float32)
    b2 = np.array([[64.0, 1.0, 1.0], [64.0, 1.5, 0.0]], dtype=np.float32)
    gi, gs = fnn.fnn_nearest_blocked(dev(a2), dev(b2), 1, 0, compute="f16", half_accumulate=True)
    assert host(gi).tolist() == [1] and host(gs).tolist() == [2050.0]
    gi, gs = fnn.fnn_nearest_blocked(dev(a2), dev(b2), 1, 0, compute="f16")
    assert host(gi).tolist() == [0] and host(gs).tolist() == [2050.0]
    # only the blocked entry point offers it, and only for fp16
    with pytest.raises(fnn.FnnError):
        fnn.fnn_nearest_blocked(dev(a), dev(b), 128, 0, compute="bf16", half_accumulate=True)
