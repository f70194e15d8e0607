"""The measurement aid that times the kernels' bare instruction mix: it must run, report plausible
figures, and the figures must order the way the instruction counts do."""
import pytest
import torch

import paper_2503_10017_amd as fnn

pytestmark = pytest.mark.gpu


def test_ceiling_figures_are_plausible_and_ordered():
    scratch = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    ns = [fnn.fnn_measure_ceiling(mix, 16384, scratch=scratch) for mix in range(5)]
    # one K=16 instruction of a 32x32 block is 32768 flops: at the published 2.5 PFLOP/s over 1024 SIMDs
    # that is 13.4 ns; nothing can be faster, and an idle-free device is not 20x slower either
    assert all(10.0 < x < 400.0 for x in ns), ns
    k16, k16_k8, k16_k16, fold8, max16 = ns
    assert k16_k8 > 1.5 * k16 and k16_k16 > 1.5 * k16           # a second matrix instruction costs about as much as the first
    assert fold8 >= 0.98 * k16_k8 and max16 >= 0.98 * fold8     # vector work never makes a block cheaper
    with pytest.raises(fnn.FnnError) as err:
        fnn.fnn_measure_ceiling(7, 16384, scratch=scratch)
    assert err.value.status == 4
    with pytest.raises(fnn.FnnError) as err:
        fnn.fnn_measure_ceiling(1, 16384, scratch=scratch[:1024])
    assert err.value.status == 5
