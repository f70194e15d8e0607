"""The measurement aid that times the kernels' bare instruction mix: it must run, report plausible
figures, and the figures must order the way the instruction counts do."""
import pytest
import torch

import paper_2503_10017_amd as fnn

pytestmark = pytest.mark.gpu


def test_ceiling_figures_are_plausible_and_ordered():
    scratch = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    ns = [fnn.fnn_measure_ceiling(mix, 65536, scratch=scratch) for mix in range(9)]
    # one K=16 instruction of a 32x32 block is 32768 flops: at the published 2.5 PFLOP/s over 1024 SIMDs
    # that is 13.4 ns; nothing can be faster, and an idle-free device is not 20x slower either
    assert all(10.0 < x < 400.0 for x in ns), ns
    k16, k16_k8, k16_k16, fold8, max16, quad16x16x32, bf_k16_k8, bf_fold8, bf_max16 = ns
    assert k16_k8 > 1.5 * k16 and k16_k16 > 1.5 * k16           # a second matrix instruction costs about as much as the first
    assert fold8 >= 0.98 * k16_k8 and max16 >= 0.98 * fold8     # vector work never makes a block cheaper
    # the 24-channel block padded to 32 channels and run as four 16x16x32 instructions is no cheaper
    # than the K=16 + K=8 pair (beyond run-to-run noise, which reaches 10 % between loops of one run while the
    # clock settles): padding does not buy matrix time back
    assert quad16x16x32 >= 0.85 * k16_k8, (quad16x16x32, k16_k8)
    # the bfloat16 instructions cost what the fp16 ones do, with and without the vector work
    assert 0.75 * k16_k8 < bf_k16_k8 < 1.25 * k16_k8
    assert bf_fold8 >= 0.98 * bf_k16_k8 and bf_max16 >= 0.98 * bf_fold8
    with pytest.raises(fnn.FnnError) as err:
        fnn.fnn_measure_ceiling(9, 16384, scratch=scratch)
    assert err.value.status == 4
    with pytest.raises(fnn.FnnError) as err:
        fnn.fnn_measure_ceiling(1, 16384, scratch=scratch[:1024])
    assert err.value.status == 5
