"""fnn_reciprocal_static (the entry point that allocates nothing: its workspace is an array the library
holds on the device) against fnn_reciprocal, through the C ABI: two calls in a row on the shared array,
the second on a smaller input, each compared with the ordinary entry point bit for bit."""
import numpy as np
import pytest
import torch

import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import dev, host

pytestmark = pytest.mark.gpu


def _outputs(batch, n_seeds):
    device = torch.device("cuda:0")
    return {
        "seed_i": torch.full((batch, n_seeds), -7, dtype=torch.int32, device=device),
        "seed_j": torch.full((batch, n_seeds), -7, dtype=torch.int32, device=device),
        "seed_iter": torch.full((batch, n_seeds), -7, dtype=torch.int32, device=device),
        "pairs": torch.full((batch, n_seeds, 2), -7, dtype=torch.int32, device=device),
        "n_pairs": torch.full((batch,), -7, dtype=torch.int32, device=device),
    }


def _compare(width, height, stride, batch, compute, seed):
    maps = [synth.warped_pair(seed + p, width, height, 24)[:2] for p in range(batch)]
    seeds = np.tile(synth.grid_seeds(width, height, stride), (batch, 1))
    t1 = [dev(m[0]) for m in maps]
    t2 = [dev(m[1]) for m in maps]
    ts = dev(seeds)
    want = fnn.fnn_reciprocal(t1, t2, ts, max_iter=10, compute=compute)
    got = fnn.fnn_reciprocal_static(t1, t2, ts, _outputs(batch, seeds.shape[1]), max_iter=10, compute=compute)
    torch.cuda.synchronize()
    for key in ("seed_i", "seed_j", "seed_iter", "pairs", "n_pairs"):
        assert np.array_equal(host(got[key]), host(want[key])), (key, width, height, compute)
    assert int(host(want["n_pairs"]).min()) > 0
    return int(host(want["n_pairs"]).sum())


def test_static_scratch_entry_point_matches_fnn_reciprocal_on_two_calls_in_a_row():
    first = _compare(320, 240, 8, 2, "f16", 71)     # 76800 pixels, 1200 seeds per pair, two pairs
    second = _compare(96, 64, 4, 1, "f16", 73)      # smaller input on the array the first call left dirty
    third = _compare(160, 120, 4, 1, "f32", 75)     # and another compute format
    assert first > second > 0 and third > 0


def test_static_scratch_limit_is_enforced_before_anything_runs():
    n = 512 * 384
    maps = torch.zeros((16, n, 24), dtype=torch.float32, device="cuda:0")   # 16 pairs need about 300 MB
    seeds = torch.zeros((16, 3072), dtype=torch.int32, device="cuda:0")
    out = _outputs(16, 3072)
    with pytest.raises(fnn.FnnError) as err:
        fnn.fnn_reciprocal_static(maps, maps, seeds, out, max_iter=10, compute="f16")
    assert err.value.status == 5
    torch.cuda.synchronize()
    assert int(out["n_pairs"][0]) == -7   # outputs untouched
