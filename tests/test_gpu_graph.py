"""fnn_reciprocal captured into a HIP graph (the library launches kernels only and clears its buffers with
kernels, so a call can be recorded once and replayed): every replay, with eager calls and new inputs in
between, must give what the eager call gives on the same inputs."""
import numpy as np
import pytest
import torch

import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import dev, unit_maps

pytestmark = pytest.mark.gpu

KEYS = ("seed_i", "seed_j", "seed_iter", "pairs", "n_pairs")


@pytest.mark.parametrize("width,height,stride,static", [(160, 120, 4, False), (256, 192, 4, False), (160, 120, 4, True)])
def test_graph_replays_match_eager_calls(width, height, stride, static):
    pairs = [synth.warped_pair(900 + i, width, height, 24)[:2] for i in range(3)]
    seeds = dev(synth.grid_seeds(width, height, stride))[None]
    n = width * height
    d1 = torch.empty((n, 24), dtype=torch.float32, device="cuda:0")
    d2 = torch.empty((n, 24), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(fnn.fnn_workspace_bytes(1, n, n, 24, seeds.shape[1], "f16"), dtype=torch.uint8, device="cuda:0")

    def call(out):
        if static:
            return fnn.fnn_reciprocal_static(d1, d2, seeds, out, max_iter=10, compute="f16")
        return fnn.fnn_reciprocal(d1, d2, seeds, max_iter=10, compute="f16", out=out, workspace=ws)

    d1.copy_(dev(pairs[0][0]))
    d2.copy_(dev(pairs[0][1]))
    out = fnn.fnn_reciprocal(d1, d2, seeds, max_iter=10, compute="f16", workspace=ws)   # eager first: fills the launch caches
    call(out)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(out)
    for a, b in pairs + pairs[:1]:
        d1.copy_(dev(a))
        d2.copy_(dev(b))
        want = fnn.fnn_reciprocal(d1, d2, seeds, max_iter=10, compute="f16")     # eager, its own buffers
        torch.cuda.synchronize()
        for k in KEYS:
            out[k].fill_(-3)
        graph.replay()
        torch.cuda.synchronize()
        for k in KEYS:
            assert torch.equal(out[k], want[k]), k
        assert int(want["n_pairs"][0]) > 0


def test_dense_graph_replays_match_eager_calls():
    """The same for fnn_mutual_dense, at a size whose interior workgroups take the staged sweep (direct
    global->LDS loads) and whose edge workgroups take the unstaged one."""
    n, m = 9000, 5000
    maps = [unit_maps(700 + i, n, m, 24) for i in range(3)]
    d1 = torch.empty((n, 24), dtype=torch.float32, device="cuda:0")
    d2 = torch.empty((m, 24), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(fnn.fnn_workspace_bytes(1, n, m, 24, 0, "f16"), dtype=torch.uint8, device="cuda:0")
    d1.copy_(dev(maps[0][0]))
    d2.copy_(dev(maps[0][1]))
    out = fnn.fnn_mutual_dense(d1, d2, "f16", workspace=ws)
    fnn.fnn_mutual_dense(d1, d2, "f16", out=out, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fnn.fnn_mutual_dense(d1, d2, "f16", out=out, workspace=ws)
    for a, b in maps + maps[:1]:
        d1.copy_(dev(a))
        d2.copy_(dev(b))
        want = fnn.fnn_mutual_dense(d1, d2, "f16")
        torch.cuda.synchronize()
        for k in out:
            out[k].fill_(-3)
        graph.replay()
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], want[k]), k
        assert int(want["n_pairs"][0]) > 0
