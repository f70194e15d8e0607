"""The search launcher picks how many query blocks a wave keeps resident (1, 2 or 4 groups of four) from the
batch size, the query count and the candidate count.  These shapes are chosen to reach each choice on an
MI355X (64 pairs leave 32 waves per pair; a wave takes more groups only while its chunk keeps >= 128 tiles,
and rows wider than 48 bytes stop at two groups); the launch reports its choice through the kernel trace, and
whatever is chosen the results must be bit-identical to single-pair calls (which use one group) and to the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import dev, exact_maps, host

pytestmark = pytest.mark.gpu


def traced_nearest(*args, **kw):
    fnn.fnn_trace_begin(16)
    try:
        out = fnn.fnn_nearest(*args, **kw)
        torch.cuda.synchronize()
    finally:
        trace = fnn.fnn_trace_end(16, details=True)
    groups = [detail for name, _, detail in trace if name == "search_kernel"]
    assert len(groups) == 1
    return out, groups[0]


@pytest.mark.parametrize("nq,m,compute,l2,want_groups", [
    (128, 262144 + 17, "f16", False, 4),     # 8193 tiles / 32 chunks = 256 per chunk: four groups
    (512, 160000, "f16", False, 4),          # 5000 tiles: 156 per chunk with four groups
    (512, 100000, "f16", False, 2),          # 3125 tiles: 97 per chunk with four groups, 195 with two
    (512, 40000, "f16", False, 1),           # 1250 tiles: short chunks, one group
    (512, 100000, "bf16", False, 2),
    (512, 160000, "bf16", True, 2),          # 32-channel rows: at most two groups (312 tiles per chunk)
    (512, 40000, "bf16", True, 1),           # 32-channel rows, 78 tiles per chunk with two groups: one
    (128, 262144 + 17, "f32", False, 2),     # fp32 rows of 24 channels: at most two groups (256 tiles per chunk)
    (128, 100000, "f32", False, 1),          # 97 tiles per chunk: one group
])
def test_every_row_group_width_gives_the_same_answers(nq, m, compute, l2, want_groups):
    batch, n, d = 64, 2048, 24
    _, cand = exact_maps(900 + nq, 1, m, d)
    tb = dev(cand)
    rng = np.random.default_rng(nq + m)
    srcs = [rng.integers(-8, 9, size=(n, d)).astype(np.float32) / 8 for _ in range(batch)]
    q = np.stack([np.sort(rng.choice(n, nq, replace=False)) for _ in range(batch)]).astype(np.int32)
    ts = [dev(x) for x in srcs]
    (gi, gs), groups = traced_nearest(ts, [tb] * batch, q_idx=dev(q), compute=compute, l2=l2)
    assert groups == want_groups, f"the launcher chose {groups} row groups per wave, the shape was built for {want_groups}"
    gi, gs = host(gi), host(gs)
    for b in (0, 17, 63):                  # single-pair calls: many waves per pair, one group per wave
        (si, ss), single_groups = traced_nearest(ts[b], tb, q_idx=dev(q[b])[None], compute=compute, l2=l2)
        assert single_groups == 1
        assert np.array_equal(gi[b], host(si)[0]) and np.array_equal(gs[b], host(ss)[0])
    for b in (0, 63):
        if l2:
            ri, rbest, _ = oracle.nearest_l2(srcs[b][q[b]], cand)
            assert np.array_equal(gi[b], ri) and np.array_equal(-2.0 * gs[b], rbest)
        else:
            ri, rbest, _ = oracle.nearest(srcs[b][q[b]], cand)
            assert np.array_equal(gi[b], ri) and np.array_equal(gs[b], rbest)


@pytest.mark.parametrize("batch,m,compute,kw", [
    (1, 30011, "f16", {}),              # one pair: chunks shorter than the ring
    (16, 196608 + 5, "f16", {}),        # the batched shape (four row groups per wave in the ordinary path)
    (16, 50000, "bf16", {"l2": True}),  # 32-channel rows
    (4, 40000, "f32", {}),              # fp32 rows
    (4, 20000, "f16", {"split": True}), # 80-channel rows of the two-term representation (ordinary ring)
])
def test_few_live_queries_take_the_streaming_path_with_the_same_answers(batch, m, compute, kw):
    """A pair with at most 128 live queries is searched by a path of its own (only the 32-query blocks
    that hold a live query are multiplied, a longer ring of candidate tiles in flight).  Live counts on
    both sides of every block boundary, mixed within one batch, against the oracle bit for bit; outputs
    past the live count stay untouched."""
    n, d, nq = 4096, 24, 160
    rng = np.random.default_rng(batch * 1000 + m)
    cand = rng.integers(-8, 9, size=(m, d)).astype(np.float32) / 8
    tb = dev(cand)
    srcs = [rng.integers(-8, 9, size=(n, d)).astype(np.float32) / 8 for _ in range(batch)]
    q = rng.integers(0, n, size=(batch, nq)).astype(np.int32)
    counts = [1, 31, 32, 33, 63, 64, 65, 96, 97, 127, 128, 129, 160, 3, 0, 106]
    active = np.array([counts[b % len(counts)] for b in range(batch)], dtype=np.int32)
    if batch == 1:
        runs = [np.array([c], dtype=np.int32) for c in (1, 32, 33, 64, 65, 128, 129)]
    else:
        runs = [active, np.roll(active, 5)]
    ts = [dev(x) for x in srcs]
    for act in runs:
        out_idx = torch.full((batch, nq), -7, dtype=torch.int32, device="cuda:0")
        out_score = torch.full((batch, nq), -7.0, dtype=torch.float32, device="cuda:0")
        fnn.fnn_nearest(ts, [tb] * batch, q_idx=dev(q), nq_active=dev(act), compute=compute,
                        out_idx=out_idx, out_score=out_score, **kw)
        torch.cuda.synchronize()
        gi, gs = host(out_idx), host(out_score)
        for b in range(batch):
            k = int(act[b])
            if kw.get("l2"):
                ri, rbest, _ = oracle.nearest_l2(srcs[b][q[b, :k]], cand)
                assert np.array_equal(gi[b, :k], ri) and np.array_equal(-2.0 * gs[b, :k], rbest), (b, k)
            else:
                ri, rbest, _ = oracle.nearest(srcs[b][q[b, :k]], cand)
                assert np.array_equal(gi[b, :k], ri) and np.array_equal(gs[b, :k], rbest), (b, k)
            assert np.all(gi[b, k:] == -7) and np.all(gs[b, k:] == -7.0), (b, k)
