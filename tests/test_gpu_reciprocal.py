"""fnn_reciprocal on the GPU against the CPU oracle."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import (GAP_F32, GAP_HALF, GAP_ROUNDED, ROUNDERS, check_reciprocal_exact, check_reciprocal_pinned,
                         dev, exact_maps, host, run_reciprocal)

pytestmark = pytest.mark.gpu

COMPUTES = ["f16", "bf16", "f32"]


@pytest.mark.parametrize("compute", COMPUTES)
def test_handworked_walks(golden_dir, compute):
    with open(os.path.join(golden_dir, "handworked_walk.json")) as f:
        g = json.load(f)
    d1 = np.asarray(g["scores"], dtype=np.float32)
    d2 = np.eye(6, dtype=np.float32)
    seeds = np.asarray(g["seeds"], dtype=np.int32)[None]
    for case in g["cases"]:
        got = run_reciprocal([d1], [d2], seeds, case["max_iter"], compute)
        n_pairs = int(got["n_pairs"][0])
        assert got["seed_i"][0].tolist() == case["seed_i"]
        assert got["seed_j"][0].tolist() == case["seed_j"]
        assert got["seed_iter"][0].tolist() == case["seed_iter"]
        assert got["pairs"][0, :n_pairs].tolist() == case["pairs"]


@pytest.mark.parametrize("compute", COMPUTES)
@pytest.mark.parametrize("w,h,d,sub,max_iter", [(64, 48, 24, 8, 10), (64, 48, 24, 1, 10), (40, 30, 8, 3, 10),
                                                  (33, 17, 24, 2, 2), (64, 48, 2, 4, 1), (64, 48, 24, 8, 0),
                                                  (100, 70, 32, 5, 4)])
def test_exact_inputs_bit_exact(compute, w, h, d, sub, max_iter):
    a, b = synth.exact_pair(10 * w + h + d, w, h, d)
    seeds = synth.grid_seeds(w, h, sub)
    ref = oracle.reciprocal(a, b, seeds, max_iter)
    got = run_reciprocal([a], [b], seeds[None], max_iter, compute)
    check_reciprocal_exact(got, 0, ref)


def test_rectangular_maps_and_duplicate_seeds():
    a, b = exact_maps(77, 900, 2500, 24)
    rng = np.random.default_rng(1)
    seeds = rng.integers(0, 900, size=400).astype(np.int32)          # with repeats
    ref = oracle.reciprocal(a, b, seeds, 10)
    for compute in COMPUTES:
        got = run_reciprocal([a], [b], seeds[None], 10, compute)
        check_reciprocal_exact(got, 0, ref)


def test_batch_of_exact_pairs():
    pairs = [synth.exact_pair(300 + b, 48, 40, 24) for b in range(5)]
    rng = np.random.default_rng(12)
    seeds = rng.integers(0, 48 * 40, size=(5, 240)).astype(np.int32)
    got = run_reciprocal([p[0] for p in pairs], [p[1] for p in pairs], seeds, 10, "f16")
    for b in range(5):
        ref = oracle.reciprocal(pairs[b][0], pairs[b][1], seeds[b], 10)
        check_reciprocal_exact(got, b, ref)


def test_all_pixel_seeds_equal_dense_mutual_on_gpu():
    # every mutual pair is found at t = 0 by its own seed, so the two entry points must agree
    a, b = synth.config_pair(1)
    seeds = np.arange(a.shape[0], dtype=np.int32)[None]
    got = run_reciprocal([a], [b], seeds, 10, "f16")
    dense = fnn.fnn_mutual_dense(dev(a), dev(b), compute="f16")
    torch.cuda.synchronize()
    n_pairs, n_dense = int(got["n_pairs"][0]), int(dense["n_pairs"][0])
    assert n_pairs == n_dense
    assert np.array_equal(got["pairs"][0, :n_pairs], host(dense["pairs"])[0, :n_dense])
    check_reciprocal_exact(got, 0, oracle.reciprocal(a, b, seeds[0], 10))


def test_no_seeds():
    a, b = exact_maps(2, 64, 64, 24)
    got = run_reciprocal([a], [b], np.zeros((1, 0), dtype=np.int32), 10, "f16")
    assert int(got["n_pairs"][0]) == 0


@pytest.mark.parametrize("compute", COMPUTES)
def test_gaussian_pair_pinned_seeds(compute):
    a, b, _ = synth.warped_pair(31, 160, 120, 24)
    seeds = synth.grid_seeds(160, 120, 4)
    got = run_reciprocal([a], [b], seeds[None], 10, compute)
    rnd = ROUNDERS[compute]
    ra, rb = rnd(a), rnd(b)
    ref = oracle.reciprocal(ra, rb, seeds, 10)
    check_reciprocal_pinned(got, 0, ref, ra, rb, GAP_ROUNDED, f"{compute} rounded inputs")
    if compute != "bf16":
        ref = oracle.reciprocal(a, b, seeds, 10)
        check_reciprocal_pinned(got, 0, ref, a, b, GAP_F32 if compute == "f32" else GAP_HALF, f"{compute} fp32 inputs")


def test_many_iterations_and_strided_half_storage():
    # long iteration cap (the launch sequence keeps going after every seed has converged) and
    # fp16 maps stored with a row stride, which takes the generic prepare path
    a, b = synth.exact_pair(91, 56, 40, 24)
    seeds = synth.grid_seeds(56, 40, 3)
    ref = oracle.reciprocal(a, b, seeds, 40)
    wide_a = torch.zeros((a.shape[0], 36), dtype=torch.float16, device=dev(a).device)
    wide_b = torch.zeros((b.shape[0], 36), dtype=torch.float16, device=dev(a).device)
    wide_a[:, :24] = dev(a).to(torch.float16)
    wide_b[:, :24] = dev(b).to(torch.float16)
    out = fnn.fnn_reciprocal(wide_a[:, :24], wide_b[:, :24], dev(seeds)[None], max_iter=40, compute="f16")
    torch.cuda.synchronize()
    check_reciprocal_exact({k: host(v) for k, v in out.items()}, 0, ref)


def test_batch_of_64_pairs():
    pairs = [synth.exact_pair(700 + b, 24, 20, 24) for b in range(64)]
    rng = np.random.default_rng(3)
    seeds = rng.integers(0, 480, size=(64, 50)).astype(np.int32)
    got = run_reciprocal([p[0] for p in pairs], [p[1] for p in pairs], seeds, 10, "bf16")
    for b in range(64):
        check_reciprocal_exact(got, b, oracle.reciprocal(pairs[b][0], pairs[b][1], seeds[b], 10))


def test_fused_normalisation_reciprocal_and_dense():
    rng = np.random.default_rng(5)
    a, b, _ = synth.warped_pair(61, 96, 64, 24)
    a = (a * rng.uniform(0.1, 9.0, size=(a.shape[0], 1))).astype(np.float32)     # undo the unit norms
    b = (b * rng.uniform(0.1, 9.0, size=(b.shape[0], 1))).astype(np.float32)
    seeds = synth.grid_seeds(96, 64, 4)
    out = fnn.fnn_reciprocal(dev(a), dev(b), dev(seeds)[None], max_iter=10, compute="f16", normalize=True)
    dense = fnn.fnn_mutual_dense(dev(a), dev(b), compute="f16", normalize=True)
    torch.cuda.synchronize()
    ra, rb = oracle.round_fp16(oracle.normalize(a)), oracle.round_fp16(oracle.normalize(b))
    ref = oracle.reciprocal(ra, rb, seeds, 10)
    check_reciprocal_pinned({k: host(v) for k, v in out.items()}, 0, ref, ra, rb, GAP_ROUNDED, "normalised")
    dref = oracle.mutual_dense(ra, rb)
    clear = dref["gap12"] > GAP_ROUNDED
    assert np.array_equal(host(dense["nn12"])[0][clear], dref["nn12"][clear])
    clear = dref["gap21"] > GAP_ROUNDED
    assert np.array_equal(host(dense["nn21"])[0][clear], dref["nn21"][clear])


def test_hip_graph_capture_and_replay():
    # the call sequence allocates nothing, never synchronises and clears its buffers with
    # kernels, so it can be captured into a HIP graph; every replay must equal the eager result
    a, b, _ = synth.warped_pair(83, 128, 96, 24)
    seeds = dev(synth.grid_seeds(128, 96, 4))[None]
    ta, tb = dev(a), dev(b)
    ws = torch.empty(fnn.fnn_workspace_bytes(1, a.shape[0], b.shape[0], 24, seeds.shape[1], "f16"),
                     dtype=torch.uint8, device=ta.device)
    eager = fnn.fnn_reciprocal(ta, tb, seeds, max_iter=10, compute="f16", workspace=ws)   # also warms the launch caches
    torch.cuda.synchronize()
    want = {k: host(v).copy() for k, v in eager.items()}
    out = {k: torch.zeros_like(v) for k, v in eager.items()}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fnn.fnn_reciprocal(ta, tb, seeds, max_iter=10, compute="f16", out=out, workspace=ws, stream=side)
    torch.cuda.synchronize()
    for rep in range(3):
        for v in out.values():
            v.fill_(-5)                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in want:
            assert np.array_equal(host(out[k]), want[k]), (rep, k)
        again = fnn.fnn_reciprocal(ta, tb, seeds, max_iter=10, compute="f16", workspace=ws)
        torch.cuda.synchronize()
        for k in want:
            assert np.array_equal(host(again[k]), want[k]), (rep, k, "eager")
