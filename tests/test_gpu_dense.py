"""fnn_mutual_dense on the GPU against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
from gpu_helpers import GAP_F32, GAP_HALF, GAP_ROUNDED, ROUNDERS, SCORE_TOL, SCORE_TOL_ROUNDED, dev, exact_maps, host, unit_maps

pytestmark = pytest.mark.gpu

COMPUTES = ["f16", "bf16", "f32"]


def run_dense(d1, d2, compute):
    out = fnn.fnn_mutual_dense([dev(x) for x in d1], [dev(x) for x in d2], compute=compute)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def check_exact(got, b, ref):
    n_pairs = int(got["n_pairs"][b])
    assert np.array_equal(got["nn12"][b], ref["nn12"])
    assert np.array_equal(got["nn21"][b], ref["nn21"])
    assert np.array_equal(got["s12"][b], ref["s12"])
    assert np.array_equal(got["s21"][b], ref["s21"])
    assert np.array_equal(got["pairs"][b, :n_pairs], ref["pairs"])
    assert np.all(got["pairs"][b, n_pairs:] == -1)


@pytest.mark.parametrize("compute", COMPUTES)
@pytest.mark.parametrize("n,m,d", [(1, 1, 1), (31, 33, 24), (64, 64, 24), (100, 7, 8), (7, 100, 16), (257, 1025, 24),
                                   (3072, 3072, 24), (5000, 4100, 24), (4097, 9000, 32), (9001, 300, 5)])
def test_exact_inputs_bit_exact(compute, n, m, d):
    a, b = exact_maps(3 * n + m + d, n, m, d)
    check_exact(run_dense([a], [b], compute), 0, oracle.mutual_dense(a, b))


def test_batch_of_exact_pairs():
    pairs = [exact_maps(900 + b, 1500, 1300, 24) for b in range(4)]
    got = run_dense([p[0] for p in pairs], [p[1] for p in pairs], "bf16")
    for b in range(4):
        check_exact(got, b, oracle.mutual_dense(*pairs[b]))


def test_permuted_copy_closed_form():
    rng = np.random.default_rng(8)
    a, _ = unit_maps(8, 3000, 1, 24)
    perm = rng.permutation(3000)
    b = np.empty_like(a)
    b[perm] = a
    for compute in COMPUTES:
        got = run_dense([a], [b], compute)
        assert np.array_equal(got["nn12"][0], perm)
        assert int(got["n_pairs"][0]) == 3000
        assert np.array_equal(got["pairs"][0], np.stack([np.arange(3000), perm], axis=1))


def check_gaussian(got, a, b, compute):
    rnd = ROUNDERS[compute]
    refs = [(oracle.mutual_dense(rnd(a), rnd(b)), GAP_ROUNDED, SCORE_TOL_ROUNDED)]
    if compute != "bf16":
        refs.append((oracle.mutual_dense(a, b), GAP_F32 if compute == "f32" else GAP_HALF, SCORE_TOL))
    for ref, gap, tol in refs:
        for nn, s, g in (("nn12", "s12", "gap12"), ("nn21", "s21", "gap21")):
            clear = ref[g] > gap
            assert clear.mean() > 0.9
            assert np.array_equal(got[nn][0][clear], ref[nn][clear]), (compute, nn)
            assert np.all(np.abs(got[s][0] - ref[s]) <= tol), (compute, s)
    # the reciprocity filter is integer logic on the GPU's own tables: check it exhaustively
    nn12, nn21 = got["nn12"][0], got["nn21"][0]
    i = np.arange(a.shape[0])
    keep = nn21[nn12] == i
    want = np.stack([i[keep], nn12[keep]], axis=1)
    n_pairs = int(got["n_pairs"][0])
    assert np.array_equal(got["pairs"][0, :n_pairs], want)


@pytest.mark.parametrize("compute", COMPUTES)
@pytest.mark.parametrize("n,m", [(6000, 6000), (4133, 9050)])
def test_gaussian_inputs(compute, n, m):
    a, b = unit_maps(n + m, n, m, 24)
    check_gaussian(run_dense([a], [b], compute), a, b, compute)


def test_empty_sides():
    a, _ = exact_maps(1, 40, 1, 24)
    out = fnn.fnn_mutual_dense(dev(a), torch.zeros((0, 24), device=dev(a).device), compute="f16")
    torch.cuda.synchronize()
    assert int(out["n_pairs"][0]) == 0 and np.all(host(out["nn12"]) == -1)


def test_strided_half_storage_and_nearest_agreement():
    # bf16 storage with a row stride (generic prepare path); the dense row table must also
    # equal what fnn_nearest returns for every pixel as a query (same arithmetic, other kernel)
    a, b = exact_maps(17, 2300, 4500, 24)
    wide_a = torch.zeros((2300, 32), dtype=torch.bfloat16, device=dev(a).device)
    wide_b = torch.zeros((4500, 32), dtype=torch.bfloat16, device=dev(a).device)
    wide_a[:, :24] = dev(a).to(torch.bfloat16)
    wide_b[:, :24] = dev(b).to(torch.bfloat16)
    out = fnn.fnn_mutual_dense(wide_a[:, :24], wide_b[:, :24], compute="bf16")
    gi, gs = fnn.fnn_nearest(wide_a[:, :24], wide_b[:, :24], compute="bf16")
    gj, _ = fnn.fnn_nearest(wide_b[:, :24], wide_a[:, :24], compute="bf16")
    torch.cuda.synchronize()
    ref = oracle.mutual_dense(a, b)
    check_exact({k: host(v) for k, v in out.items()}, 0, ref)
    assert np.array_equal(host(gi)[0], ref["nn12"]) and np.array_equal(host(gs)[0], ref["s12"])
    assert np.array_equal(host(gj)[0], ref["nn21"])


@pytest.mark.parametrize("compute,d,staged", [("f16", 24, True), ("bf16", 24, True), ("f32", 24, False), ("f16", 16, False), ("f16", 32, False)])
def test_which_pass1_kernel_ran(compute, d, staged):
    """16-bit rows of 24 channels take the kernel that stages the query blocks through LDS (trace detail
    1), everything else the one with per-wave loads; a shape with interior workgroups (staged sweep) and
    edge workgroups (padding: unstaged sweep inside the same kernel) is bit-exact either way."""
    a, b = exact_maps(77, 9000, 5000, d)
    fnn.fnn_trace_begin(64)
    got = run_dense([a], [b], compute)
    trace = fnn.fnn_trace_end(64, details=True)
    details = [detail for name, _, detail in trace if name == "dense_kernel"]
    assert details == [1 if staged else 0]
    check_exact(got, 0, oracle.mutual_dense(a, b))


def test_staged_kernel_batch_and_several_groups_per_workgroup():
    """The staged pass-1 kernel beyond the small shapes: a batch of two pairs with interior and edge
    workgroups, and one pair large enough that a workgroup sweeps several candidate groups (the query
    stream repeats per group) while its last super-block and last group still meet padding."""
    pairs = [exact_maps(300 + b, 9000, 5000, 24) for b in range(2)]
    got = run_dense([p[0] for p in pairs], [p[1] for p in pairs], "f16")
    for b in range(2):
        check_exact(got, b, oracle.mutual_dense(*pairs[b]))
    a, b = exact_maps(41, 150000, 30000, 24)
    check_exact(run_dense([a], [b], "bf16"), 0, oracle.mutual_dense(a, b))
