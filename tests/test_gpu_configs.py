"""The five workload configurations at full size, in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_10017_amd as fnn
import synth_inputs as synth
from gpu_helpers import (GAP_F32, GAP_HALF, GAP_ROUNDED, ROUNDERS, SCORE_TOL, SCORE_TOL_ROUNDED, cached_mutual_dense,
                         check_reciprocal_exact, check_reciprocal_pinned, dev, host, run_reciprocal)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("compute", ["f16", "bf16", "f32"])
def test_config1_exact(compute):
    a, b = synth.config_pair(1)
    seeds = synth.grid_seeds(64, 48, 8)
    got = run_reciprocal([a], [b], seeds[None], 10, compute)
    check_reciprocal_exact(got, 0, oracle.reciprocal(a, b, seeds, 10))
    dense = fnn.fnn_mutual_dense(dev(a), dev(b), compute=compute)
    torch.cuda.synchronize()
    ref = oracle.mutual_dense(a, b)
    n_pairs = int(dense["n_pairs"][0])
    for k in ("nn12", "nn21", "s12", "s21"):
        assert np.array_equal(host(dense[k])[0], ref[k]), k
    assert np.array_equal(host(dense["pairs"])[0, :n_pairs], ref["pairs"])


@pytest.mark.parametrize("compute", ["f16", "f32"])
def test_config2_single_pair(compute):
    a, b = synth.config_pair(2)
    seeds = synth.grid_seeds(512, 384, 8)
    got = run_reciprocal([a], [b], seeds[None], 10, compute)
    ref = oracle.reciprocal(a, b, seeds, 10)
    check_reciprocal_pinned(got, 0, ref, a, b, GAP_F32 if compute == "f32" else GAP_HALF, f"cfg2 {compute}",
                            min_pinned=0.99 if compute == "f32" else 0.9)
    if compute == "f16":
        ra, rb = oracle.round_fp16(a), oracle.round_fp16(b)
        ref = oracle.reciprocal(ra, rb, seeds, 10)
        check_reciprocal_pinned(got, 0, ref, ra, rb, GAP_ROUNDED, "cfg2 f16 rounded")


def _check_dense_sampled(a, b, compute, n_sample, seed):
    out = fnn.fnn_mutual_dense(dev(a), dev(b), compute=compute)
    torch.cuda.synchronize()
    got = {k: host(v)[0] for k, v in out.items()}
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(a.shape[0], n_sample, replace=False))
    cols = np.sort(rng.choice(b.shape[0], n_sample, replace=False))
    rnd = ROUNDERS[compute]
    ra, rb = rnd(a), rnd(b)
    checks = [(ra, rb, GAP_ROUNDED, SCORE_TOL_ROUNDED)]
    if compute == "f16":
        checks.append((a, b, GAP_HALF, SCORE_TOL))
    for xa, xb, gap, tol in checks:
        ri, rbest, rsec = oracle.nearest(xa[rows], xb)
        clear = (rbest - rsec) > gap
        assert clear.mean() > 0.9
        assert np.array_equal(got["nn12"][rows][clear], ri[clear])
        assert np.all(np.abs(got["s12"][rows] - rbest) <= tol)
        ci, cbest, csec = oracle.nearest(xb[cols], xa)
        clear = (cbest - csec) > gap
        assert clear.mean() > 0.9
        assert np.array_equal(got["nn21"][cols][clear], ci[clear])
        assert np.all(np.abs(got["s21"][cols] - cbest) <= tol)
    # properties that hold at any size: the filter and the compaction are integer logic
    nn12, nn21 = got["nn12"], got["nn21"]
    assert nn12.min() >= 0 and nn12.max() < b.shape[0] and nn21.min() >= 0 and nn21.max() < a.shape[0]
    i = np.arange(a.shape[0])
    keep = nn21[nn12] == i
    n_pairs = int(got["n_pairs"])
    assert n_pairs == int(keep.sum())
    assert np.array_equal(got["pairs"][:n_pairs], np.stack([i[keep], nn12[keep]], axis=1))
    assert np.all(got["pairs"][n_pairs:] == -1)
    # a mutual pair's score is computed twice, by the two resolve passes with the operands in
    # swapped roles (query replicated / candidate replicated): the bits must agree
    mi, mj = got["pairs"][:n_pairs, 0], got["pairs"][:n_pairs, 1]
    assert np.array_equal(got["s12"][mi], got["s21"][mj])
    # the score tables are consistent with the index tables (recomputed in float64)
    s = np.einsum("nd,nd->n", ra[rows].astype(np.float64), rb[nn12[rows]].astype(np.float64))
    assert np.all(np.abs(s - got["s12"][rows]) <= 1e-5)
    return got


def test_config3_dense_fp16_sampled():
    a, b = synth.config_pair(3)
    _check_dense_sampled(a, b, "f16", 4096, 3)


@pytest.fixture(scope="module")
def config3_gpu():
    a, b = synth.config_pair(3)
    out = fnn.fnn_mutual_dense(dev(a), dev(b), compute="f16")
    torch.cuda.synchronize()
    return a, b, {k: host(v)[0] for k, v in out.items()}


@pytest.mark.parametrize("inputs", ["rounded", "fp32"])
def test_config3_dense_fp16_full(config3_gpu, inputs):
    """Every row and every column of the 196608 x 196608 problem against the oracle: on inputs rounded
    to fp16 the way the library rounds them (only the fp32 summation order differs) and on the fp32
    inputs themselves (the stated tolerance).  The oracle's arrays are cached on disk by input hash."""
    a, b, got = config3_gpu
    if inputs == "rounded":
        xa, xb, gap, tol = oracle.round_fp16(a), oracle.round_fp16(b), GAP_ROUNDED, SCORE_TOL_ROUNDED
    else:
        xa, xb, gap, tol = a, b, GAP_HALF, SCORE_TOL
    ref = cached_mutual_dense(xa, xb, "cfg3_" + inputs)
    for side in ("12", "21"):
        clear = ref["gap" + side] > gap
        assert clear.mean() > (0.99 if inputs == "rounded" else 0.9), (side, clear.mean())
        bad = clear & (got["nn" + side] != ref["nn" + side])
        assert not bad.any(), f"{inputs} nn{side}: {bad.sum()} indices differ where the gap is clear (first {np.nonzero(bad)[0][:5]})"
        err = np.abs(got["s" + side] - ref["s" + side])
        assert err.max() <= tol, f"{inputs} s{side}: max score error {err.max()}"
    # the pair list: every oracle pair whose two searches were clear is returned, and every returned
    # pair whose two searches were clear is an oracle pair
    n_pairs = int(got["n_pairs"])
    gp = got["pairs"][:n_pairs]
    clear12, clear21 = ref["gap12"] > gap, ref["gap21"] > gap
    want = ref["pairs"][clear12[ref["pairs"][:, 0]] & clear21[ref["pairs"][:, 1]]]
    got_keys = gp[:, 0].astype(np.int64) * b.shape[0] + gp[:, 1]
    want_keys = want[:, 0].astype(np.int64) * b.shape[0] + want[:, 1]
    assert np.isin(want_keys, got_keys).all()
    sure = gp[clear12[gp[:, 0]] & clear21[gp[:, 1]]]
    ref_keys = ref["pairs"][:, 0].astype(np.int64) * b.shape[0] + ref["pairs"][:, 1]
    assert np.isin(sure[:, 0].astype(np.int64) * b.shape[0] + sure[:, 1], ref_keys).all()
    if inputs == "rounded":
        assert len(want) > 0.99 * len(ref["pairs"])


def test_config4_batch16():
    maps = [synth.config_pair(4, p) for p in range(16)]
    seeds = np.tile(synth.grid_seeds(512, 384, 8), (16, 1))
    got = run_reciprocal([m[0] for m in maps], [m[1] for m in maps], seeds, 10, "f16")
    for p in range(16):
        ra, rb = oracle.round_fp16(maps[p][0]), oracle.round_fp16(maps[p][1])
        ref = oracle.reciprocal(ra, rb, seeds[p], 10)
        check_reciprocal_pinned(got, p, ref, ra, rb, GAP_ROUNDED, f"cfg4 pair {p}")
    # the stated tolerance against unrounded inputs, on a few pairs
    for p in (0, 7, 15):
        ref = oracle.reciprocal(maps[p][0], maps[p][1], seeds[p], 10)
        check_reciprocal_pinned(got, p, ref, maps[p][0], maps[p][1], GAP_HALF, f"cfg4 pair {p} fp32 inputs")


def test_config5_large_pair_bf16():
    a, b = synth.config_pair(5)
    got = _check_dense_sampled(a, b, "bf16", 4096, 5)
    # reciprocal on the same pair: walks are independent per seed, so the oracle follows a
    # sample of the 12288 seeds and those must agree
    seeds = synth.grid_seeds(1024, 768, 8)
    assert seeds.shape == (12288,)
    out = run_reciprocal([a], [b], seeds[None], 10, "bf16")
    rng = np.random.default_rng(55)
    pick = np.sort(rng.choice(seeds.shape[0], 1536, replace=False))
    ra, rb = oracle.round_bf16(a), oracle.round_bf16(b)
    ref = oracle.reciprocal(ra, rb, seeds[pick], 10)
    pinned = ref["min_gap"] > GAP_ROUNDED
    assert pinned.mean() > 0.9
    for k in ("seed_i", "seed_j", "seed_iter"):
        assert np.array_equal(out[k][0][pick][pinned], ref[k][pinned]), k
    # pair list = sorted set of the converged seeds' pairs
    done = out["seed_iter"][0] >= 0
    want = np.unique(np.stack([out["seed_i"][0][done], out["seed_j"][0][done]], axis=1), axis=0)
    n_pairs = int(out["n_pairs"][0])
    assert np.array_equal(out["pairs"][0, :n_pairs], want)
    # reciprocal matches are mutual nearest neighbours of the dense result (same arithmetic)
    conv = pick[pinned & (ref["seed_iter"] >= 0)]
    i, j = out["seed_i"][0][conv], out["seed_j"][0][conv]
    assert np.array_equal(got["nn12"][i], j) and np.array_equal(got["nn21"][j], i)
