"""Seeded random shapes through every entry point against the oracle: whichever kernel the dispatcher picks for a
shape (stencil, grouped or chunk-parallel matrix-core path, scan, general kernels), the result has to meet the
same tolerance.  Shapes are small enough for the fp64 oracle and ragged on purpose."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_01868_amd import binding, synth

from gpu_util import TOL, check_gated, dev, host, say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    for name in ("se_vec", "se_rows", "mr_rows", "mr_waves", "se_walk"):
        binding.set_option(name, 0)


def pick(rng, xs):
    return xs[int(rng.integers(0, len(xs)))]


def gated_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        group = pick(rng, [1, 1, 2, 4, 8, 16, 16, 32, 64])
        D = group * int(rng.integers(1, 5)) * pick(rng, [1, 2, 4, 8, 16])
        D = min(D, 512)
        D -= D % group
        D = max(D, group)
        lh = pick(rng, [1, 2, 3, 7, 8, 9, 13, 17, 18, 31, 33, 50, 64, 100, 128, 129, 145, 146, 200, 257, 258])
        L = int(rng.integers(1, 1400))
        B = int(rng.integers(1, 4))
        dtype = pick(rng, ["bf16", "bf16", "bf16", "f32"])
        entry = pick(rng, ["hyena_se_fwd", "hyena_mr_fwd"])
        rows = pick(rng, [0, 0, 32, 96, 256, 512])
        out.append((i, entry, B, L, D, lh, group, dtype, rows))
    return out


@pytest.mark.parametrize("case", gated_cases(48, 2024), ids=lambda c: "%d-%s-B%dL%dD%dlh%dg%d%s-r%d" % c)
def test_gated_entry_points_on_random_shapes(case):
    i, entry, B, L, D, lh, group, dtype, rows = case
    binding.set_option("mr_rows", rows)
    binding.set_option("se_rows", rows)
    check_gated(entry, 3000 + i, B, L, D, lh, group, dtype, kind="mr" if lh > 8 else "se")


def li_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        group = pick(rng, [1, 4, 16, 16, 16, 32, 48])
        D = group * int(rng.integers(1, 9))
        if rng.random() < 0.5:
            D = max(64, D - D % 64) if group in (16, 32) else D
        D = max(group, D - D % group)
        order = int(rng.integers(1, 17))
        L = int(rng.integers(1, 1500))
        B = int(rng.integers(1, 4))
        dtype = pick(rng, ["bf16", "bf16", "f32"])
        rows = pick(rng, [0, 32, 64, 160, 512])
        out.append((i, B, L, D, order, group, dtype, rows))
    return out


@pytest.mark.parametrize("case", li_cases(20, 2025), ids=lambda c: "%d-B%dL%dD%do%dg%d%s-r%d" % c)
def test_long_implicit_entry_point_on_random_shapes(case):
    i, B, L, D, order, group, dtype, rows = case
    binding.set_option("mr_rows", rows)
    say("hyena_li_fwd random %s" % (case,))
    rng = np.random.Generator(np.random.PCG64(4000 + i))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    R, lam = synth.li_params(rng, D // group, order)
    y = host(binding.hyena_li_fwd(dev(q), dev(k), dev(v), dev(R), dev(lam), group))
    ref = oracle.li_conv(q, k, v, R, lam, group=group)
    assert np.isfinite(y).all()
    assert oracle.rel_err(y, ref) <= TOL[dtype]


def chain_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        group = pick(rng, [16, 16, 32, 8, 1])
        D = pick(rng, [64, 128, 256, 48, 40])
        D = max(group, D - D % group)
        feat_group = pick(rng, [1, 1, 2]) if D % 2 == 0 else 1
        lf = int(rng.integers(1, 9))
        lh = pick(rng, [8, 33, 64, 128, 129, 130])
        L = int(rng.integers(1, 900))
        B = int(rng.integers(1, 3))
        dtype = pick(rng, ["bf16", "bf16", "f32"])
        out.append((i, B, L, D, lf, feat_group, lh, group, dtype))
    return out


@pytest.mark.parametrize("case", chain_cases(12, 2026), ids=lambda c: "%d-B%dL%dD%dlf%dfg%dlh%dg%d%s" % c)
def test_chain_entry_point_on_random_shapes(case):
    i, B, L, D, lf, feat_group, lh, group, dtype = case
    say("hyena_chain_fwd random %s" % (case,))
    rng = np.random.Generator(np.random.PCG64(5000 + i))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    hq, hk, hv = (synth.short_filter(rng, D // feat_group, lf) for _ in range(3))
    h = synth.decay_filter(rng, D // group, lh)
    y = host(binding.hyena_chain_fwd(dev(q), dev(k), dev(v), dev(hq), dev(hk), dev(hv), dev(h), group, feat_group))
    ref = oracle.chain(q, k, v, hq, hk, hv, h, group=group, feat_group=feat_group)
    assert np.isfinite(y).all()
    assert oracle.rel_err(y, ref) <= TOL[dtype]


def fused_chain_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        D = pick(rng, [128, 128, 256, 384])
        group = pick(rng, [16, 16, 32, 64, 128])
        feat_group = pick(rng, [1, 1, 2, 4, 128])
        lf = int(rng.integers(1, 10))
        lh = int(rng.integers(1, 130))
        L = int(rng.integers(1, 2500))
        B = int(rng.integers(1, 3))
        rows = pick(rng, [0, 32, 64, 96, 160, 256, 1024])
        out.append((i, B, L, D, lf, feat_group, lh, group, rows))
    return out


@pytest.mark.parametrize("case", fused_chain_cases(16, 2027), ids=lambda c: "%d-B%dL%dD%dlf%dfg%dlh%dg%drows%d" % c)
def test_single_kernel_chain_on_random_shapes_and_tile_lengths(case):
    """Shapes the single-kernel chain takes (bf16, D a multiple of 128, groups of 16 channels or more), random
    filter lengths (featurizers up to nine taps), tile lengths and sequence ends."""
    i, B, L, D, lf, feat_group, lh, group, rows = case
    say("hyena_chain_fwd fused random %s" % (case,))
    rng = np.random.Generator(np.random.PCG64(6000 + i))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    hq, hk, hv = (synth.short_filter(rng, D // feat_group, lf) for _ in range(3))
    h = synth.decay_filter(rng, D // group, lh)
    ref = oracle.chain(q, k, v, hq, hk, hv, h, group=group, feat_group=feat_group)
    binding.set_option("mr_rows", rows)
    assert binding.lib().hyena_chain_workspace_bytes(B, L, D, lf, feat_group, lh, group, binding.HY_BF16) == 0
    y = host(binding.hyena_chain_fwd(dev(q), dev(k), dev(v), dev(hq), dev(hk), dev(hv), dev(h), group, feat_group))
    assert np.isfinite(y).all()
    assert oracle.rel_err(y, ref) <= TOL["bf16"]


def knob_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        D = pick(rng, [128, 128, 256, 384])
        group = pick(rng, [1, 2, 8, 16, 32, 64])
        lh = pick(rng, [int(rng.integers(1, 9)), int(rng.integers(9, 130)), int(rng.integers(130, 258))])
        L = int(rng.integers(1, 2600))
        B = int(rng.integers(1, 3))
        knobs = (pick(rng, [0, 32, 64, 96, 256, 1024]), pick(rng, [0, 4, 8, 16]), pick(rng, [0, 1, 2]),
                 pick(rng, [0, 32, 100, 256, 1000]), pick(rng, [0, 2, 4, 8]))
        out.append((i, pick(rng, ["hyena_se_fwd", "hyena_mr_fwd"]), B, L, D, lh, group) + knobs)
    return out


@pytest.mark.parametrize("case", knob_cases(48, 2028),
                         ids=lambda c: "%d-%s-B%dL%dD%dlh%dg%d-mr%dw%dwalk%dse%dvec%d" % c)
def test_every_tuning_knob_combination_leaves_the_result_within_tolerance(case):
    """Widths where all bf16 kernels apply (stencil, tile walker, grouped, both chunk-parallel kernels with and
    without mover waves), with the tuning options drawn at random: they may change which kernel runs and how it is
    tiled, never the result beyond rounding."""
    i, entry, B, L, D, lh, group, mr_rows, mr_waves, se_walk, se_rows, se_vec = case
    for name, value in (("mr_rows", mr_rows), ("mr_waves", mr_waves), ("se_walk", se_walk), ("se_rows", se_rows),
                        ("se_vec", se_vec)):
        binding.set_option(name, value)
    check_gated(entry, 7000 + i, B, L, D, lh, group, "bf16", kind="mr" if lh > 8 else "se")


def bwd_cases(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        group = pick(rng, [1, 1, 2, 4, 8, 16, 16, 32, 64])
        D = group * int(rng.integers(1, 5)) * pick(rng, [1, 2, 4, 8, 16])
        D = min(D, 512)
        D -= D % group
        D = max(D, group)
        if rng.random() < 0.4:  # widths the matrix-core and tile-walking paths take
            D = pick(rng, [128, 256, 384, 512])
            group = pick(rng, [g for g in (1, 2, 4, 8, 16, 32, 64) if D % g == 0])
        lh = pick(rng, [1, 2, 3, 7, 8, 9, 13, 17, 33, 48, 50, 64, 65, 66, 100, 128, 129, 130, 140])
        L = int(rng.integers(1, 1200))
        B = int(rng.integers(1, 4))
        dtype = pick(rng, ["bf16", "bf16", "bf16", "f32"])
        entry = pick(rng, ["hyena_se_bwd", "hyena_mr_bwd"])
        rows = pick(rng, [0, 0, 64, 128, 256, 512])
        walk = pick(rng, [0, 0, 1])
        out.append((i, entry, B, L, D, lh, group, dtype, rows, walk))
    return out


@pytest.mark.parametrize("case", bwd_cases(40, 2026), ids=lambda c: "%d-%s-B%dL%dD%dlh%dg%d%s-r%d-w%d" % c)
def test_backward_entry_points_on_random_shapes(case):
    """Whichever backward path a shape lands on (stencil, tile walker, one-pass matrix-core kernel, chunk-parallel
    ungrouped kernels with one or two gates, general kernels): dq, dk, dv within the storage type's tolerance; dh
    at the fp32 bar where it is summed in fp32 from unrounded products, at the matrix-core bar where u and g enter
    the contraction rounded to bf16."""
    i, entry, B, L, D, lh, group, dtype, rows, walk = case
    binding.set_option("mr_rows", rows)
    binding.set_option("se_rows", rows)
    binding.set_option("se_walk", walk)
    say("%s #%d B=%d L=%d D=%d lh=%d group=%d %s rows=%d walk=%d" % (entry, i, B, L, D, lh, group, dtype, rows, walk))
    rng = np.random.Generator(np.random.PCG64(7000 + i))
    dy, q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(4))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    outs = getattr(binding, entry)(dev(dy), dev(q), dev(k), dev(v), dev(h), group)
    ref = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    on_matrix_cores = dtype == "bf16" and 8 < lh <= 129 and (
        (group % 16 == 0 and D % 64 == 0) or (group % 16 != 0 and D % 128 == 0))
    dh_tol = 1e-2 if on_matrix_cores else TOL["f32"]
    for name, got, want, tol in zip(("dq", "dk", "dv", "dh"), outs, ref, (TOL[dtype],) * 3 + (dh_tol,)):
        g = host(got)
        assert g.shape == want.shape and np.isfinite(g).all(), name
        err = oracle.rel_err(g, want)
        assert err <= tol, (name, err)
