"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle on identical seeded inputs,
element by element.  Sizes span several tiles and ragged tails; edge cases cover the left boundary,
batch boundaries, short sequences, odd widths and every kernel family behind the entry points."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_01868_amd import binding, synth

from gpu_util import TOL, check_gated, dev, draw, gated, host, say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    for name in ("se_vec", "se_rows", "mr_rows", "mr_waves", "se_walk"):
        binding.set_option(name, 0)


# ------------------------------------------------------------------------------------------ Hyena-SE
SE_CASES = [
    # B, L, D, lh, group
    (1, 1024, 256, 7, 1),    # the tiny fp32 configuration
    (2, 777, 512, 7, 1),     # ragged L, two batch items
    (3, 100, 264, 4, 1),     # D not a multiple of the block's channel span
    (1, 5, 64, 7, 1),        # L < lh
    (1, 1, 8, 3, 1),         # single time step
    (2, 333, 96, 1, 1),      # lh = 1: elementwise
    (2, 400, 128, 8, 4),     # grouped short filter
    (1, 300, 100, 5, 2),     # D = 100: vector width falls back
    (1, 260, 33, 6, 1),      # odd D: scalar lanes
    (2, 129, 64, 2, 64),     # one filter for all channels
    (1, 513, 256, 3, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", SE_CASES)
def test_se_matches_oracle(case, dtype):
    B, L, D, lh, group = case
    check_gated("hyena_se_fwd", 11, B, L, D, lh, group, dtype)


@pytest.mark.parametrize("vec", [1, 2, 4, 8])
@pytest.mark.parametrize("rows", [1, 5, 32, 1000])
def test_se_every_lane_width_and_tile_length(vec, rows):
    binding.set_option("se_vec", vec)
    binding.set_option("se_rows", rows)
    for dtype in ("f32", "bf16"):
        check_gated("hyena_se_fwd", 12, 2, 203, 192, 7, 1, dtype)


def test_se_long_filter_falls_back_to_general_kernel():
    for dtype in ("f32", "bf16"):
        check_gated("hyena_se_fwd", 13, 2, 150, 72, 13, 1, dtype)
        check_gated("hyena_se_fwd", 13, 1, 90, 40, 40, 2, dtype)


# Long-sequence SE kernel (the MR kernel's data movement with the stencil's fp32 arithmetic), forced on small shapes.
# Tiles are at least 256 steps, so L above 256 per workgroup column gives several tiles with their warm-up chunks.
SE_WALK_CASES = [
    (1, 1000, 128, 7, 1),    # 8 waves, four tiles, ragged last chunk
    (2, 700, 256, 7, 1),     # 16 waves
    (1, 300, 512, 3, 2),
    (3, 257, 128, 8, 1),     # longest filter, one step into the second tile
    (1, 33, 128, 1, 1),      # lh = 1
    (1, 5, 256, 7, 16),      # sequence shorter than the filter
    (1, 2049, 256, 5, 1),
    (4, 64, 384, 2, 4),      # D = 3 * 128
]


@pytest.mark.parametrize("case", SE_WALK_CASES)
def test_se_long_sequence_kernel_matches_oracle(case):
    B, L, D, lh, group = case
    binding.set_option("se_walk", 1)
    check_gated("hyena_se_fwd", 14, B, L, D, lh, group, "bf16")


def test_se_long_sequence_kernel_is_bit_exact_on_impulses_and_agrees_with_the_stencil():
    """Dyadic taps, q = k = 1, unit impulses around tile and chunk boundaries: exact.  On random data both SE kernels
    do the same fp32 FMA chain in the same tap order, so they must agree bit for bit."""
    B, L, D, lh = 2, 1100, 128, 7
    say("impulse se walk")
    h = dyadic_filter(D, lh, 45)
    one = torch.ones(B, L, D, dtype=torch.bfloat16)
    v = torch.zeros(B, L, D, dtype=torch.bfloat16)
    hits = [(0, 0, 0), (0, 250, 17), (0, 255, 127), (1, 256, 64), (1, 511, 3), (1, 1099, 5), (0, 31, 9), (0, 1023, 77)]
    expect = np.zeros((B, L, D))
    for b, t0, c in hits:
        v[b, t0, c] = 1.0
        n = min(lh, L - t0)
        expect[b, t0:t0 + n, c] += h[c, :n]
    binding.set_option("se_walk", 1)
    y = host(gated("hyena_se_fwd", one, one, v, h, 1))
    assert np.array_equal(y, expect)
    q, k, vv, hr = draw(15, 2, 900, 256, 7, 1, "bf16")
    y_walk = gated("hyena_se_fwd", q, k, vv, hr, 1)
    binding.set_option("se_walk", 2)
    y_sten = gated("hyena_se_fwd", q, k, vv, hr, 1)
    torch.cuda.synchronize()
    assert torch.equal(y_walk, y_sten)


def test_se_long_sequence_kernel_guard_bands():
    B, L, D, lh = 2, 301, 256, 7
    say("guard bands se walk")
    binding.set_option("se_walk", 1)
    q, k, v, h = draw(16, B, L, D, lh, 1, "bf16")
    n = B * L * D
    guard = 4096
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    binding.hyena_se_fwd(dev(q), dev(k), dev(v), dev(h), 1, out=out)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all()
    assert not torch.isnan(out).any()
    assert oracle.rel_err(host(out), oracle.gated_conv(q, k, v, h, group=1)) <= TOL["bf16"]


# --------------------------------------------------------------------------------------- featurizer
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [(2, 300, 256, 7, 1), (1, 4, 32, 7, 1), (3, 65, 48, 3, 2), (1, 128, 40, 20, 1)])
def test_featurize_matches_oracle(case, dtype):
    B, L, D, lh, group = case
    say("featurize B=%d L=%d D=%d lh=%d group=%d %s" % (B, L, D, lh, group, dtype))
    rng = np.random.Generator(np.random.PCG64(21))
    x = synth.normal_tensor(rng, (B, L, D), dtype)
    h = synth.short_filter(rng, D // group, lh)
    y = host(binding.hyena_featurize_fwd(dev(x), dev(h), group))
    assert oracle.rel_err(y, oracle.causal_conv(x, h, group)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_featurize3_matches_three_single_calls_and_oracle(dtype):
    B, L, D, lh = 2, 211, 320, 7
    say("featurize3 %s" % dtype)
    rng = np.random.Generator(np.random.PCG64(22))
    xs = [synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3)]
    hs = [synth.short_filter(rng, D, lh) for _ in range(3)]
    outs = binding.hyena_featurize3_fwd(*[dev(x) for x in xs], *[dev(h) for h in hs], 1)
    for x, h, o in zip(xs, hs, outs):
        single = binding.hyena_featurize_fwd(dev(x), dev(h), 1)
        assert torch.equal(single, o)
        assert oracle.rel_err(host(o), oracle.causal_conv(x, h, 1)) <= TOL[dtype]


# ------------------------------------------------------------------------------------------ Hyena-MR
MR_MFMA_CASES = [
    # B, L, D, lh, group, mr_rows (0 = library's choice)
    (1, 512, 64, 128, 16, 0),
    (2, 1000, 128, 128, 16, 256),   # several time tiles with halo warm-up, ragged tail, two batch items
    (1, 333, 64, 128, 16, 32),      # tile length = one chunk: every tile is mostly halo
    (2, 97, 64, 128, 16, 64),       # L < lh
    (1, 1, 64, 128, 16, 0),
    (1, 31, 64, 7, 16, 0),
    (1, 640, 192, 33, 16, 128),     # lh = 32 + 1: exactly two source blocks
    (1, 640, 64, 34, 16, 128),      # one tap past that boundary
    (1, 500, 64, 64, 32, 96),       # group of 32 channels = two matrix tiles per filter
    (1, 500, 128, 65, 64, 160),
    (1, 300, 64, 1, 16, 64),        # lh = 1
    (1, 700, 64, 129, 16, 128),     # one tap past 128
    (1, 900, 64, 200, 16, 224),
    (1, 1100, 64, 257, 64, 288),    # longest filter at two waves per SIMD
    (3, 256, 256, 128, 16, 128),
    (1, 1300, 64, 258, 16, 0),      # filters in the hundreds (one wave per SIMD, 13 source blocks)
    (2, 1500, 128, 384, 16, 512),   # several tiles, each with 12 warm-up chunks
    (1, 900, 64, 385, 32, 416),     # last filter of 13 source blocks
    (1, 2000, 64, 386, 16, 576),    # first of 17 source blocks
    (1, 2500, 192, 513, 16, 1024),  # longest filter of the matrix-core path
    (1, 300, 64, 513, 64, 0),       # L < lh
]


@pytest.mark.parametrize("case", MR_MFMA_CASES)
def test_mr_matrix_core_path_matches_oracle(case):
    B, L, D, lh, group, rows = case
    binding.set_option("mr_rows", rows)
    check_gated("hyena_mr_fwd", 31, B, L, D, lh, group, "bf16", kind="mr")


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("case", [(2, 700, 512, 128, 16, 256), (1, 333, 256, 65, 32, 96), (1, 1500, 256, 128, 16, 0)])
def test_mr_every_workgroup_width(case, waves):
    B, L, D, lh, group, rows = case
    binding.set_option("mr_waves", waves)
    binding.set_option("mr_rows", rows)
    check_gated("hyena_mr_fwd", 34, B, L, D, lh, group, "bf16", kind="mr")


@pytest.mark.parametrize("case", [
    (1, 300, 64, 128, 16, "f32"),   # fp32: exact-to-1e-5 check of the Toeplitz indexing on the general kernel
    (2, 257, 48, 128, 8, "bf16"),   # group smaller than a matrix tile
    (1, 200, 40, 50, 1, "bf16"),    # ungrouped medium filter
    (1, 700, 64, 514, 16, "bf16"),  # filter longer than the matrix-core path takes
    (2, 130, 64, 128, 16, "f32"),
    (1, 64, 16, 128, 16, "bf16"),   # D below the 64-channel block
])
def test_mr_general_path_matches_oracle(case):
    B, L, D, lh, group, dtype = case
    check_gated("hyena_mr_fwd", 32, B, L, D, lh, group, dtype, kind="mr")


# Chunk-parallel matrix-core path (App. A.1): bf16, filters not shared by 16 channels, 9 <= lh <= 145, D % 64 == 0.
# (B, L, D, lh, group, rows): rows = 0 keeps the default tile length, 256 forces a tile boundary every iteration.
CP_CASES = [
    (1, 700, 64, 128, 1, 0),        # ungrouped medium filter, ragged last iteration
    (2, 1000, 128, 128, 1, 256),    # tiles of one iteration: every history path
    (1, 2300, 64, 145, 1, 512),     # longest filter of this path, ring wraps several times
    (1, 515, 64, 17, 1, 256),       # K = 32 exactly filled (lh + 15 = 32)
    (1, 515, 64, 18, 1, 256),       # first length that needs K = 64
    (1, 300, 64, 49, 2, 0),
    (1, 300, 64, 50, 4, 0),
    (1, 777, 128, 81, 8, 256),
    (2, 513, 64, 113, 1, 256),
    (1, 259, 64, 9, 1, 0),          # shortest filter routed here
    (1, 3, 64, 128, 1, 0),          # sequence shorter than one row group
    (1, 1, 64, 20, 1, 0),
    (1, 256, 192, 64, 3, 0),        # group that does not divide the 64-channel block evenly
    (3, 256, 64, 128, 32, 0),       # hyena_se_fwd entry with a shared filter also lands here (see test below)
]


# The same shapes with D a multiple of 128 land on the batched 4x4x4 kernel (lh <= 129); tiles are at least 256 steps.
CP4_CASES = [
    (1, 700, 128, 128, 1, 0),       # 8 waves, ragged last iteration
    (2, 1000, 256, 128, 1, 256),    # four tiles per sequence: history passes
    (1, 2300, 128, 129, 1, 512),    # longest filter of this path, ring cycles many times
    (1, 515, 256, 17, 1, 256),      # 16 waves, 5 products
    (1, 515, 256, 18, 1, 256),      # 9 products
    (1, 300, 128, 49, 2, 0),
    (1, 300, 256, 65, 4, 0),        # 17 products, 16 waves
    (1, 777, 128, 81, 8, 256),
    (2, 513, 384, 113, 1, 256),     # D = 3 * 128
    (1, 259, 128, 9, 1, 0),
    (1, 3, 128, 128, 1, 0),
    (1, 1, 256, 20, 1, 0),
    (1, 256, 384, 64, 3, 0),
    (3, 256, 128, 128, 32, 0),      # through hyena_se_fwd
    (1, 1000, 256, 100, 1, 320),    # tile length that is not a multiple of the ring
    (1, 2300, 256, 129, 1, 512),    # long filters, two and more channel blocks per tile
    (2, 513, 512, 113, 2, 256),
    (1, 777, 256, 81, 8, 256),
    (1, 3, 256, 128, 1, 0),
    (1, 130, 768, 97, 3, 0),
]


@pytest.mark.parametrize("case", CP4_CASES)
def test_batched_small_tile_path_matches_oracle(case):
    B, L, D, lh, group, rows = case
    binding.set_option("mr_rows", rows)
    entry = "hyena_se_fwd" if group == 32 else "hyena_mr_fwd"
    check_gated(entry, 36, B, L, D, lh, group, "bf16", kind="mr")


@pytest.mark.parametrize("case", [c for c in CP4_CASES if c[3] <= 65])
def test_batched_small_tile_path_with_eight_waves_matches_oracle(case):
    """Filters of up to 65 taps run 16 waves per workgroup where D allows; `mr_waves` = 8 selects the 128-channel
    workgroup for them."""
    B, L, D, lh, group, rows = case
    binding.set_option("mr_rows", rows)
    binding.set_option("mr_waves", 8)
    entry = "hyena_se_fwd" if group == 32 else "hyena_mr_fwd"
    check_gated(entry, 37, B, L, D, lh, group, "bf16", kind="mr")


@pytest.mark.parametrize("case", CP_CASES)
def test_chunk_parallel_path_matches_oracle(case):
    B, L, D, lh, group, rows = case
    binding.set_option("mr_rows", rows)
    entry = "hyena_se_fwd" if group == 32 else "hyena_mr_fwd"
    check_gated(entry, 35, B, L, D, lh, group, "bf16", kind="mr")


def test_chunk_parallel_impulse_and_tile_boundaries_are_bit_exact():
    """Ungrouped dyadic taps, q = k = 1, v = unit impulses placed so that responses cross iteration and tile
    boundaries and the ring's wrap-around: y must reproduce each channel's own taps exactly."""
    _chunk_parallel_impulse(128)


def test_chunk_parallel_impulse_with_256_channel_workgroups_is_bit_exact():
    _chunk_parallel_impulse(256)


def _chunk_parallel_impulse(D):
    B, L, lh = 2, 1500, 100
    say("impulse chunk-parallel D=%d" % D)
    binding.set_option("mr_rows", 512)
    h = dyadic_filter(D, lh, 44)
    one = torch.ones(B, L, D, dtype=torch.bfloat16)
    v = torch.zeros(B, L, D, dtype=torch.bfloat16)
    hits = [(0, 0, 0), (0, 200, 17), (0, 500, 63), (1, 511, 64), (1, 1023, 127), (1, 1450, 5), (0, 1499, 9), (0, 255, 70),
            (1, 31, D - 1), (0, 32, D - 17), (1, 63, D - 16), (0, 992, D - 33)]
    expect = np.zeros((B, L, D))
    for b, t0, c in hits:
        v[b, t0, c] = 1.0
        n = min(lh, L - t0)
        expect[b, t0:t0 + n, c] += h[c, :n]
    y = host(gated("hyena_mr_fwd", one, one, v, h, 1))
    assert np.array_equal(y, expect)


def test_chunk_parallel_guard_bands_determinism_and_no_leak_between_batch_items():
    B, L, D, lh = 2, 301, 128, 77
    say("guard bands chunk-parallel")
    q, k, v, h = draw(54, 1, L, D, lh, 1, "bf16", "mr")
    q2, k2, v2 = (torch.cat([x, x], dim=0) for x in (q, k, v))
    n = B * L * D
    guard = 4096
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    binding.hyena_mr_fwd(dev(q2), dev(k2), dev(v2), dev(h), 1, out=out)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all()
    assert not torch.isnan(out).any()
    assert torch.equal(out[0], out[1])
    again = binding.hyena_mr_fwd(dev(q2), dev(k2), dev(v2), dev(h), 1)
    torch.cuda.synchronize()
    assert torch.equal(again, out)
    assert oracle.rel_err(host(out[:1]), oracle.gated_conv(q, k, v, h, group=1)) <= TOL["bf16"]


def test_mr_and_se_entry_points_agree_on_a_short_grouped_filter():
    q, k, v, h = draw(33, 2, 300, 128, 7, 16, "bf16", kind="mr")
    y_mr = host(gated("hyena_mr_fwd", q, k, v, h, 16))
    y_se = host(gated("hyena_se_fwd", q, k, v, h, 16))
    ref = oracle.gated_conv(q, k, v, h, group=16)
    assert oracle.rel_err(y_mr, ref) <= TOL["bf16"] and oracle.rel_err(y_se, ref) <= TOL["bf16"]


# ------------------------------------------------------------------------- exact-arithmetic cases
def dyadic_filter(n, lh, seed):
    """Taps that are small multiples of 1/8: exact in bf16, and sums of a few of them exact in fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.integers(-8, 9, size=(n, lh)) / 8.0).astype(np.float32)


@pytest.mark.parametrize("entry,lh,group,dtype", [
    ("hyena_se_fwd", 7, 1, "bf16"), ("hyena_se_fwd", 7, 1, "f32"),
    ("hyena_mr_fwd", 128, 16, "bf16"), ("hyena_mr_fwd", 128, 16, "f32"),
])
def test_impulse_response_is_bit_exact(entry, lh, group, dtype):
    """q = k = 1, v = unit impulses: y must reproduce the filter taps exactly (every product and sum
    is exactly representable), at the first row, mid-sequence and across a tile boundary."""
    B, L, D = 2, 600, 64
    say("impulse %s %s" % (entry, dtype))
    binding.set_option("mr_rows", 256)
    binding.set_option("se_rows", 50)
    h = dyadic_filter(D // group, lh, 41)
    td = synth.torch_dtype(dtype)
    one = torch.ones(B, L, D, dtype=td)
    v = torch.zeros(B, L, D, dtype=td)
    hits = [(0, 0, 0), (0, 250, 17), (1, 301, 63), (1, 0, 5), (0, 599, 1)]
    expect = np.zeros((B, L, D))
    for b, t0, c in hits:
        v[b, t0, c] = 1.0
        n = min(lh, L - t0)
        expect[b, t0:t0 + n, c] += h[c // group, :n]
    y = host(gated(entry, one, one, v, h, group))
    assert np.array_equal(y, expect)


@pytest.mark.parametrize("entry,lh,group", [("hyena_se_fwd", 7, 1), ("hyena_mr_fwd", 128, 16)])
def test_sparse_signed_inputs_are_bit_exact_in_bf16(entry, lh, group):
    """k, v in {-1, 0, 1} (sparse), q in {-2, ..., 2}, dyadic taps: every partial sum is a multiple of
    1/8 below 2^8, so fp32 accumulation is exact in any order and the bf16 result is exact."""
    B, L, D = 2, 700, 128
    say("sparse exact %s" % entry)
    binding.set_option("mr_rows", 192)
    rng = np.random.Generator(np.random.PCG64(42))
    h = dyadic_filter(D // group, lh, 43) * (rng.random((D // group, lh)) < 0.25)
    h = h.astype(np.float32)
    k = torch.from_numpy(rng.integers(-1, 2, (B, L, D)).astype(np.float32)).bfloat16()
    v = torch.from_numpy((rng.integers(-1, 2, (B, L, D)) * (rng.random((B, L, D)) < 0.3)).astype(np.float32)).bfloat16()
    q = torch.from_numpy(rng.integers(-2, 3, (B, L, D)).astype(np.float32)).bfloat16()
    ref = oracle.gated_conv(q, k, v, h, group=group)
    assert np.array_equal(ref, torch.from_numpy(ref).bfloat16().double().numpy())  # the case really is exact
    y = host(gated(entry, q, k, v, h, group))
    assert np.array_equal(y, ref)


# --------------------------------------------------------------- memory safety and determinism
@pytest.mark.parametrize("entry,lh,group,kind", [("hyena_se_fwd", 7, 1, "se"), ("hyena_mr_fwd", 128, 16, "mr")])
def test_writes_stay_inside_the_output_and_cover_all_of_it(entry, lh, group, kind):
    B, L, D = 2, 301, 128
    say("guard bands %s" % entry)
    q, k, v, h = draw(51, B, L, D, lh, group, "bf16", kind)
    n = B * L * D
    guard = 4096
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    getattr(binding, entry)(dev(q), dev(k), dev(v), dev(h), group, out=out)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all()
    assert not torch.isnan(out).any()
    assert oracle.rel_err(host(out), oracle.gated_conv(q, k, v, h, group=group)) <= TOL["bf16"]


@pytest.mark.parametrize("entry,lh,group,kind", [("hyena_se_fwd", 7, 1, "se"), ("hyena_mr_fwd", 128, 16, "mr")])
def test_repeat_runs_are_bit_identical_and_batch_items_do_not_leak(entry, lh, group, kind):
    B, L, D = 2, 500, 128
    say("determinism %s" % entry)
    q, k, v, h = draw(52, 1, L, D, lh, group, "bf16", kind)
    q2, k2, v2 = (torch.cat([x, x], dim=0) for x in (q, k, v))  # two identical batch items
    y_a = gated(entry, q2, k2, v2, h, group)
    y_b = gated(entry, q2, k2, v2, h, group)
    torch.cuda.synchronize()
    assert torch.equal(y_a, y_b)
    assert torch.equal(y_a[0], y_a[1])  # item 1 must not see the tail of item 0 as its past


def test_runs_on_a_side_stream():
    q, k, v, h = draw(53, 1, 256, 128, 7, 1, "bf16")
    s = torch.cuda.Stream()
    dq, dk, dv, dh = dev(q), dev(k), dev(v), dev(h)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        y = binding.hyena_se_fwd(dq, dk, dv, dh, 1)
    s.synchronize()
    assert oracle.rel_err(host(y), oracle.gated_conv(q, k, v, h)) <= TOL["bf16"]


def test_stream_copy_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    binding.hyena_stream_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


# ------------------------------------------------------------------------------- operator chain
def draw_chain(seed, B, L, D, lf, feat_group, lh, group, dtype):
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    hq, hk, hv = (synth.short_filter(rng, D // feat_group, lf) for _ in range(3))
    h = synth.decay_filter(rng, D // group, lh)
    return q, k, v, hq, hk, hv, h


def check_chain(seed, B, L, D, lf, feat_group, lh, group, dtype, expect_fused):
    say("chain seed=%d B=%d L=%d D=%d lf=%d fg=%d lh=%d group=%d %s" % (seed, B, L, D, lf, feat_group, lh, group, dtype))
    code = binding.HY_BF16 if dtype == "bf16" else binding.HY_F32
    need = binding.lib().hyena_chain_workspace_bytes(B, L, D, lf, feat_group, lh, group, code)
    assert (need == 0) == expect_fused
    q, k, v, hq, hk, hv, h = draw_chain(seed, B, L, D, lf, feat_group, lh, group, dtype)
    y = host(binding.hyena_chain_fwd(dev(q), dev(k), dev(v), dev(hq), dev(hk), dev(hv), dev(h), group, feat_group))
    ref = oracle.chain(q, k, v, hq, hk, hv, h, group=group, feat_group=feat_group)
    err = oracle.rel_err(y, ref)
    assert np.isfinite(y).all() and err <= TOL[dtype], err
    return err


CHAIN_FUSED_CASES = [
    # B, L, D, lf, feat_group, lh, group, mr_rows
    (1, 512, 128, 7, 1, 128, 16, 0),
    (2, 1000, 256, 7, 1, 128, 16, 256),   # several tiles: look-back chunk + warm-up chunks, ragged tail
    (1, 333, 128, 7, 1, 128, 16, 32),     # one-chunk tiles
    (2, 97, 128, 7, 1, 128, 16, 64),      # L < lh
    (1, 1, 128, 7, 1, 128, 16, 0),
    (1, 300, 128, 1, 1, 33, 16, 64),      # lf = 1: featurizer is a per-channel scale
    (1, 450, 128, 8, 1, 65, 32, 96),      # longest fused featurizer
    (1, 200, 128, 3, 1, 1, 128, 64),      # lh = 1, one inner filter for all channels
    (3, 256, 384, 4, 1, 129, 16, 128),    # longest fused inner filter
    (1, 700, 128, 7, 1, 7, 16, 128),
    (1, 260, 256, 7, 2, 128, 16, 96),     # featurizer filters shared by channel pairs
    (1, 2100, 128, 7, 1, 128, 16, 1024),
]


@pytest.mark.parametrize("case", CHAIN_FUSED_CASES)
def test_chain_single_kernel_path_matches_oracle(case):
    """The single-kernel chain: featurizers and medium convolution as matrix products."""
    B, L, D, lf, fg, lh, group, rows = case
    binding.set_option("mr_rows", rows)
    check_chain(61, B, L, D, lf, fg, lh, group, "bf16", expect_fused=True)


def test_chain_nine_tap_featurizer_is_the_longest_the_single_kernel_takes():
    binding.set_option("mr_rows", 96)
    check_chain(65, 2, 500, 128, 9, 1, 100, 16, "bf16", expect_fused=True)
    check_chain(65, 2, 500, 128, 10, 1, 100, 16, "bf16", expect_fused=False)


@pytest.mark.parametrize("case", [
    (2, 200, 64, 7, 1, 128, 16, "bf16"),    # D below the 128-channel block
    (1, 150, 128, 7, 1, 128, 16, "f32"),    # fp32
    (1, 300, 128, 7, 1, 200, 16, "bf16"),   # inner filter longer than the fused kernel takes
    (1, 120, 128, 12, 1, 64, 16, "bf16"),   # featurizer longer than the fused kernel takes
    (1, 90, 96, 5, 3, 40, 8, "bf16"),       # small odd groups
])
def test_chain_two_kernel_path_matches_oracle(case):
    B, L, D, lf, fg, lh, group, dtype = case
    check_chain(62, B, L, D, lf, fg, lh, group, dtype, expect_fused=False)


def test_chain_impulse_is_bit_exact():
    """q = 1 through a delta featurizer, k = 1 through a delta featurizer, v = impulse through a dyadic
    featurizer, dyadic inner filter: y is the convolution of the two filters, exactly representable."""
    B, L, D, lf, lh, group = 1, 400, 128, 7, 128, 16
    say("chain impulse")
    binding.set_option("mr_rows", 128)
    rng = np.random.Generator(np.random.PCG64(63))
    delta = np.zeros((D, lf), dtype=np.float32)
    delta[:, 0] = 1.0
    hv = (rng.integers(-4, 5, size=(D, lf)) / 4.0).astype(np.float32)
    h = ((rng.integers(-4, 5, size=(D // group, lh)) / 4.0) * (rng.random((D // group, lh)) < 0.2)).astype(np.float32)
    one = torch.ones(B, L, D, dtype=torch.bfloat16)
    v = torch.zeros(B, L, D, dtype=torch.bfloat16)
    hits = [(0, 3, 0), (0, 130, 77), (0, 255, 127)]
    for b, t0, c in hits:
        v[b, t0, c] = 1.0
    ref = oracle.chain(one, one, v, delta, delta, hv, h, group=group)
    assert np.array_equal(ref, torch.from_numpy(ref).bfloat16().double().numpy())
    y = host(binding.hyena_chain_fwd(dev(one), dev(one), dev(v), dev(delta), dev(delta), dev(hv), dev(h), group, 1))
    assert np.array_equal(y, ref)


def test_chain_guard_bands_and_determinism():
    B, L, D = 2, 301, 128
    say("chain guard bands")
    q, k, v, hq, hk, hv, h = draw_chain(64, B, L, D, 7, 1, 128, 16, "bf16")
    n = B * L * D
    guard = 4096
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    args = [dev(x) for x in (q, k, v, hq, hk, hv, h)]
    binding.hyena_chain_fwd(*args, 16, 1, out=out)
    again = binding.hyena_chain_fwd(*args, 16, 1)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all() and not torch.isnan(out).any()
    assert torch.equal(out, again)


@pytest.mark.parametrize("case", [
    # B, L, D, strip_channels, rows, depth, waves
    (1, 1000, 256, 0, 0, 0, 0), (2, 333, 256, 64, 0, 1, 0), (1, 700, 256, 128, 96, 3, 0), (3, 129, 512, 256, 32, 4, 0),
    (1, 1, 256, 256, 0, 6, 0), (2, 77, 64, 64, 0, 6, 4), (1, 50, 24, 0, 0, 0, 0), (1, 900, 128, 128, 64, 2, 8),
    (2, 555, 512, 256, 0, 4, 8), (1, 1001, 256, 256, 40, 8, 4), (1, 301, 384, 128, 0, 4, 4), (1, 7, 256, 256, 0, 8, 8),
])
def test_bandwidth_yardstick_computes_the_elementwise_gate(case):
    """hyena_stream_gate is the operator with a one-tap unit filter: y = q*k*v, compared with the oracle as such,
    for the linear stream and every strip width, with ragged tiles."""
    B, L, D, strip, rows, depth, waves = case
    say("hyena_stream_gate B=%d L=%d D=%d strip=%d rows=%d depth=%d waves=%d" % case)
    rng = np.random.Generator(np.random.PCG64(90 + strip + L))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    n = B * L * D
    guard = 2048
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    binding.hyena_stream_gate(dev(q), dev(k), dev(v), strip, rows, depth, waves, out=out)
    y = host(out)
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all()
    ref = oracle.gated_conv(q, k, v, np.ones((D, 1), dtype=np.float32), group=1)
    assert np.isfinite(y).all() and oracle.rel_err(y, ref) <= TOL["bf16"]


# --------------------------------------------------------------------------------------- featurizer on the tile walker
@pytest.mark.parametrize("case", SE_WALK_CASES)
def test_featurizer_long_sequence_kernel_matches_oracle_and_the_stencil(case):
    """The ungated variant of the long-sequence kernel (forced on small shapes), one tensor and three tensors per
    launch, against the oracle and, bit for bit (same fp32 FMA chain in the same tap order), against the stencil."""
    B, L, D, lh, group = case
    say("featurizer walker B=%d L=%d D=%d lh=%d group=%d" % case)
    rng = np.random.Generator(np.random.PCG64(2300 + L + D))
    xs = [synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3)]
    hs = [synth.short_filter(rng, D // group, lh) for _ in range(3)]
    dx, dh = [dev(x) for x in xs], [dev(h) for h in hs]
    binding.set_option("se_walk", 1)
    one = binding.hyena_featurize_fwd(dx[0], dh[0], group)
    three = binding.hyena_featurize3_fwd(*dx, *dh, group)
    binding.set_option("se_walk", 2)
    one_s = binding.hyena_featurize_fwd(dx[0], dh[0], group)
    three_s = binding.hyena_featurize3_fwd(*dx, *dh, group)
    torch.cuda.synchronize()
    assert torch.equal(one, one_s) and torch.equal(one, three[0])
    for x, h, o, o_s in zip(xs, hs, three, three_s):
        assert torch.equal(o, o_s)
        assert oracle.rel_err(host(o), oracle.causal_conv(x, h, group)) <= TOL["bf16"]


def test_featurizer_long_sequence_kernel_guard_bands_and_chain_fallback():
    """Three outputs between NaN guard bands, and the two-kernel chain (a shape the single-kernel chain does not
    take: lh = 200) with the walker as its first kernel against the oracle."""
    B, L, D, lh = 2, 301, 256, 7
    say("guard bands featurizer walker")
    binding.set_option("se_walk", 1)
    rng = np.random.Generator(np.random.PCG64(2400))
    xs = [synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3)]
    hs = [synth.short_filter(rng, D, lh) for _ in range(3)]
    n, guard = B * L * D, 4096
    buf = torch.full((3, n + 2 * guard), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    outs = tuple(buf[i, guard:guard + n].view(B, L, D) for i in range(3))
    binding.hyena_featurize3_fwd(*[dev(x) for x in xs], *[dev(h) for h in hs], 1, out=outs)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, :guard]).all() and torch.isnan(buf[:, guard + n:]).all() and not torch.isnan(buf[:, guard:guard + n]).any()
    h = synth.decay_filter(rng, D // 16, 200)
    y = binding.hyena_chain_fwd(*[dev(x) for x in xs], *[dev(f) for f in hs], dev(h), 16, 1)
    ref = oracle.chain(*xs, *hs, h, group=16, feat_group=1)
    assert oracle.rel_err(host(y), ref) <= TOL["bf16"]
