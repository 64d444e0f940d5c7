"""The entry points launch kernels on the caller's stream and nothing else (no allocation, no memset, no
synchronisation), so a caller may record them into a HIP graph.  Each test captures a few calls, replays the
graph several times with eager work and synchronisations in between, and checks every replay against the
eager result bit for bit."""
import numpy as np
import pytest
import torch

import paper_2503_01868_amd as pkg
from paper_2503_01868_amd import binding, synth

from gpu_util import dev, say

pytestmark = pytest.mark.gpu


def capture(build_plans):
    """build_plans(stream) -> list of Plan objects bound to `stream`; returns (graph, outputs)."""
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plans = build_plans(side)
        for p in plans:  # warm-up outside the capture (loads the code objects)
            p()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        for p in plans:
            p()
    return g, plans


def replay_and_compare(g, plans, eager, refill):
    for it in range(3):
        refill(it)            # eager work between replays: new inputs written into the captured buffers
        torch.cuda.synchronize()
        want = eager()
        torch.cuda.synchronize()
        for p in plans:       # spoil the outputs so that a replay that does nothing is noticed
            outs = p.out if isinstance(p.out, tuple) else (p.out,)
            for o in outs:
                o.fill_(float("nan")) if o.dtype != torch.float32 else o.fill_(7.0)
        g.replay()
        torch.cuda.synchronize()
        got = [o.clone() for p in plans for o in (p.out if isinstance(p.out, tuple) else (p.out,))]
        assert len(got) == len(want)
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d differs from the eager result" % it


def test_forward_entry_points_replay_from_a_graph():
    say("graph: se, mr, chunk-parallel, chain, li forward")
    B, L, D = 2, 700, 256
    rng = np.random.Generator(np.random.PCG64(91))
    q, k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(3))
    h_se = dev(synth.short_filter(rng, D, 7))
    h_mr = dev(synth.decay_filter(rng, D // 16, 128))
    h_un = dev(synth.decay_filter(rng, D, 100))
    hq, hk, hv = (dev(synth.short_filter(rng, D, 7)) for _ in range(3))
    R, lam = (dev(x) for x in synth.li_params(rng, D // 16, 16))
    binding.set_option("mr_rows", 256)  # several tiles: the li scan uses its workspace

    def build(stream):
        return [
            pkg.plan_gated("hyena_se_fwd", q, k, v, h_se, 1, stream=stream),
            pkg.plan_gated("hyena_mr_fwd", q, k, v, h_mr, 16, stream=stream),
            pkg.plan_gated("hyena_mr_fwd", q, k, v, h_un, 1, stream=stream),
            pkg.plan_chain(q, k, v, hq, hk, hv, h_mr, 16, 1, stream=stream),
            pkg.plan_li(q, k, v, R, lam, 16, stream=stream),
        ]

    try:
        g, plans = capture(build)

        def eager():
            return [binding.hyena_se_fwd(q, k, v, h_se, 1), binding.hyena_mr_fwd(q, k, v, h_mr, 16),
                    binding.hyena_mr_fwd(q, k, v, h_un, 1), binding.hyena_chain_fwd(q, k, v, hq, hk, hv, h_mr, 16, 1),
                    binding.hyena_li_fwd(q, k, v, R, lam, 16)]

        def refill(it):
            for t in (q, k, v):
                t.copy_(dev(synth.normal_tensor(rng, (B, L, D), "bf16")))

        replay_and_compare(g, plans, eager, refill)
    finally:
        binding.set_option("mr_rows", 0)


def test_backward_entry_points_replay_from_a_graph():
    say("graph: se, mr (grouped and ungrouped) and featurizer backward")
    B, L, D = 2, 500, 128
    rng = np.random.Generator(np.random.PCG64(92))
    dy, q, k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(4))
    h_se = dev(synth.short_filter(rng, D, 7))
    h_mr = dev(synth.decay_filter(rng, D // 16, 128))
    h_un = dev(synth.decay_filter(rng, D, 128))     # ungrouped, long: dk and dv from one two-gate launch
    h_us = dev(synth.decay_filter(rng, D // 2, 40))  # ungrouped, short: one launch each

    def build(stream):
        return [pkg.plan_bwd("hyena_se_bwd", dy, q, k, v, h_se, 1, stream=stream),
                pkg.plan_bwd("hyena_mr_bwd", dy, q, k, v, h_mr, 16, stream=stream),
                pkg.plan_bwd("hyena_mr_bwd", dy, q, k, v, h_un, 1, stream=stream),
                pkg.plan_bwd("hyena_mr_bwd", dy, q, k, v, h_us, 2, stream=stream),
                pkg.plan_featurize_bwd(dy, k, h_se, 1, stream=stream)]

    g, plans = capture(build)

    def eager():
        return (list(binding.hyena_se_bwd(dy, q, k, v, h_se, 1)) + list(binding.hyena_mr_bwd(dy, q, k, v, h_mr, 16)) +
                list(binding.hyena_mr_bwd(dy, q, k, v, h_un, 1)) + list(binding.hyena_mr_bwd(dy, q, k, v, h_us, 2)) +
                list(binding.hyena_featurize_bwd(dy, k, h_se, 1)))

    def refill(it):
        for t in (dy, q, k, v):
            t.copy_(dev(synth.normal_tensor(rng, (B, L, D), "bf16")))

    replay_and_compare(g, plans, eager, refill)


def test_shard_entry_points_replay_from_a_graph():
    say("graph: forward and backward shard calls (windows of full tensors, halos on both sides)")
    B, L, D, t0, t1 = 2, 900, 128, 300, 700
    rng = np.random.Generator(np.random.PCG64(93))
    dy, q, k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(4))
    h_se = dev(synth.short_filter(rng, D, 7))
    h_mr = dev(synth.decay_filter(rng, D // 16, 128))
    h_un = dev(synth.decay_filter(rng, D, 100))
    w = slice(t0, t1)
    cases = [("se", h_se, 1, 6), ("mr", h_mr, 16, 127), ("mr", h_un, 1, 99)]

    def build(stream):
        plans = []
        for kind, h, group, halo in cases:
            plans.append(binding.plan_gated_shard("hyena_%s_fwd_shard" % kind, q[:, w], k[:, w], v[:, w], h, group, halo,
                                                  out=torch.empty_like(q)[:, w], stream=stream))
            plans.append(binding.plan_bwd_shard("hyena_%s_bwd_shard" % kind, dy[:, w], q[:, w], k[:, w], v[:, w], h, group,
                                                halo, halo, stream=stream))
        return plans

    g, plans = capture(build)

    def eager():
        out = []
        for kind, h, group, halo in cases:
            out.append(getattr(binding, "hyena_%s_fwd_shard" % kind)(q[:, w], k[:, w], v[:, w], h, group, halo,
                                                                     out=torch.empty_like(q)[:, w]))
            out += list(getattr(binding, "hyena_%s_bwd_shard" % kind)(dy[:, w], q[:, w], k[:, w], v[:, w], h, group,
                                                                      halo, halo))
        return out

    def refill(it):
        for t in (dy, q, k, v):
            t.copy_(dev(synth.normal_tensor(rng, (B, L, D), "bf16")))

    replay_and_compare(g, plans, eager, refill)


def test_entry_points_run_concurrently_on_separate_streams():
    """Two streams issue different entry points back to back (each call with its own outputs and workspace); the
    results must equal those of the same calls issued one after the other on the default stream."""
    say("two streams")
    B, L, D = 2, 3000, 256
    rng = np.random.Generator(np.random.PCG64(93))
    q, k, v, dy = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(4))
    h_se = dev(synth.short_filter(rng, D, 7))
    h_mr = dev(synth.decay_filter(rng, D // 16, 128))
    h_un = dev(synth.decay_filter(rng, D, 64))
    R, lam = (dev(x) for x in synth.li_params(rng, D // 16, 16))
    binding.set_option("mr_rows", 512)
    try:
        want = [binding.hyena_se_fwd(q, k, v, h_se, 1), binding.hyena_mr_fwd(q, k, v, h_mr, 16),
                binding.hyena_li_fwd(q, k, v, R, lam, 16), binding.hyena_mr_fwd(q, k, v, h_un, 1)]
        want += list(binding.hyena_mr_bwd(dy, q, k, v, h_mr, 16)) + list(binding.hyena_se_bwd(dy, q, k, v, h_se, 1))
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        a = [pkg.plan_gated("hyena_se_fwd", q, k, v, h_se, 1, stream=s1), pkg.plan_li(q, k, v, R, lam, 16, stream=s1),
             pkg.plan_bwd("hyena_mr_bwd", dy, q, k, v, h_mr, 16, stream=s1)]
        b = [pkg.plan_gated("hyena_mr_fwd", q, k, v, h_mr, 16, stream=s2),
             pkg.plan_gated("hyena_mr_fwd", q, k, v, h_un, 1, stream=s2),
             pkg.plan_bwd("hyena_se_bwd", dy, q, k, v, h_se, 1, stream=s2)]
        torch.cuda.synchronize()
        for rep in range(3):
            for pa, pb in zip(a, b):
                pa()
                pb()
        torch.cuda.synchronize()
        got = [a[0].out, b[0].out, a[1].out, b[1].out] + list(a[2].out) + list(b[2].out)
        for x, y in zip(got, want):
            assert torch.equal(x, y)
    finally:
        binding.set_option("mr_rows", 0)
