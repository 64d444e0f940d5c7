"""A sequence computed in shards (each call sees its own steps plus the rows of k and v that precede them) equals
the unsharded call: the compute half of the point-to-point scheme of Sec. 4, on one GPU.  The shards here are windows
of the full tensors, so the rows in front of a window are its history, as they would be after a halo exchange."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_01868_amd import binding, synth

from gpu_util import TOL, dev, host, say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    for name in ("se_vec", "se_rows", "mr_rows", "mr_waves", "se_walk"):
        binding.set_option(name, 0)


def run_sharded(entry, q, k, v, h, group, cuts, lh):
    """y over [B, L, D] from one shard call per stretch between consecutive cuts; q and y of a shard are windows of
    the full tensors (batch stride L * D), k and v too, with min(t0, lh - 1) rows of history in front."""
    B, L, D = q.shape
    y = torch.full_like(q, float("nan"))
    edges = [0] + list(cuts) + [L]
    for t0, t1 in zip(edges[:-1], edges[1:]):
        hist = min(t0, lh - 1)
        getattr(binding, entry)(q[:, t0:t1], k[:, t0:t1], v[:, t0:t1], h, group, hist, out=y[:, t0:t1])
    torch.cuda.synchronize()
    return y


CASES = [
    # entry, B, L, D, lh, group, dtype, cuts, options
    ("hyena_se_fwd_shard", 2, 1000, 256, 7, 1, "bf16", (300, 301, 640), {}),            # stencil; a one-step shard
    ("hyena_se_fwd_shard", 1, 900, 64, 4, 2, "f32", (3, 500), {}),                       # history shorter than lh - 1
    ("hyena_se_fwd_shard", 2, 4096, 256, 7, 1, "bf16", (1024, 3000), {"se_walk": 1}),    # tile walker
    ("hyena_se_fwd_shard", 1, 2100, 128, 8, 4, "bf16", (5, 1111), {"se_walk": 1}),       # walker refuses history 5
    ("hyena_mr_fwd_shard", 2, 1500, 128, 128, 16, "bf16", (400, 1000), {}),              # grouped matrix-core kernel
    ("hyena_mr_fwd_shard", 1, 2000, 256, 128, 16, "bf16", (50, 90, 1024), {"mr_rows": 256}),  # partial halo chunks
    ("hyena_mr_fwd_shard", 3, 700, 64, 33, 32, "bf16", (128, 129), {}),
    ("hyena_mr_fwd_shard", 1, 3000, 512, 257, 16, "bf16", (1500,), {}),                  # nine source blocks
    ("hyena_mr_fwd_shard", 2, 800, 48, 100, 1, "bf16", (333,), {}),                      # general kernel (ungrouped)
    ("hyena_mr_fwd_shard", 1, 600, 256, 128, 16, "f32", (200, 400), {}),                 # general kernel (fp32)
    ("hyena_mr_fwd_shard", 1, 640, 128, 7, 16, "bf16", (320,), {}),                      # short grouped filter
    ("hyena_mr_fwd_shard", 2, 1500, 128, 128, 1, "bf16", (400, 1000), {}),               # ungrouped: 4x4x4 kernel, long filter
    ("hyena_mr_fwd_shard", 1, 1000, 256, 40, 2, "bf16", (30, 64, 500), {"mr_rows": 256}),  # 16 waves; short histories
    ("hyena_mr_fwd_shard", 3, 700, 128, 20, 1, "bf16", (350, 351), {}),                  # 8 waves, 9 products
    ("hyena_se_fwd_shard", 2, 900, 384, 100, 8, "bf16", (450,), {}),                     # through the SE entry point
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%s-B%dL%dD%dlh%dg%d%s" % c[:7])
def test_sharded_sequence_equals_the_whole_sequence(case):
    entry, B, L, D, lh, group, dtype, cuts, opts = case
    say("%s B=%d L=%d D=%d lh=%d group=%d %s cuts=%s" % (entry, B, L, D, lh, group, dtype, cuts))
    rng = np.random.Generator(np.random.PCG64(4100 + L + lh))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    for name, value in opts.items():
        binding.set_option(name, value)
    dq, dk, dv, dh = dev(q), dev(k), dev(v), dev(h)
    y_sh = run_sharded(entry, dq, dk, dv, dh, group, cuts, lh)
    whole = getattr(binding, entry.replace("_shard", ""))(dq, dk, dv, dh, group)
    ref = oracle.gated_conv(q, k, v, h, group=group)
    got = host(y_sh)
    assert np.isfinite(got).all()
    assert oracle.rel_err(got, ref) <= TOL[dtype]
    if lh <= 8 and group % 16 != 0:
        assert torch.equal(y_sh, whole)   # fixed tap order on the short-filter paths: bit for bit
    else:
        assert oracle.rel_err(got, host(whole)) <= TOL[dtype]


def test_shard_with_its_own_halo_buffer_and_dense_q_and_y():
    """The layout a rank would really hold: k and v as [B, history + L, D] buffers whose first rows were received
    from the left neighbour, q and y dense [B, L, D]."""
    B, Ltot, D, lh, group = 2, 900, 128, 128, 16
    t0, L = 500, 400
    hist = lh - 1
    rng = np.random.Generator(np.random.PCG64(4242))
    q, k, v = (synth.normal_tensor(rng, (B, Ltot, D), "bf16") for _ in range(3))
    h = synth.decay_filter(rng, D // group, lh)
    kbuf = dev(k[:, t0 - hist:t0 + L].contiguous())
    vbuf = dev(v[:, t0 - hist:t0 + L].contiguous())
    qs = dev(q[:, t0:t0 + L].contiguous())
    guard = torch.full((B * L * D + 4096,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = guard[2048:2048 + B * L * D].view(B, L, D)
    binding.hyena_mr_fwd_shard(qs, kbuf[:, hist:], vbuf[:, hist:], dev(h), group, hist, out=out)
    torch.cuda.synchronize()
    assert torch.isnan(guard[:2048]).all() and torch.isnan(guard[2048 + B * L * D:]).all()
    ref = oracle.gated_conv(q, k, v, h, group=group)[:, t0:t0 + L]
    assert oracle.rel_err(host(out), ref) <= TOL["bf16"]


def test_zero_history_is_the_plain_call():
    B, L, D, lh, group = 2, 700, 256, 128, 16
    rng = np.random.Generator(np.random.PCG64(4343))
    q, k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(3))
    h = dev(synth.decay_filter(rng, D // group, lh))
    assert torch.equal(binding.hyena_mr_fwd_shard(q, k, v, h, group, 0), binding.hyena_mr_fwd(q, k, v, h, group))
    hs = dev(synth.short_filter(rng, D, 7))
    assert torch.equal(binding.hyena_se_fwd_shard(q, k, v, hs, 1, 0), binding.hyena_se_fwd(q, k, v, hs, 1))


# ------------------------------------------------------------------------------------------------ backward
def run_bwd_sharded(entry, dy, q, k, v, h, group, cuts, lh):
    """dq, dk, dv over [B, L, D] and the sum of the shards' filter-gradient shares, one shard call per stretch;
    every tensor of a shard is a window of the full tensor."""
    B, L, D = q.shape
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    dh = torch.zeros_like(h, dtype=torch.float64)
    edges = [0] + list(cuts) + [L]
    for t0, t1 in zip(edges[:-1], edges[1:]):
        hist, fut = min(t0, lh - 1), min(L - t1, lh - 1)
        w = slice(t0, t1)
        outs = getattr(binding, entry)(dy[:, w], q[:, w], k[:, w], v[:, w], h, group, hist, fut,
                                       out=(dq[:, w], dk[:, w], dv[:, w], torch.empty_like(h)))
        dh += outs[3].double()
    torch.cuda.synchronize()
    return dq, dk, dv, dh


BWD_CASES = [
    # entry, B, L, D, lh, group, dtype, cuts, options
    ("hyena_se_bwd_shard", 2, 1000, 256, 7, 1, "bf16", (300, 301, 640), {}),        # stencil; a one-step shard
    ("hyena_se_bwd_shard", 1, 900, 64, 4, 2, "f32", (3, 500, 898), {}),             # halos shorter than lh - 1
    ("hyena_se_bwd_shard", 2, 700, 128, 8, 4, "bf16", (350,), {"se_rows": 64}),
    ("hyena_se_bwd_shard", 2, 1000, 256, 7, 1, "bf16", (300, 301, 640), {"se_walk": 1}),   # tile walker
    ("hyena_se_bwd_shard", 1, 1500, 512, 4, 2, "bf16", (3, 700, 1497), {"se_walk": 1, "se_rows": 64}),  # ... short halos
    ("hyena_se_bwd_shard", 1, 2100, 256, 7, 1, "bf16", (1000,), {"se_walk": 1, "se_rows": 256}),  # ... several tiles
    ("hyena_mr_bwd_shard", 2, 1500, 128, 128, 16, "bf16", (400, 1000), {}),         # one-pass matrix-core kernel
    ("hyena_mr_bwd_shard", 1, 2000, 64, 128, 16, "bf16", (50, 90, 1024, 1950), {"mr_rows": 256}),  # partial halo chunks
    ("hyena_mr_bwd_shard", 3, 700, 64, 33, 32, "bf16", (128, 129), {}),
    ("hyena_mr_bwd_shard", 2, 800, 48, 100, 1, "bf16", (333,), {}),                 # general kernels (ungrouped)
    ("hyena_mr_bwd_shard", 1, 600, 128, 128, 16, "f32", (200, 400), {}),            # general kernels (fp32)
    ("hyena_mr_bwd_shard", 1, 640, 128, 100, 1, "bf16", (320,), {}),                # chunk-parallel 4x4x4 kernels
    ("hyena_mr_bwd_shard", 2, 1000, 128, 128, 1, "bf16", (300, 301, 640), {}),      # ... two post-gates; shard lengths
                                                                                    # 300, 1, 339, 360
    ("hyena_mr_bwd_shard", 1, 777, 256, 33, 2, "bf16", (130, 391), {}),             # ... 16-wave kernel, groups of 2
    ("hyena_mr_bwd_shard", 1, 1100, 128, 65, 4, "bf16", (7, 550, 1098), {"mr_rows": 256}),  # ... short halos, tiles
    ("hyena_mr_bwd_shard", 2, 515, 128, 9, 1, "bf16", (258,), {}),                  # ... shortest filter; 258 % 4 = 2
]


@pytest.mark.parametrize("case", BWD_CASES, ids=lambda c: "%s-B%dL%dD%dlh%dg%d%s" % c[:7])
def test_sharded_backward_equals_the_whole_sequence(case):
    entry, B, L, D, lh, group, dtype, cuts, opts = case
    say("%s B=%d L=%d D=%d lh=%d group=%d %s cuts=%s" % (entry, B, L, D, lh, group, dtype, cuts))
    rng = np.random.Generator(np.random.PCG64(4500 + L + lh))
    dy, q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(4))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    for name, value in opts.items():
        binding.set_option(name, value)
    got = run_bwd_sharded(entry, dev(dy), dev(q), dev(k), dev(v), dev(h), group, cuts, lh)
    ref = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    on_matrix_cores = dtype == "bf16" and 8 < lh <= 129 and ((group % 16 == 0 and D % 64 == 0) or D % 128 == 0)
    for name, g, want, tol in zip(("dq", "dk", "dv", "dh"), got, ref,
                                  (TOL[dtype],) * 3 + (1e-2 if on_matrix_cores else TOL["f32"],)):
        gh = host(g)
        assert np.isfinite(gh).all(), name
        err = oracle.rel_err(gh, want)
        assert err <= tol, (name, err)


# ------------------------------------------------------------------------------------------------ fused chain
@pytest.mark.parametrize("entry,lh,group,D,walk", [
    ("hyena_se_bwd_shard", 7, 1, 128, 0), ("hyena_se_bwd_shard", 7, 1, 256, 1), ("hyena_mr_bwd_shard", 128, 16, 128, 0),
    ("hyena_mr_bwd_shard", 100, 1, 128, 0), ("hyena_mr_bwd_shard", 40, 2, 128, 0)])
def test_backward_shards_with_their_own_halo_buffers(entry, lh, group, D, walk):
    """The layout ranks would really hold: k and v as [B, history + L, D] buffers (first rows received from the left
    neighbour), dy and q as [B, L + future, D] buffers (last rows received from the right neighbour), dq, dk, dv
    dense: three different batch strides.  Two ranks; the shares of dh add up."""
    B, Ltot, cut = 2, 900, 500
    say("%s lh=%d group=%d, buffers with halos, B=%d L=%d+%d D=%d" % (entry, lh, group, B, cut, Ltot - cut, D))
    binding.set_option("se_walk", walk)   # 1: the short-filter tile walker whatever the length
    rng = np.random.Generator(np.random.PCG64(4600 + lh))
    dy, q, k, v = (synth.normal_tensor(rng, (B, Ltot, D), "bf16") for _ in range(4))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    hd = dev(h)
    parts, dh = [], torch.zeros_like(hd, dtype=torch.float64)
    for t0, t1 in ((0, cut), (cut, Ltot)):
        L = t1 - t0
        hist, fut = min(t0, lh - 1), min(Ltot - t1, lh - 1)
        kbuf, vbuf = (dev(x[:, t0 - hist:t1].contiguous()) for x in (k, v))
        gbuf, qbuf = (dev(x[:, t0:t1 + fut].contiguous()) for x in (dy, q))
        guard = torch.full((3, B * L * D + 4096), float("nan"), dtype=torch.bfloat16, device="cuda:0")
        outs = tuple(guard[i, 2048:2048 + B * L * D].view(B, L, D) for i in range(3))
        res = getattr(binding, entry)(gbuf[:, :L], qbuf[:, :L], kbuf[:, hist:], vbuf[:, hist:], hd, group, hist, fut,
                                      out=outs + (torch.empty_like(hd),))
        torch.cuda.synchronize()
        assert torch.isnan(guard[:, :2048]).all() and torch.isnan(guard[:, 2048 + B * L * D:]).all()
        parts.append([host(o) for o in outs])
        dh += res[3].double()
    ref = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    for i, name in enumerate(("dq", "dk", "dv")):
        got = np.concatenate([parts[0][i], parts[1][i]], axis=1)
        assert np.isfinite(got).all(), name
        assert oracle.rel_err(got, ref[i]) <= TOL["bf16"], name
    assert oracle.rel_err(host(dh), ref[3]) <= (1e-2 if lh > 8 else TOL["f32"])


@pytest.mark.parametrize("case", [
    # B, L, D, lf, lh, group, cuts, mr_rows
    (2, 1500, 128, 7, 128, 16, (400, 1000), 0),
    (1, 2048, 256, 7, 128, 16, (60, 100, 1024), 256),   # histories shorter than (lh - 1) + (lf - 1) near the start
    (3, 700, 128, 9, 33, 32, (128, 129), 0),            # a one-step shard; longest featurizer
    (1, 1000, 128, 3, 129, 16, (500,), 0),
])
def test_sharded_operator_chain_equals_the_whole_sequence(case):
    """hyena_chain_fwd_shard: every shard call sees its own steps of q, k, v plus (lh - 1) + (lf - 1) rows of each in
    front of them; the shards' outputs against the oracle's chain on the whole sequence and against one call."""
    B, L, D, lf, lh, group, cuts, rows = case
    say("chain shards B=%d L=%d D=%d lf=%d lh=%d group=%d cuts=%s rows=%d" % case)
    binding.set_option("mr_rows", rows)
    rng = np.random.Generator(np.random.PCG64(4700 + L + lh))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    hq, hk, hv = (synth.short_filter(rng, D, lf) for _ in range(3))
    h = synth.decay_filter(rng, D // group, lh)
    dq, dk, dv = dev(q), dev(k), dev(v)
    dhq, dhk, dhv, dh = dev(hq), dev(hk), dev(hv), dev(h)
    y = torch.full_like(dq, float("nan"))
    edges = [0] + list(cuts) + [L]
    for t0, t1 in zip(edges[:-1], edges[1:]):
        hist = min(t0, lh - 1 + lf - 1)
        binding.hyena_chain_fwd_shard(dq[:, t0:t1], dk[:, t0:t1], dv[:, t0:t1], dhq, dhk, dhv, dh, group, 1, hist,
                                      out=y[:, t0:t1])
    torch.cuda.synchronize()
    ref = oracle.chain(q, k, v, hq, hk, hv, h, group=group, feat_group=1)
    got = host(y)
    assert np.isfinite(got).all() and oracle.rel_err(got, ref) <= TOL["bf16"]
    whole = binding.hyena_chain_fwd(dq, dk, dv, dhq, dhk, dhv, dh, group, 1)
    assert oracle.rel_err(got, host(whole)) <= TOL["bf16"]


# ------------------------------------------------------------------------------------------------ random cuts
def _pick(rng, xs):
    return xs[int(rng.integers(0, len(xs)))]


def random_shard_cases(n, seed):
    """Seeded random shapes, filter lengths, group sizes, options and cut positions (cuts may fall anywhere: next to
    each other, within lh - 1 steps of either end, off every tile and chunk boundary)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        group = _pick(rng, [1, 1, 2, 4, 16, 16, 32])
        D = _pick(rng, [64, 128, 128, 256, 256, 384, 512])
        D = max(D - D % group, group)
        lh = _pick(rng, [1, 3, 7, 8, 9, 20, 33, 64, 65, 66, 100, 128, 129])
        L = int(rng.integers(2, 1600))
        B = int(rng.integers(1, 3))
        dtype = _pick(rng, ["bf16", "bf16", "bf16", "f32"])
        ncut = int(rng.integers(1, 5))
        cuts = tuple(sorted(set(int(c) for c in rng.integers(1, L, size=ncut))))
        opts = {}
        if rng.random() < 0.5:
            opts["mr_rows"] = opts["se_rows"] = _pick(rng, [32, 64, 256, 512])
        if lh <= 7 and rng.random() < 0.5:
            opts["se_walk"] = 1
        out.append((i, B, L, D, lh, group, dtype, cuts, opts))
    return out


@pytest.mark.parametrize("case", random_shard_cases(28, 777), ids=lambda c: "%d-B%dL%dD%dlh%dg%d%s" % c[:7])
def test_random_cuts_forward_and_backward(case):
    i, B, L, D, lh, group, dtype, cuts, opts = case
    kind = "se" if lh <= 8 else "mr"
    say("random shards %d: B=%d L=%d D=%d lh=%d group=%d %s cuts=%s opts=%s" % (i, B, L, D, lh, group, dtype, cuts, opts))
    rng = np.random.Generator(np.random.PCG64(7000 + i))
    dy, q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(4))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    for name, value in opts.items():
        binding.set_option(name, value)
    d = [dev(x) for x in (dy, q, k, v, h)]
    y = run_sharded("hyena_%s_fwd_shard" % kind, d[1], d[2], d[3], d[4], group, cuts, lh)
    assert oracle.rel_err(host(y), oracle.gated_conv(q, k, v, h, group=group)) <= TOL[dtype]
    got = run_bwd_sharded("hyena_%s_bwd_shard" % kind, *d, group, cuts, lh)
    ref = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    on_matrix_cores = dtype == "bf16" and 8 < lh <= 129 and ((group % 16 == 0 and D % 64 == 0) or D % 128 == 0)
    for name, g, want, tol in zip(("dq", "dk", "dv", "dh"), got, ref,
                                  (TOL[dtype],) * 3 + (1e-2 if on_matrix_cores else TOL["f32"],)):
        gh = host(g)
        assert np.isfinite(gh).all(), name
        err = oracle.rel_err(gh, want)
        assert err <= tol, (name, err)


# ------------------------------------------------------------------------------------------------ overlap
@pytest.mark.parametrize("kind,lh,group", [("se", 7, 1), ("mr", 128, 16), ("mr", 100, 1)])
def test_interior_and_boundary_calls_hide_the_halo_exchange(kind, lh, group):
    """How a rank overlaps the exchange with compute (Sec. 4, point-to-point scheme): the steps of its shard that lie
    at least lh - 1 steps away from a cut need no neighbour data, because their halo is the shard's own rows, so
    they are launched at once; a copy on a second stream (standing in for the receive) meanwhile fills the halo
    rows in front of k, v and behind dy, q; the lh - 1 steps next to each cut follow when it has finished.  All of
    these are ordinary shard calls; forward and backward, with the shares of dh adding up."""
    B, Ltot, D, t0, n = 2, 1500, 128, 500, 700          # the rank owns steps t0 .. t0 + n - 1
    H = lh - 1
    say("overlap pattern %s lh=%d group=%d: rank owns %d..%d of %d" % (kind, lh, group, t0, t0 + n - 1, Ltot))
    rng = np.random.Generator(np.random.PCG64(5200 + lh))
    dy, q, k, v = (synth.normal_tensor(rng, (B, Ltot, D), "bf16") for _ in range(4))
    h = synth.short_filter(rng, D // group, lh) if lh <= 8 else synth.decay_filter(rng, D // group, lh)
    hd = dev(h)
    full = [dev(x) for x in (dy, q, k, v)]
    nan = float("nan")
    # the rank's buffers: k, v with room for the left halo in front, dy, q with room for the right halo behind
    kbuf, vbuf = (torch.full((B, H + n, D), nan, dtype=torch.bfloat16, device="cuda:0") for _ in range(2))
    gbuf, qbuf = (torch.full((B, n + H, D), nan, dtype=torch.bfloat16, device="cuda:0") for _ in range(2))
    kbuf[:, H:], vbuf[:, H:] = full[2][:, t0:t0 + n], full[3][:, t0:t0 + n]
    gbuf[:, :n], qbuf[:, :n] = full[0][:, t0:t0 + n], full[1][:, t0:t0 + n]
    dq, dk, dv = (torch.full((B, n, D), nan, dtype=torch.bfloat16, device="cuda:0") for _ in range(3))
    y = torch.full((B, n + H, D), nan, dtype=torch.bfloat16, device="cuda:0")[:, :n]   # q's batch stride (the forward
    #                                                                                    entry has one for q and y)
    dh_parts = [torch.empty_like(hd) for _ in range(3)]
    fwd = getattr(binding, "hyena_%s_fwd_shard" % kind)
    bwd = getattr(binding, "hyena_%s_bwd_shard" % kind)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    arrived = torch.cuda.Event()
    with torch.cuda.stream(side):   # the "receive": the neighbours' rows land in the halo regions
        kbuf[:, :H].copy_(full[2][:, t0 - H:t0], non_blocking=True)
        vbuf[:, :H].copy_(full[3][:, t0 - H:t0], non_blocking=True)
        gbuf[:, n:].copy_(full[0][:, t0 + n:t0 + n + H], non_blocking=True)
        qbuf[:, n:].copy_(full[1][:, t0 + n:t0 + n + H], non_blocking=True)
        arrived.record(side)
    kk, vv, gg, qq = kbuf[:, H:], vbuf[:, H:], gbuf[:, :n], qbuf[:, :n]    # the rank's own n steps
    # interior, launched without waiting: forward needs H own rows of history, backward also H own rows of future
    fwd(qq[:, H:], kk[:, H:], vv[:, H:], hd, group, H, out=y[:, H:])
    inner = slice(H, n - H)
    bwd(gg[:, inner], qq[:, inner], kk[:, inner], vv[:, inner], hd, group, H, H,
        out=(dq[:, inner], dk[:, inner], dv[:, inner], dh_parts[0]))
    torch.cuda.current_stream().wait_event(arrived)
    # the steps next to the cuts
    fwd(qq[:, :H], kk[:, :H], vv[:, :H], hd, group, H, out=y[:, :H])
    first, last = slice(0, H), slice(n - H, n)
    bwd(gg[:, first], qq[:, first], kk[:, first], vv[:, first], hd, group, H, H,
        out=(dq[:, first], dk[:, first], dv[:, first], dh_parts[1]))
    bwd(gg[:, last], qq[:, last], kk[:, last], vv[:, last], hd, group, H, H,
        out=(dq[:, last], dk[:, last], dv[:, last], dh_parts[2]))
    torch.cuda.synchronize()

    ref_y = oracle.gated_conv(q, k, v, h, group=group)[:, t0:t0 + n]
    assert oracle.rel_err(host(y), ref_y) <= TOL["bf16"]
    ref = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    for name, got, want in zip(("dq", "dk", "dv"), (dq, dk, dv), ref[:3]):
        g = host(got)
        assert np.isfinite(g).all(), name
        assert oracle.rel_err(g, want[:, t0:t0 + n]) <= TOL["bf16"], name
    # the rank's share of dh in one unsplit shard call: the three shares of the split add up to it
    _, _, _, dh_one = bwd(gg, qq, kk, vv, hd, group, H, H)
    share = sum(p.double() for p in dh_parts)
    scale = float(dh_one.abs().max())
    assert float((share - dh_one.double()).abs().max()) <= (1e-2 if lh > 8 else 1e-5) * scale
