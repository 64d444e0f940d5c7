"""GPU parity of hyena_li_fwd (Hyena-LI, Sec. 2.1: filter = sum of real exponentials, as long as the sequence)
against the oracle's definition: filter materialised in fp64 over the whole sequence, direct convolution.  The two
full-size workloads are compared over every output against the oracle's recurrent form as well."""
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


def draw_li(seed, B, L, D, order, group, dtype):
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    R, lam = synth.li_params(rng, D // group, order)
    return q, k, v, R, lam


def check_li(seed, B, L, D, order, group, dtype, tol=None, params=None):
    say("hyena_li_fwd seed=%d B=%d L=%d D=%d order=%d group=%d dtype=%s" % (seed, B, L, D, order, group, dtype))
    q, k, v, R, lam = draw_li(seed, B, L, D, order, group, dtype)
    if params is not None:
        R, lam = params
    y = host(binding.hyena_li_fwd(dev(q), dev(k), dev(v), dev(R), dev(lam), group))
    ref = oracle.li_conv(q, k, v, R, lam, group=group)
    err = oracle.rel_err(y, ref)
    assert np.isfinite(y).all()
    assert err <= (TOL[dtype] if tol is None else tol), err
    return err


# (B, L, D, order, group, rows): rows = 0 keeps the default tile length; small values force many tiles, i.e. the
# two-pass scan with its workspace
LI_MFMA_CASES = [
    (1, 700, 64, 16, 16, 0),        # one tile, ragged last chunk
    (2, 1000, 128, 16, 16, 128),    # 8 tiles per sequence: pass 1 + Horner over up to 7 states
    (1, 2300, 256, 8, 32, 256),     # two matrix tiles per filter group, order below 16
    (1, 515, 64, 1, 16, 32),        # a single exponential, one chunk per tile
    (3, 96, 64, 16, 64, 32),
    (1, 1, 64, 16, 16, 0),          # one step
    (1, 33, 64, 5, 16, 32),         # second tile holds a single step
    (2, 4096, 64, 16, 16, 1024),
]


@pytest.mark.parametrize("case", LI_MFMA_CASES)
def test_scan_on_matrix_cores_matches_the_definition(case):
    B, L, D, order, group, rows = case
    binding.set_option("mr_rows", rows)
    check_li(61, B, L, D, order, group, "bf16")


@pytest.mark.parametrize("waves", [4, 8, 16])
def test_every_workgroup_width(waves):
    binding.set_option("mr_waves", waves)
    binding.set_option("mr_rows", 160)
    check_li(62, 2, 900, 512, 16, 16, "bf16")


def test_slow_poles_negative_poles_and_a_pole_at_one():
    """Poles next to the unit circle keep the whole past alive: the state must survive thousands of steps in
    fp32 and enter the products without losing its low bits.  Negative poles alternate in sign."""
    B, L, D, order, group = 1, 6000, 64, 4, 16
    G = D // group
    lam = np.tile(np.array([0.9999, 1.0, -0.97, 0.5], dtype=np.float32), (G, 1))
    R = np.tile(np.array([0.5, 0.05, 1.0, -2.0], dtype=np.float32), (G, 1))
    binding.set_option("mr_rows", 512)
    check_li(63, B, L, D, order, group, "bf16", params=(R, lam))


def test_nearly_cancelling_exponentials_keep_their_difference():
    """Two close poles with opposite residues: the filter, about t * 2e-4 * lambda^t, is some 50 times smaller than
    either exponential.  Each exponential's running sum and output weights therefore have to be carried well
    beyond bf16 precision, or their individual rounding errors (0.4% of an exponential = 20% of the filter) show
    at full size."""
    B, L, D, group = 1, 1800, 128, 16
    n = D // group
    l1 = np.linspace(0.9900, 0.9960, n)
    lam = np.stack([l1, l1 - 2e-4, np.full(n, 0.9), np.full(n, 0.5)], axis=1).astype(np.float32)
    R = np.stack([np.full(n, 1.0), np.full(n, -1.0), np.full(n, 1e-3), np.full(n, -1e-3)], axis=1).astype(np.float32)
    for rows in (0, 256):
        binding.set_option("mr_rows", rows)
        err = check_li(26, B, L, D, 4, group, "bf16", params=(R, lam))
        assert err <= 1e-2, err


def test_random_poles_and_residues_including_close_pairs():
    """Seeded sweep over what the precision depends on: decay rates over four decades, poles of either sign,
    residues over four decades, and (every other case) pole pairs 1e-4 to 1e-2 apart with nearly opposite
    residues.  The largest error over such a sweep was 2.6e-2 before the pole powers were carried as two bf16
    parts, 7e-3 since."""
    rng = np.random.Generator(np.random.PCG64(2701))
    worst = 0.0
    for i in range(60):
        group = (16, 32, 64)[i % 3]
        D = max(group, (64, 128, 256)[(i // 3) % 3])
        order = int(rng.integers(1, 17))
        L = int(rng.integers(1, 1200))
        G = D // group
        a = np.exp(rng.uniform(np.log(1e-4), np.log(3.0), size=(G, order)))
        lam = (np.exp(-a) * rng.choice([1.0, 1.0, -1.0], size=(G, order))).astype(np.float32)
        R = (rng.normal(size=(G, order)) * 10.0 ** rng.uniform(-2, 2, size=(G, order))).astype(np.float32)
        if i % 2 == 1 and order >= 2:
            half = order // 2
            lam[:, 1:2 * half:2] = lam[:, 0:2 * half:2] * (1 - 10.0 ** rng.uniform(-4, -2))
            R[:, 1:2 * half:2] = -R[:, 0:2 * half:2] * (1 + rng.uniform(-0.05, 0.05))
        binding.set_option("mr_rows", (0, 32, 128, 256, 512)[i % 5])
        worst = max(worst, check_li(2702 + i, 1, L, D, order, group, "bf16", tol=1.5e-2, params=(R, lam)))
    say("worst error of the sweep %.3e" % worst)


@pytest.mark.parametrize("case", [
    (1, 300, 64, 16, 16, "f32"),    # fp32 storage: the plain recurrence
    (2, 257, 48, 7, 8, "bf16"),     # group smaller than a matrix tile
    (1, 200, 40, 3, 1, "bf16"),     # one filter per channel
    (1, 129, 16, 16, 16, "bf16"),   # width below the 64-channel block
    (2, 500, 32, 2, 4, "f32"),
])
def test_general_recurrence_matches_the_definition(case):
    B, L, D, order, group, dtype = case
    check_li(64, B, L, D, order, group, dtype)


@pytest.mark.parametrize("case", [
    (1, 400, 64, 17, 16, "bf16"),   # one exponential more than the matrix-core scan takes
    (2, 300, 48, 40, 8, "bf16"),
    (1, 257, 64, 64, 16, "f32"),    # the most the general kernel holds
    (1, 100, 32, 33, 1, "f32"),
])
def test_more_than_sixteen_exponentials_run_the_general_recurrence(case):
    B, L, D, order, group, dtype = case
    check_li(66, B, L, D, order, group, dtype)


def test_impulse_response_is_bit_exact_across_chunks_and_tiles():
    """Dyadic residues and poles +-1/2: every coefficient, state and product is a power of two times a small
    integer, so the response to unit impulses must equal sum_n R_n lambda_n^j bit for bit, through chunk
    boundaries, tile boundaries (workspace states) and the two-part split of the state.  Compared exactly over
    the first 100 lags (2^-100 is still a normal number), loosely where the response sinks below that."""
    B, L, D, group = 2, 700, 64, 16
    say("impulse hyena_li_fwd")
    binding.set_option("mr_rows", 128)
    G = D // group
    R = np.tile(np.array([1.0, -0.5], dtype=np.float32), (G, 1)) * np.arange(1, G + 1, dtype=np.float32)[:, None]
    lam = np.tile(np.array([0.5, -0.5], dtype=np.float32), (G, 1))
    one = torch.ones(B, L, D, dtype=torch.bfloat16)
    v = torch.zeros(B, L, D, dtype=torch.bfloat16)
    hits = [(0, 0, 0), (0, 250, 17), (1, 127, 63), (1, 640, 33)]
    h = oracle.li_filter(R, lam, L)
    for b, t0, c in hits:
        v[b, t0, c] = 1.0
    y = host(binding.hyena_li_fwd(dev(one), dev(one), dev(v), dev(R), dev(lam), group))
    mask = np.ones((B, L, D), dtype=bool)
    for b, t0, c in hits:
        n = min(100, L - t0)
        want = h[c // group, :n]
        assert np.array_equal(want, torch.from_numpy(want).bfloat16().double().numpy())  # the case really is exact
        assert np.array_equal(y[b, t0:t0 + n, c], want)
        assert np.all(np.abs(y[b, t0 + n:, c]) <= 2.0 ** -98)
        mask[b, t0:, c] = False
    assert np.all(y[mask] == 0.0)


def test_guard_bands_determinism_and_no_leak_between_batch_items():
    B, L, D, order, group = 2, 301, 128, 16, 16
    say("guard bands hyena_li_fwd")
    binding.set_option("mr_rows", 96)
    q, k, v, R, lam = draw_li(65, 1, L, D, order, group, "bf16")
    q2, k2, v2 = (torch.cat([x, x], dim=0) for x in (q, k, v))
    n = B * L * D
    guard = 4096
    buf = torch.full((n + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    out = buf[guard:guard + n].view(B, L, D)
    binding.hyena_li_fwd(dev(q2), dev(k2), dev(v2), dev(R), dev(lam), group, out=out)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + n:]).all()
    assert not torch.isnan(out).any()
    assert torch.equal(out[0], out[1])  # item 1 must start from a zero state
    again = binding.hyena_li_fwd(dev(q2), dev(k2), dev(v2), dev(R), dev(lam), group)
    torch.cuda.synchronize()
    assert torch.equal(again, out)
    assert oracle.rel_err(host(out[:1]), oracle.li_conv(q, k, v, R, lam, group=group)) <= TOL["bf16"]


def _all_outputs_against_the_recurrent_form(w, y, slab=256):
    """max|y - y_ref| / max|y_ref| over every output, y_ref from the oracle's recurrent form in channel slabs."""
    dg = w["group"]
    num = den = 0.0
    n = 0
    for c0 in range(0, w["D"], slab):
        c1 = min(w["D"], c0 + slab)
        ref = oracle.li_recurrent(*(w[key][:, :, c0:c1].contiguous() for key in ("q", "k", "v")),
                                  w["R"][c0 // dg:c1 // dg], w["lam"][c0 // dg:c1 // dg], group=dg)
        got = y[:, :, c0:c1].float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        den = max(den, float(np.abs(ref).max()))
        np.subtract(got, ref, out=got)
        num = max(num, float(np.abs(got).max()))
        n += ref.size
    return num / den, n


def _definition_at_points(w, y, seed, n_pts):
    """Sampled outputs against the definition (filter materialised over the whole sequence, one direct sum per
    output), and the recurrent-form oracle against the definition at the same outputs of the same inputs."""
    pts = synth.sample_points(seed, w["B"], w["L"], w["D"], n_pts, 128)
    ref = oracle.li_conv_points(w["q"], w["k"], w["v"], w["R"], w["lam"], pts, group=w["group"])
    got = y[pts[:, 0], pts[:, 1], pts[:, 2]].float().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= TOL["bf16"] * scale
    # the channels the points fall in, through the recurrent form
    chans = np.unique(pts[:, 2])
    dg = w["group"]
    idx = torch.from_numpy(chans)
    sub = [w[key].index_select(2, idx).contiguous() for key in ("q", "k", "v")]
    rec = oracle.li_recurrent(*sub, w["R"][chans // dg], w["lam"][chans // dg], group=1)
    pos = np.searchsorted(chans, pts[:, 2])
    assert np.abs(rec[pts[:, 0], pts[:, 1], pos] - ref).max() <= 1e-10 * scale


@pytest.mark.timeout(600)
def test_full_size_config_all_outputs():
    """li2 (B=1, L=8192, D=4096, 16 exponentials per group of 16) in the launch configuration bench.py times: all
    33 554 432 outputs against the oracle's recurrent form, and sampled outputs against the definition, which
    also ties the recurrent form to the definition on these inputs."""
    w = synth.make("li2")
    say("li2 full size")
    y = binding.hyena_li_fwd(dev(w["q"]), dev(w["k"]), dev(w["v"]), dev(w["R"]), dev(w["lam"]), w["group"])
    torch.cuda.synchronize()
    _definition_at_points(w, y, 777, 3000)
    err, n = _all_outputs_against_the_recurrent_form(w, y)
    say("li2 all %d outputs rel_err=%.3e" % (n, err))
    assert n == 33554432 and err <= TOL["bf16"]


@pytest.mark.timeout(900)
def test_long_sequence_config_all_outputs():
    """li3 (B=1, L=131072, D=4096): the running sums cross 15 tile boundaries and 4096 chunks.  All 536 870 912
    outputs against the oracle's recurrent form (the definition is quadratic in L: 3.5e13 multiply-adds for this
    tensor), sampled outputs against the definition with the filter materialised over all 131072 steps."""
    w = synth.make("li3")
    say("li3 full size")
    y = binding.hyena_li_fwd(dev(w["q"]), dev(w["k"]), dev(w["v"]), dev(w["R"]), dev(w["lam"]), w["group"])
    torch.cuda.synchronize()
    _definition_at_points(w, y, 778, 2000)
    err, n = _all_outputs_against_the_recurrent_form(w, y)
    say("li3 all %d outputs rel_err=%.3e" % (n, err))
    assert n == 536870912 and err <= TOL["bf16"]
    del y
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ a sequence handed on in stretches
def _state_as_oracle(state, B, D, order):
    """[B][D/16][lq 4][li 16][r 4] floats -> [B, D, order]: element (b, 16 g + li, 4 lq + r)."""
    s = state.float().cpu().numpy().astype(np.float64).reshape(B, D // 16, 4, 16, 4)
    return s.transpose(0, 1, 3, 2, 4).reshape(B, D, 16)[:, :, :order]


@pytest.mark.parametrize("case", [
    # B, L, D, order, group, cuts, mr_rows
    (2, 1024, 128, 16, 16, (512,), 0),
    (1, 2048, 256, 7, 32, (256, 1280), 128),       # stretches of several tiles each
    (3, 960, 64, 16, 16, (32, 64, 480), 32),       # one-chunk stretches and one-chunk tiles
    (1, 4096, 256, 16, 16, (1024, 2048, 3072), 0),
])
def test_sequence_in_stretches_with_carried_state_equals_the_whole_sequence(case):
    """hyena_li_fwd_carry: y of every stretch against the oracle on the whole sequence, the state handed on after
    every stretch against the definition of the running sums, and the chained result against one hyena_li_fwd call."""
    B, L, D, order, group, cuts, rows = case
    say("li carry B=%d L=%d D=%d order=%d group=%d cuts=%s rows=%d" % case)
    binding.set_option("mr_rows", rows)
    rng = np.random.Generator(np.random.PCG64(600 + L))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    R, lam = synth.li_params(rng, D // group, order)
    dq, dk, dv, dR, dl = dev(q), dev(k), dev(v), dev(R), dev(lam)
    edges = [0] + list(cuts) + [L]
    state, parts = None, []
    for t0, t1 in zip(edges[:-1], edges[1:]):
        y, state = binding.hyena_li_fwd_carry(dq[:, t0:t1].contiguous(), dk[:, t0:t1].contiguous(),
                                              dv[:, t0:t1].contiguous(), dR, dl, group, state_in=state)
        parts.append(y)
        want = oracle.li_state(k[:, :t1], v[:, :t1], lam, group=group)
        got = _state_as_oracle(state, B, D, order)
        assert np.isfinite(got).all() and oracle.rel_err(got, want) <= TOL["bf16"], (t1, oracle.rel_err(got, want))
    y_cat = torch.cat(parts, dim=1)
    ref = oracle.li_recurrent(q, k, v, R, lam, group=group)
    assert oracle.rel_err(host(y_cat), ref) <= TOL["bf16"]
    whole = binding.hyena_li_fwd(dq, dk, dv, dR, dl, group)
    assert oracle.rel_err(host(y_cat), host(whole)) <= TOL["bf16"]


def test_carry_without_states_is_the_plain_call_and_bad_requests_are_refused():
    B, L, D, order, group = 2, 640, 128, 16, 16
    rng = np.random.Generator(np.random.PCG64(611))
    q, k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(3))
    R, lam = (dev(x) for x in synth.li_params(rng, D // group, order))
    y, none = binding.hyena_li_fwd_carry(q, k, v, R, lam, group, want_state=False)
    assert none is None and torch.equal(y, binding.hyena_li_fwd(q, k, v, R, lam, group))
    with pytest.raises(binding.HyenaError):   # a state after a length that is no multiple of 32
        binding.hyena_li_fwd_carry(q[:, :100].contiguous(), k[:, :100].contiguous(), v[:, :100].contiguous(), R, lam, group)
    with pytest.raises(binding.HyenaError):   # the general kernel keeps no such state
        binding.hyena_li_fwd_carry(q.float(), k.float(), v.float(), R, lam, group)


# ------------------------------------------------------------------ stretches that run at the same time
@pytest.mark.parametrize("case", [
    # B, L, D, order, group, number of equal stretches, mr_rows
    (2, 2048, 128, 16, 16, 4, 0),
    (1, 3072, 256, 7, 32, 3, 128),        # several tiles per stretch
    (3, 256, 64, 16, 16, 8, 32),          # one-chunk stretches
    (1, 8192, 512, 16, 16, 4, 0),
])
def test_stretches_from_zero_states_plus_a_fold_equal_the_whole_sequence(case):
    """What ranks that hold consecutive stretches of one sequence do (Sec. 4 applied to the recurrent form):
    hyena_li_state on every stretch from a zero state (independent of each other), hyena_li_state_fold of the
    stretches before a rank into its start state, then hyena_li_fwd_carry from there, here in reverse order to show
    that no stretch waits for another.  States and outputs against the oracle on the whole sequence."""
    B, L, D, order, group, n, rows = case
    say("li parallel stretches B=%d L=%d D=%d order=%d group=%d n=%d rows=%d" % case)
    binding.set_option("mr_rows", rows)
    rng = np.random.Generator(np.random.PCG64(650 + L + n))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    R, lam = synth.li_params(rng, D // group, order)
    dq, dk, dv, dR, dl = dev(q), dev(k), dev(v), dev(R), dev(lam)
    T = L // n
    cut = lambda x, i: x[:, i * T:(i + 1) * T].contiguous()
    local = [binding.hyena_li_state(cut(dk, i), cut(dv, i), dl, group) for i in range(n)]
    for i in (0, n - 1):   # a stretch's own end state is the definition's on that stretch alone
        want = oracle.li_state(k[:, i * T:(i + 1) * T], v[:, i * T:(i + 1) * T], lam, group=group)
        assert oracle.rel_err(_state_as_oracle(local[i], B, D, order), want) <= TOL["bf16"]
    parts = [None] * n
    for i in reversed(range(n)):
        start = binding.hyena_li_state_fold(local[:i], T, dl, B, D, group)
        want = oracle.li_state(k[:, :i * T], v[:, :i * T], lam, group=group) if i > 0 else np.zeros((B, D, order))
        got = _state_as_oracle(start, B, D, order)
        assert np.isfinite(got).all()
        assert np.abs(got - want).max() <= TOL["bf16"] * max(np.abs(want).max(), 1e-30), i
        parts[i], _ = binding.hyena_li_fwd_carry(cut(dq, i), cut(dk, i), cut(dv, i), dR, dl, group, state_in=start,
                                                 want_state=False)
    y = torch.cat(parts, dim=1)
    ref = oracle.li_recurrent(q, k, v, R, lam, group=group)
    assert oracle.rel_err(host(y), ref) <= TOL["bf16"]
    assert oracle.rel_err(host(y), host(binding.hyena_li_fwd(dq, dk, dv, dR, dl, group))) <= TOL["bf16"]
    # the state-only walk continues a sequence like the carry call does
    chained = None
    for i in range(n):
        chained = binding.hyena_li_state(cut(dk, i), cut(dv, i), dl, group, state_in=chained)
    want = oracle.li_state(k, v, lam, group=group)
    assert oracle.rel_err(_state_as_oracle(chained, B, D, order), want) <= TOL["bf16"]
    folded = binding.hyena_li_state_fold(local, T, dl, B, D, group)
    assert oracle.rel_err(_state_as_oracle(folded, B, D, order), want) <= TOL["bf16"]


def test_state_calls_refuse_what_they_cannot_do():
    B, L, D, order, group = 1, 640, 128, 16, 16
    rng = np.random.Generator(np.random.PCG64(612))
    k, v = (dev(synth.normal_tensor(rng, (B, L, D), "bf16")) for _ in range(2))
    _, lam = (dev(x) for x in synth.li_params(rng, D // group, order))
    with pytest.raises(binding.HyenaError):   # a length that is no multiple of 32
        binding.hyena_li_state(k[:, :100].contiguous(), v[:, :100].contiguous(), lam, group)
    with pytest.raises(binding.HyenaError):   # fp32: the general kernel keeps no such state
        binding.hyena_li_state(k.float(), v.float(), lam, group)
    zero = binding.hyena_li_state_fold([], 512, lam, B, D, group)
    assert torch.count_nonzero(zero) == 0
    s = binding.hyena_li_state(k, v, lam, group)
    same = binding.hyena_li_state_fold([], 512, lam, B, D, group, state_in=s)    # nothing to fold: the state itself
    assert torch.equal(same, s)
