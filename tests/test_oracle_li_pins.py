"""Pins of the Hyena-LI part of the oracle (Sec. 2.1: h_t = sum_n R_n lambda_n^(t-1)) against things that are not
the oracle: SciPy's recursive filter, closed forms of geometric sums, hand-computed taps, special poles."""
import numpy as np
import pytest
import scipy.signal

import oracle


def rng_for(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_taps_of_a_hand_computed_example_and_first_tap_is_the_sum_of_residues():
    # R = (1, 2), lambda = (1/2, -1/2): h = 3, -1/2, 3/4, -1/8, 3/16 (t = 1 gives exponent 0)
    h = oracle.li_filter([[1.0, 2.0]], [[0.5, -0.5]], 5)
    assert np.array_equal(h, np.array([[3.0, -0.5, 0.75, -0.125, 0.1875]]))
    R = rng_for(1).standard_normal((3, 7))
    lam = rng_for(2).uniform(-1, 1, (3, 7))
    assert np.allclose(oracle.li_filter(R, lam, 4)[:, 0], R.sum(axis=1), rtol=0, atol=1e-15)


def test_zero_pole_is_the_identity_and_unit_pole_a_running_sum():
    rng = rng_for(3)
    k = rng.standard_normal((2, 50, 3))
    one = np.ones_like(k)
    y0 = oracle.li_conv(one, k, one, np.full((3, 1), 2.5), np.zeros((3, 1)))
    assert np.array_equal(y0, 2.5 * k)                                    # lambda = 0: 0 ** 0 = 1, later taps vanish
    y1 = oracle.li_conv(one, k, one, np.ones((3, 1)), np.ones((3, 1)))
    assert np.allclose(y1, np.cumsum(k, axis=1), rtol=1e-13, atol=1e-13)  # lambda = 1: prefix sums
    ym = oracle.li_conv(one, k, one, np.ones((3, 1)), -np.ones((3, 1)))
    sign = (-1.0) ** np.arange(50)[None, :, None]
    assert np.allclose(ym, sign * np.cumsum(sign * k, axis=1), rtol=1e-13, atol=1e-13)  # lambda = -1: alternating sums


@pytest.mark.parametrize("d", [1, 2, 5])
def test_matches_scipy_recursive_filters_in_parallel_form(d):
    """y = sum_n R_n s_n with s_n[t] = lambda_n s_n[t-1] + u[t]: SciPy's lfilter runs each first-order recursion."""
    rng = rng_for(10 + d)
    B, L, D, group = 2, 300, 6, 2
    q, k, v = (rng.standard_normal((B, L, D)) for _ in range(3))
    R = rng.standard_normal((D // group, d))
    lam = rng.uniform(-0.99, 0.99, (D // group, d))
    u = k * v
    want = np.zeros_like(u)
    for c in range(D):
        g = c // group
        for n in range(d):
            want[:, :, c] += R[g, n] * scipy.signal.lfilter([1.0], [1.0, -lam[g, n]], u[:, :, c], axis=1)
    want *= q
    got = oracle.li_conv(q, k, v, R, lam, group=group)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-10)


def test_matches_one_rational_transfer_function():
    """Two exponentials combine into b(z)/a(z) with a = (1 - l1 z^-1)(1 - l2 z^-1); SciPy filters with the
    second-order recursion, which never forms the two first-order states."""
    rng = rng_for(20)
    R, lam = np.array([[0.7, -1.3]]), np.array([[0.9, -0.4]])
    u = rng.standard_normal((1, 400, 1))
    b = [R[0, 0] + R[0, 1], -(R[0, 0] * lam[0, 1] + R[0, 1] * lam[0, 0])]
    a = np.convolve([1.0, -lam[0, 0]], [1.0, -lam[0, 1]])
    want = scipy.signal.lfilter(b, a, u[0, :, 0])
    got = oracle.li_conv(np.ones_like(u), u, np.ones_like(u), R, lam)[0, :, 0]
    assert np.allclose(got, want, rtol=1e-11, atol=1e-11)


def test_step_response_is_the_geometric_sum():
    R = np.array([[1.5, -0.5, 2.0]])
    lam = np.array([[0.5, 0.9, -0.8]])
    L = 64
    one = np.ones((1, L, 1))
    t = np.arange(L)
    want = sum(R[0, n] * (1 - lam[0, n] ** (t + 1)) / (1 - lam[0, n]) for n in range(3))
    got = oracle.li_conv(one, one, one, R, lam)[0, :, 0]
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_filter_reaches_back_to_the_first_step_and_not_beyond_the_batch_item():
    """An impulse at t = 0 is still felt at the last step (filter as long as the sequence), scaled by lambda^(L-1);
    batch items do not see each other."""
    L = 200
    v = np.zeros((2, L, 1))
    v[0, 0, 0] = 1.0
    one = np.ones_like(v)
    y = oracle.li_conv(one, one, v, np.array([[2.0]]), np.array([[0.97]]))
    assert y[0, L - 1, 0] == pytest.approx(2.0 * 0.97 ** (L - 1), rel=1e-12)
    assert np.all(y[1] == 0.0)


def test_points_agree_with_the_full_tensor_and_groups_share_parameters():
    rng = rng_for(30)
    B, L, D, group, d = 2, 120, 8, 4, 3
    q, k, v = (rng.standard_normal((B, L, D)).astype(np.float32) for _ in range(3))
    R = rng.standard_normal((D // group, d))
    lam = rng.uniform(0.5, 1.0, (D // group, d))
    full = oracle.li_conv(q, k, v, R, lam, group=group)
    pts = np.array([[0, 0, 0], [1, 119, 7], [0, 57, 3], [1, 1, 4]])
    got = oracle.li_conv_points(q, k, v, R, lam, pts, group=group)
    assert np.array_equal(got, full[pts[:, 0], pts[:, 1], pts[:, 2]])
    same = oracle.li_conv(q, k, v, np.repeat(R, group, axis=0), np.repeat(lam, group, axis=0), group=1)
    assert np.array_equal(full, same)


def _mutants():
    def base(R, lam, L, shift=0, drop=0, absval=False, square=False):
        R = np.asarray(R, dtype=np.float64)
        lam = np.asarray(lam, dtype=np.float64)
        if absval:
            lam = np.abs(lam)
        j = np.arange(int(L)) + shift
        h = np.zeros((R.shape[0], int(L)))
        for n in range(R.shape[1] - drop):
            p = np.power(lam[:, n, None], j[None, :])
            h += (R[:, n, None] ** 2 if square else R[:, n, None]) * p
        return h

    return {
        "exponent counted from t instead of t-1": lambda R, lam, L: base(R, lam, L, shift=1),
        "last exponential dropped": lambda R, lam, L: base(R, lam, L, drop=1),
        "sign of the poles lost": lambda R, lam, L: base(R, lam, L, absval=True),
        "residues squared": lambda R, lam, L: base(R, lam, L, square=True),
        "filter one tap short": lambda R, lam, L: np.concatenate(
            [base(R, lam, L)[:, :-1], np.zeros((np.asarray(R).shape[0], 1))], axis=1) if L > 1 else base(R, lam, L),
    }


def test_planted_mistakes_in_the_filter_are_caught(monkeypatch):
    """Each plausible mistake, planted in a copy of li_filter, must fail at least one of the pins above."""
    pins = [
        test_taps_of_a_hand_computed_example_and_first_tap_is_the_sum_of_residues,
        test_zero_pole_is_the_identity_and_unit_pole_a_running_sum,
        lambda: test_matches_scipy_recursive_filters_in_parallel_form(2),
        test_matches_one_rational_transfer_function,
        test_step_response_is_the_geometric_sum,
        test_filter_reaches_back_to_the_first_step_and_not_beyond_the_batch_item,
    ]
    for name, mutant in _mutants().items():
        monkeypatch.setattr(oracle, "li_filter", mutant)
        caught = 0
        for pin in pins:
            try:
                pin()
            except AssertionError:
                caught += 1
        assert caught > 0, "no pin notices: " + name
    monkeypatch.undo()
    for pin in pins:  # and the real filter passes them all
        pin()


# ------------------------------------------------------------------ the recurrent form (oracle.li_recurrent)
@pytest.mark.parametrize("case", [(1, 1, 1, 1, 1), (2, 257, 12, 5, 4), (3, 64, 33, 16, 1), (1, 500, 70, 3, 35)])
def test_recurrent_form_equals_the_definition(case):
    """Exchanging the two sums of the definition changes fp64 rounding only."""
    B, L, D, d, group = case
    rng = rng_for(40 + L)
    q, k, v = (rng.standard_normal((B, L, D)) for _ in range(3))
    R = rng.standard_normal((D // group, d))
    lam = rng.uniform(-1.0, 1.0, (D // group, d))
    want = oracle.li_conv(q, k, v, R, lam, group=group)
    got = oracle.li_recurrent(q, k, v, R, lam, group=group)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * max(1.0, np.abs(want).max()))


def test_recurrent_form_takes_the_stored_bits_of_bf16_and_fp32_inputs():
    import torch

    rng = rng_for(50)
    B, L, D, d, group = 2, 90, 32, 4, 16
    q, k, v = (torch.from_numpy(rng.standard_normal((B, L, D)).astype(np.float32)).bfloat16() for _ in range(3))
    R = rng.standard_normal((D // group, d)).astype(np.float32)
    lam = rng.uniform(0.0, 1.0, (D // group, d)).astype(np.float32)
    want = oracle.li_conv(q, k, v, R, lam, group=group)
    got = oracle.li_recurrent(q, k, v, R, lam, group=group)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.abs(want).max())


def test_recurrent_form_against_scipy_and_closed_forms():
    """The same outside pins as the definition: SciPy's first-order recursions, the geometric step response,
    poles 0, 1 and -1, and batch items that do not see each other."""
    rng = rng_for(60)
    B, L, D, group, d = 2, 300, 6, 2, 3
    q, k, v = (rng.standard_normal((B, L, D)) for _ in range(3))
    R = rng.standard_normal((D // group, d))
    lam = rng.uniform(-0.99, 0.99, (D // group, d))
    u = k * v
    want = np.zeros_like(u)
    for c in range(D):
        g = c // group
        for n in range(d):
            want[:, :, c] += R[g, n] * scipy.signal.lfilter([1.0], [1.0, -lam[g, n]], u[:, :, c], axis=1)
    assert np.allclose(oracle.li_recurrent(q, k, v, R, lam, group=group), want * q, rtol=1e-10, atol=1e-10)
    one = np.ones((1, 64, 1))
    Rs, ls = np.array([[1.5, -0.5, 2.0]]), np.array([[0.5, 0.9, -0.8]])
    t = np.arange(64)
    step = sum(Rs[0, n] * (1 - ls[0, n] ** (t + 1)) / (1 - ls[0, n]) for n in range(3))
    assert np.allclose(oracle.li_recurrent(one, one, one, Rs, ls)[0, :, 0], step, rtol=1e-12, atol=1e-12)
    kk = rng.standard_normal((2, 50, 3))
    o3 = np.ones_like(kk)
    assert np.array_equal(oracle.li_recurrent(o3, kk, o3, np.full((3, 1), 2.5), np.zeros((3, 1))), 2.5 * kk)
    assert np.allclose(oracle.li_recurrent(o3, kk, o3, np.ones((3, 1)), np.ones((3, 1))), np.cumsum(kk, axis=1),
                       rtol=1e-13, atol=1e-13)
    imp = np.zeros((2, 200, 1))
    imp[0, 0, 0] = 1.0
    y = oracle.li_recurrent(np.ones_like(imp), np.ones_like(imp), imp, np.array([[2.0]]), np.array([[0.97]]))
    assert y[0, 199, 0] == pytest.approx(2.0 * 0.97 ** 199, rel=1e-12)
    assert np.all(y[1] == 0.0)


# ------------------------------------------------------------------ the state a cut sequence hands on (oracle.li_state)
def test_end_state_reproduces_the_last_output_and_the_continuation():
    """Three things the running sums must satisfy, none of which uses their own formula: (1) weighted by the
    residues they give the last output of the definition; (2) they obey the first-order recursion in L (SciPy's
    recursive filter evaluated at its last step); (3) a sequence continued from them equals the uncut sequence:
    y[t >= L0] = q[t] * (sum_n R_n lam_n^(t - L0 + 1) s_n  +  the definition on the steps from L0 on)."""
    rng = rng_for(70)
    B, L, D, group, d = 2, 120, 6, 2, 3
    q, k, v = (rng.standard_normal((B, L, D)) for _ in range(3))
    R = rng.standard_normal((D // group, d))
    lam = rng.uniform(-0.95, 0.95, (D // group, d))
    s = oracle.li_state(k, v, lam, group=group)
    assert s.shape == (B, D, d)
    Rc, lc = np.repeat(R, group, axis=0), np.repeat(lam, group, axis=0)  # per channel
    one = np.ones_like(q)
    assert np.allclose((s * Rc[None]).sum(-1), oracle.li_conv(one, k, v, R, lam, group=group)[:, -1, :], rtol=1e-12, atol=1e-12)
    u = k * v
    for c in range(D):
        for n in range(d):
            rec = scipy.signal.lfilter([1.0], [1.0, -lc[c, n]], u[:, :, c], axis=1)[:, -1]
            assert np.allclose(s[:, c, n], rec, rtol=1e-11, atol=1e-11)
    L0 = 70
    s0 = oracle.li_state(k[:, :L0], v[:, :L0], lam, group=group)
    tail = oracle.li_conv(q[:, L0:], k[:, L0:], v[:, L0:], R, lam, group=group)
    j = np.arange(1, L - L0 + 1)
    carry = np.einsum("bcn,cnj->bjc", s0, Rc[:, :, None] * np.power(lc[:, :, None], j[None, None, :]))
    whole = oracle.li_conv(q, k, v, R, lam, group=group)
    assert np.allclose(tail + q[:, L0:] * carry, whole[:, L0:], rtol=1e-11, atol=1e-11)


def test_end_state_closed_forms_and_stored_bits():
    import torch

    one = np.ones((1, 40, 2))
    s = oracle.li_state(one, one, np.array([[0.5, 1.0, 0.0]]), group=2)
    assert np.allclose(s[0, 0], [(1 - 0.5 ** 40) / 0.5, 40.0, 1.0], rtol=1e-13) and np.array_equal(s[0, 0], s[0, 1])
    rng = rng_for(71)
    k, v = (torch.from_numpy(rng.standard_normal((1, 30, 4)).astype(np.float32)).bfloat16() for _ in range(2))
    lam = rng.uniform(0, 1, (4, 2)).astype(np.float32)
    want = oracle.li_state(k.float().numpy().astype(np.float64), v.float().numpy().astype(np.float64), lam, group=1)
    assert np.array_equal(oracle.li_state(k, v, lam, group=1), want)
