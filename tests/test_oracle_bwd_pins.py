"""Pins for the backward oracle: it must be the gradient of the (already pinned) forward oracle.
Checked by central finite differences, by the adjoint identity, by closed forms and against numpy
correlations; none of these re-uses the backward formulas."""
import numpy as np
import pytest

import oracle


def rng(seed):
    return np.random.default_rng(seed)


def loss(q, k, v, h, w, group):
    return float(np.sum(w * oracle.gated_conv(q, k, v, h, group=group)))


@pytest.mark.parametrize("B,L,D,lh,group", [(1, 9, 2, 3, 1), (2, 12, 4, 5, 2), (1, 7, 4, 9, 4), (1, 10, 2, 1, 1)])
def test_matches_central_finite_differences(B, L, D, lh, group):
    """The forward is multilinear in (q), (k), (v), (h) separately, so a central difference in one argument
    is exact up to rounding."""
    r = rng(B * 100 + L * 10 + lh)
    q, k, v, w = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D // group, lh))
    dq, dk, dv, dh = oracle.gated_conv_bwd(w, q, k, v, h, group=group)
    eps = 1e-3
    for name, arr, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv), ("h", h, dh)):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = loss(q, k, v, h, w, group)
            arr[idx] = old - eps
            lm = loss(q, k, v, h, w, group)
            arr[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=0, atol=1e-8, err_msg=name)


def test_adjoint_identity():
    """<dy, J_v . delta> = <J_v^T dy, delta> for the linear map v -> y, and likewise for k, q and h."""
    r = rng(3)
    B, L, D, lh, group = 2, 40, 6, 11, 3
    q, k, v, dy = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D // group, lh))
    dq, dk, dv, dh = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    zero = np.zeros((B, L, D))
    for arr, grad, which in ((q, dq, "q"), (k, dk, "k"), (v, dv, "v")):
        delta = r.standard_normal((B, L, D))
        args = dict(q=q, k=k, v=v)
        args[which] = delta
        jd = oracle.gated_conv(args["q"], args["k"], args["v"], h, group=group)
        assert abs(np.sum(dy * jd) - np.sum(grad * delta)) < 1e-9
    dlt = r.standard_normal(h.shape)
    assert abs(np.sum(dy * oracle.gated_conv(q, k, v, dlt, group=group)) - np.sum(dh * dlt)) < 1e-9
    assert zero.shape == dq.shape


def test_filter_gradient_is_a_correlation():
    """dh[j] = sum_t g[t] u[t-j] with g = dy*q, u = k*v: numpy.correlate per channel, summed over the group."""
    r = rng(4)
    B, L, D, lh, group = 2, 50, 4, 8, 2
    q, k, v, dy = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D // group, lh))
    _, _, _, dh = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    g, u = dy * q, k * v
    ref = np.zeros_like(dh)
    for b in range(B):
        for c in range(D):
            full = np.correlate(g[b, :, c], u[b, :, c], mode="full")  # lag j at index L-1+j
            ref[c // group] += full[L - 1:L - 1 + lh]
    np.testing.assert_allclose(dh, ref, rtol=0, atol=1e-10)


def test_input_gradients_against_numpy_convolutions():
    r = rng(5)
    L, D, lh = 33, 3, 6
    q, k, v, dy = (r.standard_normal((1, L, D)) for _ in range(4))
    h = r.standard_normal((D, lh))
    dq, dk, dv, _ = oracle.gated_conv_bwd(dy, q, k, v, h)
    for c in range(D):
        z = np.convolve(k[0, :, c] * v[0, :, c], h[c])[:L]
        np.testing.assert_allclose(dq[0, :, c], dy[0, :, c] * z, rtol=0, atol=1e-12)
        g = dy[0, :, c] * q[0, :, c]
        du = np.convolve(g[::-1], h[c])[:L][::-1]  # anti-causal = causal on the reversed signal
        np.testing.assert_allclose(dk[0, :, c], du * v[0, :, c], rtol=0, atol=1e-12)
        np.testing.assert_allclose(dv[0, :, c], du * k[0, :, c], rtol=0, atol=1e-12)


def test_closed_form_length_one_filter():
    r = rng(6)
    q, k, v, dy = (r.standard_normal((2, 8, 3)) for _ in range(4))
    h = r.standard_normal((3, 1))
    dq, dk, dv, dh = oracle.gated_conv_bwd(dy, q, k, v, h)
    np.testing.assert_allclose(dq, dy * h[:, 0] * k * v, rtol=1e-14)
    np.testing.assert_allclose(dk, dy * q * h[:, 0] * v, rtol=1e-14)
    np.testing.assert_allclose(dv, dy * q * h[:, 0] * k, rtol=1e-14)
    np.testing.assert_allclose(dh[:, 0], np.sum(dy * q * k * v, axis=(0, 1)), rtol=1e-13)


def test_anti_causality_of_input_gradients():
    """dk[s], dv[s] depend on dy and q only at times >= s, and on nothing before s."""
    r = rng(7)
    B, L, D, lh, s = 1, 40, 2, 7, 20
    q, k, v, dy = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D, lh))
    _, dk0, dv0, _ = oracle.gated_conv_bwd(dy, q, k, v, h)
    dy2, q2 = dy.copy(), q.copy()
    dy2[:, :s] = r.standard_normal((B, s, D))
    q2[:, :s] = r.standard_normal((B, s, D))
    _, dk1, dv1, _ = oracle.gated_conv_bwd(dy2, q2, k, v, h)
    assert np.array_equal(dk0[:, s:], dk1[:, s:]) and np.array_equal(dv0[:, s:], dv1[:, s:])
    assert not np.array_equal(dk0[:, :s], dk1[:, :s])


def test_batch_and_group_sums_in_filter_gradient():
    r = rng(8)
    L, D, lh, group = 20, 4, 5, 2
    q, k, v, dy = (r.standard_normal((3, L, D)) for _ in range(4))
    h = r.standard_normal((D // group, lh))
    _, _, _, dh = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    per_item = sum(oracle.gated_conv_bwd(dy[b:b + 1], q[b:b + 1], k[b:b + 1], v[b:b + 1], h, group=group)[3] for b in range(3))
    np.testing.assert_allclose(dh, per_item, rtol=0, atol=1e-12)
    per_chan = oracle.gated_conv_bwd(dy, q, k, v, np.repeat(h, group, axis=0), group=1)[3]
    np.testing.assert_allclose(dh, per_chan.reshape(D // group, group, lh).sum(axis=1), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------- featurizer backward
@pytest.mark.parametrize("B,L,D,lh,group", [(1, 6, 2, 3, 1), (2, 7, 4, 4, 2), (1, 5, 4, 8, 4), (2, 4, 2, 1, 1)])
def test_featurizer_backward_is_the_adjoint_of_the_forward_on_every_basis_vector(B, L, D, lh, group):
    """The forward x -> h * x is linear in x and in h, so its gradient given dy is fixed element by element:
    dx[i] = <dy, h * e_i> and dh[m] = <dy, e_m * x>, computed here with the pinned forward oracle on unit inputs."""
    r = rng(700 + L + lh)
    x, dy = r.standard_normal((B, L, D)), r.standard_normal((B, L, D))
    h = r.standard_normal((D // group, lh))
    dx, dh = oracle.causal_conv_bwd(dy, x, h, group=group)
    want_dx = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        e = np.zeros_like(x)
        e[idx] = 1.0
        want_dx[idx] = np.sum(dy * oracle.causal_conv(e, h, group=group))
    want_dh = np.zeros_like(h)
    for idx in np.ndindex(*h.shape):
        e = np.zeros_like(h)
        e[idx] = 1.0
        want_dh[idx] = np.sum(dy * oracle.causal_conv(x, e, group=group))
    np.testing.assert_allclose(dx, want_dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dh, want_dh, rtol=0, atol=1e-12)


def test_featurizer_backward_against_numpy_correlations():
    """Per channel: dx is dy correlated with h (np.correlate, taps reaching forward in time), dh[j] the lag-j
    correlation of dy with x, summed over the batch and the channels of a group."""
    r = rng(711)
    B, L, D, lh, group = 2, 40, 6, 7, 3
    x, dy = r.standard_normal((B, L, D)), r.standard_normal((B, L, D))
    h = r.standard_normal((D // group, lh))
    dx, dh = oracle.causal_conv_bwd(dy, x, h, group=group)
    want_dh = np.zeros_like(h)
    for b in range(B):
        for c in range(D):
            g = c // group
            full = np.correlate(np.concatenate([dy[b, :, c], np.zeros(lh - 1)]), h[g], mode="valid")
            np.testing.assert_allclose(dx[b, :, c], full, rtol=0, atol=1e-12)
            for j in range(lh):
                want_dh[g, j] += np.dot(dy[b, j:, c], x[b, :L - j, c])
    np.testing.assert_allclose(dh, want_dh, rtol=0, atol=1e-11)


def test_featurizer_backward_is_the_gated_backward_with_unit_gates():
    """With q = v = 1 the gated operator is the featurizer of k, so dk and dh of the (separately pinned) gated
    backward are dx and dh."""
    r = rng(712)
    B, L, D, lh, group = 2, 30, 8, 5, 2
    x, dy = r.standard_normal((B, L, D)), r.standard_normal((B, L, D))
    h = r.standard_normal((D // group, lh))
    one = np.ones_like(x)
    _, dk, _, dh_g = oracle.gated_conv_bwd(dy, one, x, one, h, group=group)
    dx, dh = oracle.causal_conv_bwd(dy, x, h, group=group)
    np.testing.assert_allclose(dx, dk, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dh, dh_g, rtol=0, atol=1e-12)


def test_featurizer_backward_closed_forms():
    """A filter that is one tap at lag j0 shifts: dx[s] = dy[s + j0] (zero past the end); with dy = x = 1 the filter
    gradient counts the terms: dh[g, j] = B * group * (L - j), zero once the lag reaches L."""
    B, L, D, lh, group, j0 = 2, 9, 4, 12, 2, 3
    r = rng(713)
    dy = r.standard_normal((B, L, D))
    h = np.zeros((D // group, lh))
    h[:, j0] = 1.0
    dx, _ = oracle.causal_conv_bwd(dy, np.zeros_like(dy), h, group=group)
    want = np.zeros_like(dy)
    want[:, :L - j0] = dy[:, j0:]
    np.testing.assert_array_equal(dx, want)
    one = np.ones((B, L, D))
    _, dh = oracle.causal_conv_bwd(one, one, h, group=group)
    np.testing.assert_array_equal(dh, np.tile(np.maximum(L - np.arange(lh), 0) * B * group, (D // group, 1)).astype(float))


def test_featurizer_backward_reads_bf16_and_fp32_inputs_exactly():
    r = rng(714)
    B, L, D, lh = 1, 20, 4, 4
    x32 = r.standard_normal((B, L, D)).astype(np.float32)
    dy32 = r.standard_normal((B, L, D)).astype(np.float32)
    h = r.standard_normal((D, lh)).astype(np.float32)
    a = oracle.causal_conv_bwd(dy32, x32, h)
    b = oracle.causal_conv_bwd(dy32.astype(np.float64), x32.astype(np.float64), h.astype(np.float64))
    for u, w in zip(a, b):
        np.testing.assert_array_equal(u, w)


# ---------------------------------------------------------------------------------------- chain backward
@pytest.mark.parametrize("B,L,D,lf,fg,lh,group", [(1, 8, 2, 3, 1, 4, 1), (2, 9, 4, 2, 2, 6, 4), (1, 6, 4, 4, 1, 9, 2)])
def test_chain_backward_matches_central_finite_differences_of_the_chain(B, L, D, lf, fg, lh, group):
    """The chain is linear in each of q, k, v, hq, hk, hv, h separately, so a central difference of the (pinned)
    forward chain in one argument is exact up to rounding."""
    r = rng(900 + L + lh)
    q, k, v, w = (r.standard_normal((B, L, D)) for _ in range(4))
    hq, hk, hv = (r.standard_normal((D // fg, lf)) for _ in range(3))
    h = r.standard_normal((D // group, lh))
    grads = oracle.chain_bwd(w, q, k, v, hq, hk, hv, h, group=group, feat_group=fg)
    args = [q, k, v, hq, hk, hv, h]
    eps = 1e-3

    def f():
        return float(np.sum(w * oracle.chain(*args, group=group, feat_group=fg)))

    for name, arr, grad in zip(("q", "k", "v", "hq", "hk", "hv", "h"), args, grads):
        num = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            old = arr[idx]
            arr[idx] = old + eps
            lp = f()
            arr[idx] = old - eps
            lm = f()
            arr[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=0, atol=1e-8, err_msg=name)


def test_chain_backward_with_identity_featurizers_is_the_gated_backward():
    """Featurizers that are a single unit tap at lag 0 leave q, k, v unchanged: dq, dk, dv and dh are those of the
    gated operator, and the featurizer gradients at tap 0 are <dq, q>, <dk, k>, <dv, v> per channel."""
    r = rng(950)
    B, L, D, lf, lh, group = 2, 12, 4, 3, 5, 2
    q, k, v, dy = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D // group, lh))
    ident = np.zeros((D, lf))
    ident[:, 0] = 1.0
    dq, dk, dv, dhq, dhk, dhv, dh = oracle.chain_bwd(dy, q, k, v, ident, ident, ident, h, group=group, feat_group=1)
    want = oracle.gated_conv_bwd(dy, q, k, v, h, group=group)
    for a, b in zip((dq, dk, dv, dh), want):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dhq[:, 0], np.sum(want[0] * q, axis=(0, 1)), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dhk[:, 0], np.sum(want[1] * k, axis=(0, 1)), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dhv[:, 0], np.sum(want[2] * v, axis=(0, 1)), rtol=0, atol=1e-11)
