"""Pins for the fp64 CPU oracle against things other than itself: the worked example the paper
prints, library routines (numpy.convolve, FFT), a literal dense Toeplitz product, closed forms and
invariants.  None of these needs a GPU."""
import os

import numpy as np
import pytest
import torch

import oracle


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- helpers (test side)
def read_index_matrices(path):
    mats, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                mats[cur] = []
                continue
            mats[cur].append([-1 if tok == "." else int(tok) for tok in line.split()])
    return {k: np.asarray(v, dtype=np.int64) for k, v in mats.items()}


def fill(idx, h):
    out = np.zeros(idx.shape, dtype=np.float64)
    m = idx >= 0
    out[m] = np.asarray(h, dtype=np.float64)[idx[m]]
    return out


def dense_toeplitz(h, L):
    """Literal matrix of Sec. 3.1 Eq. 3: T[t][s] = h[t - s] inside the band, else 0 (python loops)."""
    T = [[0.0] * L for _ in range(L)]
    for t in range(L):
        for s in range(L):
            if 0 <= t - s < len(h):
                T[t][s] = float(h[t - s])
    return np.asarray(T, dtype=np.float64).reshape(L, L)


def ones_like_gate(shape):
    return np.ones(shape, dtype=np.float64)


# ------------------------------------------------------------------- the paper's worked example
def test_worked_example_factors_sum_to_printed_T(golden_dir):
    m = read_index_matrices(os.path.join(golden_dir, "two_stage_worked_example.txt"))
    h = np.array([2.0, 3.0, 5.0, 7.0])
    H0, H1, T = fill(m["H0"], h), fill(m["H1"], h), fill(m["T"], h)
    Z = np.zeros((3, 3))
    np.testing.assert_array_equal(np.block([[H0, Z], [Z, H0]]) + np.block([[Z, Z], [H1, Z]]), T)


def test_oracle_reproduces_printed_T_column_by_column(golden_dir):
    """Impulse at time s must return column s of the printed 6x6 matrix."""
    m = read_index_matrices(os.path.join(golden_dir, "two_stage_worked_example.txt"))
    h = np.array([[2.0, 3.0, 5.0, 7.0]])
    T = fill(m["T"], h[0])
    L = 6
    for s in range(L):
        x = np.zeros((1, L, 1))
        x[0, s, 0] = 1.0
        np.testing.assert_array_equal(oracle.causal_conv(x, h)[0, :, 0], T[:, s])
        one = np.ones((1, L, 1))
        np.testing.assert_array_equal(oracle.gated_conv(one, one, x, h)[0, :, 0], T[:, s])


def test_oracle_matches_general_printed_factor_corners(golden_dir):
    """Corner entries of H_0 / H_1 as displayed in Sec. 3.1, for several block sizes."""
    rows = []
    with open(os.path.join(golden_dir, "block_factors_general.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    for lb in (3, 4, 8):
        lh = 2 * lb
        h = rng(lb).standard_normal((1, lh))
        L = 2 * lb
        # columns of T from the oracle (impulse responses); T[lb + i][j] is H_1[i][j], T[i][j] is H_0[i][j]
        T = np.zeros((L, L))
        for s in range(L):
            x = np.zeros((1, L, 1))
            x[0, s, 0] = 1.0
            T[:, s] = oracle.causal_conv(x, h)[0, :, 0]
        for fac, r, c, a, b in rows:
            r = lb - 1 if r == "last" else int(r)
            c = lb - 1 if c == "last" else int(c)
            tap = int(a) * lb + int(b)
            got = T[r + (lb if fac == "H1" else 0), c]
            assert got == h[0, tap], (lb, fac, r, c, tap)


# ------------------------------------------------------------------------- library special cases
@pytest.mark.parametrize("L,lh", [(1, 1), (5, 1), (9, 4), (16, 7), (40, 13), (33, 40), (64, 128)])
def test_matches_numpy_convolve_per_channel(L, lh):
    r = rng(100 + L + lh)
    D, B = 3, 2
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    h = r.standard_normal((D, lh))
    y = oracle.gated_conv(q, k, v, h)
    z = oracle.causal_conv(v, h)
    for b in range(B):
        for c in range(D):
            ref = np.convolve(k[b, :, c] * v[b, :, c], h[c])[:L]
            np.testing.assert_allclose(y[b, :, c], q[b, :, c] * ref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(z[b, :, c], np.convolve(v[b, :, c], h[c])[:L], rtol=0, atol=1e-12)


@pytest.mark.parametrize("L,lh,dg", [(257, 7, 1), (512, 128, 4), (300, 200, 2)])
def test_matches_fft_convolution(L, lh, dg):
    """(x*h) = F^-1(F(x) o F(h)) with zero padding to >= L + l_h - 1 (Sec. 4, FFT identity)."""
    r = rng(7 * L + lh)
    D, B = 8, 2
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    h = r.standard_normal((D // dg, lh))
    n = 1
    while n < L + lh - 1:
        n *= 2
    u = k * v
    hf = np.fft.rfft(np.repeat(h, dg, axis=0).T, n=n, axis=0)  # [n/2+1, D]
    zf = np.fft.irfft(np.fft.rfft(u, n=n, axis=1) * hf[None], n=n, axis=1)[:, :L, :]
    y = oracle.gated_conv(q, k, v, h, group=dg)
    np.testing.assert_allclose(y, q * zf, rtol=0, atol=1e-10)


@pytest.mark.parametrize("L,lh", [(1, 3), (4, 1), (7, 3), (12, 5), (16, 16), (10, 25)])
def test_matches_literal_dense_toeplitz_product(L, lh):
    r = rng(L * 31 + lh)
    D = 4
    q, k, v = (r.standard_normal((1, L, D)) for _ in range(3))
    h = r.standard_normal((D, lh))
    y = oracle.gated_conv(q, k, v, h)
    for c in range(D):
        T = dense_toeplitz(h[c], L)
        ref = np.array([sum(T[t, s] * k[0, s, c] * v[0, s, c] for s in range(L)) for t in range(L)])
        np.testing.assert_allclose(y[0, :, c], q[0, :, c] * ref, rtol=0, atol=1e-12)


# ------------------------------------------------------------------------------------ invariants
def test_impulse_response_returns_the_filter():
    L, D, dg, lh, t0 = 50, 8, 4, 9, 11
    h = rng(1).standard_normal((D // dg, lh))
    one = np.ones((1, L, D))
    for c in (0, 3, 4, 7):
        v = np.zeros((1, L, D))
        v[0, t0, c] = 1.0
        y = oracle.gated_conv(one, one, v, h, group=dg)
        expect = np.zeros((L, D))
        expect[t0:t0 + lh, c] = h[c // dg]
        np.testing.assert_array_equal(y[0], expect)


def test_linearity_in_v():
    r = rng(2)
    B, L, D, lh = 2, 70, 6, 11
    q, k, v1, v2 = (r.standard_normal((B, L, D)) for _ in range(4))
    h = r.standard_normal((D, lh))
    a, b = 0.75, -2.5
    lhs = oracle.gated_conv(q, k, a * v1 + b * v2, h)
    rhs = a * oracle.gated_conv(q, k, v1, h) + b * oracle.gated_conv(q, k, v2, h)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)


def test_not_linear_in_joint_scaling_of_k_and_v():
    """u = k (.) v is a product: scaling both k and v by a scales y by a^2 (catches u = k + v)."""
    r = rng(3)
    q, k, v = (r.standard_normal((1, 30, 2)) for _ in range(3))
    h = r.standard_normal((2, 5))
    np.testing.assert_allclose(oracle.gated_conv(q, 3 * k, 3 * v, h), 9 * oracle.gated_conv(q, k, v, h),
                               rtol=1e-13, atol=1e-13)


def test_causality_bitwise():
    r = rng(4)
    B, L, D, lh, t = 2, 64, 5, 9, 37
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    h = r.standard_normal((D, lh))
    y0 = oracle.gated_conv(q, k, v, h)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for a in (q2, k2, v2):
        a[:, t + 1:, :] = r.standard_normal((B, L - t - 1, D))
    y1 = oracle.gated_conv(q2, k2, v2, h)
    assert np.array_equal(y0[:, :t + 1], y1[:, :t + 1])
    assert not np.array_equal(y0[:, t + 1:], y1[:, t + 1:])


def test_post_gate_uses_q_at_the_output_time():
    """y[t] depends on q only through q[t]: zeroing q at one time zeroes exactly that row."""
    r = rng(5)
    q, k, v = (r.standard_normal((1, 20, 3)) + 3.0 for _ in range(3))
    h = np.abs(r.standard_normal((3, 4))) + 0.1
    q[0, 9] = 0.0
    y = oracle.gated_conv(q, k, v, h)
    assert np.all(y[0, 9] == 0.0) and np.all(y[0, :9] != 0.0) and np.all(y[0, 10:] != 0.0)


def test_closed_form_saturating_prefix_sum():
    L, lh = 40, 7
    h = rng(6).standard_normal((1, lh))
    one = np.ones((1, L, 1))
    y = oracle.gated_conv(one, one, one, h)[0, :, 0]
    ref = np.array([h[0, : min(t, lh - 1) + 1].sum() for t in range(L)])
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-14)


def test_closed_form_geometric_filter():
    L, lh, alpha = 300, 128, 0.05
    h = np.exp(-alpha * np.arange(lh))[None, :]
    one = np.ones((1, L, 1))
    y = oracle.gated_conv(one, one, one, h)[0, :, 0]
    n = np.minimum(np.arange(L), lh - 1) + 1
    ref = (1.0 - np.exp(-alpha * n)) / (1.0 - np.exp(-alpha))
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=0)


def test_length_one_filter_is_elementwise():
    r = rng(7)
    q, k, v = (r.standard_normal((2, 9, 4)) for _ in range(3))
    h = r.standard_normal((4, 1))
    np.testing.assert_allclose(oracle.gated_conv(q, k, v, h), h[:, 0] * q * k * v, rtol=1e-15, atol=0)
    np.testing.assert_allclose(oracle.causal_conv(v, h), h[:, 0] * v, rtol=1e-15, atol=0)


@pytest.mark.parametrize("dg", [2, 4, 16])
def test_grouped_filter_equals_replicated_filter(dg):
    """Sec. 2.2: every channel of a contiguous group of d_g channels uses the group's filter."""
    r = rng(8 + dg)
    B, L, D, lh = 2, 48, 32, 10
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    h = r.standard_normal((D // dg, lh))
    y_g = oracle.gated_conv(q, k, v, h, group=dg)
    y_r = oracle.gated_conv(q, k, v, np.repeat(h, dg, axis=0), group=1)
    assert np.array_equal(y_g, y_r)
    # and the groups are contiguous: channel c uses filter c // dg, not c % (D // dg)
    c = dg  # first channel of the second group
    ref = np.convolve(k[0, :, c] * v[0, :, c], h[1])[:L] * q[0, :, c]
    np.testing.assert_allclose(y_g[0, :, c], ref, rtol=0, atol=1e-12)


def test_shift_equivariance():
    r = rng(9)
    L, D, lh, s = 60, 3, 8, 13
    k, v = (r.standard_normal((1, L, D)) for _ in range(2))
    h = r.standard_normal((D, lh))
    one = np.ones((1, L, D))
    z = oracle.gated_conv(one, k, v, h)
    ks, vs = np.zeros_like(k), np.zeros_like(v)
    ks[:, s:], vs[:, s:] = k[:, : L - s], v[:, : L - s]
    zs = oracle.gated_conv(one, ks, vs, h)
    assert np.array_equal(zs[:, s:], z[:, : L - s]) and np.all(zs[:, :s] == 0)


def test_batch_items_are_independent():
    r = rng(10)
    L, D, lh = 20, 4, 6
    q, k, v = (r.standard_normal((3, L, D)) for _ in range(3))
    h = r.standard_normal((D, lh))
    y = oracle.gated_conv(q, k, v, h)
    for b in range(3):
        assert np.array_equal(y[b:b + 1], oracle.gated_conv(q[b:b + 1], k[b:b + 1], v[b:b + 1], h))
    perm = [2, 0, 1]
    assert np.array_equal(oracle.gated_conv(q[perm], k[perm], v[perm], h), y[perm])


# --------------------------------------------------------------- block convolution (Sec. 3.1-3.2)
def blocked_conv(x, h, lb, n_blocks=None):
    """hat y_n = sum_k H_k hat x_{n-k}, H_k[i][j] = h[k*lb + i - j]; numpy, written for this test."""
    L, lh = len(x), len(h)
    nb = -(-(lh - 1) // lb) if n_blocks is None else n_blocks
    n_chunks = -(-L // lb)
    xp = np.zeros(n_chunks * lb)
    xp[:L] = x
    y = np.zeros(n_chunks * lb)
    for n in range(n_chunks):
        for kk in range(nb + 1):
            if n - kk < 0:
                continue
            H = np.zeros((lb, lb))
            for i in range(lb):
                for j in range(lb):
                    tap = kk * lb + i - j
                    if 0 <= tap < lh:
                        H[i, j] = h[tap]
            y[n * lb:(n + 1) * lb] += H @ xp[(n - kk) * lb:(n - kk + 1) * lb]
    return y[:L]


@pytest.mark.parametrize("L,lh,lb", [(6, 4, 3), (50, 7, 16), (37, 12, 5), (64, 33, 8), (100, 128, 32), (45, 9, 8)])
def test_block_convolution_identity(L, lh, lb):
    r = rng(L + lh + lb)
    x, h = r.standard_normal(L), r.standard_normal(lh)
    ref = oracle.causal_conv(x.reshape(1, L, 1), h.reshape(1, lh))[0, :, 0]
    np.testing.assert_allclose(blocked_conv(x, h, lb), ref, rtol=0, atol=1e-12)


def test_two_stage_needs_filter_length_at_most_block_plus_one():
    """With l_h = l_b + 2 a third factor H_2 is non-zero, so H_0, H_1 alone fall short; with
    l_h = l_b + 1 they suffice (the worked example sits exactly there)."""
    r = rng(11)
    L, lb = 40, 8
    x = r.standard_normal(L)
    for lh, ok in ((lb + 1, True), (lb + 2, False)):
        h = r.standard_normal(lh)
        ref = oracle.causal_conv(x.reshape(1, L, 1), h.reshape(1, lh))[0, :, 0]
        two = blocked_conv(x, h, lb, n_blocks=1)
        assert np.allclose(two, ref, atol=1e-12) == ok


# ------------------------------------------------------------------------------------------ chain
def test_chain_equals_composition_and_single_long_filter():
    r = rng(12)
    B, L, D, lf, lh, dg = 2, 80, 8, 7, 20, 4
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    hq, hk, hv = (r.standard_normal((D, lf)) for _ in range(3))
    h = r.standard_normal((D // dg, lh))
    y = oracle.chain(q, k, v, hq, hk, hv, h, group=dg)
    # by hand with numpy.convolve
    for c in (0, 5, 7):
        qf = np.convolve(q[1, :, c], hq[c])[:L]
        kf = np.convolve(k[1, :, c], hk[c])[:L]
        vf = np.convolve(v[1, :, c], hv[c])[:L]
        ref = qf * np.convolve(kf * vf, h[c // dg])[:L]
        np.testing.assert_allclose(y[1, :, c], ref, rtol=0, atol=1e-11)
    # gating-free path: featurizer followed by the inner conv is one conv with h_G * h_f
    one = np.ones((B, L, D))
    delta = np.zeros((D, lf))
    delta[:, 0] = 1.0
    z = oracle.chain(one, one, v, delta, delta, hv, np.repeat(h, dg, axis=0), group=1)
    for c in range(D):
        hh = np.convolve(h[c // dg], hv[c])
        ref = np.convolve(v[0, :, c], hh)[:L]
        np.testing.assert_allclose(z[0, :, c], ref, rtol=0, atol=1e-11)


def test_point_evaluators_agree_with_full_tensors():
    r = rng(13)
    B, L, D, lf, lh, dg = 2, 40, 8, 7, 12, 4
    q, k, v = (r.standard_normal((B, L, D)) for _ in range(3))
    hq, hk, hv = (r.standard_normal((D, lf)) for _ in range(3))
    h = r.standard_normal((D // dg, lh))
    pts = np.array([(b, t, c) for b in range(B) for t in (0, 1, 6, 11, 12, 39) for c in (0, 3, 4, 7)])
    y = oracle.gated_conv(q, k, v, h, group=dg)
    np.testing.assert_allclose(oracle.gated_conv_points(q, k, v, h, pts, group=dg),
                               y[pts[:, 0], pts[:, 1], pts[:, 2]], rtol=0, atol=1e-13)
    yc = oracle.chain(q, k, v, hq, hk, hv, h, group=dg)
    np.testing.assert_allclose(oracle.chain_points(q, k, v, hq, hk, hv, h, pts, group=dg),
                               yc[pts[:, 0], pts[:, 1], pts[:, 2]], rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------- storage dtypes, API
def test_bf16_and_fp32_inputs_are_widened_exactly():
    r = rng(14)
    B, L, D, lh = 1, 33, 4, 7
    q32, k32, v32 = (torch.from_numpy(r.standard_normal((B, L, D)).astype(np.float32)) for _ in range(3))
    h = r.standard_normal((D, lh)).astype(np.float32)
    qb, kb, vb = (t.to(torch.bfloat16) for t in (q32, k32, v32))
    y_b = oracle.gated_conv(qb, kb, vb, h)
    y_d = oracle.gated_conv(qb.double().numpy(), kb.double().numpy(), vb.double().numpy(), h.astype(np.float64))
    assert np.array_equal(y_b, y_d)
    y_f = oracle.gated_conv(q32, k32, v32, h)
    y_fd = oracle.gated_conv(q32.double().numpy(), k32.double().numpy(), v32.double().numpy(), h.astype(np.float64))
    assert np.array_equal(y_f, y_fd)
    # known bit patterns: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3E80 = 0.25
    bits = np.array([0x3F80, 0xC000, 0x3E80], dtype=np.uint16).reshape(1, 3, 1)
    z = oracle.causal_conv(bits, np.ones((1, 1)))
    assert z[0, :, 0].tolist() == [1.0, -2.0, 0.25]


def test_argument_errors():
    x = np.zeros((1, 4, 6))
    with pytest.raises(ValueError):
        oracle.gated_conv(x, x, x, np.zeros((2, 3)), group=4)  # 6 % 4 != 0
    with pytest.raises(ValueError):
        oracle.gated_conv(x, x, x, np.zeros((3, 3)), group=3)  # wrong number of filters
    with pytest.raises(ValueError):
        oracle.gated_conv(x, x, x[:, :3], np.zeros((6, 3)))
    with pytest.raises(ValueError):
        oracle.gated_conv_points(x, x, x, np.zeros((6, 3)), [(0, 4, 0)])
    with pytest.raises(TypeError):
        oracle.gated_conv(x, x.astype(np.float32), x, np.zeros((6, 3)))


def test_empty_and_short_sequences():
    h = rng(15).standard_normal((2, 5))
    assert oracle.gated_conv(*(np.zeros((0, 3, 2)),) * 3, h).shape == (0, 3, 2)
    r = rng(16)
    q, k, v = (r.standard_normal((1, 2, 2)) for _ in range(3))  # L < l_h
    y = oracle.gated_conv(q, k, v, h)
    u = k * v
    ref0 = q[0, 0] * h[:, 0] * u[0, 0]
    ref1 = q[0, 1] * (h[:, 0] * u[0, 1] + h[:, 1] * u[0, 0])
    np.testing.assert_allclose(y[0, 0], ref0, rtol=1e-14)
    np.testing.assert_allclose(y[0, 1], ref1, rtol=1e-14)
