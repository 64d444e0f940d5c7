"""The pins must notice a plausible mistake anywhere in the oracle.  Each case below plants one mistake in a
COPY of the oracle's C source (on the CPU, in a temporary directory), builds it, and checks that at least one
of the independent references used by the pin tests (numpy.convolve / numpy.correlate, finite differences)
disagrees with the mutant, while the unmodified source agrees.  Nothing here touches the GPU."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle

SRC = os.path.join(os.path.dirname(oracle.__file__), "hyena_oracle.c")

# (what is planted, text to replace, replacement, how many occurrences are replaced: 0 = all)
MUTATIONS = [
    ("tap reaches forward instead of back", "(b * L + (t - j)) * D + c", "(b * L + (t + j < L ? t + j : t)) * D + c", 0),
    ("channel-major filter index", "(size_t)(g * lh + j)", "(size_t)(j * (D / dg) + g)", 0),
    ("groups interleaved instead of contiguous", "int64_t g = c / dg;", "int64_t g = c % (D / dg);", 0),
    ("pre-gate is a sum", "orc_load(k, x_dtype, src) * orc_load(v, x_dtype, src)", "orc_load(k, x_dtype, src) + orc_load(v, x_dtype, src)", 0),
    ("post-gate dropped", "y[dst] = orc_load(q, x_dtype, dst) * z;", "y[dst] = z;", 1),
    ("post-gate taken at the source step", "y[dst] = orc_load(q, x_dtype, dst) * z;", "y[dst] = orc_load(q, x_dtype, (size_t)((b * L + (t > 0 ? t - 1 : 0)) * D + c)) * z;", 1),
    ("one tap short", "j < lh && j <= t", "j < lh - 1 && j <= t", 0),
    ("left boundary leaks one step", "j < lh && j <= t", "j < lh && j <= t + 1 && (b * L + t - j) >= 0", 0),
    ("no batch isolation", "int64_t b = r / L, t = r % L;", "int64_t b = 0, t = r;", 0),
    ("du reaches back instead of forward", "(b * L + (t + j)) * D + c", "(b * L + (t - j >= 0 ? t - j : t)) * D + c", 0),
    ("dk and dv swapped", "dk[at] = du * orc_load(v, x_dtype, at);", "dk[at] = du * orc_load(k, x_dtype, at);", 1),
    ("dh lag sign", "size_t src = (size_t)((b * L + (t - j)) * D + c);\n                        s +=", "size_t src = (size_t)((b * L + (t - j)) * D + c); src = (size_t)((b * L + (L - 1 - t + j)) * D + c);\n                        s +=", 1),
    ("dq misses the upstream gradient", "dq[at] = orc_load(dy, x_dtype, at) * z;", "dq[at] = z;", 1),
    ("featurizer dx reaches back instead of forward", "(b * L + (s + j)) * D + c", "(b * L + (s - j >= 0 ? s - j : s)) * D + c", 1),
    ("featurizer dx one tap short", "j < lh && s + j < L", "j < lh - 1 && s + j < L", 1),
    ("featurizer dx clipped at the sequence start like the forward", "j < lh && s + j < L; ++j)", "j < lh && s + j < L && j <= s; ++j)", 1),
    ("featurizer dh starts at lag 0 rows", "for (int64_t t = j; t < L; ++t)\n                        acc +=", "for (int64_t t = j + 1; t < L; ++t)\n                        acc +=", 1),
    ("featurizer dh forgets the group's channels", "for (int64_t c = g * dg; c < (g + 1) * dg; ++c)\n                    for (int64_t t = j; t < L; ++t)\n                        acc +=", "for (int64_t c = g * dg; c < g * dg + 1; ++c)\n                    for (int64_t t = j; t < L; ++t)\n                        acc +=", 1),
]


def build(src_text, tmp_path, tag):
    c = tmp_path / ("m_%s.c" % tag)
    so = tmp_path / ("m_%s.so" % tag)
    c.write_text(src_text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c)])
    lib = ctypes.CDLL(str(so))
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.oracle_gated_conv.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, ci]
    lib.oracle_gated_conv_bwd.argtypes = [vp] * 9 + [i64] * 5 + [ci, ci]
    lib.oracle_causal_conv_bwd.argtypes = [vp] * 5 + [i64] * 5 + [ci, ci]
    return lib


def ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def disagreements(lib):
    """Number of independent reference checks the library fails (forward vs numpy.convolve; backward vs
    numpy.convolve / numpy.correlate on the reversed signals).  The shape has L not a multiple of anything,
    two batch items and groups of 2 so that index mix-ups show."""
    r = np.random.default_rng(5)
    B, L, D, lh, dg = 2, 23, 6, 5, 2
    q, k, v, dy = (np.ascontiguousarray(r.standard_normal((B, L, D))) for _ in range(4))
    h = np.ascontiguousarray(r.standard_normal((D // dg, lh)))
    bad = 0
    y = np.empty((B, L, D))
    assert lib.oracle_gated_conv(ptr(q), ptr(k), ptr(v), ptr(h), ptr(y), B, L, D, lh, dg, 0, 0) == 0
    dq, dk, dv = (np.empty((B, L, D)) for _ in range(3))
    dh = np.empty((D // dg, lh))
    assert lib.oracle_gated_conv_bwd(ptr(dy), ptr(q), ptr(k), ptr(v), ptr(h), ptr(dq), ptr(dk), ptr(dv), ptr(dh),
                                     B, L, D, lh, dg, 0, 0) == 0
    dh_ref = np.zeros_like(dh)
    for b in range(B):
        for c in range(D):
            u, g, hh = k[b, :, c] * v[b, :, c], dy[b, :, c] * q[b, :, c], h[c // dg]
            z = np.convolve(u, hh)[:L]
            du = np.convolve(g[::-1], hh)[:L][::-1]
            bad += not np.allclose(y[b, :, c], q[b, :, c] * z, atol=1e-10)
            bad += not np.allclose(dq[b, :, c], dy[b, :, c] * z, atol=1e-10)
            bad += not np.allclose(dk[b, :, c], du * v[b, :, c], atol=1e-10)
            bad += not np.allclose(dv[b, :, c], du * k[b, :, c], atol=1e-10)
            dh_ref[c // dg] += np.correlate(g, u, mode="full")[L - 1:L - 1 + lh]
    bad += not np.allclose(dh, dh_ref, atol=1e-9)
    # featurizer backward: dx and dh of x -> h * x
    dx = np.empty((B, L, D))
    dhf = np.empty((D // dg, lh))
    assert lib.oracle_causal_conv_bwd(ptr(dy), ptr(k), ptr(h), ptr(dx), ptr(dhf), B, L, D, lh, dg, 0, 0) == 0
    dhf_ref = np.zeros_like(dhf)
    for b in range(B):
        for c in range(D):
            bad += not np.allclose(dx[b, :, c], np.convolve(dy[b, ::-1, c], h[c // dg])[:L][::-1], atol=1e-10)
            dhf_ref[c // dg] += np.correlate(dy[b, :, c], k[b, :, c], mode="full")[L - 1:L - 1 + lh]
    bad += not np.allclose(dhf, dhf_ref, atol=1e-9)
    return bad


def test_unmodified_source_agrees(tmp_path):
    assert disagreements(build(open(SRC).read(), tmp_path, "orig")) == 0


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_planted_mistake_is_caught(idx, tmp_path):
    what, old, new, count = MUTATIONS[idx]
    text = open(SRC).read()
    assert old in text, "mutation target vanished from the oracle source: " + what
    mutated = text.replace(old, new) if count == 0 else text.replace(old, new, count)
    assert mutated != text
    assert disagreements(build(mutated, tmp_path, str(idx))) > 0, what
