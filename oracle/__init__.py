"""TEST INFRASTRUCTURE: Python face of the fp64 CPU parity oracle (``hyena_oracle.c``).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It imports nothing from the HIP package and shares no code with it.

What it computes (paper Sec. 2.1 Eq. 1, Sec. 2.2 filter grouping, Sec. 3.1 Eq. 2):
``y[b,t,c] = q[b,t,c] * sum_{j<l_h, j<=t} h[c // d_g, j] * k[b,t-j,c] * v[b,t-j,c]`` in fp64, inputs
widened exactly from the bits handed over (fp64, fp32 or bf16).  For Hyena-LI (Sec. 2.1) the filter is the sum
of real exponentials ``h[g, j] = sum_n R[g, n] lam[g, n]^j``, materialised over the whole sequence and fed to the
same direct convolution (``li_filter``, ``li_conv``): the definition, not the recurrence and not an FFT.
``li_recurrent`` is the same sum with its two summations exchanged (the recurrent form Sec. 2.1 mentions), linear
in the sequence length, for sequences the quadratic definition cannot cover in full; it is pinned to ``li_conv``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

import hashlib

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hyena_oracle.c")

# -O3 -march=native: the oracle doubles as the CPU baseline of bench.py and is built for the host it runs on.
# -ffp-contract=off keeps every multiply and add of the C source a separately rounded fp64 operation (no fused
# multiply-add is formed), so the arithmetic is the written sum on any host.
CFLAGS = ["-O3", "-march=native", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]

F64, F32, BF16 = 0, 1, 2


def _host_tag() -> str:
    """A short tag of this host's CPU feature flags: code built with -march=native must not be carried to a
    host with another instruction set, so every distinct CPU gets a library of its own."""
    flags = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    flags = " ".join(sorted(line.split(":", 1)[1].split()))
                    break
    except OSError:
        pass
    return hashlib.sha1(flags.encode()).hexdigest()[:10]


_SO = os.path.join(_HERE, "liboracle_%s.so" % _host_tag())


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (+OpenMP) next to its source; returns the .so path."""
    stale = not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + ".%d.tmp" % os.getpid()
        subprocess.check_call(["gcc"] + CFLAGS + ["-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_num_threads.restype = ci
        lib.oracle_causal_conv.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, ci, ci]
        lib.oracle_gated_conv.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, ci]
        lib.oracle_gated_conv_points.argtypes = [vp, vp, vp, vp, vp, i64, vp] + [i64] * 5 + [ci, ci]
        lib.oracle_chain_points.argtypes = [vp] * 8 + [i64, vp] + [i64] * 7 + [ci, ci]
        lib.oracle_gated_conv_bwd.argtypes = [vp] * 9 + [i64] * 5 + [ci, ci]
        lib.oracle_causal_conv_bwd.argtypes = [vp] * 5 + [i64] * 5 + [ci, ci]
        lib.oracle_li_recurrent.argtypes = [vp] * 7 + [i64] * 5 + [ci, ci]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _arr(x):
    """Return (contiguous numpy array, dtype code) holding exactly the bits of ``x``.

    Accepts numpy float64/float32 arrays, numpy uint16 arrays (taken as bf16 bit patterns) and CPU
    torch tensors of dtype float64/float32/bfloat16.
    """
    if not isinstance(x, np.ndarray):
        import torch

        if not isinstance(x, torch.Tensor):
            raise TypeError("oracle input must be a numpy array or a CPU torch tensor")
        if x.device.type != "cpu":
            raise ValueError("oracle inputs live on the host")
        x = x.contiguous()
        if x.dtype == torch.bfloat16:
            x = x.view(torch.int16).numpy().view(np.uint16)
        elif x.dtype in (torch.float32, torch.float64):
            x = x.numpy()
        else:
            raise TypeError("unsupported tensor dtype %s" % x.dtype)
    x = np.ascontiguousarray(x)
    if x.dtype == np.float64:
        return x, F64
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:
        return x, BF16
    raise TypeError("unsupported array dtype %s" % x.dtype)


def _same(*codes):
    if len(set(codes)) != 1:
        raise TypeError("activation arrays must share one dtype")
    return codes[0]


def _filt(h, n_filters, lh=None):
    h = np.ascontiguousarray(h)
    if h.dtype not in (np.float64, np.float32):
        raise TypeError("filters are float32 or float64")
    if h.ndim != 2 or h.shape[0] != n_filters or (lh is not None and h.shape[1] != lh):
        raise ValueError("filter array must be [D // group, l_h]; got %s" % (h.shape,))
    return h, (F64 if h.dtype == np.float64 else F32)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _ok(rc, what):
    if rc != 0:
        raise ValueError("%s rejected its arguments (code %d)" % (what, rc))


def causal_conv(x, h, group: int = 1) -> np.ndarray:
    """Featurizer convolution (Eq. 1 lines 1-3 with Eq. 2): y = h * x per channel, no gating."""
    xa, xd = _arr(x)
    B, L, D = xa.shape
    ha, hd = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    y = np.empty((B, L, D), dtype=np.float64)
    _ok(_load().oracle_causal_conv(_ptr(xa), _ptr(ha), _ptr(y), B, L, D, ha.shape[1], group, xd, hd),
        "oracle_causal_conv")
    return y


def gated_conv(q, k, v, h, group: int = 1) -> np.ndarray:
    """Hyena-SE / Hyena-MR inner operator: y = q (.) (h * (k (.) v)) (Eq. 1 last line, Eq. 2)."""
    qa, qd = _arr(q)
    ka, kd = _arr(k)
    va, vd = _arr(v)
    xd = _same(qd, kd, vd)
    if not (qa.shape == ka.shape == va.shape) or qa.ndim != 3:
        raise ValueError("q, k, v must share one [B, L, D] shape")
    B, L, D = qa.shape
    ha, hd = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    y = np.empty((B, L, D), dtype=np.float64)
    _ok(_load().oracle_gated_conv(_ptr(qa), _ptr(ka), _ptr(va), _ptr(ha), _ptr(y), B, L, D,
                                  ha.shape[1], group, xd, hd), "oracle_gated_conv")
    return y


def _points(pts, n_dims=3):
    p = np.ascontiguousarray(np.asarray(pts, dtype=np.int64))
    if p.ndim != 2 or p.shape[1] != n_dims:
        raise ValueError("points are an [n, 3] array of (b, t, c)")
    return p


def gated_conv_points(q, k, v, h, pts, group: int = 1) -> np.ndarray:
    """``gated_conv`` evaluated only at the listed (b, t, c) outputs."""
    qa, qd = _arr(q)
    ka, kd = _arr(k)
    va, vd = _arr(v)
    xd = _same(qd, kd, vd)
    B, L, D = qa.shape
    ha, hd = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    p = _points(pts)
    out = np.empty(p.shape[0], dtype=np.float64)
    _ok(_load().oracle_gated_conv_points(_ptr(qa), _ptr(ka), _ptr(va), _ptr(ha), _ptr(p), p.shape[0],
                                         _ptr(out), B, L, D, ha.shape[1], group, xd, hd),
        "oracle_gated_conv_points")
    return out


def chain(q, k, v, hq, hk, hv, h, group: int = 1, feat_group: int = 1) -> np.ndarray:
    """Operator chain of Eq. 1 minus the dense projections: featurize q, k, v, then the gated inner
    convolution; intermediates stay in fp64 (composition of the two functions above)."""
    qf = causal_conv(q, hq, feat_group)
    kf = causal_conv(k, hk, feat_group)
    vf = causal_conv(v, hv, feat_group)
    return gated_conv(qf, kf, vf, h, group)


def chain_points(q, k, v, hq, hk, hv, h, pts, group: int = 1, feat_group: int = 1) -> np.ndarray:
    """``chain`` evaluated only at the listed (b, t, c) outputs (nested sums written out in C)."""
    qa, qd = _arr(q)
    ka, kd = _arr(k)
    va, vd = _arr(v)
    xd = _same(qd, kd, vd)
    B, L, D = qa.shape
    nf = D // feat_group if feat_group > 0 and D % feat_group == 0 else -1
    hqa, d1 = _filt(hq, nf)
    hka, d2 = _filt(hk, nf, hqa.shape[1])
    hva, d3 = _filt(hv, nf, hqa.shape[1])
    ha, d4 = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    hd = _same(d1, d2, d3, d4)
    p = _points(pts)
    out = np.empty(p.shape[0], dtype=np.float64)
    _ok(_load().oracle_chain_points(_ptr(qa), _ptr(ka), _ptr(va), _ptr(hqa), _ptr(hka), _ptr(hva),
                                    _ptr(ha), _ptr(p), p.shape[0], _ptr(out), B, L, D, hqa.shape[1],
                                    feat_group, ha.shape[1], group, xd, hd), "oracle_chain_points")
    return out


def gated_conv_bwd(dy, q, k, v, h, group: int = 1):
    """Gradients of ``gated_conv`` w.r.t. q, k, v (each [B, L, D]) and h ([D // group, l_h]) given dy: the
    chain rule of Eq. 1 / Eq. 2 written out in fp64.  Returns (dq, dk, dv, dh)."""
    ga, gd = _arr(dy)
    qa, qd = _arr(q)
    ka, kd = _arr(k)
    va, vd = _arr(v)
    xd = _same(gd, qd, kd, vd)
    if not (ga.shape == qa.shape == ka.shape == va.shape) or qa.ndim != 3:
        raise ValueError("dy, q, k, v must share one [B, L, D] shape")
    B, L, D = qa.shape
    ha, hd = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    dq, dk, dv = (np.empty((B, L, D), dtype=np.float64) for _ in range(3))
    dh = np.empty(ha.shape, dtype=np.float64)
    _ok(_load().oracle_gated_conv_bwd(_ptr(ga), _ptr(qa), _ptr(ka), _ptr(va), _ptr(ha), _ptr(dq), _ptr(dk), _ptr(dv),
                                      _ptr(dh), B, L, D, ha.shape[1], group, xd, hd), "oracle_gated_conv_bwd")
    return dq, dk, dv, dh


def causal_conv_bwd(dy, x, h, group: int = 1):
    """Gradients of ``causal_conv`` (the featurizers of Eq. 1) w.r.t. x ([B, L, D]) and h ([D // group, l_h]) given
    dy: the chain rule of Eq. 2 written out in fp64.  Returns (dx, dh)."""
    ga, gd = _arr(dy)
    xa, xd = _arr(x)
    cd = _same(gd, xd)
    if ga.shape != xa.shape or xa.ndim != 3:
        raise ValueError("dy and x must share one [B, L, D] shape")
    B, L, D = xa.shape
    ha, hd = _filt(h, D // group if group > 0 and D % group == 0 else -1)
    dx = np.empty((B, L, D), dtype=np.float64)
    dh = np.empty(ha.shape, dtype=np.float64)
    _ok(_load().oracle_causal_conv_bwd(_ptr(ga), _ptr(xa), _ptr(ha), _ptr(dx), _ptr(dh), B, L, D, ha.shape[1], group,
                                       cd, hd), "oracle_causal_conv_bwd")
    return dx, dh


def chain_bwd(dy, q, k, v, hq, hk, hv, h, group: int = 1, feat_group: int = 1):
    """Gradients of ``chain`` w.r.t. q, k, v and the four filters given dy: the chain rule of Eq. 1 through the two
    backward functions above, intermediates in fp64.  Returns (dq, dk, dv, dhq, dhk, dhv, dh)."""
    qf = causal_conv(q, hq, feat_group)
    kf = causal_conv(k, hk, feat_group)
    vf = causal_conv(v, hv, feat_group)
    dqf, dkf, dvf, dh = gated_conv_bwd(_wide(dy), qf, kf, vf, h, group)
    dq, dhq = causal_conv_bwd(dqf, _wide(q), hq, feat_group)
    dk, dhk = causal_conv_bwd(dkf, _wide(k), hk, feat_group)
    dv, dhv = causal_conv_bwd(dvf, _wide(v), hv, feat_group)
    return dq, dk, dv, dhq, dhk, dhv, dh


def li_filter(R, lam, L: int) -> np.ndarray:
    """Hyena-LI inner filter (Sec. 2.1, "long implicit"): a sum of real exponentials per filter group,
    ``h[g, j] = sum_n R[g, n] * lam[g, n] ** j`` for j = 0 .. L-1, i.e. the paper's ``h_t = sum_n R_n lambda_n^(t-1)``
    with t counted from 1, so tap 0 is ``sum_n R_n`` (0 ** 0 = 1).  R, lam: [G, d]; returns fp64 [G, L]."""
    R = np.asarray(R, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    if R.ndim != 2 or R.shape != lam.shape:
        raise ValueError("R and lam must share one [G, d] shape")
    j = np.arange(int(L), dtype=np.int64)
    h = np.zeros((R.shape[0], int(L)), dtype=np.float64)
    for n in range(R.shape[1]):  # one exponential at a time: [G, L] temporaries only
        h += R[:, n, None] * np.power(lam[:, n, None], j[None, :])
    return h


def _wide(x) -> np.ndarray:
    """The values of ``x`` in fp64, widened exactly from its stored bits (bf16 bit patterns become the fp32 with
    the same upper half)."""
    a, code = _arr(x)
    if code == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def li_state(k, v, lam, group: int = 1) -> np.ndarray:
    """Running sums of the Hyena-LI recurrent form (Sec. 2.1) after the last step of the sequence:
    ``s[b, c, n] = sum_{i=0}^{L-1} lam[c // group, n] ** (L - 1 - i) * k[b, i, c] * v[b, i, c]``: what a sequence cut
    after step L - 1 hands to its continuation.  fp64 [B, D, d]."""
    ka, va = _wide(k), _wide(v)
    lam = np.asarray(lam, dtype=np.float64)
    if ka.shape != va.shape or ka.ndim != 3 or lam.ndim != 2:
        raise ValueError("k, v must share one [B, L, D] shape and lam be [G, d]")
    B, L, D = ka.shape
    if group < 1 or D % group != 0 or lam.shape[0] != D // group:
        raise ValueError("lam must have one row per group of channels")
    u = ka * va
    e = np.arange(L - 1, -1, -1, dtype=np.int64)  # exponent of step i
    out = np.empty((B, D, lam.shape[1]), dtype=np.float64)
    for n in range(lam.shape[1]):  # one exponential at a time: [L, D] temporaries only
        w = np.power(np.repeat(lam[:, n], group)[None, :], e[:, None])  # [L, D]
        out[:, :, n] = np.einsum("bld,ld->bd", u, w)
    return out


def li_conv(q, k, v, R, lam, group: int = 1) -> np.ndarray:
    """Hyena-LI inner operator: ``gated_conv`` with the filter of ``li_filter`` as long as the sequence."""
    return gated_conv(q, k, v, li_filter(R, lam, int(q.shape[1])), group=group)


def li_conv_points(q, k, v, R, lam, pts, group: int = 1) -> np.ndarray:
    """``li_conv`` evaluated only at the listed (b, t, c) outputs."""
    return gated_conv_points(q, k, v, li_filter(R, lam, int(q.shape[1])), pts, group=group)


def li_recurrent(q, k, v, R, lam, group: int = 1) -> np.ndarray:
    """Hyena-LI inner operator through its recurrent form (``s_n[t] = lam_n s_n[t-1] + k[t] v[t]``,
    ``y[t] = q[t] sum_n R_n s_n[t]``): the sum of ``li_conv`` with the order of summation exchanged."""
    qa, qd = _arr(q)
    ka, kd = _arr(k)
    va, vd = _arr(v)
    xd = _same(qd, kd, vd)
    if not (qa.shape == ka.shape == va.shape) or qa.ndim != 3:
        raise ValueError("q, k, v must share one [B, L, D] shape")
    B, L, D = qa.shape
    Ra, rd = _filt(R, D // group if group > 0 and D % group == 0 else -1)
    la, ld = _filt(lam, Ra.shape[0], Ra.shape[1])
    hd = _same(rd, ld)
    y = np.empty((B, L, D), dtype=np.float64)
    state = np.empty(B * D * Ra.shape[1], dtype=np.float64)
    _ok(_load().oracle_li_recurrent(_ptr(qa), _ptr(ka), _ptr(va), _ptr(Ra), _ptr(la), _ptr(y), _ptr(state), B, L, D,
                                    Ra.shape[1], group, xd, hd), "oracle_li_recurrent")
    return y


def rel_err(y, y_ref) -> float:
    """Acceptance metric: max|y - y_ref| / max|y_ref| over the whole tensor."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    den = float(np.max(np.abs(y_ref))) if y_ref.size else 0.0
    num = float(np.max(np.abs(y - y_ref))) if y_ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
