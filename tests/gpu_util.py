"""Shared helpers of the GPU parity tests: draw a case, run it through the C ABI, compare to the oracle."""
import sys

import numpy as np
import torch

import oracle
from paper_2503_01868_amd import binding, synth

TOL = {"f32": 1e-5, "bf16": 2e-2}  # max|y - y_ref| / max|y_ref|, the acceptance bar


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def draw(seed, B, L, D, lh, group, dtype, kind="se"):
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
    n = D // group
    h = synth.short_filter(rng, n, lh) if kind == "se" else synth.decay_filter(rng, n, lh)
    return q, k, v, h


def dev(x):
    if isinstance(x, np.ndarray):
        x = torch.from_numpy(x)
    return x.to("cuda:0")


def host(y):
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


def gated(entry, q, k, v, h, group):
    fn = getattr(binding, entry)
    return fn(dev(q), dev(k), dev(v), dev(h), group)


def check_gated(entry, seed, B, L, D, lh, group, dtype, kind="se", tol=None):
    say("%s seed=%d B=%d L=%d D=%d lh=%d group=%d dtype=%s" % (entry, seed, B, L, D, lh, group, dtype))
    q, k, v, h = draw(seed, B, L, D, lh, group, dtype, kind)
    y = host(gated(entry, q, k, v, h, group))
    ref = oracle.gated_conv(q, k, v, h, group=group)
    err = oracle.rel_err(y, ref)
    assert np.isfinite(y).all()
    assert err <= (TOL[dtype] if tol is None else tol), err
    return err
