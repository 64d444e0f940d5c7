"""hyena_li_fwd_static: the Hyena-LI forward whose scan scratch is a static buffer inside the library, for callers
that cannot allocate.  Called through the C ABI on caller-provided inputs and outputs and compared with
hyena_li_fwd (bit for bit: same kernels) and with the oracle, on two calls in a row, the second smaller, so that
whatever the first call left in the shared buffer must not leak into the second."""
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


def draw(seed, B, L, D, order, group):
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v = (synth.normal_tensor(rng, (B, L, D), "bf16") for _ in range(3))
    R, lam = synth.li_params(rng, D // group, order)
    return q, k, v, R, lam


def call_static(lib, t, y, B, L, D, order, group):
    """The raw C-ABI call: device pointers and sizes only, output buffer allocated by the caller beforehand."""
    stream = torch.cuda.current_stream().cuda_stream
    return lib.hyena_li_fwd_static(t["q"].data_ptr(), t["k"].data_ptr(), t["v"].data_ptr(), t["R"].data_ptr(),
                                   t["lam"].data_ptr(), y.data_ptr(), B, L, D, order, group, binding.HY_BF16, stream)


def test_static_scratch_calls_match_the_workspace_entry_point_twice_in_a_row():
    lib = binding.lib()
    # first call: 3 sequences x 8 tiles (the scan's first pass leaves 21 x 16 records of end states in the buffer);
    # second call: smaller in every dimension, 2 sequences x 4 tiles, so it overwrites only part of those records
    shapes = [(3, 2000, 256, 16, 16, 256), (2, 900, 128, 7, 32, 256)]
    outs = []
    for i, (B, L, D, order, group, rows) in enumerate(shapes):
        say("hyena_li_fwd_static call %d B=%d L=%d D=%d order=%d group=%d rows=%d" % (i, B, L, D, order, group, rows))
        binding.set_option("mr_rows", rows)
        q, k, v, R, lam = draw(9100 + i, B, L, D, order, group)
        t = dict(q=dev(q), k=dev(k), v=dev(v), R=dev(R), lam=dev(lam))
        assert lib.hyena_li_workspace_bytes(B, L, D, order, group, binding.HY_BF16) > 0   # the scan does use scratch
        y_static = torch.full((B, L, D), float("nan"), dtype=torch.bfloat16, device="cuda:0")
        outs.append((t, y_static, (q, k, v, R, lam), (B, L, D, order, group)))
    torch.cuda.synchronize()
    # the two calls back to back on one stream, nothing in between
    for (t, y_static, _, (B, L, D, order, group)), (_, _, _, _, _, rows) in zip(outs, shapes):
        binding.set_option("mr_rows", rows)
        rc = call_static(lib, t, y_static, B, L, D, order, group)
        assert rc == 0, binding.status_string(rc)
    torch.cuda.synchronize()
    for (t, y_static, (q, k, v, R, lam), (B, L, D, order, group)), (_, _, _, _, _, rows) in zip(outs, shapes):
        binding.set_option("mr_rows", rows)
        y_ws = binding.hyena_li_fwd(t["q"], t["k"], t["v"], t["R"], t["lam"], group)
        torch.cuda.synchronize()
        assert torch.equal(y_static, y_ws)
        ref = oracle.li_conv(q, k, v, R, lam, group=group)
        got = host(y_static)
        assert np.isfinite(got).all()
        assert oracle.rel_err(got, ref) <= TOL["bf16"]


def test_static_scratch_serves_the_general_recurrence_and_single_tiles_too():
    """Shapes whose scan needs no scratch (one tile per sequence; fp32 and small groups on the plain recurrence)."""
    for seed, (B, L, D, order, group, dtype) in enumerate([(1, 300, 64, 16, 16, "bf16"), (2, 257, 48, 7, 8, "bf16"),
                                                            (1, 200, 32, 4, 16, "f32")]):
        say("hyena_li_fwd_static no-scratch B=%d L=%d D=%d order=%d group=%d %s" % (B, L, D, order, group, dtype))
        rng = np.random.Generator(np.random.PCG64(9200 + seed))
        q, k, v = (synth.normal_tensor(rng, (B, L, D), dtype) for _ in range(3))
        R, lam = synth.li_params(rng, D // group, order)
        y = host(binding.hyena_li_fwd_static(dev(q), dev(k), dev(v), dev(R), dev(lam), group))
        assert oracle.rel_err(y, oracle.li_conv(q, k, v, R, lam, group=group)) <= TOL[dtype]


def test_static_scratch_refuses_a_scan_that_does_not_fit():
    B, L, D, order, group = 1, 1 << 16, 512, 16, 16
    binding.set_option("mr_rows", 32)
    assert binding.lib().hyena_li_workspace_bytes(B, L, D, order, group, binding.HY_BF16) > 4 * 1024 * 1024
    q, k, v, R, lam = draw(9300, B, L, D, order, group)
    with pytest.raises(binding.HyenaError) as e:
        binding.hyena_li_fwd_static(dev(q), dev(k), dev(v), dev(R), dev(lam), group)
    assert e.value.code == 7
