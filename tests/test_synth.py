"""The seeded input generators: reproducible, right shapes and distributions, no hidden arithmetic."""
import numpy as np
import torch

from paper_2503_01868_amd import synth


def test_five_configs_as_named():
    c = synth.CONFIGS
    assert list(c)[:5] == ["c0", "c1", "c2", "c3", "c4"]  # the five named configurations keep their seeds
    assert {k: v for k, v in c["c2u"].items() if k != "group"} == {k: v for k, v in c["c2"].items() if k != "group"}
    assert c["c2u"]["group"] == 1
    assert (c["c0"]["B"], c["c0"]["L"], c["c0"]["D"], c["c0"]["lh"], c["c0"]["dtype"]) == (1, 1024, 256, 7, "f32")
    assert (c["c1"]["L"], c["c1"]["D"], c["c1"]["lh"], c["c1"]["group"], c["c1"]["dtype"]) == (8192, 4096, 7, 1, "bf16")
    assert (c["c2"]["L"], c["c2"]["D"], c["c2"]["lh"], c["c2"]["group"]) == (8192, 4096, 128, 16)
    assert (c["c3"]["L"], c["c3"]["lh"], c["c3"]["group"]) == (131072, 128, 16)
    assert (c["c4"]["B"], c["c4"]["L"], c["c4"]["lf"], c["c4"]["lh"]) == (4, 32768, 7, 128)


def test_reproducible_and_seed_dependent():
    a = synth.make("c0")
    b = synth.make("c0")
    c = synth.make("c0", variant=1)
    for key in ("q", "k", "v"):
        assert torch.equal(a[key], b[key]) and not torch.equal(a[key], c[key])
    assert np.array_equal(a["h"], b["h"])


def test_distributions():
    w = synth.make("c2", L=256, D=1024)
    assert w["q"].dtype == torch.bfloat16 and w["q"].shape == (1, 256, 1024)
    q = w["q"].float().numpy()
    assert abs(q.mean()) < 0.02 and abs(q.std() - 1.0) < 0.02
    h = w["h"]
    assert h.shape == (64, 128) and h.dtype == np.float32
    # tap 0 is undecayed: variance 1/l_h; late taps are damped by at least exp(-0.01*j)
    assert abs(h[:, 0].std() * np.sqrt(128) - 1.0) < 0.3
    assert np.abs(h[:, 120:]).mean() < np.abs(h[:, :8]).mean() * np.exp(-0.01 * 112) * 1.5
    s = synth.make("c1", L=64, D=2048)
    assert abs(s["h"].std() * np.sqrt(7) - 1.0) < 0.05
    ch = synth.make("c4", B=1, L=32, D=64)
    assert ch["hq"].shape == (64, 7) and not np.array_equal(ch["hq"], ch["hk"])


def test_sample_points_cover_the_edges():
    pts = synth.sample_points(1, B=2, L=100, D=32, n=50, lh=7)
    assert pts.shape[1] == 3 and len(pts) > 50
    assert pts[:, 0].max() < 2 and pts[:, 1].max() < 100 and pts[:, 2].max() < 32
    have = {tuple(p) for p in pts.tolist()}
    for need in [(0, 0, 0), (1, 99, 31), (0, 6, 0), (1, 5, 31)]:
        assert need in have
