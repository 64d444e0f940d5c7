"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2503_01868_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        src = open(os.path.join(ROOT, "include", fn)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(hyena_\w+)\s*\(", src)
    return sorted(set(names))


def test_header_declares_the_three_required_entry_points():
    names = declared_functions()
    for need in ("hyena_se_fwd", "hyena_mr_fwd", "hyena_featurize_fwd"):
        assert need in names


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_exposes_the_same_names():
    import paper_2503_01868_amd as pkg

    for name in ("hyena_se_fwd", "hyena_mr_fwd", "hyena_featurize_fwd", "hyena_featurize3_fwd", "hyena_chain_fwd",
                 "hyena_se_bwd", "hyena_mr_bwd", "hyena_li_fwd", "hyena_li_fwd_static", "hyena_stream_copy"):
        assert callable(getattr(pkg, name))


def test_version_and_status_strings():
    assert binding.version() >= 100
    seen = {binding.status_string(c) for c in range(8)}
    assert len(seen) == 8 and "ok" in seen


# fake but well-formed device addresses: validation must finish before any of them is dereferenced
P = [0x10000 * (i + 1) for i in range(9)]


def conv(entry, q=P[0], k=P[1], v=P[2], h=P[3], y=P[4], B=1, L=8, D=16, lh=3, group=1, dtype=0):
    return getattr(binding.lib(), entry)(q, k, v, h, y, B, L, D, lh, group, dtype, None)


@pytest.mark.parametrize("entry", ["hyena_se_fwd", "hyena_mr_fwd"])
def test_gated_entry_points_reject_bad_arguments(entry):
    assert conv(entry, q=None) == 1
    assert conv(entry, k=None) == 1
    assert conv(entry, v=None) == 1
    assert conv(entry, h=None) == 1
    assert conv(entry, y=None) == 1
    assert conv(entry, B=-1) == 2
    assert conv(entry, L=-5) == 2
    assert conv(entry, lh=0) == 2
    assert conv(entry, group=0) == 2
    assert conv(entry, D=16, group=3) == 2
    assert conv(entry, dtype=7) == 3
    assert conv(entry, q=P[0] + 4) == 4
    assert conv(entry, y=P[4] + 2) == 4
    assert conv(entry, h=P[3] + 8) == 4
    assert conv(entry, y=P[1]) == 4  # output aliases k
    assert conv(entry, y=P[1] + 16) == 4  # partial overlap
    assert conv(entry, h=P[4] + 32) == 4  # the filter table lies inside the output
    assert conv(entry, y=P[3] - 16) == 4  # the output's last bytes run into the filter table
    assert conv(entry, B=1 << 40, L=1 << 40, D=16) == 2  # size overflows 64-bit offsets
    # empty problems are valid and launch nothing
    assert conv(entry, B=0) == 0
    assert conv(entry, L=0) == 0
    assert conv(entry, D=0, group=1) == 0


def test_featurizer_entry_points_reject_bad_arguments():
    lib = binding.lib()
    f = lambda x=P[0], h=P[1], y=P[2], B=1, L=8, D=16, lh=3, group=1, dtype=1: lib.hyena_featurize_fwd(
        x, h, y, B, L, D, lh, group, dtype, None)
    assert f(x=None) == 1 and f(h=None) == 1 and f(y=None) == 1
    assert f(lh=-1) == 2 and f(D=10, group=4) == 2 and f(dtype=2) == 3
    assert f(x=P[0] + 1) == 4 and f(y=P[0]) == 4 and f(L=0) == 0

    def f3(**kw):
        a = dict(q=P[0], k=P[1], v=P[2], hq=P[3], hk=P[4], hv=P[5], qo=P[6], ko=P[7], vo=P[8],
                 B=1, L=8, D=16, lh=3, group=1, dtype=1)
        a.update(kw)
        return lib.hyena_featurize3_fwd(*[a[n] for n in ("q", "k", "v", "hq", "hk", "hv", "qo", "ko", "vo", "B",
                                                            "L", "D", "lh", "group", "dtype")], None)

    assert f3(hv=None) == 1 and f3(vo=None) == 1 and f3(group=5) == 2 and f3(dtype=-1) == 3
    assert f3(ko=P[6]) == 4  # two outputs alias
    assert f3(qo=P[2]) == 4 and f3(B=0) == 0


def test_stream_copy_and_options_reject_bad_arguments():
    lib = binding.lib()
    assert lib.hyena_stream_copy(None, P[1], 16, None) == 1
    assert lib.hyena_stream_copy(P[0], P[1], 24, None) == 2
    assert lib.hyena_stream_copy(P[0], P[0] + 16, 64, None) == 4
    assert lib.hyena_stream_copy(P[0], P[1], 0, None) == 0
    assert lib.hyena_set_option(b"no_such_knob", 1) == 5
    assert lib.hyena_set_option(None, 1) == 1
    assert lib.hyena_set_option(b"se_vec", 3) == 2
    assert lib.hyena_set_option(b"mr_rows", 48) == 2
    assert lib.hyena_set_option(b"se_vec", 0) == 0


def test_bandwidth_yardstick_rejects_bad_arguments():
    lib = binding.lib()
    g = lambda q=P[0], k=P[1], v=P[2], y=P[3], B=1, L=8, D=256, strip=0, rows=0, depth=0, waves=0: lib.hyena_stream_gate(
        q, k, v, y, B, L, D, strip, rows, depth, waves, None)
    assert g(depth=5) == 5 and g(depth=6, strip=64, B=0) == 0 and g(depth=8, strip=256, waves=4, B=0) == 0
    assert g(waves=8) == 5 and g(strip=64, waves=8) == 5 and g(strip=256, waves=12) == 5
    assert g(q=None) == 1 and g(y=None) == 1 and g(L=-1) == 2 and g(D=12) == 2 and g(rows=-1) == 2
    assert g(strip=32) == 5 and g(strip=128, D=192) == 2 and g(y=P[1]) == 4 and g(k=P[1] + 8) == 4
    assert g(B=0) == 0 and g(L=0, strip=256) == 0


def test_binding_refuses_cpu_tensors():
    import torch

    x = torch.zeros(1, 4, 8)
    with pytest.raises(ValueError):
        binding.hyena_se_fwd(x, x, x, torch.zeros(8, 3))


def test_chain_entry_point_rejects_bad_arguments_and_sizes_its_workspace():
    lib = binding.lib()

    def ch(**kw):
        a = dict(q=P[0], k=P[1], v=P[2], hq=P[3], hk=P[4], hv=P[5], h=P[6], y=P[7], ws=P[8], wsb=1 << 20,
                 B=1, L=8, D=128, lf=7, fg=1, lh=128, group=16, dtype=1)
        a.update(kw)
        return lib.hyena_chain_fwd(*[a[n] for n in ("q", "k", "v", "hq", "hk", "hv", "h", "y", "ws", "wsb", "B", "L",
                                                    "D", "lf", "fg", "lh", "group", "dtype")], None)

    assert ch(q=None) == 1 and ch(hv=None) == 1 and ch(h=None) == 1 and ch(y=None) == 1
    assert ch(lf=0) == 2 and ch(fg=3) == 2 and ch(group=24) == 2 and ch(lh=0) == 2 and ch(dtype=9) == 3
    assert ch(y=P[2]) == 4 and ch(hq=P[3] + 4) == 4
    assert ch(B=0) == 0 and ch(L=0, ws=None) == 0
    # problems outside the single-kernel domain need a workspace
    assert ch(dtype=0, ws=None) == 1 and ch(D=64, group=16, ws=None) == 1 and ch(dtype=0, ws=P[8] + 2) == 4
    assert ch(dtype=0, ws=P[0]) == 4  # workspace overlaps an input
    assert ch(dtype=0, wsb=3 * 8 * 128 * 4 - 1) == 2 and ch(wsb=-1) == 2  # workspace too small / negative size
    assert ch(dtype=0, ws=P[4] - 4096) == 4  # workspace runs into a featurizer filter table
    assert ch(h=P[7] + 64) == 4  # inner filter table inside the output
    wb = lib.hyena_chain_workspace_bytes
    assert wb(4, 32768, 4096, 7, 1, 128, 16, 1) == 0
    assert wb(1, 100, 64, 7, 1, 128, 16, 1) == 3 * 100 * 64 * 2
    assert wb(1, 100, 128, 7, 1, 128, 16, 0) == 3 * 100 * 128 * 4
    assert wb(1, 100, 128, 7, 1, 130, 16, 1) == 3 * 100 * 128 * 2
    assert wb(1, 100, 128, 9, 1, 128, 16, 1) == 0   # up to nine taps: single kernel
    assert wb(1, 100, 128, 10, 1, 128, 16, 1) == 3 * 100 * 128 * 2
    assert wb(1, 100, 128, 7, 1, 128, 24, 1) == -1 and wb(1, 100, 128, 0, 1, 128, 16, 1) == -1
    assert wb(0, 100, 128, 7, 1, 128, 16, 0) == 0


def test_backward_entry_points_reject_bad_arguments_and_size_their_workspace():
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(11)]

    def bw(entry="hyena_se_bwd", **kw):
        a = dict(dy=Q[0], q=Q[1], k=Q[2], v=Q[3], h=Q[4], dq=Q[5], dk=Q[6], dv=Q[7], dh=Q[8], ws=Q[9], wsb=1 << 19,
                 B=1, L=8, D=16, lh=3, group=1, dtype=1)
        a.update(kw)
        return getattr(lib, entry)(*[a[n] for n in ("dy", "q", "k", "v", "h", "dq", "dk", "dv", "dh", "ws", "wsb",
                                                    "B", "L", "D", "lh", "group", "dtype")], None)

    for entry in ("hyena_se_bwd", "hyena_mr_bwd"):
        for name in ("dy", "q", "k", "v", "h", "dq", "dk", "dv", "dh"):
            assert bw(entry, **{name: None}) == 1
        assert bw(entry, lh=0) == 2 and bw(entry, group=3) == 2 and bw(entry, dtype=4) == 3 and bw(entry, wsb=-1) == 2
        assert bw(entry, dq=Q[1]) == 4 and bw(entry, dk=Q[5]) == 4 and bw(entry, dh=Q[4]) == 4 and bw(entry, dv=Q[7] + 2) == 4
        assert bw(entry, dh=Q[6] + 64) == 4 and bw(entry, h=Q[5] + 64) == 4  # filter tables inside written tensors
        assert bw(entry, ws=None) == 1 and bw(entry, wsb=16) == 2 and bw(entry, ws=Q[9] + 4) == 4 and bw(entry, ws=Q[0]) == 4
    wb = lib.hyena_bwd_workspace_bytes
    assert wb(1, 8, 16, 3, 1, 1) == 1 * 1 * 16 * 3 * 4        # one tile
    assert wb(2, 1000, 256, 7, 1, 1) % (256 * 7 * 4) == 0 and wb(2, 1000, 256, 7, 1, 1) > 0
    assert wb(1, 100, 64, 128, 16, 1) == 1 * 1 * (64 // 16) * 128 * 4   # matrix-core path: one row per tile and slice
    assert wb(1, 100, 64, 128, 16, 0) == 0 and wb(1, 100, 40, 50, 1, 1) == 0  # general kernel: no workspace
    assert wb(1, 100, 128, 50, 1, 1) == 1 * 1 * 128 * 50 * 4   # chunk-parallel matrix-core path: one row per tile and channel
    assert wb(0, 100, 64, 7, 1, 1) == 0 and wb(1, 100, 64, 0, 1, 1) == -1 and wb(1, 100, 64, 7, 5, 1) == -1


def test_featurizer_backward_rejects_bad_arguments_and_sizes_its_workspace():
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(7)]

    def fb(**kw):
        a = dict(dy=Q[0], x=Q[1], h=Q[2], dx=Q[3], dh=Q[4], ws=Q[5], wsb=1 << 19, B=1, L=8, D=16, lh=3, group=1, dtype=1)
        a.update(kw)
        return lib.hyena_featurize_bwd(*[a[n] for n in ("dy", "x", "h", "dx", "dh", "ws", "wsb", "B", "L", "D", "lh",
                                                        "group", "dtype")], None)

    for name in ("dy", "x", "h", "dx", "dh"):
        assert fb(**{name: None}) == 1
    assert fb(lh=0) == 2 and fb(group=3) == 2 and fb(dtype=4) == 3 and fb(wsb=-1) == 2 and fb(L=-1) == 2
    assert fb(dx=Q[0]) == 4 and fb(dx=Q[1] + 16) == 4 and fb(dh=Q[2]) == 4 and fb(dx=Q[3] + 2) == 4
    assert fb(dh=Q[3] + 64) == 4 and fb(h=Q[3] + 64) == 4      # filter tables inside the written tensor
    assert fb(dh=Q[0] + 64) == 4                               # the filter gradient inside a tensor that is read
    assert fb(ws=None) == 1 and fb(wsb=16) == 2 and fb(ws=Q[5] + 4) == 4 and fb(ws=Q[1]) == 4
    wb = lib.hyena_featurize_bwd_workspace_bytes
    assert wb(1, 8, 16, 3, 1, 1) == 16 * 3 * 4 and wb(1, 8, 16, 3, 1, 0) == 16 * 3 * 4
    assert wb(2, 1000, 256, 7, 1, 1) == lib.hyena_bwd_shard_workspace_bytes(2, 1000, 256, 7, 1, 1)   # the stencil's tiles
    assert wb(1, 100, 64, 20, 1, 1) == 0 and wb(0, 100, 64, 7, 1, 1) == 0
    assert wb(1, 100, 64, 0, 1, 1) == -1 and wb(1, 100, 64, 7, 5, 1) == -1 and wb(1, 100, 64, 7, 1, 7) == -1


def test_chain_backward_rejects_bad_arguments_and_sizes_its_workspace():
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(17)]
    names = ("dy", "q", "k", "v", "hq", "hk", "hv", "h", "dq", "dk", "dv", "dhq", "dhk", "dhv", "dh", "ws")

    def cb(**kw):
        a = dict(zip(names, Q))
        a.update(wsb=1 << 19, B=1, L=8, D=16, lf=3, fg=1, lh=5, group=1, dtype=1)
        a.update(kw)
        return lib.hyena_chain_bwd(*[a[n] for n in names + ("wsb", "B", "L", "D", "lf", "fg", "lh", "group", "dtype")], None)

    for name in names[:15]:
        assert cb(**{name: None}) == 1
    assert cb(lf=0) == 2 and cb(fg=3) == 2 and cb(lh=0) == 2 and cb(group=5) == 2 and cb(dtype=7) == 3 and cb(wsb=-1) == 2
    assert cb(dq=Q[1]) == 4 and cb(dk=Q[8]) == 4 and cb(dv=Q[0] + 16) == 4        # activations
    assert cb(dhq=Q[4]) == 4 and cb(dhk=Q[11]) == 4 and cb(dh=Q[7]) == 4 and cb(dhv=Q[9] + 64) == 4 and cb(dh=Q[2] + 32) == 4
    need = lib.hyena_chain_bwd_workspace_bytes(1, 8, 16, 3, 1, 5, 1, 1)
    assert need == 6 * 256 + max(lib.hyena_bwd_workspace_bytes(1, 8, 16, 5, 1, 1),
                                 lib.hyena_featurize_bwd_workspace_bytes(1, 8, 16, 3, 1, 1))
    assert cb(ws=None) == 1 and cb(wsb=need - 1) == 2 and cb(ws=Q[15] + 4) == 4 and cb(ws=Q[3]) == 4
    wb = lib.hyena_chain_bwd_workspace_bytes
    assert wb(0, 8, 16, 3, 1, 5, 1, 1) == 0 and wb(1, 8, 16, 0, 1, 5, 1, 1) == -1 and wb(1, 8, 16, 3, 5, 5, 1, 1) == -1
    assert wb(1, 8, 16, 3, 1, 5, 1, 9) == -1
    # six tensors of 2 GiB-ish each plus the inner calls' share
    assert wb(4, 32768, 4096, 7, 1, 128, 16, 1) >= 6 * 4 * 32768 * 4096 * 2


def li(q=P[0], k=P[1], v=P[2], R=P[3], lam=P[5], y=P[4], ws=P[6], ws_bytes=1 << 30, B=1, L=8, D=16, order=4, group=1,
       dtype=0):
    return binding.lib().hyena_li_fwd(q, k, v, R, lam, y, ws, ws_bytes, B, L, D, order, group, dtype, None)


def test_long_implicit_entry_point_rejects_bad_arguments():
    lib = binding.lib()
    assert li(q=None) == 1 and li(R=None) == 1 and li(lam=None) == 1 and li(y=None) == 1
    assert li(B=-1) == 2 and li(order=0) == 2 and li(group=0) == 2 and li(D=16, group=3) == 2
    assert li(dtype=9) == 3
    assert li(lam=P[5] + 4) == 4 and li(y=P[2]) == 4
    assert li(order=65) == 5                      # more exponentials than the kernels hold
    assert li(ws_bytes=-1) == 2
    assert li(B=0) == 0 and li(L=0) == 0          # empty problems launch nothing
    # matrix-core shapes that span several tiles need the workspace: present, aligned, large enough, disjoint
    big = dict(B=1, L=1 << 16, D=256, order=16, group=16, dtype=1)
    need = lib.hyena_li_workspace_bytes(big["B"], big["L"], big["D"], big["order"], big["group"], big["dtype"])
    assert need > 0 and need % 1024 == 0
    far = 1 << 40
    ptrs = dict(q=far, k=2 * far, v=3 * far, y=4 * far, R=P[3], lam=P[5])
    assert li(ws=None, **ptrs, **big) == 1
    assert li(ws=5 * far + 8, **ptrs, **big) == 4
    assert li(ws=5 * far, ws_bytes=need - 1, **ptrs, **big) == 2
    assert li(ws=far + 64, **ptrs, **big) == 4    # inside q
    assert lib.hyena_li_workspace_bytes(1, 1 << 16, 256, 16, 16, 0) == 0   # fp32: general kernel, no workspace
    assert lib.hyena_li_workspace_bytes(1, 64, 256, 16, 16, 1) == 0        # one tile
    assert lib.hyena_li_workspace_bytes(1, 64, 256, 0, 16, 1) == -1
    assert lib.hyena_li_workspace_bytes(1, 64, 250, 16, 16, 1) == -1


def li_static(q=P[0], k=P[1], v=P[2], R=P[3], lam=P[5], y=P[4], B=1, L=8, D=16, order=4, group=1, dtype=0):
    return binding.lib().hyena_li_fwd_static(q, k, v, R, lam, y, B, L, D, order, group, dtype, None)


def test_static_scratch_entry_point_rejects_bad_arguments_and_oversized_scans():
    lib = binding.lib()
    assert li_static(q=None) == 1 and li_static(lam=None) == 1 and li_static(y=None) == 1
    assert li_static(order=0) == 2 and li_static(D=16, group=3) == 2 and li_static(dtype=9) == 3
    assert li_static(R=P[3] + 4) == 4 and li_static(y=P[2]) == 4 and li_static(order=65) == 5
    assert li_static(B=0) == 0 and li_static(L=0) == 0
    # the scan of this problem needs more end-of-tile records than the static buffer holds: refused, nothing launched
    far = 1 << 40
    big = dict(q=far, k=2 * far, v=3 * far, y=4 * far, B=1, L=1 << 16, D=256, order=16, group=16, dtype=1)
    assert lib.hyena_set_option(b"mr_rows", 32) == 0
    try:
        assert lib.hyena_li_workspace_bytes(1, 1 << 16, 256, 16, 16, 1) > 4 * 1024 * 1024
        assert li_static(**big) == 7
    finally:
        assert lib.hyena_set_option(b"mr_rows", 0) == 0
    # with the built-in tile choice no shape needs more than the buffer holds
    for B, L, D in ((1, 131072, 4096), (4, 32768, 4096), (3, 100000, 1024), (1, 1 << 20, 256), (7, 5000, 128), (1, 1 << 22, 64)):
        assert 0 <= lib.hyena_li_workspace_bytes(B, L, D, 16, 16, 1) <= 4 * 1024 * 1024, (B, L, D)


def test_options_are_snapshotted_per_call_and_safe_to_set_from_other_threads():
    """Workspace queries read one consistent snapshot of the options; setting options from other threads while
    queries run never yields a size that belongs to neither setting."""
    import threading

    lib = binding.lib()
    a = lib.hyena_li_workspace_bytes(1, 1 << 16, 256, 16, 16, 1)
    assert lib.hyena_set_option(b"mr_rows", 1024) == 0
    b = lib.hyena_li_workspace_bytes(1, 1 << 16, 256, 16, 16, 1)
    assert lib.hyena_set_option(b"mr_rows", 0) == 0
    assert a != b and a > 0 and b > 0
    stop = threading.Event()

    def flip():
        while not stop.is_set():
            lib.hyena_set_option(b"mr_rows", 1024)
            lib.hyena_set_option(b"mr_rows", 0)

    t = threading.Thread(target=flip)
    t.start()
    try:
        seen = {lib.hyena_li_workspace_bytes(1, 1 << 16, 256, 16, 16, 1) for _ in range(20000)}
    finally:
        stop.set()
        t.join()
        lib.hyena_set_option(b"mr_rows", 0)
    assert seen <= {a, b}


def test_long_implicit_state_entry_points_reject_bad_arguments():
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(6)]

    def st(k=Q[0], v=Q[1], lam=Q[2], s_in=None, s_out=Q[3], ws=Q[4], wsb=1 << 20, B=1, L=64, D=64, order=4, group=16,
           dtype=1):
        return lib.hyena_li_state(k, v, lam, s_in, s_out, ws, wsb, B, L, D, order, group, dtype, None)

    assert st(k=None) == 1 and st(v=None) == 1 and st(lam=None) == 1 and st(s_out=None) == 1
    assert st(order=0) == 2 and st(group=5) == 2 and st(dtype=3) == 3 and st(wsb=-1) == 2
    assert st(s_out=Q[3] + 4) == 4 and st(s_in=Q[5] + 8) == 4 and st(s_out=Q[0]) == 4 and st(s_in=Q[3]) == 4
    assert st(L=100) == 5 and st(dtype=0) == 5 and st(group=8) == 5 and st(order=17) == 5 and st(L=0) == 5
    need = lib.hyena_li_state_workspace_bytes(1, 64, 64, 4, 16, 1)
    assert need == 1 * 1 * (64 // 16) * 256 * 4            # one tile: one record per 16 channels
    assert st(ws=None) == 1 and st(wsb=need - 1) == 2 and st(ws=Q[4] + 4) == 4 and st(ws=Q[1]) == 4
    assert lib.hyena_li_state_workspace_bytes(1, 64, 64, 4, 16, 0) == 0 and lib.hyena_li_state_workspace_bytes(1, 64, 64, 0, 16, 1) == -1

    def fold(states=Q[0], n=3, steps=512, lam=Q[2], s_in=None, s_out=Q[3], B=1, D=64, order=4, group=16):
        return lib.hyena_li_state_fold(states, n, steps, lam, s_in, s_out, B, D, order, group, None)

    assert fold(states=None) == 1 and fold(lam=None) == 1 and fold(s_out=None) == 1
    assert fold(n=-1) == 2 and fold(steps=-1) == 2 and fold(order=0) == 2 and fold(group=5) == 2
    assert fold(D=24, group=8) == 5 and fold(order=17) == 5
    assert fold(states=Q[0] + 4) == 4 and fold(s_out=Q[3] + 8) == 4 and fold(s_in=Q[5] + 4) == 4
    assert fold(s_out=Q[0] + 2 * 64 * 64) == 4      # the result inside the third state that is read
    assert fold(s_out=Q[2]) == 4 and fold(s_in=Q[3]) == 4
    assert fold(B=0) == 0 and fold(D=0, group=1) == 0


@pytest.mark.parametrize("entry", ["hyena_se_fwd_shard", "hyena_mr_fwd_shard"])
def test_shard_entry_points_reject_bad_layouts(entry):
    lib = binding.lib()

    def call(q=P[0], k=P[1], v=P[2], h=P[3], y=P[4], B=2, L=8, D=16, lh=3, group=1, dtype=1, skv=10 * 16, sqy=8 * 16,
             hist=2):
        return getattr(lib, entry)(q, k, v, h, y, B, L, D, lh, group, dtype, skv, sqy, hist, None)

    assert call(hist=-1) == 2 and call(skv=-16) == 2 and call(sqy=-16) == 2
    assert call(skv=9 * 16) == 2          # k, v stride shorter than history + L rows
    assert call(sqy=7 * 16) == 2          # q, y stride shorter than L rows
    assert call(skv=10 * 16 + 4) == 4     # batch items of bf16 rows must start on 16-byte boundaries
    assert call(q=None) == 1 and call(L=-1) == 2 and call(dtype=9) == 3
    # overlap is judged on what is really touched: y inside the history rows in front of k
    assert call(y=P[1] - 2 * 16 * 2) == 4
    # and across the batch stride: y between k's two batch items is inside k's span
    assert call(y=P[1] + 8 * 16 * 2, skv=64 * 16) == 4
    assert call(B=0) == 0 and call(L=0) == 0   # empty problems: nothing to do, nothing launched
    assert call(B=1, skv=0, sqy=0, L=0) == 0   # strides are ignored for a single batch item


def test_long_implicit_carry_entry_point_rejects_bad_arguments():
    lib = binding.lib()

    def call(q=P[0], k=P[1], v=P[2], R=P[3], lam=P[4], y=P[5], s_in=P[6], s_out=P[7], ws=P[8], ws_bytes=1 << 20, B=1,
             L=64, D=64, order=4, group=16, dtype=1):
        return lib.hyena_li_fwd_carry(q, k, v, R, lam, y, s_in, s_out, ws, ws_bytes, B, L, D, order, group, dtype, None)

    assert call(q=None) == 1 and call(L=-1) == 2 and call(dtype=7) == 3
    assert call(s_in=P[6] + 4) == 4 and call(s_out=P[7] + 8) == 4      # states are 16-byte aligned
    assert call(s_out=P[5]) == 4 and call(s_in=P[7]) == 4              # and disjoint from y and from each other
    assert call(L=40) == 5                                             # a state after a ragged last chunk
    assert call(dtype=0) == 5 and call(group=8) == 5 and call(order=17) == 5 and call(D=48, group=16) == 5
    assert call(L=0) == 5                                              # an empty stretch has no state of its own
    assert lib.hyena_li_state_bytes(2, 64) == 2 * 64 * 64 and lib.hyena_li_state_bytes(1, 24) == -1


@pytest.mark.parametrize("entry", ["hyena_se_bwd_shard", "hyena_mr_bwd_shard"])
def test_backward_shard_entry_points_reject_bad_layouts(entry):
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(10)]

    def call(dy=Q[0], q=Q[1], k=Q[2], v=Q[3], h=Q[4], dq=Q[5], dk=Q[6], dv=Q[7], dh=Q[8], ws=Q[9], wsb=1 << 20, B=2, L=8,
             D=16, lh=3, group=1, dtype=1, skv=10 * 16, sgq=10 * 16, sout=8 * 16, hist=2, fut=2):
        return getattr(lib, entry)(dy, q, k, v, h, dq, dk, dv, dh, ws, wsb, B, L, D, lh, group, dtype, skv, sgq, sout,
                                   hist, fut, None)

    assert call(hist=-1) == 2 and call(fut=-1) == 2 and call(skv=-16) == 2
    assert call(skv=9 * 16) == 2 and call(sgq=9 * 16) == 2 and call(sout=7 * 16) == 2   # strides shorter than the rows
    assert call(sgq=10 * 16 + 4) == 4
    assert call(dy=None) == 1 and call(L=-1) == 2 and call(dtype=9) == 3 and call(wsb=-1) == 2
    assert call(dk=Q[2] - 2 * 16 * 2) == 4      # an output inside the history rows in front of k
    assert call(dq=Q[0] + 8 * 16 * 2) == 4      # an output inside the future rows behind dy
    assert call(dh=Q[1] + 9 * 16 * 2) == 4      # the filter gradient inside q's future rows
    assert lib.hyena_bwd_shard_workspace_bytes(1, 4096, 256, 7, 1, 1) > 0
    assert lib.hyena_bwd_shard_workspace_bytes(1, 4096, 128, 100, 1, 1) > 0     # ungrouped medium: 4x4x4 kernels
    assert lib.hyena_bwd_shard_workspace_bytes(1, 4096, 96, 100, 1, 1) == 0     # ... at D % 128 != 0: general kernels
    assert lib.hyena_bwd_shard_workspace_bytes(1, 64, 30, 3, 4, 1) == -1


def test_chain_shard_entry_point_rejects_bad_layouts():
    lib = binding.lib()
    Q = [0x100000 * (i + 1) for i in range(8)]

    def call(q=Q[0], k=Q[1], v=Q[2], hq=Q[3], hk=Q[4], hv=Q[5], h=Q[6], y=Q[7], B=2, L=64, D=128, lf=7, fg=1, lh=128,
             group=16, dtype=1, sin=200 * 128, sy=64 * 128, hist=133):
        return lib.hyena_chain_fwd_shard(q, k, v, hq, hk, hv, h, y, B, L, D, lf, fg, lh, group, dtype, sin, sy, hist, None)

    assert call(hist=-1) == 2 and call(sin=-1) == 2 and call(sin=196 * 128) == 2 and call(sy=63 * 128) == 2
    assert call(sin=200 * 128 + 4) == 4 and call(q=None) == 1 and call(lf=0) == 2 and call(fg=3) == 2
    assert call(y=Q[0] - 133 * 128 * 2) == 4          # y inside q's history rows
    assert call(dtype=0) == 5 and call(group=8) == 5 and call(lh=130) == 5 and call(lf=10) == 5   # single-kernel path only
    assert call(B=0) == 0 and call(L=0) == 0
