"""Thin ctypes binding of the C ABI declared in ``include/hyena.h``.

Argument marshalling only: every step of the operators runs inside ``libhyena.so``.  PyTorch supplies
device memory and the HIP stream.  There is no CPU or PyTorch fallback: if the library is missing and
cannot be built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

HY_OK = 0
HY_F32, HY_BF16 = 0, 1

_lib = None


class HyenaError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__("%s failed: %s (status %d)" % (what, status_string(code), code))


def lib() -> ctypes.CDLL:
    """Load ``libhyena.so`` from the package directory, building it first if it is absent or older than any of
    its sources (so that an edited kernel is never tested through a stale library)."""
    global _lib
    if _lib is None:
        if _build.stale():
            _build.build_library()
        L = ctypes.CDLL(_build.LIB)
        vp, i64, i32, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int
        conv_args = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_se_fwd.argtypes = conv_args
        L.hyena_mr_fwd.argtypes = conv_args
        shard_args = [vp] * 5 + [i64, i64, i64, i32, i32, ci, i64, i64, i32, vp]
        L.hyena_se_fwd_shard.argtypes = shard_args
        L.hyena_mr_fwd_shard.argtypes = shard_args
        L.hyena_featurize_fwd.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_featurize3_fwd.argtypes = [vp] * 9 + [i64, i64, i64, i32, i32, ci, vp]
        L.hyena_chain_fwd.argtypes = [vp] * 9 + [i64, i64, i64, i64, i32, i32, i32, i32, ci, vp]
        L.hyena_chain_fwd_shard.argtypes = [vp] * 8 + [i64, i64, i64, i32, i32, i32, i32, ci, i64, i64, i32, vp]
        L.hyena_chain_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, i32, i32, ci]
        L.hyena_chain_workspace_bytes.restype = i64
        bwd_args = [vp] * 10 + [i64, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_se_bwd.argtypes = bwd_args
        L.hyena_mr_bwd.argtypes = bwd_args
        L.hyena_bwd_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ci]
        L.hyena_bwd_workspace_bytes.restype = i64
        bwd_shard_args = [vp] * 10 + [i64, i64, i64, i64, i32, i32, ci, i64, i64, i64, i32, i32, vp]
        L.hyena_se_bwd_shard.argtypes = bwd_shard_args
        L.hyena_mr_bwd_shard.argtypes = bwd_shard_args
        L.hyena_bwd_shard_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ci]
        L.hyena_bwd_shard_workspace_bytes.restype = i64
        L.hyena_featurize_bwd.argtypes = [vp] * 6 + [i64, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_featurize_bwd_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ci]
        L.hyena_featurize_bwd_workspace_bytes.restype = i64
        L.hyena_chain_bwd.argtypes = [vp] * 16 + [i64, i64, i64, i64, i32, i32, i32, i32, ci, vp]
        L.hyena_chain_bwd_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, i32, i32, ci]
        L.hyena_chain_bwd_workspace_bytes.restype = i64
        L.hyena_li_fwd.argtypes = [vp] * 7 + [i64, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_li_fwd_static.argtypes = [vp] * 6 + [i64, i64, i64, i32, i32, ci, vp]
        L.hyena_li_fwd_carry.argtypes = [vp] * 9 + [i64, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_li_state_bytes.argtypes = [i64, i64]
        L.hyena_li_state_bytes.restype = i64
        L.hyena_li_state.argtypes = [vp] * 6 + [i64, i64, i64, i64, i32, i32, ci, vp]
        L.hyena_li_state_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ci]
        L.hyena_li_state_workspace_bytes.restype = i64
        L.hyena_li_state_fold.argtypes = [vp, i64, i64, vp, vp, vp, i64, i64, i32, i32, vp]
        L.hyena_li_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ci]
        L.hyena_li_workspace_bytes.restype = i64
        L.hyena_stream_copy.argtypes = [vp, vp, i64, vp]
        L.hyena_stream_gate.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i64, i32, i32, vp]
        L.hyena_set_option.argtypes = [ctypes.c_char_p, i32]
        for name in ("hyena_se_fwd", "hyena_mr_fwd", "hyena_se_fwd_shard", "hyena_mr_fwd_shard", "hyena_featurize_fwd",
                     "hyena_featurize3_fwd",
                     "hyena_chain_fwd", "hyena_chain_fwd_shard", "hyena_se_bwd", "hyena_mr_bwd", "hyena_se_bwd_shard",
                     "hyena_mr_bwd_shard", "hyena_featurize_bwd", "hyena_chain_bwd", "hyena_li_fwd",
                     "hyena_li_fwd_static", "hyena_li_fwd_carry", "hyena_li_state", "hyena_li_state_fold",
                     "hyena_stream_copy", "hyena_stream_gate", "hyena_set_option"):
            getattr(L, name).restype = ci
        L.hyena_status_string.argtypes = [ci]
        L.hyena_status_string.restype = ctypes.c_char_p
        L.hyena_version.argtypes = []
        L.hyena_version.restype = i32
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().hyena_status_string(int(code)).decode()


def version() -> int:
    return int(lib().hyena_version())


def set_option(name: str, value: int) -> None:
    rc = lib().hyena_set_option(name.encode(), int(value))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_set_option(%s)" % name)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HY_F32
    if t.dtype == torch.bfloat16:
        return HY_BF16
    raise TypeError("activations must be float32 or bfloat16, got %s" % t.dtype)


def _check_act(name: str, t: torch.Tensor, ref: torch.Tensor | None = None) -> None:
    if not isinstance(t, torch.Tensor) or t.device.type != "cuda":
        raise ValueError("%s must be a tensor on the GPU" % name)
    if t.dim() != 3 or not t.is_contiguous():
        raise ValueError("%s must be a contiguous [B, L, D] tensor" % name)
    if ref is not None and (t.shape != ref.shape or t.dtype != ref.dtype or t.device != ref.device):
        raise ValueError("%s must match the shape, dtype and device of the first activation" % name)


def _check_filter(name: str, h: torch.Tensor, x: torch.Tensor, group: int) -> int:
    if not isinstance(h, torch.Tensor) or h.device != x.device or h.dtype != torch.float32:
        raise ValueError("%s must be a float32 tensor on the same GPU" % name)
    if h.dim() != 2 or not h.is_contiguous() or group < 1 or x.shape[2] % group != 0 or h.shape[0] != x.shape[2] // group:
        raise ValueError("%s must be a contiguous [D // group, l_h] tensor" % name)
    return int(h.shape[1])


def _stream(x: torch.Tensor, stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _gated(entry: str, q, k, v, h, group, out, stream):
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    lh = _check_filter("h", h, q, group)
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    with torch.cuda.device(q.device):
        rc = getattr(lib(), entry)(q.data_ptr(), k.data_ptr(), v.data_ptr(), h.data_ptr(), y.data_ptr(),
                                   B, L, D, lh, int(group), _dtype_code(q), _stream(q, stream))
    if rc != HY_OK:
        raise HyenaError(rc, entry)
    return y


class Plan:
    """A fully marshalled call: ``plan()`` re-issues the same C-ABI call on the same buffers and stream.

    Nothing is computed or cached here; it only keeps the ctypes arguments (and references to the
    tensors, so they stay alive) to take Python's per-call checks out of a launch loop."""

    __slots__ = ("_fn", "_args", "_what", "_keep", "out")

    def __init__(self, fn, args, what, keep, out):
        self._fn, self._args, self._what, self._keep, self.out = fn, args, what, keep, out

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != HY_OK:
            raise HyenaError(rc, self._what)
        return self.out


def plan_gated(entry: str, q, k, v, h, group: int, out=None, stream=None) -> Plan:
    """Marshal one ``hyena_se_fwd`` / ``hyena_mr_fwd`` call (``entry`` names which) for repeated issue."""
    if entry not in ("hyena_se_fwd", "hyena_mr_fwd"):
        raise ValueError("entry must be hyena_se_fwd or hyena_mr_fwd")
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    lh = _check_filter("h", h, q, group)
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    c = ctypes
    args = (c.c_void_p(q.data_ptr()), c.c_void_p(k.data_ptr()), c.c_void_p(v.data_ptr()), c.c_void_p(h.data_ptr()),
            c.c_void_p(y.data_ptr()), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lh), c.c_int32(int(group)),
            c.c_int(_dtype_code(q)), c.c_void_p(_stream(q, stream)))
    return Plan(getattr(lib(), entry), args, entry, (q, k, v, h, y), y)


def _check_rows(name: str, t: torch.Tensor, ref: torch.Tensor | None = None) -> None:
    """A [B, L, D] window of rows: D contiguous, rows D apart, any distance between batch items."""
    if not isinstance(t, torch.Tensor) or t.device.type != "cuda":
        raise ValueError("%s must be a tensor on the GPU" % name)
    if t.dim() != 3 or t.stride(2) != 1 or t.stride(1) != t.shape[2]:
        raise ValueError("%s must be a [B, L, D] tensor or view with contiguous rows" % name)
    if ref is not None and (t.shape != ref.shape or t.dtype != ref.dtype or t.device != ref.device):
        raise ValueError("%s must match the shape, dtype and device of the first activation" % name)


def plan_gated_shard(entry: str, q, k, v, h, group: int, history: int, out=None, stream=None) -> Plan:
    """Marshal one ``hyena_se_fwd_shard`` / ``hyena_mr_fwd_shard`` call.  q, k, v (and out) are [B, L, D] windows
    with contiguous rows, e.g. ``x[:, t0:t0 + L]`` of a longer tensor; k and v must have ``history`` valid rows in
    front of their first row in memory and share one batch stride, q and out another."""
    if entry not in ("hyena_se_fwd_shard", "hyena_mr_fwd_shard"):
        raise ValueError("entry must be hyena_se_fwd_shard or hyena_mr_fwd_shard")
    _check_rows("q", q)
    _check_rows("k", k, q)
    _check_rows("v", v, q)
    lh = _check_filter("h", h, q, group)
    y = torch.empty_like(q, memory_format=torch.contiguous_format) if out is None else out
    _check_rows("out", y, q)
    B, L, D = q.shape
    if B > 1 and (k.stride(0) != v.stride(0) or q.stride(0) != y.stride(0)):
        raise ValueError("k and v must share a batch stride, q and out too")
    c = ctypes
    args = (c.c_void_p(q.data_ptr()), c.c_void_p(k.data_ptr()), c.c_void_p(v.data_ptr()), c.c_void_p(h.data_ptr()),
            c.c_void_p(y.data_ptr()), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lh), c.c_int32(int(group)),
            c.c_int(_dtype_code(q)), c.c_int64(k.stride(0)), c.c_int64(q.stride(0)), c.c_int32(int(history)),
            c.c_void_p(_stream(q, stream)))
    return Plan(getattr(lib(), entry), args, entry, (q, k, v, h, y), y)


def hyena_se_fwd_shard(q, k, v, h, group: int = 1, history: int = 0, out=None, stream=None) -> torch.Tensor:
    """One sequence shard of ``hyena_se_fwd``; see ``hyena_se_fwd_shard`` in hyena.h."""
    with torch.cuda.device(q.device):
        return plan_gated_shard("hyena_se_fwd_shard", q, k, v, h, group, history, out, stream)()


def hyena_mr_fwd_shard(q, k, v, h, group: int = 1, history: int = 0, out=None, stream=None) -> torch.Tensor:
    """One sequence shard of ``hyena_mr_fwd``; see ``hyena_mr_fwd_shard`` in hyena.h."""
    with torch.cuda.device(q.device):
        return plan_gated_shard("hyena_mr_fwd_shard", q, k, v, h, group, history, out, stream)()


def plan_featurize3(q, k, v, hq, hk, hv, group: int = 1, out=None, stream=None) -> Plan:
    """Marshal one ``hyena_featurize3_fwd`` call for repeated issue."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    lh = _check_filter("hq", hq, q, group)
    if _check_filter("hk", hk, q, group) != lh or _check_filter("hv", hv, q, group) != lh:
        raise ValueError("the three featurizer filters must share one length")
    outs = tuple(torch.empty_like(q) for _ in range(3)) if out is None else tuple(out)
    for name, o in zip(("qo", "ko", "vo"), outs):
        _check_act(name, o, q)
    B, L, D = q.shape
    c = ctypes
    ptrs = [t.data_ptr() for t in (q, k, v, hq, hk, hv) + outs]
    args = tuple(c.c_void_p(p) for p in ptrs) + (c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lh),
                                                  c.c_int32(int(group)), c.c_int(_dtype_code(q)),
                                                  c.c_void_p(_stream(q, stream)))
    return Plan(lib().hyena_featurize3_fwd, args, "hyena_featurize3_fwd", (q, k, v, hq, hk, hv) + outs, outs)


def hyena_se_fwd(q, k, v, h, group: int = 1, out=None, stream=None) -> torch.Tensor:
    """y = q * (h conv (k * v)), short filters; see ``hyena_se_fwd`` in hyena.h."""
    return _gated("hyena_se_fwd", q, k, v, h, group, out, stream)


def hyena_mr_fwd(q, k, v, h, group: int = 16, out=None, stream=None) -> torch.Tensor:
    """y = q * (h conv (k * v)), medium grouped filters; see ``hyena_mr_fwd`` in hyena.h."""
    return _gated("hyena_mr_fwd", q, k, v, h, group, out, stream)


def hyena_featurize_fwd(x, h, group: int = 1, out=None, stream=None) -> torch.Tensor:
    """y = h conv x, no gating; see ``hyena_featurize_fwd`` in hyena.h."""
    _check_act("x", x)
    lh = _check_filter("h", h, x, group)
    y = torch.empty_like(x) if out is None else out
    _check_act("out", y, x)
    B, L, D = x.shape
    with torch.cuda.device(x.device):
        rc = lib().hyena_featurize_fwd(x.data_ptr(), h.data_ptr(), y.data_ptr(), B, L, D, lh, int(group),
                                       _dtype_code(x), _stream(x, stream))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_featurize_fwd")
    return y


def hyena_featurize3_fwd(q, k, v, hq, hk, hv, group: int = 1, out=None, stream=None):
    """(hq conv q, hk conv k, hv conv v) in one launch; see ``hyena_featurize3_fwd`` in hyena.h."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    lh = _check_filter("hq", hq, q, group)
    if _check_filter("hk", hk, q, group) != lh or _check_filter("hv", hv, q, group) != lh:
        raise ValueError("the three featurizer filters must share one length")
    outs = tuple(torch.empty_like(q) for _ in range(3)) if out is None else tuple(out)
    for name, o in zip(("qo", "ko", "vo"), outs):
        _check_act(name, o, q)
    B, L, D = q.shape
    with torch.cuda.device(q.device):
        rc = lib().hyena_featurize3_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), hq.data_ptr(), hk.data_ptr(),
                                        hv.data_ptr(), outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(),
                                        B, L, D, lh, int(group), _dtype_code(q), _stream(q, stream))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_featurize3_fwd")
    return outs


def _chain_args(q, k, v, hq, hk, hv, h, group, feat_group, out, workspace, stream):
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    lf = _check_filter("hq", hq, q, feat_group)
    if _check_filter("hk", hk, q, feat_group) != lf or _check_filter("hv", hv, q, feat_group) != lf:
        raise ValueError("the three featurizer filters must share one length")
    lh = _check_filter("h", h, q, group)
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    need = int(lib().hyena_chain_workspace_bytes(B, L, D, lf, int(feat_group), lh, int(group), _dtype_code(q)))
    if need < 0:
        raise ValueError("not a valid chain problem")
    if need > 0 and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)  # device memory from PyTorch
    if need > 0 and (workspace.device != q.device or not workspace.is_contiguous()
                     or workspace.numel() * workspace.element_size() < need):
        raise ValueError("workspace must be a contiguous tensor of at least %d bytes on the same GPU" % need)
    c = ctypes
    ptrs = [t.data_ptr() for t in (q, k, v, hq, hk, hv, h, y)] + [workspace.data_ptr() if need > 0 else None]
    ws_bytes = workspace.numel() * workspace.element_size() if need > 0 else 0
    args = tuple(c.c_void_p(p) for p in ptrs) + (c.c_int64(ws_bytes), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lf),
                                                  c.c_int32(int(feat_group)), c.c_int32(lh), c.c_int32(int(group)),
                                                  c.c_int(_dtype_code(q)), c.c_void_p(_stream(q, stream)))
    return args, (q, k, v, hq, hk, hv, h, y, workspace), y


def hyena_chain_fwd(q, k, v, hq, hk, hv, h, group: int = 16, feat_group: int = 1, out=None, workspace=None,
                    stream=None) -> torch.Tensor:
    """Featurize q, k, v and apply the gated medium convolution; see ``hyena_chain_fwd`` in hyena.h."""
    args, _, y = _chain_args(q, k, v, hq, hk, hv, h, group, feat_group, out, workspace, stream)
    with torch.cuda.device(q.device):
        rc = lib().hyena_chain_fwd(*args)
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_chain_fwd")
    return y


def plan_chain(q, k, v, hq, hk, hv, h, group: int = 16, feat_group: int = 1, out=None, workspace=None,
               stream=None) -> Plan:
    """Marshal one ``hyena_chain_fwd`` call for repeated issue."""
    args, keep, y = _chain_args(q, k, v, hq, hk, hv, h, group, feat_group, out, workspace, stream)
    return Plan(lib().hyena_chain_fwd, args, "hyena_chain_fwd", keep, y)


def hyena_chain_fwd_shard(q, k, v, hq, hk, hv, h, group: int = 16, feat_group: int = 1, history: int = 0, out=None,
                          stream=None) -> torch.Tensor:
    """One sequence shard of ``hyena_chain_fwd``: q, k, v are [B, L, D] windows with contiguous rows and ``history``
    valid rows in front of each in memory; see ``hyena_chain_fwd_shard`` in hyena.h."""
    _check_rows("q", q)
    _check_rows("k", k, q)
    _check_rows("v", v, q)
    lf = _check_filter("hq", hq, q, feat_group)
    if _check_filter("hk", hk, q, feat_group) != lf or _check_filter("hv", hv, q, feat_group) != lf:
        raise ValueError("the three featurizer filters must share one length")
    lh = _check_filter("h", h, q, group)
    y = torch.empty_like(q, memory_format=torch.contiguous_format) if out is None else out
    _check_rows("out", y, q)
    B, L, D = q.shape
    if B > 1 and (q.stride(0) != k.stride(0) or q.stride(0) != v.stride(0)):
        raise ValueError("q, k, v must share a batch stride")
    c = ctypes
    with torch.cuda.device(q.device):
        rc = lib().hyena_chain_fwd_shard(
            *(c.c_void_p(t.data_ptr()) for t in (q, k, v, hq, hk, hv, h, y)), c.c_int64(B), c.c_int64(L), c.c_int64(D),
            c.c_int32(lf), c.c_int32(int(feat_group)), c.c_int32(lh), c.c_int32(int(group)), c.c_int(_dtype_code(q)),
            c.c_int64(q.stride(0)), c.c_int64(y.stride(0)), c.c_int32(int(history)), c.c_void_p(_stream(q, stream)))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_chain_fwd_shard")
    return y


def plan_bwd(entry: str, dy, q, k, v, h, group: int, out=None, workspace=None, stream=None) -> Plan:
    """Marshal one ``hyena_se_bwd`` / ``hyena_mr_bwd`` call for repeated issue; ``out`` = (dq, dk, dv, dh)."""
    if entry not in ("hyena_se_bwd", "hyena_mr_bwd"):
        raise ValueError("entry must be hyena_se_bwd or hyena_mr_bwd")
    _check_act("dy", dy)
    _check_act("q", q, dy)
    _check_act("k", k, dy)
    _check_act("v", v, dy)
    lh = _check_filter("h", h, dy, group)
    B, L, D = dy.shape
    code = _dtype_code(dy)
    need = int(lib().hyena_bwd_workspace_bytes(B, L, D, lh, int(group), code))
    if need < 0:
        raise ValueError("not a valid backward problem")
    if need > 0 and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dy.device)
    if out is None:
        out = tuple(torch.empty_like(dy) for _ in range(3)) + (torch.empty_like(h),)
    for name, o in zip(("dq", "dk", "dv"), out[:3]):
        _check_act(name, o, dy)
    _check_filter("dh", out[3], dy, group)
    c = ctypes
    ptrs = [t.data_ptr() for t in (dy, q, k, v, h) + tuple(out)]
    ws_ptr = workspace.data_ptr() if need > 0 else None
    ws_bytes = workspace.numel() * workspace.element_size() if need > 0 else 0
    args = tuple(c.c_void_p(p) for p in ptrs) + (c.c_void_p(ws_ptr), c.c_int64(ws_bytes), c.c_int64(B), c.c_int64(L),
                                                  c.c_int64(D), c.c_int32(lh), c.c_int32(int(group)), c.c_int(code),
                                                  c.c_void_p(_stream(dy, stream)))
    return Plan(getattr(lib(), entry), args, entry, (dy, q, k, v, h, workspace) + tuple(out), tuple(out))


def plan_bwd_shard(entry: str, dy, q, k, v, h, group: int, history: int, future: int, out=None, stream=None) -> Plan:
    """Marshal one ``hyena_se_bwd_shard`` / ``hyena_mr_bwd_shard`` call; dy, q, k, v are [B, L, D] windows with
    contiguous rows (k, v with ``history`` valid rows in front of them in memory, dy, q with ``future`` valid rows
    behind them); ``out`` = (dq, dk, dv, dh), the first three windows too, dh this shard's share."""
    if entry not in ("hyena_se_bwd_shard", "hyena_mr_bwd_shard"):
        raise ValueError("entry must be hyena_se_bwd_shard or hyena_mr_bwd_shard")
    _check_rows("dy", dy)
    _check_rows("q", q, dy)
    _check_rows("k", k, dy)
    _check_rows("v", v, dy)
    lh = _check_filter("h", h, dy, group)
    B, L, D = dy.shape
    code = _dtype_code(dy)
    need = int(lib().hyena_bwd_shard_workspace_bytes(B, L, D, lh, int(group), code))
    if need < 0:
        raise ValueError("not a valid backward problem")
    workspace = torch.empty(need, dtype=torch.uint8, device=dy.device) if need > 0 else None
    if out is None:
        out = tuple(torch.empty_like(dy, memory_format=torch.contiguous_format) for _ in range(3)) + (torch.empty_like(h),)
    for name, o in zip(("dq", "dk", "dv"), out[:3]):
        _check_rows(name, o, dy)
    _check_filter("dh", out[3], dy, group)
    if B > 1 and (k.stride(0) != v.stride(0) or dy.stride(0) != q.stride(0) or
                  out[0].stride(0) != out[1].stride(0) or out[0].stride(0) != out[2].stride(0)):
        raise ValueError("k, v / dy, q / dq, dk, dv must each share a batch stride")
    c = ctypes
    ptrs = [t.data_ptr() for t in (dy, q, k, v, h) + tuple(out)]
    args = tuple(c.c_void_p(p) for p in ptrs) + (
        c.c_void_p(workspace.data_ptr() if need > 0 else None), c.c_int64(need), c.c_int64(B), c.c_int64(L),
        c.c_int64(D), c.c_int32(lh), c.c_int32(int(group)), c.c_int(code), c.c_int64(k.stride(0)),
        c.c_int64(dy.stride(0)), c.c_int64(out[0].stride(0)), c.c_int32(int(history)), c.c_int32(int(future)),
        c.c_void_p(_stream(dy, stream)))
    return Plan(getattr(lib(), entry), args, entry, (dy, q, k, v, h, workspace) + tuple(out), tuple(out))


def hyena_se_bwd_shard(dy, q, k, v, h, group: int = 1, history: int = 0, future: int = 0, out=None, stream=None):
    """One sequence shard of ``hyena_se_bwd``: (dq, dk, dv, this shard's share of dh)."""
    with torch.cuda.device(dy.device):
        return plan_bwd_shard("hyena_se_bwd_shard", dy, q, k, v, h, group, history, future, out, stream)()


def hyena_mr_bwd_shard(dy, q, k, v, h, group: int = 1, history: int = 0, future: int = 0, out=None, stream=None):
    """One sequence shard of ``hyena_mr_bwd``: (dq, dk, dv, this shard's share of dh)."""
    with torch.cuda.device(dy.device):
        return plan_bwd_shard("hyena_mr_bwd_shard", dy, q, k, v, h, group, history, future, out, stream)()


def _bwd(entry: str, dy, q, k, v, h, group, workspace, stream):
    _check_act("dy", dy)
    _check_act("q", q, dy)
    _check_act("k", k, dy)
    _check_act("v", v, dy)
    lh = _check_filter("h", h, dy, group)
    B, L, D = dy.shape
    code = _dtype_code(dy)
    need = int(lib().hyena_bwd_workspace_bytes(B, L, D, lh, int(group), code))
    if need < 0:
        raise ValueError("not a valid backward problem")
    if need > 0 and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dy.device)  # device memory from PyTorch
    ws_ptr = workspace.data_ptr() if workspace is not None and workspace.numel() > 0 else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    dq, dk, dv = (torch.empty_like(dy) for _ in range(3))
    dh = torch.empty_like(h)
    with torch.cuda.device(dy.device):
        rc = getattr(lib(), entry)(dy.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), h.data_ptr(), dq.data_ptr(),
                                   dk.data_ptr(), dv.data_ptr(), dh.data_ptr(), ws_ptr, ws_bytes, B, L, D, lh,
                                   int(group), code, _stream(dy, stream))
    if rc != HY_OK:
        raise HyenaError(rc, entry)
    return dq, dk, dv, dh


def hyena_se_bwd(dy, q, k, v, h, group: int = 1, workspace=None, stream=None):
    """(dq, dk, dv, dh) of ``hyena_se_fwd``; see ``hyena_se_bwd`` in hyena.h."""
    return _bwd("hyena_se_bwd", dy, q, k, v, h, group, workspace, stream)


def hyena_mr_bwd(dy, q, k, v, h, group: int = 16, workspace=None, stream=None):
    """(dq, dk, dv, dh) of ``hyena_mr_fwd``; see ``hyena_mr_bwd`` in hyena.h."""
    return _bwd("hyena_mr_bwd", dy, q, k, v, h, group, workspace, stream)


def plan_featurize_bwd(dy, x, h, group: int = 1, out=None, workspace=None, stream=None) -> Plan:
    """Marshal one ``hyena_featurize_bwd`` call for repeated issue; ``out`` = (dx, dh)."""
    _check_act("dy", dy)
    _check_act("x", x, dy)
    lh = _check_filter("h", h, dy, group)
    B, L, D = dy.shape
    code = _dtype_code(dy)
    need = int(lib().hyena_featurize_bwd_workspace_bytes(B, L, D, lh, int(group), code))
    if need < 0:
        raise ValueError("not a valid backward problem")
    if need > 0 and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dy.device)  # device memory from PyTorch
    if out is None:
        out = (torch.empty_like(dy), torch.empty_like(h))
    _check_act("dx", out[0], dy)
    _check_filter("dh", out[1], dy, group)
    c = ctypes
    ws_ptr = workspace.data_ptr() if need > 0 else None
    ws_bytes = workspace.numel() * workspace.element_size() if need > 0 else 0
    args = tuple(c.c_void_p(t.data_ptr()) for t in (dy, x, h) + tuple(out)) + (
        c.c_void_p(ws_ptr), c.c_int64(ws_bytes), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lh),
        c.c_int32(int(group)), c.c_int(code), c.c_void_p(_stream(dy, stream)))
    return Plan(lib().hyena_featurize_bwd, args, "hyena_featurize_bwd", (dy, x, h, workspace) + tuple(out), tuple(out))


def hyena_featurize_bwd(dy, x, h, group: int = 1, workspace=None, stream=None):
    """(dx, dh) of ``hyena_featurize_fwd``; see ``hyena_featurize_bwd`` in hyena.h."""
    with torch.cuda.device(dy.device):
        return plan_featurize_bwd(dy, x, h, group, None, workspace, stream)()


def plan_chain_bwd(dy, q, k, v, hq, hk, hv, h, group: int = 16, feat_group: int = 1, out=None, workspace=None,
                   stream=None) -> Plan:
    """Marshal one ``hyena_chain_bwd`` call for repeated issue; ``out`` = (dq, dk, dv, dhq, dhk, dhv, dh)."""
    _check_act("dy", dy)
    _check_act("q", q, dy)
    _check_act("k", k, dy)
    _check_act("v", v, dy)
    lf = _check_filter("hq", hq, dy, feat_group)
    if _check_filter("hk", hk, dy, feat_group) != lf or _check_filter("hv", hv, dy, feat_group) != lf:
        raise ValueError("the three featurizer filters must share one length")
    lh = _check_filter("h", h, dy, group)
    B, L, D = dy.shape
    code = _dtype_code(dy)
    need = int(lib().hyena_chain_bwd_workspace_bytes(B, L, D, lf, int(feat_group), lh, int(group), code))
    if need < 0:
        raise ValueError("not a valid chain problem")
    if need > 0 and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dy.device)  # device memory from PyTorch
    if out is None:
        out = tuple(torch.empty_like(dy) for _ in range(3)) + tuple(torch.empty_like(f) for f in (hq, hk, hv, h))
    for name, o in zip(("dq", "dk", "dv"), out[:3]):
        _check_act(name, o, dy)
    for name, o in zip(("dhq", "dhk", "dhv"), out[3:6]):
        _check_filter(name, o, dy, feat_group)
    _check_filter("dh", out[6], dy, group)
    c = ctypes
    ws_ptr = workspace.data_ptr() if need > 0 else None
    ws_bytes = workspace.numel() * workspace.element_size() if need > 0 else 0
    args = tuple(c.c_void_p(t.data_ptr()) for t in (dy, q, k, v, hq, hk, hv, h) + tuple(out)) + (
        c.c_void_p(ws_ptr), c.c_int64(ws_bytes), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(lf),
        c.c_int32(int(feat_group)), c.c_int32(lh), c.c_int32(int(group)), c.c_int(code), c.c_void_p(_stream(dy, stream)))
    return Plan(lib().hyena_chain_bwd, args, "hyena_chain_bwd", (dy, q, k, v, hq, hk, hv, h, workspace) + tuple(out),
                tuple(out))


def hyena_chain_bwd(dy, q, k, v, hq, hk, hv, h, group: int = 16, feat_group: int = 1, workspace=None, stream=None):
    """(dq, dk, dv, dhq, dhk, dhv, dh) of ``hyena_chain_fwd``; see ``hyena_chain_bwd`` in hyena.h."""
    with torch.cuda.device(dy.device):
        return plan_chain_bwd(dy, q, k, v, hq, hk, hv, h, group, feat_group, None, workspace, stream)()


def plan_li(q, k, v, R, lam, group: int = 16, out=None, workspace=None, stream=None) -> Plan:
    """Marshal one ``hyena_li_fwd`` call for repeated issue (workspace sized under the current options)."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    order = _check_filter("R", R, q, group)
    if _check_filter("lam", lam, q, group) != order:
        raise ValueError("R and lam must share one [D // group, order] shape")
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    code = _dtype_code(q)
    need = int(lib().hyena_li_workspace_bytes(B, L, D, order, int(group), code))
    if need < 0:
        raise ValueError("not a valid Hyena-LI problem")
    if need > 0 and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    c = ctypes
    ws_ptr = workspace.data_ptr() if need > 0 else None
    ws_bytes = workspace.numel() * workspace.element_size() if need > 0 else 0
    args = tuple(c.c_void_p(t.data_ptr()) for t in (q, k, v, R, lam, y)) + (
        c.c_void_p(ws_ptr), c.c_int64(ws_bytes), c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(order),
        c.c_int32(int(group)), c.c_int(code), c.c_void_p(_stream(q, stream)))
    return Plan(lib().hyena_li_fwd, args, "hyena_li_fwd", (q, k, v, R, lam, y, workspace), y)


def hyena_li_fwd(q, k, v, R, lam, group: int = 16, out=None, workspace=None, stream=None) -> torch.Tensor:
    """y = q * (h conv (k * v)) with h[g, j] = sum_n R[g, n] lam[g, n]^j; see ``hyena_li_fwd`` in hyena.h."""
    with torch.cuda.device(q.device):
        return plan_li(q, k, v, R, lam, group, out, workspace, stream)()


def hyena_li_fwd_carry(q, k, v, R, lam, group: int = 16, state_in=None, want_state: bool = True, out=None,
                       stream=None):
    """One stretch of a longer sequence: returns (y, state_out); ``state_in`` is the state the previous stretch
    returned (None at the start of a sequence); see ``hyena_li_fwd_carry`` in hyena.h."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    order = _check_filter("R", R, q, group)
    if _check_filter("lam", lam, q, group) != order:
        raise ValueError("R and lam must share one [D // group, order] shape")
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    code = _dtype_code(q)
    nstate = int(lib().hyena_li_state_bytes(B, D))
    if nstate < 0:
        raise ValueError("D must be a multiple of 16")
    if state_in is not None and (state_in.dtype != torch.float32 or state_in.numel() * 4 != nstate or
                                 not state_in.is_contiguous() or state_in.device != q.device):
        raise ValueError("state_in must be the float32 state a previous call returned")
    state_out = torch.empty(nstate // 4, dtype=torch.float32, device=q.device) if want_state else None
    need = int(lib().hyena_li_workspace_bytes(B, L, D, order, int(group), code))
    if need < 0:
        raise ValueError("not a valid Hyena-LI problem")
    workspace = torch.empty(need, dtype=torch.uint8, device=q.device) if need > 0 else None
    c = ctypes
    with torch.cuda.device(q.device):
        rc = lib().hyena_li_fwd_carry(
            *(c.c_void_p(t.data_ptr()) for t in (q, k, v, R, lam, y)),
            c.c_void_p(state_in.data_ptr() if state_in is not None else None),
            c.c_void_p(state_out.data_ptr() if state_out is not None else None),
            c.c_void_p(workspace.data_ptr() if workspace is not None else None), c.c_int64(need), c.c_int64(B),
            c.c_int64(L), c.c_int64(D), c.c_int32(order), c.c_int32(int(group)), c.c_int(code),
            c.c_void_p(_stream(q, stream)))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_li_fwd_carry")
    return y, state_out


def hyena_li_state(k, v, lam, group: int = 16, state_in=None, stream=None) -> torch.Tensor:
    """The running sums after the steps of k, v (no q, no y): the state ``hyena_li_fwd_carry`` would return; see
    ``hyena_li_state`` in hyena.h."""
    _check_act("k", k)
    _check_act("v", v, k)
    order = _check_filter("lam", lam, k, group)
    B, L, D = k.shape
    code = _dtype_code(k)
    nstate = int(lib().hyena_li_state_bytes(B, D))
    if nstate < 0:
        raise ValueError("D must be a multiple of 16")
    if state_in is not None and (state_in.dtype != torch.float32 or state_in.numel() * 4 != nstate or
                                 not state_in.is_contiguous() or state_in.device != k.device):
        raise ValueError("state_in must be a float32 state of this shape")
    state_out = torch.empty(nstate // 4, dtype=torch.float32, device=k.device)
    need = int(lib().hyena_li_state_workspace_bytes(B, L, D, order, int(group), code))
    if need < 0:
        raise ValueError("not a valid Hyena-LI problem")
    workspace = torch.empty(need, dtype=torch.uint8, device=k.device) if need > 0 else None   # device memory from PyTorch
    c = ctypes
    with torch.cuda.device(k.device):
        rc = lib().hyena_li_state(
            c.c_void_p(k.data_ptr()), c.c_void_p(v.data_ptr()), c.c_void_p(lam.data_ptr()),
            c.c_void_p(state_in.data_ptr() if state_in is not None else None), c.c_void_p(state_out.data_ptr()),
            c.c_void_p(workspace.data_ptr() if workspace is not None else None), c.c_int64(need), c.c_int64(B),
            c.c_int64(L), c.c_int64(D), c.c_int32(order), c.c_int32(int(group)), c.c_int(code),
            c.c_void_p(_stream(k, stream)))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_li_state")
    return state_out


def hyena_li_state_fold(states, steps: int, lam, B: int, D: int, group: int = 16, state_in=None, stream=None) -> torch.Tensor:
    """The state after ``len(states)`` consecutive stretches of ``steps`` steps whose zero-start end states are given
    (``states``: a float32 tensor [n, state floats] or a list of states); see ``hyena_li_state_fold`` in hyena.h."""
    if isinstance(states, (list, tuple)):
        states = torch.stack(list(states)) if len(states) > 0 else torch.empty((0, B * D * 16), dtype=torch.float32,
                                                                              device=lam.device)
    nstate = int(lib().hyena_li_state_bytes(B, D))
    if nstate < 0:
        raise ValueError("D must be a multiple of 16")
    if (states.dtype != torch.float32 or states.dim() != 2 or states.shape[1] * 4 != nstate or not states.is_contiguous()
            or states.device.type != "cuda"):
        raise ValueError("states must be a contiguous float32 [n, B * D * 16] tensor on the GPU")
    if lam.dtype != torch.float32 or lam.dim() != 2 or not lam.is_contiguous() or lam.shape[0] * int(group) != D:
        raise ValueError("lam must be a contiguous float32 [D // group, order] tensor")
    if state_in is not None and (state_in.dtype != torch.float32 or state_in.numel() * 4 != nstate or
                                 not state_in.is_contiguous() or state_in.device != states.device):
        raise ValueError("state_in must be a float32 state of this shape")
    out = torch.empty(nstate // 4, dtype=torch.float32, device=states.device)
    n = int(states.shape[0])
    c = ctypes
    with torch.cuda.device(states.device):
        rc = lib().hyena_li_state_fold(
            c.c_void_p(states.data_ptr() if n > 0 else None), c.c_int64(n), c.c_int64(int(steps)),
            c.c_void_p(lam.data_ptr()), c.c_void_p(state_in.data_ptr() if state_in is not None else None),
            c.c_void_p(out.data_ptr()), c.c_int64(B), c.c_int64(D), c.c_int32(int(lam.shape[1])), c.c_int32(int(group)),
            c.c_void_p(_stream(states, stream)))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_li_state_fold")
    return out


def hyena_li_fwd_static(q, k, v, R, lam, group: int = 16, out=None, stream=None) -> torch.Tensor:
    """``hyena_li_fwd`` with the scan's scratch inside the library (no workspace, no allocation in the call when
    ``out`` is given); see ``hyena_li_fwd_static`` in hyena.h."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    order = _check_filter("R", R, q, group)
    if _check_filter("lam", lam, q, group) != order:
        raise ValueError("R and lam must share one [D // group, order] shape")
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    with torch.cuda.device(q.device):
        rc = lib().hyena_li_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), R.data_ptr(), lam.data_ptr(),
                                       y.data_ptr(), B, L, D, order, int(group), _dtype_code(q), _stream(q, stream))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_li_fwd_static")
    return y


def hyena_stream_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> torch.Tensor:
    """Plain streaming copy (bandwidth yardstick); see ``hyena_stream_copy`` in hyena.h."""
    if src.device.type != "cuda" or not src.is_contiguous() or not dst.is_contiguous():
        raise ValueError("src and dst must be contiguous GPU tensors")
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or dst.device != src.device:
        raise ValueError("src and dst must have the same size and device")
    with torch.cuda.device(src.device):
        rc = lib().hyena_stream_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(src, stream))
    if rc != HY_OK:
        raise HyenaError(rc, "hyena_stream_copy")
    return dst


def plan_stream_gate(q, k, v, strip_channels: int = 0, rows: int = 0, depth: int = 0, waves: int = 0, out=None,
                     stream=None) -> Plan:
    """Marshal one ``hyena_stream_gate`` call (y = q*k*v, the bandwidth yardstick) for repeated issue."""
    _check_act("q", q)
    _check_act("k", k, q)
    _check_act("v", v, q)
    if q.dtype != torch.bfloat16:
        raise TypeError("hyena_stream_gate takes bfloat16 tensors")
    y = torch.empty_like(q) if out is None else out
    _check_act("out", y, q)
    B, L, D = q.shape
    c = ctypes
    args = tuple(c.c_void_p(t.data_ptr()) for t in (q, k, v, y)) + (
        c.c_int64(B), c.c_int64(L), c.c_int64(D), c.c_int32(int(strip_channels)), c.c_int64(int(rows)),
        c.c_int32(int(depth)), c.c_int32(int(waves)), c.c_void_p(_stream(q, stream)))
    return Plan(lib().hyena_stream_gate, args, "hyena_stream_gate", (q, k, v, y), y)


def hyena_stream_gate(q, k, v, strip_channels: int = 0, rows: int = 0, depth: int = 0, waves: int = 0, out=None,
                      stream=None) -> torch.Tensor:
    """y = q*k*v elementwise, linearly or through column strips; see ``hyena_stream_gate`` in hyena.h."""
    with torch.cuda.device(q.device):
        return plan_stream_gate(q, k, v, strip_channels, rows, depth, waves, out, stream)()
