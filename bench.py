#!/usr/bin/env python3
"""Throughput of the Hyena-SE / Hyena-MR forward path on one MI355X, against the HBM roofline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1|c2|c3|c4|...]

A step is one pass of the hot path over one synthetic batch that already sits in HBM:
  c1  Hyena-SE  bf16 B1 L8192   D4096 lh7            hyena_se_fwd            (default; the headline case)
  c2  Hyena-MR  bf16 B1 L8192   D4096 lh128 group16  hyena_mr_fwd
  c3  Hyena-MR  bf16 B1 L131072 D4096 lh128 group16  hyena_mr_fwd
  c4  chain     bf16 B4 L32768  D4096                hyena_chain_fwd (featurizers + MR in one kernel)
  c1_bwd / c2_bwd / c3_bwd / c2u_bwd: the backward entry points (hyena_se_bwd / hyena_mr_bwd) on the shapes of
      c1 / c2 / c3 / c2u; c4_bwd: hyena_chain_bwd on c4's shape (featurizers recomputed, inner backward, three
      featurizer backward calls; 6 tensors of workspace); c4_feat: the three featurizer convolutions of c4 alone
      (hyena_featurize3_fwd, 12 bytes per element: three tensors read and written)
  c1_shards / c2_shards / c3_shards: c1 / c2 / c3 computed as four consecutive sequence shards (hyena_se_fwd_shard /
      hyena_mr_fwd_shard: each call sees its quarter of the steps plus the lh - 1 rows of k and v before it), the
      compute half of a sequence-sharded run on one GPU; a step is the four launches.  c3_bwd_shards: the same for
      the backward pass (hyena_mr_bwd_shard: halos on both sides, every shard its share of the filter gradient).
      c3_overlap: c3_shards with every shard after the first split into the call that needs no neighbour data (all
      but its first lh - 1 steps) and the call for those first steps, the split that lets a rank hide the exchange
Successive steps rotate through several independent input/output sets so that every launch streams from
HBM instead of re-hitting the 256 MB last-level cache (c1 and c2 move exactly 256 MiB per step).
  c2u c2 with one filter per channel; li2 / li3: Hyena-LI at the shapes of c2 / c3
  stream / strip64 / strip128 / strip256: the bandwidth yardstick hyena_stream_gate (y = q*k*v: the operator's
      3-read/1-write traffic without its arithmetic) on c1's shape, streamed linearly or walked in column strips
      of 64 / 128 / 256 channels (128 / 256 / 512-byte row pieces) the way the matrix-core kernels move their data;
      strip256w8 / strip256w4: 512-byte strips walked by 8 / 4 waves with 4 / 8 chunks in flight per lane
Prints ONE JSON line.  The CPU oracle is timed beside it on a bounded slice of the same workload.  With the default
workload the line also carries, under "also", the same roofline figures for c2, c3, c4, c2u, li2 and both backward
workloads (a quarter of the steps each, after a warm-up of their own, which each entry states).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "Hyena-SE/MR fwd tokens/s at D=4096; achieved HBM GB/s and MFMA % of peak"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# bandwidth yardsticks: workload name -> (channels per workgroup strip (0 = linear stream), waves per workgroup
# (0 = one per 16 channels), chunks of loads in flight per lane (0 = 2)); the first four have the shape of the
# operator kernels, the last two keep the same bytes in flight with fewer, fatter streams
YARDSTICKS = {"stream": (0, 0, 0), "strip64": (64, 0, 0), "strip128": (128, 0, 0), "strip256": (256, 0, 0),
              "strip256w8": (256, 8, 4), "strip256w4": (256, 4, 8)}
TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c1",
                    choices=["c1", "c2", "c3", "c4", "c2u", "li2", "li3", "c1_bwd", "c2_bwd", "c3_bwd", "c2u_bwd", "c1_shards",
                             "c2_shards", "c3_shards", "c3_overlap", "c1_bwd_shards", "c3_bwd_shards", "c4_bwd", "c4_feat", "copy"] + list(YARDSTICKS),
                    help="'copy' only issues the plain copy kernel used to calibrate hardware byte counters")
    ap.add_argument("--seq-len", type=int, default=0,
                    help="override L of the workload (the paper sweeps its operator benchmark over L at batch 1, "
                         "width 4096); the JSON line then names the changed shape and carries no stored traffic figure")
    ap.add_argument("--batch", type=int, default=0,
                    help="override B of the workload (like --seq-len: the line names the changed shape, no stored traffic)")
    ap.add_argument("--width", type=int, default=0, help="override D of the workload (likewise)")
    ap.add_argument("--sets", type=int, default=0, help="independent buffer sets to rotate through (0 = auto)")
    ap.add_argument("--depth", type=int, default=0,
                    help="strip yardsticks only: chunks of loads in flight per lane (0 = the workload's own: 2 as in the operator kernels, 4 / 8 for strip256w8 / strip256w4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle slice")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob (hyena_set_option), may repeat; results never depend on these")
    ap.add_argument("--also", default="c2,c3,c4,c2u,li2,c1_bwd,c2_bwd",
                    help="comma list of further workloads to time briefly (c1 only)")
    ap.add_argument("--settle", type=int, default=300,
                    help="launches issued right after set-up, before the --warmup steps, so that the clocks have left "
                         "their idle state when warm-up and timing begin (uploading the inputs leaves the GPU idle for "
                         "seconds; measured: the first few hundred launches after that run up to 5%% slower); part "
                         "of set-up, never timed, stated in the JSON line")
    ap.add_argument("--also-warmup", type=int, default=200,
                    help="untimed launches before each --also workload (at least --warmup): the matrix-heavy kernels run "
                         "several percent slower until the clocks have settled after an idle period")
    return ap.parse_args()


def upload(w, torch):
    """Copy one workload to the GPU.  q, k, v and the output y of a buffer set are carved back to back out
    of ONE allocation: measured on MI355X, four separately allocated 1 GiB tensors ran the long-context
    kernel ~7% slower than the same tensors laid out contiguously."""
    d = {}
    n_bytes = w["q"].numel() * w["q"].element_size()
    arena = torch.empty(4 * n_bytes, dtype=torch.uint8, device="cuda")
    d["_arena"] = arena
    for i, key in enumerate(("q", "k", "v", "y")):
        t = arena[i * n_bytes:(i + 1) * n_bytes].view(w["q"].dtype).view(w["q"].shape)
        if key != "y":
            t.copy_(w[key])
        d[key] = t
    for key in ("h", "hq", "hk", "hv", "R", "lam"):
        if key in w:
            d[key] = torch.from_numpy(w[key]).cuda()
    return d


class Workload:
    """Device-resident rotating buffer sets plus the pre-marshalled launches of one configuration."""

    def __init__(self, name, nsets, torch, pkg, synth, seq_len=0, depth=0, batch=0, width=0):
        self.name, self.torch, self.pkg = name, torch, pkg
        self.overlap = name.endswith("_overlap")   # shards split into an interior call and a boundary call
        name = name[:-8] + "_shards" if self.overlap else name
        self.shards = 4 if name.endswith("_shards") else 0
        name = name[:-7] if self.shards else name
        self.bwd = name.endswith("_bwd")
        self.feat = name.endswith("_feat")   # the three featurizer convolutions of the chain alone
        name = name[:-5] if self.feat else name
        self.strip, self.ywaves, ydepth = YARDSTICKS.get(name, (None, 0, 0))
        depth = depth or ydepth
        name = name[:-4] if self.bwd else name
        over = {"L": seq_len} if seq_len > 0 else {}
        if batch > 0:
            over["B"] = batch
        if width > 0:
            over["D"] = width
        if self.strip is not None:
            name = "c1"  # the yardsticks run on c1's tensors (its filter is not used)
        self.cfg = synth.config(name, **over)
        c = self.cfg
        self.n_out = c["B"] * c["L"] * c["D"]
        self.tokens = c["B"] * c["L"]
        bytes_set = self.n_out * 2 * (8 if self.bwd else 4)
        if nsets <= 0:
            nsets = max(1, min(6, int((1.5 * 2 ** 30) // bytes_set) + 1))
        self.host0 = None
        self.sets, self.main = [], []
        for i in range(nsets):
            w = synth.make(name, variant=i, **over)
            if i == 0:
                self.host0 = w
            d = upload(w, torch)
            if self.bwd:
                # dy is drawn like the activations; dq, dk, dv share one more allocation
                rng = np.random.Generator(np.random.PCG64(synth.seed_for(name, i) + 500000))
                dy_host = synth.normal_tensor(rng, tuple(d["q"].shape), c["dtype"])
                if i == 0:
                    self.host0["dy"] = dy_host
                d["dy"] = dy_host.cuda()
                grads = torch.empty((3,) + tuple(d["q"].shape), dtype=d["q"].dtype, device="cuda")
                d["dq"], d["dk"], d["dv"] = grads[0], grads[1], grads[2]
                d["dh"] = torch.empty_like(d["h"])
                if c["kind"] == "chain":
                    d["dhf"] = [torch.empty_like(d["hq"]) for _ in range(3)]
                    self.main.append(pkg.plan_chain_bwd(d["dy"], d["q"], d["k"], d["v"], d["hq"], d["hk"], d["hv"], d["h"],
                                                        c["group"], c["feat_group"],
                                                        out=(d["dq"], d["dk"], d["dv"]) + tuple(d["dhf"]) + (d["dh"],)))
                elif self.shards:
                    # the sequence as consecutive shard calls: lh - 1 rows of k, v before and of dy, q behind each
                    # shard; every call leaves its share of dh in a buffer of its own
                    entry = "hyena_se_bwd_shard" if c["kind"] == "se" else "hyena_mr_bwd_shard"
                    n = c["L"] // self.shards
                    d["dh_parts"] = [torch.empty_like(d["h"]) for _ in range(self.shards)]
                    plans = []
                    for i in range(self.shards):
                        w = slice(i * n, (i + 1) * n)
                        plans.append(pkg.plan_bwd_shard(entry, d["dy"][:, w], d["q"][:, w], d["k"][:, w], d["v"][:, w],
                                                        d["h"], c["group"], min(i * n, c["lh"] - 1),
                                                        min(c["L"] - (i + 1) * n, c["lh"] - 1),
                                                        out=(d["dq"][:, w], d["dk"][:, w], d["dv"][:, w],
                                                             d["dh_parts"][i])))
                    self.main.append(lambda plans=plans: [p() for p in plans])
                else:
                    self.main.append(pkg.plan_bwd("hyena_se_bwd" if c["kind"] == "se" else "hyena_mr_bwd", d["dy"], d["q"],
                                                  d["k"], d["v"], d["h"], c["group"],
                                                  out=(d["dq"], d["dk"], d["dv"], d["dh"])))
            elif self.strip is not None:
                self.main.append(pkg.plan_stream_gate(d["q"], d["k"], d["v"], self.strip, 0, depth, self.ywaves,
                                                      out=d["y"]))
            elif self.feat:
                d["feat_out"] = tuple(torch.empty_like(d["q"]) for _ in range(3))
                self.main.append(pkg.plan_featurize3(d["q"], d["k"], d["v"], d["hq"], d["hk"], d["hv"], c["feat_group"],
                                                     out=d["feat_out"]))
            elif c["kind"] == "li":
                self.main.append(pkg.plan_li(d["q"], d["k"], d["v"], d["R"], d["lam"], c["group"], out=d["y"]))
            elif c["kind"] == "chain":
                self.main.append(pkg.plan_chain(d["q"], d["k"], d["v"], d["hq"], d["hk"], d["hv"], d["h"],
                                                c["group"], c["feat_group"], out=d["y"]))
            elif self.shards:
                # the sequence as `shards` consecutive shard calls, each with the lh - 1 rows before it as history
                entry = "hyena_se_fwd_shard" if c["kind"] == "se" else "hyena_mr_fwd_shard"
                n = c["L"] // self.shards
                def shard(t0, t1):
                    w = slice(t0, t1)
                    return pkg.plan_gated_shard(entry, d["q"][:, w], d["k"][:, w], d["v"][:, w], d["h"], c["group"],
                                                min(t0, c["lh"] - 1), out=d["y"][:, w])

                H = c["lh"] - 1
                plans = []
                for i in range(self.shards):
                    if self.overlap and i > 0:
                        # what a rank does to hide the exchange: the steps at least lh - 1 in first (their history is
                        # the shard's own rows), the lh - 1 steps next to the cut once the halo is there
                        plans += [shard(i * n + H, (i + 1) * n), shard(i * n, i * n + H)]
                    else:
                        plans.append(shard(i * n, (i + 1) * n))
                self.main.append(lambda plans=plans: [p() for p in plans])
            else:
                entry = "hyena_se_fwd" if c["kind"] == "se" else "hyena_mr_fwd"
                self.main.append(pkg.plan_gated(entry, d["q"], d["k"], d["v"], d["h"], c["group"], out=d["y"]))
            self.sets.append(d)
        self.i = 0

    def step(self):
        j = self.i % len(self.sets)
        self.i += 1
        self.main[j]()

    def run(self, steps, warmup, settle=0):
        """Returns (wall seconds for `steps` steps, average duration in ms of the dominant kernel)."""
        torch = self.torch
        ev = torch.cuda.Event
        for _ in range(settle):  # set-up: brings the clocks out of idle (see --settle)
            self.step()
        torch.cuda.synchronize()
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        # bracket the whole timed region with two events on the launch stream; (elapsed / steps) is the average
        # launch period of the entry point's kernel(s), an upper bound of their duration
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            self.step()
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) / steps

    def launch_stats(self, n=60):
        """Outside the timed region: an event pair around every one of n launches rotating through the buffer
        sets (median and minimum duration), then n launches on buffer set 0 alone, which is the cache-warm
        figure where one set fits the 256 MB memory-side cache.  Microseconds."""
        torch = self.torch
        ev = torch.cuda.Event

        def series(pick):
            pairs = [(ev(enable_timing=True), ev(enable_timing=True)) for _ in range(n)]
            for i, (a, b) in enumerate(pairs):
                j = pick(i)
                a.record()
                self.main[j]()
                b.record()
            torch.cuda.synchronize()
            return sorted(1e3 * a.elapsed_time(b) for a, b in pairs)

        rot = series(lambda i: i % len(self.sets))
        same = series(lambda i: 0)
        return {"unit": "us", "launches": n, "median": rot[n // 2], "min": rot[0],
                "same_buffers_median": same[n // 2], "same_buffers_min": same[0]}

    # algorithmic work of the dominant kernel per launch
    def algo_bytes(self):
        if self.feat:
            return 12.0 * self.n_out  # bf16: three tensors read once and written once
        if self.bwd:
            return 14.0 * self.n_out  # bf16: dy, q, k, v read once, dq, dk, dv written once
        return 8.0 * self.n_out  # bf16: q, k, v read once, y written once

    def algo_flops(self):
        if self.cfg["kind"] == "li":
            # recurrent form: per exponential one FMA for the running sum and one for the output, plus two gates
            return (4.0 * self.cfg["order"] + 2.0) * self.n_out
        if self.feat:
            return 3 * 2.0 * self.cfg["lf"] * self.n_out
        f = 2.0 * self.cfg["lh"] + 2.0
        if self.bwd:
            f = 3 * 2.0 * self.cfg["lh"] + 5.0  # z, du, dh contractions + five gates
            if self.cfg["kind"] == "chain":
                f += 3 * 3 * 2.0 * self.cfg["lf"]  # per featurizer: the recomputed forward, dx and its filter gradient
            return f * self.n_out
        if self.cfg["kind"] == "chain":
            f += 3 * 2.0 * self.cfg["lf"]
        return f * self.n_out


def cpu_baseline(wl, target_s, np, oracle):
    """Time the fp64 oracle as it stands on a bounded slice of buffer set 0 (all channels, the first rows
    of batch item 0), sized for about target_s seconds; a slice that finishes sooner is repeated."""
    w, c = wl.host0, wl.cfg
    L = c["L"]

    def run(rows):
        q, k, v = (w[key][:1, :rows].contiguous() for key in ("q", "k", "v"))
        t0 = time.perf_counter()
        if wl.feat:
            y = oracle.causal_conv(q, w["hq"], c["feat_group"])
        elif wl.bwd:
            # dq[t] only looks at the past, so the first rows of the slice's dq equal those of the full problem
            dy = w["dy"][:1, :rows].contiguous()
            if c["kind"] == "chain":
                # ... except for the last lf - 1 rows, which the featurizer's transpose reaches past
                y = oracle.chain_bwd(dy, q, k, v, w["hq"], w["hk"], w["hv"], w["h"], group=c["group"],
                                     feat_group=c["feat_group"])[0][:, :max(rows - (c["lf"] - 1), 1)]
            else:
                y = oracle.gated_conv_bwd(dy, q, k, v, w["h"], group=c["group"])[0]
        elif c["kind"] == "li":
            y = oracle.li_conv(q, k, v, w["R"], w["lam"], group=c["group"])
        elif c["kind"] == "chain":
            y = oracle.chain(q, k, v, w["hq"], w["hk"], w["hv"], w["h"], group=c["group"], feat_group=c["feat_group"])
        else:
            y = oracle.gated_conv(q, k, v, w["h"], group=c["group"])
        return time.perf_counter() - t0, y

    probe_rows = min(L, 128)
    t_probe, _ = run(probe_rows)
    grow = target_s / max(t_probe, 1e-4)
    if c["kind"] == "li":
        grow = grow ** 0.5  # the filter is as long as the slice: the oracle's work grows with rows squared
    rows = int(min(L, max(probe_rows, probe_rows * grow)))
    t, y = run(rows)
    times = [t]
    while sum(times) < 0.8 * target_s and len(times) < 200:
        times.append(run(rows)[0])
    t_avg = sum(times) / len(times)
    return {
        "value": rows / t_avg, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "first %d of %d time steps of batch item 0, all %d channels, fp64, %d run(s) of %.2f s" % (
            rows, L, c["D"], len(times), t_avg),
    }, rows, y


def gpu_clocks():
    """Current shader and memory clock as the driver's sysfs tables mark them (None where unreadable)."""
    import glob

    out = {}
    for key, pat in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk")):
        out[key] = None
        for path in sorted(glob.glob("/sys/class/drm/card*/device/" + pat)):
            try:
                with open(path) as f:
                    marked = [ln.split(":", 1)[1].replace("*", "").strip() for ln in f if ln.rstrip().endswith("*")]
            except OSError:
                continue
            if marked:
                out[key] = marked[0]
                break
    return out


def stored_traffic(workload, seq_len):
    """HBM bytes per step as hardware counters saw them in an EARLIER profiled run of this workload (this run takes
    no counters): (bytes or None, where the figure comes from)."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if seq_len > 0 or not os.path.exists(path):
        return None, None
    with open(path) as f:
        entry = json.load(f).get(workload)
    if not entry:
        return None, None
    return entry.get("bytes_per_launch"), ("stored: %s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                           "workload, scaled by the copy-kernel calibration; see profiles/%s)"
                                           % (TRAFFIC_FILE, entry.get("profile", "")))


def entry_point(wl):
    if wl.strip is not None:
        return "hyena_stream_gate (strip_channels=%d, waves=%d)" % (wl.strip, wl.ywaves or wl.strip // 16)
    if wl.feat:
        return "hyena_featurize3_fwd"
    name = {"se": "hyena_se_fwd", "mr": "hyena_mr_fwd", "chain": "hyena_chain_fwd",
            "li": "hyena_li_fwd (both passes of the scan)"}[wl.cfg["kind"]]
    if wl.bwd:
        name = name.replace("_fwd", "_bwd")
    if wl.shards:
        if wl.overlap:
            return "%s_shard x %d (consecutive shards, each after the first as an interior and a boundary call)" % (
                name, 2 * wl.shards - 1)
        return "%s_shard x %d (the sequence in consecutive shards, one call each)" % (name, wl.shards)
    return name + " (all launches of the entry point)" if wl.bwd else name


def measure(name, args, torch, pkg, synth, steps, warmup, settle=0):
    """Times one workload; returns it with the figures every line and every "also" entry carries."""
    wl = Workload(name, args.sets, torch, pkg, synth, args.seq_len, args.depth, args.batch, args.width)
    wall, kern_ms = wl.run(steps, warmup, settle)
    ms_step = 1e3 * wall / steps
    gbs = wl.algo_bytes() / (kern_ms * 1e-3) / 1e9
    traffic, source = stored_traffic(name, args.seq_len if args.batch <= 0 and args.width <= 0 else 1)
    res = {
        "tokens_per_s": wl.tokens * steps / wall, "ms_per_step": ms_step, "steps": steps, "warmup": warmup,
        "settle_launches_before_warmup": settle, "buffer_sets": len(wl.sets),
        "roofline": {"bound": "hbm", "kernel": entry_point(wl), "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
                     "kernel_ms_avg": kern_ms, "algorithmic_bytes_per_launch": wl.algo_bytes(),
                     # the same fraction from the wall clock of the timed region (launch overhead included)
                     "frac_wall_clock": wl.algo_bytes() / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if wl.cfg["kind"] != "se" and wl.strip is None and not wl.feat:
        tf = wl.algo_flops() / (kern_ms * 1e-3) / 1e12
        res["mfma"] = {"tflops_algorithmic": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": tf / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops_per_launch": wl.algo_flops()}
    return wl, res


def calibrate_copy(args, torch, pkg):
    """Plain copy of known size for scaling the rocprofv3 byte counters: 128 MiB read + 128 MiB written."""
    n = 128 * 2 ** 20
    src = [torch.empty(n, dtype=torch.uint8, device="cuda").random_() for _ in range(6)]
    dst = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(6)]
    for i in range(args.warmup + args.steps):
        pkg.hyena_stream_copy(src[i % 6], dst[i % 6])
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "hyena_stream_copy", "bytes_read_per_launch": n, "bytes_written_per_launch": n,
                      "launches": args.warmup + args.steps}), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one MI355X; --gpus %d is not supported (this build has no multi-GPU path)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2503_01868_amd as pkg
    from paper_2503_01868_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    for item in args.opt:
        name, value = item.split("=")
        pkg.set_option(name, int(value))
    if args.workload == "copy":
        calibrate_copy(args, torch, pkg)
        return

    wl, res = measure(args.workload, args, torch, pkg, synth, args.steps, args.warmup, args.settle)
    cfg = wl.cfg
    what = "bandwidth yardstick y=q*k*v," if wl.strip is not None else "three featurizer convolutions," if wl.feat else {
        "se": "Hyena-SE", "mr": "Hyena-MR", "chain": "featurizers + Hyena-MR, one kernel,", "li": "Hyena-LI"}[cfg["kind"]]
    out = {
        "metric": METRIC, "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s%s bf16 B=%d L=%d D=%d %s=%d group=%d" % (
            args.workload, what, " backward" if wl.bwd else "",
            cfg["B"], cfg["L"], cfg["D"], "order" if cfg["kind"] == "li" else "lf" if wl.feat else "lh",
            cfg["order"] if cfg["kind"] == "li" else cfg["lf"] if wl.feat else cfg["lh"],
            cfg["feat_group"] if wl.feat else cfg["group"]), "buffer_sets": res["buffer_sets"],
            "settle_launches_before_warmup": args.settle},
        "roofline": res["roofline"],
    }
    out["launch_stats"] = wl.launch_stats()
    out["launch_stats"]["clocks_after_run"] = gpu_clocks()
    if "mfma" in res:
        out["mfma"] = res["mfma"]

    if not args.no_cpu_baseline and wl.strip is None:
        import oracle

        base, rows, y_ref = cpu_baseline(wl, args.cpu_seconds, np, oracle)
        out["cpu_baseline"] = base
        # the slice the oracle just computed doubles as an end-of-run parity check of buffer set 0
        d = wl.sets[0]
        wl.i = 0
        wl.step()
        torch.cuda.synchronize()
        out0 = d["feat_out"][0] if wl.feat else (d["dq"] if wl.bwd else d["y"])
        got = out0[:1, :y_ref.shape[1]].float().cpu().numpy().astype(np.float64)
        out["parity_rel_err"] = oracle.rel_err(got, y_ref)

    if args.workload == "c1" and args.also and args.seq_len <= 0 and args.batch <= 0 and args.width <= 0:
        del wl
        torch.cuda.empty_cache()
        out["also"] = {}
        for name in [s for s in args.also.split(",") if s]:
            wl2, r2 = measure(name, args, torch, pkg, synth, max(10, args.steps // 4), max(args.also_warmup, args.warmup))
            out["also"][name] = r2
            del wl2
            torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
