#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic activations:
every tensor of the workload is compressed in forward order, then every
container is decompressed in reverse order, all on ONE stream (the forward /
backward pattern of Section 4.4 of the paper, as the benchmark configuration
states it).  Inputs are resident in HBM before the timed region starts.
Prints ONE JSON line.

  value      = fp32 bytes compressed + fp32 bytes decompressed, per second (GB/s)
  roofline   = the kernel with the largest share of the step: its algorithmic
               HBM bytes per second against the 8 TB/s peak, durations measured
               with HIP events around each of its launches on the stream it runs
               on (a second pass over the same steps, so that the events do not
               perturb `value`)
  cpu_baseline = the CPU oracle, one core, on a bounded sample of the workload;
               the same leg compares the oracle's containers and reconstructions
               with the GPU's, byte for byte (`parity_checked_tensors`)

The whole workload is one cmp_compress_batch call and one cmp_decompress_batch
call per step (--api single: one call per tensor).

Extra keys (context, not the headline): `multi_stream` (single calls dealt over
several streams), `sparse_variant` (the 85 %-zeros variant of the workload, also
with the sparsity-aware front end), `other_configs` (the single-tensor
configurations).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# Algorithmic HBM bytes per element of each kernel (cbar = compressed bytes per element,
# measured): what the kernel must read and write once if nothing is re-read.
KERNEL_BYTES = {
    "k_quant_lorenzo_split_hist": lambda cbar: 4.0 + 2.0,      # read x, write u16 symbols
    "k_encode": lambda cbar: 2.0 + cbar,                       # read symbols, write container payload
    "k_lengths": lambda cbar: 2.0,                             # read symbols (bit counts are 1/16 byte per element)
    "k_pack": lambda cbar: 2.0 + cbar,                         # read symbols, write container payload
    "k_decode_fused": lambda cbar: cbar + 4.0,                 # read container, write fp32
    "k_decode": lambda cbar: cbar + 4.0,                       # unfused path: read payload, write int32 residuals
    "k_row_scan": lambda cbar: 8.0,
    "k_col_scan_dequant": lambda cbar: 8.0,
}

# HBM bytes per element actually moved, from rocprofv3 FETCH_SIZE / WRITE_SIZE counters scaled by a
# plain copy of known size (the named file under profiles/ has the commands and the readings).
# Counters cannot be read from inside this process, so the figures are only reported for the
# configuration they were measured on, with the date of that measurement.
MEASURED_TRAFFIC = {
    ("cfg5_resnet18_stream", 32, 1e-2): {
        "profile": "profiles/hbm_traffic_cfg5_resnet18_stream.txt",
        "per_elem": {
            "k_quant_lorenzo_split_hist": 4.0178 + 1.0509,     # 8-bit symbols in the scratch
            "k_lengths": 1.0088 + 0.0672,
            "k_pack": 1.0138 + 0.6639,
            "k_decode_fused": 0.8330 + 4.0086,
        },
        # vector instructions per element and the fraction of the kernel's time its vector units are busy
        # (profiles/instruction_counters_cfg5_resnet18_stream.txt)
        "valu": {
            "k_quant_lorenzo_split_hist": (26.48, 0.688),
            "k_lengths": (2.98, 0.355),
            "k_pack": (12.27, 0.831),
            "k_decode_fused": (46.83, 0.829),
        },
    },
}
ALU_PEAK_LANE_INST_PER_S = 256 * 4 * 16 * 2.4e9       # CUs x SIMDs x lanes x clock: 39.3 T lane-instructions/s


class Run:
    """One workload resident on the GPU: inputs, containers, outputs, contexts."""

    def __init__(self, binding, torch, wl, eb, sub, nstreams, dev, api="batch", zero_blocks=0):
        self.b, self.torch, self.wl, self.eb, self.sub = binding, torch, wl, eb, sub
        self.api = api if nstreams == 1 else "single"          # batches are one call on one stream
        self.xs = [wl.tensor(i, device=dev) for i in range(len(wl.shapes))]
        self.numels = [x.numel() for x in self.xs]
        self.total = sum(self.numels)
        S = self.S = max(1, min(nstreams, len(self.xs)))
        if self.api == "batch":
            self.ctxs = [binding.Context(sub=sub, max_numel=self.total, zero_blocks=zero_blocks)]
        else:
            self.ctxs = [binding.Context(sub=sub, max_numel=max(self.numels[k::S]), zero_blocks=zero_blocks) for k in range(S)]
        self.bounds = [self.ctxs[0].bound(x.shape) for x in self.xs]
        self.arena = [torch.empty(b, dtype=torch.uint8, device=dev) for b in self.bounds]
        self.outs = [torch.empty_like(x) for x in self.xs]
        # default-priority streams; with one stream, torch's current one
        self.tstreams = [torch.cuda.current_stream(dev)] if S == 1 else [torch.cuda.Stream(dev) for _ in range(S)]
        self.streams = [t.cuda_stream for t in self.tstreams]
        self.order = list(range(len(self.xs)))

    def compress_all(self, stream=None):
        b, S = self.b, self.S
        if self.api == "batch":
            rc, _ = b.cmp_compress_batch(self.ctxs[0]._h, [x.data_ptr() for x in self.xs], [x.shape for x in self.xs],
                                         [self.eb] * len(self.xs), [a.data_ptr() for a in self.arena],
                                         [a.numel() for a in self.arena], False, self.streams[0])
            assert rc == 0, b.cmp_strerror(rc)
            return
        for i in self.order:
            x, buf = self.xs[i], self.arena[i]
            rc, _ = b.cmp_compress(self.ctxs[i % S]._h, x.data_ptr(), x.shape, self.eb, buf.data_ptr(), buf.numel(),
                                   False, self.streams[i % S])
            assert rc == 0, b.cmp_strerror(rc)

    def decompress_all(self):
        b, S = self.b, self.S
        if self.api == "batch":
            rev = list(reversed(self.order))
            rc = b.cmp_decompress_batch(self.ctxs[0]._h, [self.arena[i].data_ptr() for i in rev],
                                        [self.bounds[i] for i in rev], [self.xs[i].shape for i in rev],
                                        [self.eb] * len(rev), [self.outs[i].data_ptr() for i in rev], self.streams[0])
            assert rc == 0, b.cmp_strerror(rc)
            return
        for i in reversed(self.order):
            rc = b.cmp_decompress(self.ctxs[i % S]._h, self.arena[i].data_ptr(), self.bounds[i], self.xs[i].shape,
                                  self.eb, self.outs[i].data_ptr(), self.streams[i % S])
            assert rc == 0, b.cmp_strerror(rc)

    def step(self):
        self.compress_all()
        self.decompress_all()

    def check(self):
        """After at least one step: status words, container sizes, the error bound."""
        torch = self.torch
        torch.cuda.synchronize()
        for c in self.ctxs:
            st = c.last_status(self.streams[0])
            assert st == 0, self.b.cmp_strerror(st)
        self.sizes, self.outliers = [], 0
        for buf in self.arena:
            rc, size = self.ctxs[0].compressed_size(buf)
            assert rc == 0
            self.sizes.append(size)
            self.outliers += int(buf[60:64].cpu().numpy().view("<u4")[0])      # header field n_outliers
        self.comp_bytes = sum(self.sizes)
        self.cbar = self.comp_bytes / self.total
        worst = 0.0
        for x, out in zip(self.xs, self.outs):
            worst = max(worst, float((x.double() - out.double()).abs().max()))
        assert worst <= float(torch.tensor(self.eb, dtype=torch.float32)), worst
        self.max_abs_err = worst

    def time_steps(self, steps):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def time_graph(self, steps):
        """One step captured into a HIP graph (the calls allocate nothing and never wait), replayed."""
        torch = self.torch
        assert self.api == "batch"
        side = torch.cuda.Stream(self.xs[0].device)          # default priority
        saved = self.streams
        self.streams = [side.cuda_stream]
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step()                                      # once eagerly on the capturing stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            self.step()
        self.streams = saved
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        self.check()                                         # what the replays left is a valid round trip
        return ms

    def time_phases(self, steps):
        """Per-phase times (host clock, a device-wide wait after each phase)."""
        torch = self.torch
        tc = td = 0.0
        for _ in range(steps):
            a = time.perf_counter(); self.compress_all(); torch.cuda.synchronize()
            b = time.perf_counter(); self.decompress_all(); torch.cuda.synchronize()
            c = time.perf_counter()
            tc += (b - a) * 1e3; td += (c - b) * 1e3
        return tc / steps, td / steps

    def kernel_times(self, steps):
        """Events around every launch, all calls on stream 0, back to back."""
        for c in self.ctxs:
            c.profile(True)
        S0 = self.streams[0]
        b = self.b
        for _ in range(steps):
            if self.api == "batch":
                self.compress_all()
            for i in (self.order if self.api != "batch" else []):
                rc, _ = b.cmp_compress(self.ctxs[i % self.S]._h, self.xs[i].data_ptr(), self.xs[i].shape, self.eb,
                                       self.arena[i].data_ptr(), self.arena[i].numel(), False, S0)
                assert rc == 0, b.cmp_strerror(rc)
            if self.api == "batch":
                self.decompress_all()
            for i in (reversed(self.order) if self.api != "batch" else []):
                rc = b.cmp_decompress(self.ctxs[i % self.S]._h, self.arena[i].data_ptr(), self.bounds[i],
                                      self.xs[i].shape, self.eb, self.outs[i].data_ptr(), S0)
                assert rc == 0, b.cmp_strerror(rc)
        self.torch.cuda.synchronize()
        kern = {}
        for c in self.ctxs:
            for name, (ms, launches) in c.profile_read(S0).items():
                e = kern.setdefault(name, {"ms": 0.0, "launches": 0})
                e["ms"] += ms; e["launches"] += launches
            c.profile(False)
        return {name: {"ms_per_step": e["ms"] / steps, "launches_per_step": e["launches"] // steps,
                       "avg_us": 1e3 * e["ms"] / e["launches"]} for name, e in kern.items()}

    def summary(self, ms_per_step, tc, td):
        total = self.total
        return {"ms_per_step": round(ms_per_step, 4), "GBps": round(2 * 4.0 * total / (ms_per_step * 1e-3) / 1e9, 2),
                "compress_ms": round(tc, 4), "decompress_ms": round(td, 4),
                "compress_GBps": round(4.0 * total / (tc * 1e-3) / 1e9, 2),
                "decompress_GBps": round(4.0 * total / (td * 1e-3) / 1e9, 2),
                "compression_ratio": round(4.0 * total / self.comp_bytes, 4),
                "compressed_bytes_held": self.comp_bytes, "outliers": self.outliers,
                "hbm_frac_algorithmic": round((12.0 + 2 * self.cbar) * total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}

    def free(self):
        for c in self.ctxs:
            c.close()
        self.xs = self.arena = self.outs = self.ctxs = None
        self.torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (ten steps give the same figure to within 0.3 %; a hundred keep the timed region at 0.2 s)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5_resnet18_stream")
    ap.add_argument("--eb", type=float, default=None)
    ap.add_argument("--sub", type=int, default=32, help="codes per sub-block (decode parallelism vs. 16 bits of metadata each)")
    ap.add_argument("--streams", type=int, default=1,
                    help="streams of the headline schedule (the benchmark configuration says one)")
    ap.add_argument("--extra-streams", type=int, default=6, help="streams of the `multi_stream` extra (0 = skip)")
    ap.add_argument("--api", default="batch", choices=["batch", "single"],
                    help="batch: one cmp_compress_batch call per step (one launch per stage over all tensors); "
                         "single: one cmp_compress call per tensor")
    ap.add_argument("--no-extras", action="store_true", help="skip sparse_variant and other_configs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of tensor 0 (numel*4 bytes read and written): "
                         "the known traffic against which hardware counter readings are scaled")
    ap.add_argument("--cpu-sample", type=int, default=2, help="tensors of the workload the oracle is timed on and compared with")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; the path shards with no communication "
              "(see DESIGN.md), so only --gpus 1 is measured", file=sys.stderr)
        return 2

    import torch
    from paper_2011_09017_amd import binding
    from paper_2011_09017_amd.workloads import WORKLOADS

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    binding.lib()                                    # fails loudly if libcmpz.so is missing
    wl = WORKLOADS[args.workload]
    eb = args.eb if args.eb is not None else wl.ebs[0]
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    run = Run(binding, torch, wl, eb, args.sub, args.streams, dev, args.api)
    run.step()
    run.check()                                      # (reads sizes and status back: the GPU idles meanwhile)
    if args.calib_copy:
        run.outs[0].copy_(run.xs[0])
        torch.cuda.synchronize()
    # the warm-up steps run right before the timed ones: after some milliseconds without work the
    # GPU's clocks are down, and the first steps behind such a pause take about a millisecond more
    for _ in range(args.warmup):
        run.step()

    # ---- timed region: exactly K steps -------------------------------------------------
    ms_per_step = run.time_steps(args.steps)
    tc, td = run.time_phases(args.steps)
    kern = run.kernel_times(args.steps)
    total, cbar = run.total, run.cbar

    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    bytes_fn = KERNEL_BYTES.get(dom)
    roofline = None
    if bytes_fn is not None:
        alg_bytes_step = bytes_fn(cbar) * total                 # over all launches of one step
        achieved = alg_bytes_step / (kern[dom]["ms_per_step"] * 1e-3) / 1e9
        meas = MEASURED_TRAFFIC.get((wl.name, args.sub, eb), {})
        per_elem = meas.get("per_elem", {}).get(dom)
        # measured HBM bytes per launch (average over the launches of a step), like `achieved`
        traffic = round(per_elem * total / kern[dom]["launches_per_step"]) if per_elem else None
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                    "traffic_source": meas.get("profile") if per_elem else None,
                    "alg_bytes_per_launch": round(alg_bytes_step / kern[dom]["launches_per_step"]),
                    "alg_bytes_per_elem": round(bytes_fn(cbar), 4),
                    "avg_launch_us": round(kern[dom]["avg_us"], 2),
                    "launches_per_step": kern[dom]["launches_per_step"]}
        valu = meas.get("valu", {}).get(dom)
        if valu:
            # context, not the bound reported: what the kernel's vector instructions alone would take
            roofline["alu"] = {"valu_inst_per_elem": valu[0], "valu_busy": valu[1],
                               "floor_us": round(valu[0] * total / kern[dom]["launches_per_step"] / ALU_PEAK_LANE_INST_PER_S * 1e6, 1),
                               "source": "profiles/instruction_counters_cfg5_resnet18_stream.txt"}

    # what a plain device copy of the largest tensor reaches on this machine (bytes read + written)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    run.outs[0].copy_(run.xs[0])
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(5):
        run.outs[0].copy_(run.xs[0])
    ev[1].record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * 4.0 * run.numels[0] / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9

    # the error-bound estimator (Sections 4.1-4.3; it runs every W = 1000 iterations, so it is not
    # part of a step): one streaming pass over an activation, a loss of the same shape and a momentum
    ctl_ctx = run.ctxs[0]
    mom = run.xs[-1].reshape(-1)[: 512 * 512 * 9].contiguous()
    ctl_ctx.estimate_eb(run.xs[0], run.outs[0], mom)
    ctl_ctx.profile(True)
    for _ in range(5):
        rc_ctl, eb_ctl, st_ctl = ctl_ctx.estimate_eb(run.xs[0], run.outs[0], mom)
    ctl_ms, ctl_n = ctl_ctx.profile_read()["k_controller_stats"]
    ctl_ctx.profile(False)
    ctl_bytes = 4.0 * (2 * run.numels[0] + mom.numel())
    ctl_gbps = ctl_bytes / (ctl_ms / ctl_n * 1e-3) / 1e9

    value = 2 * 4.0 * total / (ms_per_step * 1e-3) / 1e9
    head = run.summary(ms_per_step, tc, td)
    result = {
        "metric": "compress+decompress GB/s of fp32 activations (frac. of HBM peak); compression ratio",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32 quantiser, i32/bit codec", "data": "synthetic",
        "config": {"workload": wl.name, "tensors": len(run.xs), "numel": total, "eb": eb, "radius": 512,
                   "chunk": 4096, "sub": args.sub, "streams": run.S, "api": run.api, "schedule": "compress all in forward order, "
                   "then decompress all in reverse order", "p_zero": wl.p_zero, "box_k": wl.k,
                   "seed_base": wl.seed(0)},
        "compression_ratio": head["compression_ratio"],
        "compressed_bytes_held": head["compressed_bytes_held"],
        "compress_ms": head["compress_ms"], "decompress_ms": head["decompress_ms"],
        "compress_GBps": head["compress_GBps"], "decompress_GBps": head["decompress_GBps"],
        "hbm_frac_algorithmic": head["hbm_frac_algorithmic"],
        "payload_frac_of_peak": round(value / HBM_PEAK_GBPS, 4),
        "copy_ceiling_GBps": round(copy_gbps, 1),
        "controller": {"kernel": "k_controller_stats", "bound": "hbm", "achieved": round(ctl_gbps, 1),
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ctl_gbps / HBM_PEAK_GBPS, 4),
                       "avg_launch_us": round(1e3 * ctl_ms / ctl_n, 2), "alg_bytes_per_launch": int(ctl_bytes),
                       "eb": eb_ctl, "R": st_ctl[0]},
        "max_abs_err": run.max_abs_err,
        "kernels": {k: {kk: round(vv, 3) for kk, vv in v.items()} for k, v in kern.items()},
        "roofline": roofline,
    }

    # ---- CPU baseline: the oracle as it stands, one core, bounded sample; and parity ---------
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        run.step()
        torch.cuda.synchronize()
        n_s, t_c, t_d, checked = 0, 0.0, 0.0, 0
        for i in range(min(args.cpu_sample, len(run.xs))):
            xh = run.xs[i].cpu().numpy()
            a = time.perf_counter()
            rc, obuf, osize, _ = oracle.compress(xh, eb, oracle.Config(sub=args.sub))
            b = time.perf_counter()
            rc2, oy = oracle.decompress(obuf, xh.shape, eb, oracle.Config(sub=args.sub))
            c = time.perf_counter()
            assert rc == 0 and rc2 == 0
            n_s += xh.size; t_c += b - a; t_d += c - b
            # parity of what was timed: container and reconstruction, byte for byte
            assert osize == run.sizes[i], (i, osize, run.sizes[i])
            assert np.array_equal(run.arena[i][:osize].cpu().numpy(), obuf), f"container {i} differs from the oracle"
            assert np.array_equal(run.outs[i].cpu().numpy().view(np.uint32), oy.view(np.uint32)), \
                f"reconstruction {i} differs from the oracle"
            checked += 1
        result["cpu_baseline"] = {
            "value": round(2 * 4.0 * n_s / (t_c + t_d) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {checked} tensors of {wl.name} ({n_s} elements), "
                      f"compress {t_c:.2f} s + decompress {t_d:.2f} s, host has {os.cpu_count()} cpus"}
        result["parity_checked_tensors"] = checked
    if not args.no_extras and run.api == "batch":
        g_ms = run.time_graph(args.steps)
        result["graph_replay"] = {"ms_per_step": round(g_ms, 4), "GBps": round(2 * 4.0 * total / (g_ms * 1e-3) / 1e9, 2),
                                  "what": "the same step (both batch calls) captured once into a HIP graph and replayed"}
    run.free()

    # ---- extras ------------------------------------------------------------------------
    def measure(wl2, eb2, nstreams, zero_blocks=0):
        r = Run(binding, torch, wl2, eb2, args.sub, nstreams, dev, args.api, zero_blocks)
        r.step()
        r.check()
        for _ in range(args.warmup):
            r.step()
        ms = r.time_steps(args.steps)
        c_ms, d_ms = r.time_phases(args.steps)
        out = r.summary(ms, c_ms, d_ms)
        out["streams"] = r.S
        r.free()
        return out

    if args.extra_streams > 1 and len(wl.shapes) > 1:
        result["multi_stream"] = measure(wl, eb, args.extra_streams)
    if not args.no_extras:
        sparse = WORKLOADS.get(wl.name + "_sparse")
        if sparse is not None:
            result["sparse_variant"] = dict(measure(sparse, eb, args.streams), workload=sparse.name, p_zero=sparse.p_zero)
            # the same with the sparsity-aware front end (container version 2)
            result["sparse_variant_zero_blocks"] = dict(measure(sparse, eb, args.streams, 1), workload=sparse.name,
                                                        p_zero=sparse.p_zero, container_version=2)
        others = {}
        for name in ("cfg2_vgg16_conv1_2", "cfg3_resnet50_bottleneck", "cfg4_alexnet_conv1"):
            for eb2 in WORKLOADS[name].ebs:
                others[f"{name}@eb={eb2:g}"] = measure(WORKLOADS[name], eb2, 1)
        result["other_configs"] = others
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
