#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic activations:
every tensor of the workload is compressed in forward order, then every
container is decompressed in reverse order (the forward / backward pattern of
Section 4.4 of the paper).  Tensor i is handled by context i mod S on stream
i mod S (--streams S): tensors are independent, so the serial parts of one
tensor's codec (codebook construction, kernel tails) overlap with the bulk
kernels of its neighbours, as they overlap with the layers' own kernels in
training.  Inputs are resident in HBM before the timed region starts.  Prints
ONE JSON line.

  value      = fp32 bytes compressed + fp32 bytes decompressed, per second (GB/s)
  roofline   = the kernel with the largest share of the step: its algorithmic
               HBM bytes per second against the 8 TB/s peak, durations measured
               with HIP events around each of its launches (a second pass over
               the same steps, one call at a time, so that the events do not
               perturb `value` and concurrent streams do not stretch a kernel)
  cpu_baseline = the CPU oracle, one core, on a bounded sample of the workload
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
    "k_decode_fused": lambda cbar: cbar + 4.0,                 # read container, write fp32
    "k_decode": lambda cbar: cbar + 4.0,                       # unfused path: read payload, write int32 residuals
    "k_row_scan": lambda cbar: 8.0,
    "k_col_scan_dequant": lambda cbar: 8.0,
}


# HBM bytes per element actually moved, from rocprofv3 FETCH_SIZE / WRITE_SIZE counters scaled by a
# plain copy of known size (profiles/hbm_traffic_cfg5_resnet18_stream.txt has the commands and the
# readings).  Counters cannot be read from inside this process, so the figures are only reported
# for the configuration they were measured on.
MEASURED_TRAFFIC = {
    ("cfg5_resnet18_stream", 32, 1e-2): {
        "k_quant_lorenzo_split_hist": 4.0121 + 2.0323,
        "k_encode": 2.0330 + 0.7218,
        "k_decode_fused": 0.8244 + 4.0115,
    },
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5_resnet18_stream")
    ap.add_argument("--eb", type=float, default=None)
    ap.add_argument("--sub", type=int, default=32, help="codes per sub-block (decode parallelism vs. 16 bits of metadata each)")
    ap.add_argument("--streams", type=int, default=6, help="contexts/streams the tensors are dealt over, round robin")
    ap.add_argument("--contexts", type=int, default=6, help="compress contexts (tensors in flight) of the pipelined schedule")
    ap.add_argument("--pipeline", action="store_true",
                    help="all first sweeps (cmp_compress_begin) on one stream and the codebook / second sweep "
                         "(cmp_compress_finish) of alternate tensors on two others, instead of whole cmp_compress "
                         "calls dealt round robin over the streams (measured: no faster, 3.55 against 3.45 ms)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of tensor 0 (numel*4 bytes read and written): "
                         "the known traffic against which hardware counter readings are scaled")
    ap.add_argument("--cpu-sample", type=int, default=2, help="tensors of the workload the oracle is timed on")
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

    xs = [wl.tensor(i, device=dev) for i in range(len(wl.shapes))]
    numels = [x.numel() for x in xs]
    total = sum(numels)
    S = max(1, min(args.streams, len(xs)))
    K = max(S, args.contexts) if args.pipeline and S >= 3 else S       # compress contexts (tensors in flight)
    ctxs = [binding.Context(sub=args.sub, max_numel=max(numels[k::K])) for k in range(K)]
    # decompression gets contexts of its own: calls of one context must not overlap, and in the
    # pipelined schedule a context's next compress may start while the last decompress still runs
    dctxs = [binding.Context(sub=args.sub, max_numel=max(numels[k::S])) for k in range(S)]
    bounds = [ctxs[0].bound(x.shape) for x in xs]
    arena = [torch.empty(b, dtype=torch.uint8, device=dev) for b in bounds]
    outs = [torch.empty_like(x) for x in xs]
    # default-priority streams; with one stream, torch's current one
    tstreams = [torch.cuda.current_stream(dev)] if S == 1 else [torch.cuda.Stream(dev) for _ in range(S)]
    streams = [t.cuda_stream for t in tstreams]
    order = list(range(len(xs)))

    pipeline = args.pipeline and S >= 3
    # pipelined forward pass: stream 0 runs every first sweep (cmp_compress_begin), streams 1 and 2
    # take the codebook and second sweep (cmp_compress_finish) of alternate tensors, so that the
    # one-workgroup codebook kernel of a tensor always has the first sweep of the next one beside it
    fin_ev = [None] * len(xs)                       # container i complete
    dec_ev = [None] * len(xs)                       # container i consumed by the last decompress
    ctx_free = [None] * K                           # last finish issued on context k

    def compress_all():
        if not pipeline:
            for i in order:
                x, buf = xs[i], arena[i]
                rc, _ = binding.cmp_compress(ctxs[i % K]._h, x.data_ptr(), x.shape, eb, buf.data_ptr(), buf.numel(),
                                             False, streams[i % S])
                assert rc == 0, binding.cmp_strerror(rc)
            return
        for i in order:
            k = i % K
            side = 1 + (i & 1)
            if ctx_free[k] is not None:
                tstreams[0].wait_event(ctx_free[k])
            rc = binding.cmp_compress_begin(ctxs[k]._h, xs[i].data_ptr(), xs[i].shape, eb, streams[0])
            assert rc == 0, binding.cmp_strerror(rc)
            began = torch.cuda.Event()
            began.record(tstreams[0])
            tstreams[side].wait_event(began)
            if dec_ev[i] is not None:
                tstreams[side].wait_event(dec_ev[i])
            rc, _ = binding.cmp_compress_finish(ctxs[k]._h, arena[i].data_ptr(), arena[i].numel(), False, streams[side])
            assert rc == 0, binding.cmp_strerror(rc)
            fin_ev[i] = torch.cuda.Event()
            fin_ev[i].record(tstreams[side])
            ctx_free[k] = fin_ev[i]

    def decompress_all():
        for i in reversed(order):
            x = xs[i]
            if pipeline:
                tstreams[i % S].wait_event(fin_ev[i])
            rc = binding.cmp_decompress(dctxs[i % S]._h, arena[i].data_ptr(), bounds[i], x.shape, eb,
                                        outs[i].data_ptr(), streams[i % S])
            assert rc == 0, binding.cmp_strerror(rc)
            if pipeline:
                dec_ev[i] = torch.cuda.Event()
                dec_ev[i].record(tstreams[i % S])

    def step():
        compress_all()
        decompress_all()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calib_copy:
        outs[0].copy_(xs[0])
        torch.cuda.synchronize()
    for c in ctxs + dctxs:
        st = c.last_status(streams[0])
        assert st == 0, binding.cmp_strerror(st)
    sizes = []
    for buf in arena:
        rc, size = ctxs[0].compressed_size(buf)
        assert rc == 0
        sizes.append(size)
    comp_bytes = sum(sizes)
    cbar = comp_bytes / total

    # correctness gate inside the bench: the error bound on the last warm-up pass
    worst = 0.0
    for x, out in zip(xs, outs):
        worst = max(worst, float((x.double() - out.double()).abs().max()))
    assert worst <= float(torch.tensor(eb, dtype=torch.float32)), worst

    # ---- timed region: exactly K steps -------------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-phase times (host clock, a device-wide wait after each phase)
    tc = td = 0.0
    for _ in range(args.steps):
        a = time.perf_counter(); compress_all(); torch.cuda.synchronize()
        b = time.perf_counter(); decompress_all(); torch.cuda.synchronize()
        c = time.perf_counter()
        tc += (b - a) * 1e3; td += (c - b) * 1e3
    tc /= args.steps; td /= args.steps

    # ---- per-kernel durations (events around every launch), same K steps ----------------
    # All calls on one stream, back to back: kernels of one stream run in order, so a kernel's
    # duration is its own and not that of whatever another stream ran beside it, and no launch
    # starts on an idle GPU (an event pair around the first kernel after a device-wide wait also
    # times the wake-up: 10-20 us, which a rocprofv3 kernel trace does not show).
    for c in ctxs:
        c.profile(True)
    for _ in range(args.steps):
        for i in order:
            rc, _ = binding.cmp_compress(ctxs[i % K]._h, xs[i].data_ptr(), xs[i].shape, eb, arena[i].data_ptr(),
                                         arena[i].numel(), False, streams[0])
            assert rc == 0, binding.cmp_strerror(rc)
        for i in reversed(order):
            rc = binding.cmp_decompress(ctxs[i % K]._h, arena[i].data_ptr(), bounds[i], xs[i].shape, eb,
                                        outs[i].data_ptr(), streams[0])
            assert rc == 0, binding.cmp_strerror(rc)
    torch.cuda.synchronize()
    kern = {}
    for k, c in enumerate(ctxs):
        for name, (ms, launches) in c.profile_read(streams[0]).items():
            e = kern.setdefault(name, {"ms": 0.0, "launches": 0})
            e["ms"] += ms; e["launches"] += launches
        c.profile(False)
    kern = {name: {"ms_per_step": e["ms"] / args.steps, "launches_per_step": e["launches"] // args.steps,
                   "avg_us": 1e3 * e["ms"] / e["launches"]} for name, e in kern.items()}
    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    bytes_fn = KERNEL_BYTES.get(dom)
    roofline = None
    if bytes_fn is not None:
        alg_bytes_step = bytes_fn(cbar) * total                 # over all launches of one step
        achieved = alg_bytes_step / (kern[dom]["ms_per_step"] * 1e-3) / 1e9
        per_elem = MEASURED_TRAFFIC.get((wl.name, args.sub, eb), {}).get(dom)
        # measured HBM bytes per launch (average over the launches of a step), like `achieved`
        traffic = round(per_elem * total / kern[dom]["launches_per_step"]) if per_elem else None
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                    "alg_bytes_per_launch": round(alg_bytes_step / kern[dom]["launches_per_step"]),
                    "alg_bytes_per_elem": round(bytes_fn(cbar), 4),
                    "avg_launch_us": round(kern[dom]["avg_us"], 2),
                    "launches_per_step": kern[dom]["launches_per_step"]}

    # what a plain device copy of the largest tensor reaches on this machine (bytes read + written)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    outs[0].copy_(xs[0])
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(5):
        outs[0].copy_(xs[0])
    ev[1].record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * 4.0 * numels[0] / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9

    # the error-bound estimator (Sections 4.1-4.3; it runs every W = 1000 iterations, so it is not
    # part of a step): one streaming pass over an activation, a loss of the same shape and a momentum
    ctl_ctx = ctxs[0]
    mom = xs[-1].reshape(-1)[: 512 * 512 * 9].contiguous()
    ctl_ctx.estimate_eb(xs[0], outs[0], mom)
    ctl_ctx.profile(True)
    for _ in range(5):
        rc_ctl, eb_ctl, st_ctl = ctl_ctx.estimate_eb(xs[0], outs[0], mom)
    ctl_ms, ctl_n = ctl_ctx.profile_read()["k_controller_stats"]
    ctl_ctx.profile(False)
    ctl_bytes = 4.0 * (2 * numels[0] + mom.numel())
    ctl_gbps = ctl_bytes / (ctl_ms / ctl_n * 1e-3) / 1e9

    value = 2 * 4.0 * total / (ms_per_step * 1e-3) / 1e9
    alg_roundtrip = (12.0 + 2 * cbar) * total                  # 8 + cbar compress, 4 + cbar decompress
    result = {
        "metric": "compress+decompress GB/s of fp32 activations (frac. of HBM peak); compression ratio",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32 quantiser, i32/bit codec", "data": "synthetic",
        "config": {"workload": wl.name, "tensors": len(xs), "numel": total, "eb": eb, "radius": 512,
                   "chunk": 4096, "sub": args.sub, "streams": S, "pipeline": pipeline, "p_zero": wl.p_zero, "box_k": wl.k,
                   "seed_base": wl.seed(0)},
        "compression_ratio": round(4.0 * total / comp_bytes, 4),
        "compressed_bytes_held": comp_bytes,
        "compress_ms": round(tc, 4), "decompress_ms": round(td, 4),
        "compress_GBps": round(4.0 * total / (tc * 1e-3) / 1e9, 2),
        "decompress_GBps": round(4.0 * total / (td * 1e-3) / 1e9, 2),
        "hbm_frac_algorithmic": round(alg_roundtrip / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "copy_ceiling_GBps": round(copy_gbps, 1),
        "controller": {"kernel": "k_controller_stats", "bound": "hbm", "achieved": round(ctl_gbps, 1),
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ctl_gbps / HBM_PEAK_GBPS, 4),
                       "avg_launch_us": round(1e3 * ctl_ms / ctl_n, 2), "alg_bytes_per_launch": int(ctl_bytes),
                       "eb": eb_ctl, "R": st_ctl[0]},
        "max_abs_err": worst,
        "kernels": {k: {kk: round(vv, 3) for kk, vv in v.items()} for k, v in kern.items()},
        "roofline": roofline,
    }

    # ---- CPU baseline: the oracle as it stands, one core, bounded sample ------------------
    if not args.no_cpu_baseline:
        import oracle
        n_s, t_c, t_d = 0, 0.0, 0.0
        for i in range(min(args.cpu_sample, len(xs))):
            xh = xs[i].cpu().numpy()
            a = time.perf_counter()
            rc, obuf, osize, _ = oracle.compress(xh, eb, oracle.Config(sub=args.sub))
            b = time.perf_counter()
            rc2, oy = oracle.decompress(obuf, xh.shape, eb, oracle.Config(sub=args.sub))
            c = time.perf_counter()
            assert rc == 0 and rc2 == 0
            n_s += xh.size; t_c += b - a; t_d += c - b
        result["cpu_baseline"] = {
            "value": round(2 * 4.0 * n_s / (t_c + t_d) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {min(args.cpu_sample, len(xs))} tensors of {wl.name} ({n_s} elements), "
                      f"compress {t_c:.2f} s + decompress {t_d:.2f} s, host has {os.cpu_count()} cpus"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
