#!/usr/bin/env python3
"""Benchmark of the SMaLL hot path on one MI355X.

A step = one pass of the whole path over one batch of the residual CNN workload (batch 256,
32x32x3 fp32 images, seeded synthetic): the NCHW input (already resident in HBM) goes through
small_network_run_plain (at this batch one image-resident launch: a workgroup takes an image through the first
convolution, which reads the plain input, the conv 3x3 / 1x1 layers with ReLU and residual add, average pool and
dense, every tensor between them in LDS). The logits [N][10] have one pixel and one channel block per image, so
their blocked layout IS the plain one and the run writes them where the caller wants them (SMALL_RUN_PLAIN_OUTPUT):
the layout changes of both network boundaries happen inside the first and last layer, no small_pack / small_unpack
launch. Where a table or batch does not allow that the step falls back to small_network_run_plain + small_unpack,
then to small_pack + small_network_run + small_unpack. value = images/s.

Also reported on the same JSON line:
  roofline      the kernel with the largest share of the step (per-layer HIP-event timing of the
                same launches through the per-layer entry points), algorithmic flops / duration;
  sweep         the roofline layer sweep (batch 64, Cb = 16): conv GFLOP/s against the fp32 MFMA peak,
                depthwise / max-pool / ReLU GB/s against the HBM peak, buffers rotated so that
                at least 512 MB are touched between reuses of a buffer;
  networks_u8   the CNN stand-ins on the quantized path (small_network_run_u8), the quantized oracle beside them
  sweep_u8      the same layers on the quantized path (uint8 codes, int32 sums): conv TOP/s against the int8
                MFMA peak and GB/s against the HBM peak;
  networks      images/s of the four stand-in networks at batch 1 and at their large batch;
  cpu_baseline  the CPU oracle (as it stands) on a bounded sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3e12     # MI355X dense fp32 matrix, flop/s
PEAK_MFMA_I8 = 5.0e15        # MI355X dense int8 matrix, op/s
PEAK_HBM = 8.0e12            # MI355X HBM3E, B/s
ROTATE_BYTES = 512e6         # touched between reuses of a buffer in HBM-bound timings (> 256 MB Infinity Cache)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The GPU raises its clocks only after some tens of milliseconds of sustained load: the defaults warm up
    # for about 0.3 s (a step is about 0.14 ms) and time about 0.7 s.
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--only", default="", help="comma-separated sweep layers to run (e.g. dw3x3,relu); skips the rest")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-networks", action="store_true")
    ap.add_argument("--resident-timing", action="store_true",
                    help="per-layer cycle stamps of the image-resident run (needs a library built with SMALL_RES_TIMING=1)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target wall time of the CPU-oracle sample")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    import paper_2303_04769_amd as S
    import workloads as WL

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    S.binding.load()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        """Average seconds per call of fn over reps back-to-back launches between two events on the launch stream."""
        a, b = ev(), ev()
        a.record()
        for r in range(reps):
            fn(r)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    if args.only:   # developer shortcut: selected sweep rows only, one JSON row per line ("u8" = the quantized sweep)
        only = set(args.only.split(","))
        if only != {"u8"}:
            for row in sweep(S, WL, torch, np, dev, timed, only - {"u8"}, cpu=not args.no_cpu):
                print(json.dumps(row))
        if "u8" in only:
            for row in sweep_u8(S, WL, torch, dev, timed):
                print(json.dumps(row))
            for row in networks_u8(S, WL, torch, dev, timed, cpu=not args.no_cpu):
                print(json.dumps(row))
        return

    # ------------------------------------------------------------------ the step
    net = WL.residual_cnn()
    N = args.batch
    x, ws = WL.network_tensors(net, N, WL.BASE_SEED + 2)
    pn = S.PackedNetwork(net, ws, dev)
    x_d = torch.from_numpy(x).to(dev)
    xb = torch.empty(x_d.numel(), dtype=torch.float32, device=dev)
    last = net.layers[-1]
    out_b = torch.empty(pn.out_elems(N), dtype=torch.float32, device=dev)
    logits = torch.empty(pn.out_elems(N), dtype=torch.float32, device=dev)
    pn.workspace(N)

    # The first layer reads the plain NCHW input itself where its kernel can (batch >= 16 here); otherwise the
    # input is packed by a launch of its own. Decided once, before the warm-up.
    S.small_pack(x_d, xb, N, net.C0, net.H0, net.W0, net.layers[0].Cib)     # also feeds the per-launch replays below
    try:
        pn.run_plain(x_d, out_b, N)
        plain = True
    except S.SmallError as e:
        if e.code != 7:
            raise
        plain = False
    # The logits [N][10] are one pixel and one channel block per image: blocked and plain layout coincide, and the run
    # can hand them over as the plain tensor (SMALL_RUN_PLAIN_OUTPUT) with no small_unpack launch. Checked once against
    # small_unpack of a run without the flag.
    plain_out = False
    if plain:
        try:
            pn.run_opt(x_d, logits, N, S.SMALL_RUN_PLAIN_INPUT | S.SMALL_RUN_PLAIN_OUTPUT)
            check = torch.empty_like(logits)
            S.small_unpack(out_b, check, N, last.Co, 1, 1, last.Cob)
            torch.cuda.synchronize()
            plain_out = bool(torch.equal(check, logits))
        except S.SmallError as e:
            if e.code != 7:
                raise

    def step(_=0):
        if plain_out:
            pn.run_opt(x_d, logits, N, S.SMALL_RUN_PLAIN_INPUT | S.SMALL_RUN_PLAIN_OUTPUT)
            return
        if plain:
            pn.run_plain(x_d, out_b, N)
        else:
            S.small_pack(x_d, xb, N, net.C0, net.H0, net.W0, net.layers[0].Cib)
            pn.run(xb, out_b, N)
        S.small_unpack(out_b, logits, N, last.Co, 1, 1, last.Cob)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.resident_timing:
        resident_timing(S, net, N)
        return
    t0 = time.perf_counter()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    value = N * args.steps / wall
    assert torch.isfinite(logits).all()

    # ------------------------------------------------------------------ per-launch timing of the same launches
    # small_network_run folds ReLU / residual add into the producing convolution; every launch of the
    # step is replayed on its own through small_network_run_range between two events.
    heads = pn.launches_at(N)
    groups = [net.layers[h:(heads[k + 1] if k + 1 < len(heads) else len(net.layers))] for k, h in enumerate(heads)]

    def kernel_of(L, g=()):
        if sum(x.op == "conv" for x in g) > 1:
            return "resident_run"          # several convolutions in one launch: the image-resident run
        if L.op == "conv":
            return S.small_conv2d_kernel(N, L.Ci, L.Co, L.H, L.W, L.kh, L.kw, L.stride, L.pad, L.Cib, L.Cob)
        if L.op == "dense":
            return S.small_conv2d_kernel(N, L.Ci, L.Co, 1, 1, 1, 1, 1, (0, 0, 0, 0), L.Cib, L.Cob)
        return L.op

    prof_steps = max(10, min(args.steps, 50))
    REP = 8
    per_kernel = {}
    for it in range(prof_steps + 3):
        evs = []
        for h, g in zip(heads, groups):
            a, b = ev(), ev()
            a.record()
            for _ in range(REP):         # back-to-back repeats of one launch: the event overhead is amortised
                pn.run_range(xb, out_b, N, h, 1)
            b.record()
            evs.append((g, a, b))
        torch.cuda.synchronize()
        if it < 3:
            continue
        for g, a, b in evs:
            L = g[0]
            k = per_kernel.setdefault(kernel_of(L, g), {"time": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0,
                                                     "fused": "+".join(x.op for x in g)})
            k["time"] += a.elapsed_time(b) * 1e-3 / REP
            k["launches"] += 1
            n_in, n_out = N * L.Ci * L.H * L.W, N * L.Co * L.Ho * L.Wo
            if kernel_of(L, g) == "resident_run":
                # HBM sees the run's input, its last result and the filters once; the flops are those of every layer
                convs = [x for x in g if x.op == "conv"]
                k["flops"] += sum(2.0 * N * x.Co * x.Ho * x.Wo * x.Ci * x.kh * x.kw for x in convs)
                n_in += sum(x.Co * x.Ci * x.kh * x.kw for x in convs)
                n_out = N * convs[-1].Co * convs[-1].Ho * convs[-1].Wo
            elif L.op in ("conv", "dense"):
                k["flops"] += 2.0 * N * L.Co * L.Ho * L.Wo * L.Ci * L.kh * L.kw
                n_in += L.Co * L.Ci * L.kh * L.kw
                if any(x.op == "add" for x in g[1:]):
                    n_in += n_out
            elif L.op == "add":
                n_in += n_out
            k["bytes"] += 4.0 * (n_in + n_out)
    dom_name, dom = max(per_kernel.items(), key=lambda kv: kv[1]["time"])
    isolated_us = dom["time"] / dom["launches"] * 1e6
    # When the timed step IS one launch of that kernel (nothing else on the stream), the events around the timed region
    # are its launches back to back: region / steps bounds the kernel's duration from above, in the conditions `value`
    # is measured in (the isolated passes above sit between synchronisations, where the clocks sag: a few per cent more).
    if plain_out and len(heads) == 1:
        dom = dict(dom, time=e0.elapsed_time(e1) * 1e-3 / args.steps * dom["launches"])
    if dom["flops"] > 0:
        achieved = dom["flops"] / dom["time"] / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_MFMA_F32 / 1e12, "unit": "TFLOP/s",
                    "frac": round(achieved * 1e12 / PEAK_MFMA_F32, 4)}
    else:
        achieved = dom["bytes"] / dom["time"] / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                    "frac": round(achieved * 1e9 / PEAK_HBM, 4)}
    roofline.update({"kernel": dom_name, "avg_launch_us": round(dom["time"] / dom["launches"] * 1e6, 2),
                     "launches_per_step": dom["launches"] // prof_steps,
                     "share_of_layer_time": round(per_kernel[dom_name]["time"] / sum(k["time"] for k in per_kernel.values()), 3),
                     "avg_launch_us_isolated": round(isolated_us, 2),
                     "traffic": _traffic(dom_name)})

    result = {
        "metric": "network images/s (residual CNN, batch %d); sweep: conv GFLOP/s + dw/pool GB/s vs roofline" % N,
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "residual CNN 32x32x3, batch %d: %s"
                               % (N, "small_network_run_opt, NCHW input read by the first layer, logits [N][10] written by "
                                     "the last (blocked = plain layout there): no pack / unpack launch" if plain_out
                                  else ("small_network_run_plain (NCHW input read by the first layer) + unpack" if plain
                                        else "pack + small_network_run + unpack")),
                   "global_batch": N, "seed": WL.BASE_SEED + 2, "layers": len(net.layers),
                   "gflop_per_step": round(2e-9 * net.macs_per_image() * N, 3)},
        "event_ms_per_step": round(e0.elapsed_time(e1) / args.steps, 4),
        "roofline": roofline,
        "kernels": {k: {"avg_us": round(v["time"] / v["launches"] * 1e6, 2), "per_step": v["launches"] // prof_steps,
                        "layers": v["fused"], "tflops": round(v["flops"] / v["time"] / 1e12, 2),
                        "gbs": round(v["bytes"] / v["time"] / 1e9, 1)}
                    for k, v in sorted(per_kernel.items(), key=lambda kv: -kv[1]["time"])},
        "launches_per_step": len(heads) + (0 if plain_out else (1 if plain else 2)),
    }

    # ------------------------------------------------------------------ what this machine sustains
    peaks = measured_peaks(S, torch, dev, timed)
    result["measured_peaks"] = peaks
    if roofline["bound"] == "mfma":
        roofline["frac_of_measured_peak"] = round(roofline["achieved"] / peaks["mfma_f32_tflops"], 4)
    else:
        roofline["frac_of_measured_peak"] = round(roofline["achieved"] / peaks["hbm_copy_gbs"], 4)

    # ------------------------------------------------------------------ roofline layer sweep
    if not args.no_sweep:
        result["sweep"] = sweep(S, WL, torch, np, dev, timed, cpu=not args.no_cpu)
        c = [r for r in result["sweep"] if r["layer"] == "conv3x3" and not r.get("paper_layer_study")]
        best = max(c, key=lambda r: r["frac"])
        result["roofline_sweep_conv3x3"] = {"bound": "mfma", "achieved": best["tflops"], "peak": PEAK_MFMA_F32 / 1e12,
                                            "unit": "TFLOP/s", "frac": best["frac"], "shape": best["shape"],
                                            "kernel": best["kernel"]}

        result["sweep_u8"] = sweep_u8(S, WL, torch, dev, timed)

    # ------------------------------------------------------------------ networks
    if not args.no_networks:
        result["networks"] = networks(S, WL, torch, dev, timed)
        result["networks_u8"] = networks_u8(S, WL, torch, dev, timed, cpu=not args.no_cpu)

    # ------------------------------------------------------------------ CPU oracle beside it
    if not args.no_cpu:
        from oracle import oracle as O
        cores = len(os.sched_getaffinity(0))
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        used = O.set_threads(cores)
        t = time.perf_counter()
        O.run_network(net, x[:2], ws)
        per_img = (time.perf_counter() - t) / 2
        n_s = int(max(2, min(N, args.cpu_seconds / max(per_img, 1e-6))))
        t = time.perf_counter()
        passes = 0
        while passes == 0 or (time.perf_counter() - t < args.cpu_seconds and passes < 64):
            ref = O.run_network(net, x[:n_s], ws)
            passes += 1
        dt = (time.perf_counter() - t) / passes
        got = logits[:n_s * last.Co].cpu().numpy().reshape(n_s, last.Co)
        err = float(np.abs(got - ref).max())
        # and on one thread, on a smaller slice (images are independent: the rate scales linearly)
        O.set_threads(1)
        n_1 = max(1, min(n_s, 8))
        t = time.perf_counter()
        O.run_network(net, x[:n_1], ws)
        dt1 = time.perf_counter() - t
        O.set_threads(used)
        others = []
        for oname, oidx, n_all, n_one in (("dsep_cnn", 3, 64, 4), ("audio_cnn", 4, 256, 16), ("dense_autoencoder", 5, 8192, 512)):
            onet = getattr(WL, oname)()
            ox, ows = WL.network_tensors(onet, n_all, WL.BASE_SEED + oidx)
            O.run_network(onet, ox[:2], ows)
            t = time.perf_counter()
            O.run_network(onet, ox, ows)
            ta = time.perf_counter() - t
            O.set_threads(1)
            t = time.perf_counter()
            O.run_network(onet, ox[:n_one], ows)
            t1 = time.perf_counter() - t
            O.set_threads(used)
            others.append({"network": oname, "images_per_s": round(n_all / ta, 1), "cores": used,
                           "sample": "%d seeded images, one pass of %.2f s" % (n_all, ta),
                           "single_thread_images_per_s": round(n_one / t1, 2),
                           "single_thread_sample": "%d images, one pass of %.2f s" % (n_one, t1)})
        result["cpu_baseline"] = {"value": round(n_s / dt, 2), "unit": "images/s", "cores": used, "kind": "oracle",
                                  "networks": others,
                                  "sample": "first %d of the %d images of the same batch, %d passes of %.2f s" % (n_s, N, passes, dt),
                                  "single_thread_value": round(n_1 / dt1, 2),
                                  "single_thread_sample": "first %d images, one pass of %.2f s" % (n_1, dt1),
                                  "max_abs_diff_vs_gpu": err}
    print(json.dumps(result))


def resident_timing(S, net, N):
    """Developer aid: cycle stamps that a library built with SMALL_RES_TIMING=1 leaves behind (workgroups 0 and 100, every
    wave, per layer of the last image-resident launch): time in the layer's own code, in the work after it (border
    clearing, requests for the next layer) and at the barrier, in shader clock cycles."""
    import ctypes as C
    import numpy as np
    lib = S.binding.load()
    if not hasattr(lib, "small_debug_resident_timing"):
        sys.exit("bench.py --resident-timing: the library was built without SMALL_RES_TIMING=1")
    buf = (C.c_ulonglong * (2 * 8 * 64))()
    lib.small_debug_resident_timing.argtypes = [C.POINTER(C.c_ulonglong)]
    if lib.small_debug_resident_timing(buf) != 0:
        sys.exit("bench.py --resident-timing: reading the stamps failed")
    t = np.array(buf[:], dtype=np.int64).reshape(2, 8, 64)
    n_launch_layers = sum(1 for k in range(15) if t[0, 0, 2 + 4 * k] > 0)
    for b, wg in enumerate((0, 100)):
        t0 = int(t[b, :, 0].min())
        print("workgroup %d: input staged after %d cycles" % (wg, int(t[b, :, 1].max()) - t0))
        for li in range(n_launch_layers):
            e, c, pb, ab = (t[b, :, 2 + 4 * li + k] for k in range(4))
            print("  layer %2d: wall %6d | per wave: code %s  after %s  barrier %s"
                  % (li, int((ab - e).max()), (c - e).tolist(), (pb - c).tolist(), (ab - pb).tolist()))
        print("  total %d cycles" % (int(t[b, :, 5 + 4 * (n_launch_layers - 1)].max()) - t0))


def spin(fn, seconds=0.12):
    """Untimed warm-up: keeps the GPU busy with fn long enough for its clocks to settle."""
    import torch
    t0 = time.perf_counter()
    r = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn(r)
            r += 1
        torch.cuda.synchronize()


def measured_peaks(S, torch, dev, timed):
    """Reference points measured in this run: a register-resident loop of fp32 matrix instructions
    (small_probe_mfma) and a plain device-to-device copy of 1 GiB (2 GiB of traffic), next to the published
    157.3 TFLOP/s and 8 TB/s the fractions are quoted against."""
    wgs, iters = 256 * 8, 4096
    out = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    fn = lambda r: S.small_probe_mfma(out, wgs, iters)
    spin(fn)
    t = min(timed(fn, 10) for _ in range(3))
    mfma = wgs * 4 * iters * 8 * 2048.0 / t / 1e12
    n = 1 << 28                                              # 1 GiB of floats
    src = torch.empty(n, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    fc = lambda r: dst.copy_(src)
    spin(fc)
    tc = min(timed(fc, 10) for _ in range(3))
    fr = lambda r: S.small_relu(src, dst, n)
    spin(fr)
    tr = min(timed(fr, 10) for _ in range(3))
    del src, dst
    # what a vector instruction costs next to the matrix pipe: rounds of sixteen matrix instructions (512 pipe cycles)
    # with 0 / 32 / 64 / 96 multiply-adds beside them, four waves per SIMD; cycles per round and wave at 2.4 GHz
    wgs4, it4 = 256 * 4, 2048
    out4 = torch.empty(wgs4 * 256, dtype=torch.float32, device=dev)
    mix = {}
    for valu in (0, 32, 64, 96):
        fm = lambda r: S.small_probe_mfma_valu(out4, wgs4, it4, valu)
        spin(fm, 0.2)
        mix[str(valu)] = round(min(timed(fm, 10) for _ in range(3)) * 2.4e9 / it4 / 4, 1)
    return {"mfma_f32_tflops": round(mfma, 1), "hbm_copy_gbs": round(8.0 * n / tc / 1e9, 1),
            "hbm_relu_gbs": round(8.0 * n / tr / 1e9, 1),
            "cycles_per_16_mfma_with_valu": mix,
            "note": "small_probe_mfma (register-resident 16x16x4 fp32 MFMA loop); torch copy_ and small_relu over 1 GiB in + 1 GiB out; "
                    "small_probe_mfma_valu (the same loop with independent fp32 multiply-adds beside it)"}


def _traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, if one covers it."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(kernel)
    except (OSError, ValueError):
        return None


def sweep(S, WL, torch, np, dev, timed, only=None, cpu=False):
    """Layer sweep at batch 64: every layer on its own, HBM-bound layers with rotated buffers. cpu: the CPU oracle is
    timed beside every row on the first 4 of the 64 images (one thread, then all cores), scaled to 64."""
    def want(name):
        return not only or name in only
    Nb = WL.SWEEP_N
    rng = np.random.default_rng(WL.BASE_SEED + 5)
    rows = []
    ORACLE_N = 4

    def oracle_beside(row, fn):
        """fn(): the oracle on an N = 4 slice of the row's layer; adds its time scaled to the 64 images of the row."""
        if not cpu:
            return row
        from oracle import oracle as O
        cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", 1 << 20)))
        used = O.set_threads(cores)
        fn()                                   # first touch of the arrays
        t = time.perf_counter()
        fn()
        t_all = time.perf_counter() - t
        O.set_threads(1)
        t = time.perf_counter()
        fn()
        t_one = time.perf_counter() - t
        O.set_threads(used)
        k = Nb / ORACLE_N
        row["oracle"] = {"ms_all_cores": round(t_all * k * 1e3, 2), "cores": used, "ms_one_thread": round(t_one * k * 1e3, 2),
                         "sample": "first %d of the %d images, time scaled by %d" % (ORACLE_N, Nb, int(k)),
                         "gpu_over_all_cores": round(t_all * k / (row["us"] * 1e-6), 1)}
        return row

    def rand(n):
        return (torch.rand(n, device=dev, dtype=torch.float32) * 2 - 1)

    def best_of(fn, reps, trials=3, per_graph=24):
        """These kernels take a few microseconds, less than the host needs to enqueue one through Python, so
        `per_graph` calls (rotating over the buffer sets) are recorded into a HIP graph and the graph is replayed."""
        for r in range(per_graph):
            fn(r)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for r in range(per_graph):
                fn(r)
        gfn = lambda r: graph.replay()
        spin(gfn)
        n = max(1, reps // per_graph)
        ts = [timed(gfn, n) / per_graph for _ in range(trials)]
        return min(ts), statistics.median(ts)

    shapes = WL.sweep_shapes()
    for C, H in shapes["conv"] + shapes["paper_layer_study"]:
        n_act = Nb * C * H * H
        act_bytes = 8.0 * n_act
        sets = max(2, int(-(-ROTATE_BYTES // act_bytes)))
        ins = [rand(n_act) for _ in range(sets)]
        outs = [torch.empty(n_act, device=dev, dtype=torch.float32) for _ in range(sets)]
        for k, name in ((3, "conv3x3"), (1, "conv1x1")):
            if not want(name):
                continue
            w = torch.from_numpy(WL.uniform_pm1(rng, (C * C * k * k,))).to(dev)   # already "blocked": random values
            pad = (1, 1, 1, 1) if k == 3 else (0, 0, 0, 0)
            fn = lambda r: S.small_conv2d(ins[r % sets], w, outs[r % sets], Nb, C, C, H, H, k, k, 1, pad, 16, 16)
            tmin, tmed = best_of(fn, 30 if k == 3 else 100)
            flops = 2.0 * Nb * C * H * H * C * k * k
            byts = 4.0 * (2 * n_act + C * C * k * k)
            row = {"layer": name, "shape": "N64 C%d %dx%d" % (C, H, H), "paper_layer_study": (C, H) in shapes["paper_layer_study"],
                   "us": round(tmin * 1e6, 2),
                   "us_median": round(tmed * 1e6, 2), "tflops": round(flops / tmin / 1e12, 2),
                   "frac": round(flops / tmin / PEAK_MFMA_F32, 4), "gbs": round(byts / tmin / 1e9, 1),
                   "frac_hbm": round(byts / tmin / PEAK_HBM, 4),
                   "kernel": S.small_conv2d_kernel(Nb, C, C, H, H, k, k, 1, pad, 16, 16)}
            if cpu:
                from oracle import oracle as O
                xo, wo = WL.uniform_pm1(rng, (ORACLE_N, C, H, H)), WL.uniform_pm1(rng, (C, C, k, k))
                oracle_beside(row, lambda: O.conv2d(xo, wo, 1, pad))
            rows.append(row)
        if want("dw3x3"):
            wd = torch.from_numpy(WL.uniform_pm1(rng, (C * 9,))).to(dev)
            fn = lambda r: S.small_dwconv2d(ins[r % sets], wd, outs[r % sets], Nb, C, H, H, 3, 3, 1, (1, 1, 1, 1), 16)
            tmin, tmed = best_of(fn, 100)
            # the same layer on one buffer pair: the tensors then stay in the 256 MB Infinity Cache (not an HBM figure)
            twarm, _ = best_of(lambda r: S.small_dwconv2d(ins[0], wd, outs[0], Nb, C, H, H, 3, 3, 1, (1, 1, 1, 1), 16), 100)
            byts = 4.0 * (2 * n_act + 9 * C)
            row = {"layer": "dw3x3", "shape": "N64 C%d %dx%d" % (C, H, H), "us": round(tmin * 1e6, 2),
                   "us_median": round(tmed * 1e6, 2), "gbs": round(byts / tmin / 1e9, 1),
                   "frac": round(byts / tmin / PEAK_HBM, 4), "buffer_sets": sets,
                   "us_cache_warm": round(twarm * 1e6, 2), "gbs_cache_warm": round(byts / twarm / 1e9, 1)}
            if cpu:
                from oracle import oracle as O
                xo, wo = WL.uniform_pm1(rng, (ORACLE_N, C, H, H)), WL.uniform_pm1(rng, (C, 1, 3, 3))
                oracle_beside(row, lambda: O.dwconv2d(xo, wo, 1, (1, 1, 1, 1)))
            rows.append(row)
        del ins, outs
    C, H = WL.sweep_shapes()["pool_relu"]
    n_act = Nb * C * H * H
    n_pool = Nb * C * 27 * 27
    sets = 2
    ins = [rand(n_act) for _ in range(sets)]
    outs = [torch.empty(n_act, device=dev, dtype=torch.float32) for _ in range(sets)]
    if not (want("relu") or want("maxpool3x3s2") or want("pack") or want("table2")):
        return rows
    if cpu:
        from oracle import oracle as O
        xo = WL.uniform_pm1(rng, (ORACLE_N, C, H, H))
    fn = lambda r: S.small_relu(ins[r % sets], outs[r % sets], n_act)
    tmin, tmed = best_of(fn, 50)
    rows.append(oracle_beside({"layer": "relu", "shape": "N64 C%d %dx%d" % (C, H, H), "us": round(tmin * 1e6, 2),
                               "us_median": round(tmed * 1e6, 2), "gbs": round(8.0 * n_act / tmin / 1e9, 1),
                               "frac": round(8.0 * n_act / tmin / PEAK_HBM, 4), "buffer_sets": sets}, lambda: O.relu(xo)))
    ins.append(rand(n_act))
    fn = lambda r: S.small_pool2d(ins[r % 3], outs[r % sets], Nb, C, H, H, 3, 3, 2, (0, 0, 0, 0), 16, S.POOL_MAX)
    tmin, tmed = best_of(fn, 50)
    byts = 4.0 * (n_act + n_pool)
    rows.append(oracle_beside({"layer": "maxpool3x3s2", "shape": "N64 C%d %dx%d" % (C, H, H), "us": round(tmin * 1e6, 2),
                               "us_median": round(tmed * 1e6, 2), "gbs": round(byts / tmin / 1e9, 1),
                               "frac": round(byts / tmin / PEAK_HBM, 4), "buffer_sets": 3}, lambda: O.pool2d(xo, (3, 3), 2)))
    # pack / unpack of the largest activation (network boundary only)
    fn = lambda r: S.small_pack(ins[r % 3], outs[r % sets], Nb, C, H, H, 16)
    tmin, tmed = best_of(fn, 30)
    rows.append(oracle_beside({"layer": "pack", "shape": "N64 C%d %dx%d" % (C, H, H), "us": round(tmin * 1e6, 2),
                               "us_median": round(tmed * 1e6, 2), "gbs": round(8.0 * n_act / tmin / 1e9, 1),
                               "frac": round(8.0 * n_act / tmin / PEAK_HBM, 4), "buffer_sets": 3}, lambda: O.pack(xo, 16)))
    # ---- the remaining layers of Table 2 at the same size: batch normalization (one FMA per element, HBM-bound),
    # nearest-neighbour upsampling by 2 x 2 (input N64 C256 28x28), group convolution (8 groups of 32 channels, 3x3)
    scale, shift = rand(C) + 1.5, rand(C)
    fn = lambda r: S.small_batchnorm(ins[r % 3], scale, shift, outs[r % sets], Nb, C, H, H, 16)
    tmin, tmed = best_of(fn, 50)
    rows.append(oracle_beside({"layer": "batchnorm", "shape": "N64 C%d %dx%d" % (C, H, H), "us": round(tmin * 1e6, 2),
                               "us_median": round(tmed * 1e6, 2), "gbs": round(8.0 * n_act / tmin / 1e9, 1),
                               "frac": round(8.0 * n_act / tmin / PEAK_HBM, 4), "buffer_sets": 3},
                              lambda: O.batchnorm(xo, np.full(C, 1.5, np.float32), np.zeros(C, np.float32))))
    Hu = H // 2
    n_small = Nb * C * Hu * Hu
    fn = lambda r: S.small_upsample(ins[r % 3][:n_small], outs[r % sets], Nb, C, Hu, Hu, 2, 2, 16)
    tmin, tmed = best_of(fn, 50)
    byts = 4.0 * (n_small + n_act)
    rows.append(oracle_beside({"layer": "upsample2x2", "shape": "N64 C%d %dx%d" % (C, Hu, Hu), "us": round(tmin * 1e6, 2),
                               "us_median": round(tmed * 1e6, 2), "gbs": round(byts / tmin / 1e9, 1),
                               "frac": round(byts / tmin / PEAK_HBM, 4), "buffer_sets": 3},
                              lambda: O.upsample(xo[:, :, :Hu, :Hu], 2, 2)))
    Hg, FC = 28, 32
    n_g = Nb * C * Hg * Hg
    wg = rand(C * FC * 9)
    fn = lambda r: S.small_group_conv2d(ins[r % 3][:n_g], wg, outs[r % sets][:n_g], Nb, C, FC, FC, FC, Hg, Hg, 3, 3, 1, (1, 1, 1, 1), 16, 16, 16)
    tmin, tmed = best_of(fn, 30)
    flops = 2.0 * Nb * C * Hg * Hg * FC * 9
    row = {"layer": "groupconv3x3", "shape": "N64 C%d %dx%d, %d groups of %d" % (C, Hg, Hg, C // FC, FC), "us": round(tmin * 1e6, 2),
           "us_median": round(tmed * 1e6, 2), "tflops": round(flops / tmin / 1e12, 2), "frac": round(flops / tmin / PEAK_MFMA_F32, 4),
           "gbs": round(4.0 * (2 * n_g + C * FC * 9) / tmin / 1e9, 1),
           "kernel": "the 3x3 matrix-core convolution kernel, every tile inside one group"}
    if cpu:
        wo = WL.uniform_pm1(rng, (C, FC, 3, 3))
        oracle_beside(row, lambda: O.group_conv2d(xo[:, :, :Hg, :Hg], wo, FC, FC, FC, 1, (1, 1, 1, 1)))
    rows.append(row)
    return rows


def sweep_u8(S, WL, torch, dev, timed):
    """The sweep layers on the quantized path: uint8 codes in and out, int32 sums, both zero-point corrections on."""
    from paper_2303_04769_amd.binding import small_quant
    Nb = WL.SWEEP_N
    rows = []

    def codes(n):
        return torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev)

    def best_of(fn, reps, trials=3, per_graph=24):
        """These kernels take a few microseconds, less than the host needs to enqueue one through Python, so
        `per_graph` calls (rotating over the buffer sets) are recorded into a HIP graph and the graph is replayed."""
        for r in range(per_graph):
            fn(r)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for r in range(per_graph):
                fn(r)
        gfn = lambda r: graph.replay()
        spin(gfn)
        n = max(1, reps // per_graph)
        ts = [timed(gfn, n) / per_graph for _ in range(trials)]
        return min(ts), statistics.median(ts)

    for C, H in WL.sweep_shapes()["conv"]:
        n_act = Nb * C * H * H
        sets = max(2, min(48, int(-(-ROTATE_BYTES // (2.0 * n_act)))))
        ins = [codes(n_act) for _ in range(sets)]
        outs = [torch.empty(n_act, dtype=torch.uint8, device=dev) for _ in range(sets)]
        shape = "N64 C%d %dx%d" % (C, H, H)
        for k, name in ((3, "conv3x3"), (1, "conv1x1")):
            w = codes(C * C * k * k)
            mult, shift = WL.u8_multiplier(C * k * k)
            q = small_quant(120, 131, 128, mult, shift, 0, 255)
            pad = (1, 1, 1, 1) if k == 3 else (0, 0, 0, 0)
            sums = torch.empty(C, dtype=torch.int32, device=dev)
            S.small_filter_sums_u8(w, sums, C, C, k, k, 16, 16)     # kept with the filter, like the filter itself
            fn = lambda r: S.small_conv2d_u8(ins[r % sets], w, outs[r % sets], Nb, C, C, H, H, k, k, 1, pad, 16, 16, q, sums)
            tmin, tmed = best_of(fn, 240)
            ops = 2.0 * Nb * C * H * H * C * k * k
            byts = 2.0 * n_act + C * C * k * k
            rows.append({"layer": name, "shape": shape, "us": round(tmin * 1e6, 2), "us_median": round(tmed * 1e6, 2),
                         "tops": round(ops / tmin / 1e12, 1), "frac": round(ops / tmin / PEAK_MFMA_I8, 4),
                         "gbs": round(byts / tmin / 1e9, 1), "frac_hbm": round(byts / tmin / PEAK_HBM, 4)})
        wd = codes(C * 9)
        q = small_quant(120, 131, 128, WL.u8_multiplier(9)[0], 31, 0, 255)
        fn = lambda r: S.small_dwconv2d_u8(ins[r % sets], wd, outs[r % sets], Nb, C, H, H, 3, 3, 1, (1, 1, 1, 1), 16, q)
        tmin, tmed = best_of(fn, 240)
        rows.append({"layer": "dw3x3", "shape": shape, "us": round(tmin * 1e6, 2), "us_median": round(tmed * 1e6, 2),
                     "gbs": round(2.0 * n_act / tmin / 1e9, 1), "frac": round(2.0 * n_act / tmin / PEAK_HBM, 4),
                     "buffer_sets": sets})
        del ins, outs
    C, H = WL.sweep_shapes()["pool_relu"]
    n_act, n_pool = Nb * C * H * H, Nb * C * 27 * 27
    sets = 6
    ins = [codes(n_act) for _ in range(sets)]
    outs = [torch.empty(n_act, dtype=torch.uint8, device=dev) for _ in range(sets)]
    shape = "N64 C%d %dx%d" % (C, H, H)
    fn = lambda r: S.small_relu_u8(ins[r % sets], outs[r % sets], n_act, 128)
    tmin, tmed = best_of(fn, 240)
    rows.append({"layer": "relu", "shape": shape, "us": round(tmin * 1e6, 2), "us_median": round(tmed * 1e6, 2),
                 "gbs": round(2.0 * n_act / tmin / 1e9, 1), "frac": round(2.0 * n_act / tmin / PEAK_HBM, 4), "buffer_sets": sets})
    fn = lambda r: S.small_pool2d_u8(ins[r % sets], outs[r % sets], Nb, C, H, H, 3, 3, 2, (0, 0, 0, 0), 16, S.POOL_MAX)
    tmin, tmed = best_of(fn, 240)
    rows.append({"layer": "maxpool3x3s2", "shape": shape, "us": round(tmin * 1e6, 2), "us_median": round(tmed * 1e6, 2),
                 "gbs": round((n_act + n_pool) / tmin / 1e9, 1), "frac": round((n_act + n_pool) / tmin / PEAK_HBM, 4),
                 "buffer_sets": sets})
    from paper_2303_04769_amd.binding import small_quant_add
    qa = small_quant_add(120, 131, 128, 3 << 28, 1 << 29, 30, 0, 255)
    fn = lambda r: S.small_add_u8(ins[r % sets], ins[(r + 1) % sets], outs[r % sets], n_act, qa)
    tmin, tmed = best_of(fn, 240)
    rows.append({"layer": "add", "shape": shape, "us": round(tmin * 1e6, 2), "us_median": round(tmed * 1e6, 2),
                 "gbs": round(3.0 * n_act / tmin / 1e9, 1), "frac": round(3.0 * n_act / tmin / PEAK_HBM, 4), "buffer_sets": sets})
    return rows


def networks_u8(S, WL, torch, dev, timed, cpu=False):
    """The stand-in networks on the quantized path (uint8 codes, seeded parameters): small_network_run_u8 from the
    blocked input to the blocked logits; cpu: the quantized oracle beside it (all cores, a bounded slice of the batch)."""
    out = []
    for name, idx, N in (("residual_cnn", 2, 256), ("dsep_cnn", 3, 256), ("audio_cnn", 4, 1024)):
        net = getattr(WL, name)()
        x, ws, qs = WL.quantized_network_tensors(net, N, WL.BASE_SEED + 300 + idx)
        pn = S.PackedNetworkU8(net, ws, qs, dev)
        xb = pn.pack_input(torch.from_numpy(x).to(dev))
        o = torch.empty(pn.out_elems(N), dtype=torch.uint8, device=dev)
        fn = lambda r: pn.run(xb, o, N)
        spin(fn)
        t = min(timed(fn, 100) for _ in range(3))
        row = {"network": name, "batch": N, "ms": round(t * 1e3, 4), "images_per_s": round(N / t, 1),
               "tops": round(2.0 * net.macs_per_image() * N / t / 1e12, 3), "layers": len(net.layers)}
        if cpu:
            from oracle import oracle_u8 as Q
            n_s = min(N, 64)
            Q.run_network(net, x[:2], ws, qs)
            t0 = time.perf_counter()
            ref = Q.run_network(net, x[:n_s], ws, qs)
            dt = time.perf_counter() - t0
            L = net.layers[-1]
            got = o.cpu().numpy()[:n_s * L.Co].reshape(n_s, L.Co)
            row["oracle"] = {"images_per_s": round(n_s / dt, 1), "cores": len(os.sched_getaffinity(0)),
                             "sample": "first %d images, one pass of %.2f s" % (n_s, dt),
                             "codes_equal": bool((got == ref.reshape(n_s, L.Co)).all())}
        out.append(row)
    return out


def networks(S, WL, torch, dev, timed):
    out = []
    for name, idx, batches in (("residual_cnn", 2, (1, 256)), ("dsep_cnn", 3, (1, 256)), ("audio_cnn", 4, (1, 1024)),
                               ("dense_autoencoder", 5, (1, 256, 262144))):
        net = getattr(WL, name)()
        for N in batches:
            x, ws = WL.network_tensors(net, N, WL.BASE_SEED + idx)
            pn = S.PackedNetwork(net, ws, dev)
            xb = pn.pack_input(torch.from_numpy(x).to(dev))
            o = torch.empty(pn.out_elems(N), dtype=torch.float32, device=dev)
            fn = lambda r: pn.run(xb, o, N)
            spin(fn)
            ts = [timed(fn, 100) for _ in range(3)]
            t = min(ts)
            row = {"network": name, "batch": N, "ms": round(t * 1e3, 4), "images_per_s": round(N / t, 1),
                   "tflops": round(2.0 * net.macs_per_image() * N / t / 1e12, 3), "layers": len(net.layers),
                   "launches": len(pn.launches_at(N))}
            if N == 1:      # the same run replayed from a HIP graph: no per-launch host cost
                graph = pn.capture(xb, o, N)
                gfn = lambda r: graph.replay()
                spin(gfn)
                tg = min(timed(gfn, 100) for _ in range(3))
                row.update({"graph_ms": round(tg * 1e3, 4), "graph_images_per_s": round(N / tg, 1)})
            out.append(row)
    return out


if __name__ == "__main__":
    main()
