#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: one step = forward + loss + backward (+ SGD) of a workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
    python bench.py --calibrate          # only the ceilings: MFMA-only loop, read / write / copy streams, SGD update

Default workload (config 3): VGG-A, all conv + FC layers, per-GPU minibatch 64, fp32, forward + softmax
cross-entropy + backward + SGD (momentum 0.9; lr 0.001 where the configuration names 0.01, which diverges from a
He-normal start within five steps -- see `config.lr_note` in the output), synthetic N(0,1) images, He-normal
weights -- the workload BASELINE.json's metric ("VGG-A conv+FC fwd+bwd images/sec on 1 MI355X") is quoted on.
Prints ONE JSON line.  Inputs are resident in HBM before the timed region starts.

Timing: `value` = images of the K timed steps / wall-clock between two device synchronisations.  Beside it,
`step_ms` gives mean / median / best of the K per-step durations (HIP events between the steps, on the stream the
library launches on), and `clocks` the engine / memory clocks read from sysfs before the warm-up (idle) and right
after the timed region (the GPU has just been busy); no read sits between warm-up and timed region or inside it: one
takes milliseconds, during which an idle GPU drops its clocks.
`roofline` describes the dominant kernel (largest share of the timed region): achieved = algorithmic FLOPs of its
launches / their summed duration, measured with HIP events that the library records on its own stream around every
kernel launch, inside the timed region, on every 10th timed step (`--profile-every`, `profiled_steps` in the
output): the event records cost ~2 % of a step.  `frac` is against the published peak (157.3 TFLOP/s fp32 matrix,
8 TB/s HBM); `frac_of_sustained` against what this run's own calibration (`calibration`: a register-only MFMA loop
and plain streams, run after the timed region) reached on this machine.
`layers` lists every call of a step with its time, TFLOP/s, algorithmic bytes, arithmetic intensity, the roof that
bounds it (HBM below 19.7 FLOP/byte, else the fp32 matrix cores) and the fraction of both roofs.
`cpu_baseline` is the CPU oracle (the plain fp64 loop nest, untuned) timed on this machine's host cores on a bounded
sample: a small minibatch (about 15 s of CPU work) through every layer of the same network.
"""
import argparse
import glob
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # 256 CUs x 256 FLOP/clk x 2.4 GHz (published dense fp32 matrix peak)
PEAK_HBM_GBS = 8000.0
RIDGE_FLOP_PER_BYTE = PEAK_FP32_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)


def csrc_sha():
    """Fingerprint of the kernel sources: a traffic figure read from a committed profile is only quoted when the
    profile was taken from these very sources."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1602_06709_amd", "csrc")
    for f in sorted(os.listdir(d)):
        h.update(f.encode())
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


class Clocks:
    """The current engine (sclk) and memory (mclk) clock levels from sysfs: host-side file reads that go through the
    driver to the power controller and take milliseconds, so none sits inside the timed region or just before it."""

    def __init__(self, pci_bus_id=None):
        self.files = {}
        devs = sorted(glob.glob("/sys/class/drm/card*/device"))
        if pci_bus_id:
            match = [d for d in devs if os.path.realpath(d).lower().endswith(pci_bus_id.lower())]
            devs = match or devs
        for d in devs:
            for key, fn in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk")):
                p = os.path.join(d, fn)
                if key not in self.files and os.access(p, os.R_OK):
                    self.files[key] = p

    def read(self):
        out = {}
        for key, path in self.files.items():
            out[key + "_mhz"] = None
            try:
                for line in open(path):
                    if line.rstrip().endswith("*"):
                        m = re.search(r"(\d+)\s*mhz", line, re.I)
                        if m:
                            out[key + "_mhz"] = int(m.group(1))
            except OSError:
                pass
        return out


def calibrate(cnn, ctx, torch, n_floats, reps=5):
    """The box's own ceilings, each the best of `reps` launches timed by the library's HIP events: a register-only
    fp32 MFMA loop, and read / write / copy streams plus both SGD updates over arrays of n_floats floats."""
    from paper_1602_06709_amd.net import carve_arrays
    n = n_floats // 4 * 4
    a, b, c = carve_arrays(n, 3, "cuda")          # laid out as the network lays out weights / gradients / momentum
    a.fill_(1.0)
    sink = torch.empty(cnn.PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    was = ctx.profile_count()
    ctx.profile(True)
    runs = [("mfma", lambda: cnn.cnn_probe_mfma(ctx, 4000, sink), None),
            ("read", lambda: cnn.cnn_probe_stream(ctx, cnn.STREAM_READ, a, b), 4 * n),
            ("write", lambda: cnn.cnn_probe_stream(ctx, cnn.STREAM_WRITE, None, b), 4 * n),
            ("copy", lambda: cnn.cnn_probe_stream(ctx, cnn.STREAM_COPY, a, b), 8 * n),
            ("sgd_momentum", lambda: cnn.cnn_sgd_update(ctx, b, a, c, 1e-6, 0.9), 20 * n),
            ("sgd_plain", lambda: cnn.cnn_sgd_update(ctx, b, a, None, 1e-6, 0.0), 12 * n)]
    spans = []
    for name, fn, nbytes in runs:
        fn()                                    # one untimed launch first
        lo = ctx.profile_count()
        for _ in range(reps):
            fn()
        spans.append((name, nbytes, lo, ctx.profile_count()))
    ctx.profile(False)
    torch.cuda.synchronize()
    ent = ctx.profile_entries()
    out = {"array_floats": n, "launches_each": reps}
    for name, nbytes, lo, hi in spans:
        # every probe is a single kernel: one entry per launch (the untimed first launch sits just before lo)
        ms = [e[2] for e in ent[lo:hi]]
        best, med = min(ms), statistics.median(ms)
        if name == "mfma":
            fl = ent[lo][1]
            out["mfma_fp32"] = {"kernel": ent[lo][0], "best_tflops": fl / (best * 1e-3) / 1e12,
                                "median_tflops": fl / (med * 1e-3) / 1e12, "ms_best": best,
                                "frac_of_published_peak": fl / (best * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
        else:
            out[name] = {"kernel": ent[lo][0], "bytes": nbytes, "best_gbs": nbytes / (best * 1e-3) / 1e9,
                         "median_gbs": nbytes / (med * 1e-3) / 1e9, "ms_best": best,
                         "frac_of_published_peak": nbytes / (best * 1e-3) / 1e9 / PEAK_HBM_GBS}
    assert ctx.profile_count() >= was
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=None, help="override the per-GPU minibatch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="leave the per-kernel events out of the timed region")
    ap.add_argument("--no-calibration", action="store_true", help="skip the ceilings measured after the timed region")
    ap.add_argument("--profile-every", type=int, default=10,
                    help="record the per-kernel HIP events on every P-th step of the timed region (the two event "
                         "records around each launch cost about 0.5 ms per VGG-A step; default: steps 0, 10, ...)")
    ap.add_argument("--separate-sgd", action="store_true",
                    help="store the weight gradients and update in one pass at the end instead of inside their reductions")
    ap.add_argument("--per-kernel", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--calibrate", action="store_true",
                    help="instead of the benchmark: the ceilings alone (register-only MFMA loop; read, write and copy "
                         "streams and both SGD updates over arrays of VGG-A's 132.9 M parameters), as one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark: three plain 1 GiB device-to-device copies (cnn_probe_stream), the "
                         "known-size kernel that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share of the minibatch only; "
              "nothing here uses a second GPU (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1602_06709_amd import binding as cnn, synth
    from paper_1602_06709_amd.net import Net

    cnn.ensure_built()
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        ctx = cnn.Context()
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written per launch
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.zeros(n, dtype=torch.float32, device="cuda")
        for _ in range(3):
            cnn.cnn_probe_stream(ctx, cnn.STREAM_COPY, src, dst)
        torch.cuda.synchronize()
        assert bool((dst[:: 1 << 20] == 1).all())
        print(json.dumps({"calibrate_copy": {"kernel": "k_probe_stream<2>", "launches": 3, "bytes_read_per_launch": 4 * n,
                                             "bytes_written_per_launch": 4 * n}}))
        return
    if args.calibrate:
        ctx = cnn.Context()
        print(json.dumps({"calibration": calibrate(cnn, ctx, torch, 132851392)}))
        return
    wl = synth.workload(args.config, args.batch)
    N = wl.input_shape[0]
    ctx = cnn.Context()
    net = Net(ctx, wl, synth.make_weights(wl), fuse_sgd=not args.separate_sgd)
    net.set_input(synth.make_input(wl), synth.make_labels(wl) if wl.loss else None)
    upstream = None if wl.loss else torch.from_numpy(synth.make_upstream(wl)).cuda()

    def step():
        if upstream is not None:
            net.gact[-1].copy_(upstream)     # device-to-device; the gradient buffer is overwritten by backward
        net.step()

    bus = getattr(torch.cuda.get_device_properties(0), "pci_bus_id", None)
    clocks = Clocks("%02x:00.0" % bus if isinstance(bus, int) else None)
    clock_report = {"idle_before_warmup": clocks.read()}
    for i in range(args.warmup):
        # the last warm-up step runs with the per-kernel events on: the library creates its event objects the first
        # time a launch is recorded, and that must not happen inside the timed region
        ctx.profile(not args.no_profile and i == args.warmup - 1)
        step()
    ctx.profile(False)
    torch.cuda.synchronize()
    prof_steps = [] if args.no_profile else [i for i in range(args.steps) if i % max(1, args.profile_every) == 0]
    ctx.profile_reset()
    marks = []
    # per-step events on the stream the library launches on (its context was bound to torch's current stream)
    assert ctx.stream.cuda_stream == torch.cuda.current_stream().cuda_stream
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i].record()
        ctx.profile(i in prof_steps)         # a host-side flag: no GPU work, no synchronisation
        net.marks = marks if i in prof_steps else None     # which profile entries belong to which call (host list)
        step()
    ev[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    clock_report["right_after_timed_region"] = clocks.read()
    clock_report["source"] = clocks.files or "no readable pp_dpm_sclk / pp_dpm_mclk under /sys/class/drm"
    ctx.profile(False)
    net.marks = None
    ms_per_step = dt / args.steps * 1e3
    per_step = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    plain = [t for i, t in enumerate(per_step) if i not in prof_steps] or per_step
    step_ms = {"mean": sum(per_step) / len(per_step), "median": statistics.median(per_step), "best": min(per_step),
               "worst": max(per_step), "median_of_steps_without_kernel_events": statistics.median(plain),
               "all": [round(t, 4) for t in per_step]}
    loss = float(net.loss_per_sample.mean().item()) if wl.loss else None
    # a run whose numbers have left the finite range has timed something else (zeros and NaNs also change the clocks)
    finite = all(bool(torch.isfinite(w).all()) for w in net.w) and (loss is None or np.isfinite(loss))
    if not finite:
        print("bench.py: non-finite weights or loss after the timed steps: the measurement is void", file=sys.stderr)
        sys.exit(1)
    entries = [] if args.no_profile else ctx.profile_entries()

    # ---- the box's own ceilings and the stand-alone SGD update (the default step folds the update into the weight
    # gradients), measured after the timed region
    calib = None
    if not args.no_calibration:
        ctx.profile_reset()
        calib = calibrate(cnn, ctx, torch, net.arena_elems if wl.sgd else 132851392)
    sustained_tf = calib["mfma_fp32"]["best_tflops"] if calib else None
    sgd_alone = None
    if calib and wl.sgd:
        c = calib["sgd_momentum" if net.v_arena is not None else "sgd_plain"]
        sgd_alone = {"kernel": c["kernel"], "bound": "hbm", "achieved": c["best_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": c["best_gbs"] / PEAK_HBM_GBS, "frac_of_measured_copy_stream": c["best_gbs"] / calib["copy"]["best_gbs"],
                     "bytes_per_param": 20 if net.v_arena is not None else 12, "avg_launch_ms": c["ms_best"],
                     "median_gbs": c["median_gbs"],
                     "note": "cnn_sgd_update over arrays of the parameter arena's size, outside the timed region (best of 5)"}

    # ---- algorithmic FLOPs of one step (Section 3.1 formula; first layer has no backpropagation)
    shp = [tuple(wl.input_shape)] + synth.shapes(wl)
    flops, first = 0.0, True
    for i, L in enumerate(wl.layers):
        if L[0] == "conv":
            f = 2.0 * N * L[1] * L[2] * L[3] * L[4] * shp[i + 1][2] * shp[i + 1][3]
        elif L[0] == "fc":
            f = 2.0 * N * L[1] * L[2]
        else:
            continue
        flops += f * (2 if first else 3)
        first = False

    # ---- HBM traffic per launch of each kernel, from the committed rocprofv3 --pmc summary of this same command:
    # quoted only when that summary was taken from the kernel sources this run was built from
    traffic, traffic_note = {}, None
    tpath = os.path.join(ROOT, "profiles", "vgg_a_full_n64_hbm_traffic.txt")
    if args.config == 3 and args.batch is None and os.path.exists(tpath):
        sha = None
        for line in open(tpath):
            if line.startswith("csrc_sha |"):
                sha = line.split("|")[1].strip()
            if line.startswith("traffic_bytes_per_launch |"):
                _, name, val = [t.strip() for t in line.split("|")]
                traffic[name] = int(val)
        if sha != csrc_sha():
            traffic, traffic_note = {}, (f"profiles/vgg_a_full_n64_hbm_traffic.txt was taken from kernel sources {sha}, "
                                         f"this run is built from {csrc_sha()}: not quoted")
        else:
            traffic_note = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, profiles/vgg_a_full_n64_hbm_traffic.txt"

    # ---- per-kernel table from the library's own events
    kern = {}
    layers_out = []
    if entries:
        for name, fl, ms in entries:
            k = kern.setdefault(name, [0, 0.0, 0.0])
            k[0] += 1; k[1] += fl; k[2] += ms
        # per layer and pass: every kernel a call launched (second-stage reductions, weight transposes included)
        per_call, lo = {}, 0
        for op, layer, hi, nbytes in marks:
            c = per_call.setdefault((layer, op), [0.0, 0.0, 0])
            for name, fl, ms in entries[lo:hi]:
                c[0] += fl; c[1] += ms
            c[2] += nbytes
            lo = hi
        for (layer, op), (fl, ms, nbytes) in sorted(per_call.items(), key=lambda kv: (kv[0][0] < 0, kv[0])):
            ms_step = ms / len(prof_steps)
            desc = "-" if layer < 0 else " ".join(str(t) for t in wl.layers[layer])
            tf = fl / (ms * 1e-3) / 1e12 if fl and ms > 0 else None
            gbs = nbytes / (ms * 1e-3) / 1e9 if nbytes and ms > 0 else None
            ai = fl / nbytes if fl and nbytes else None
            layers_out.append({"layer": layer, "desc": desc, "call": op, "ms": ms_step, "tflops": tf,
                               "algorithmic_bytes": nbytes // len(prof_steps) if nbytes else None,
                               "flop_per_byte": ai,
                               "bound": None if not (fl or nbytes) else ("hbm" if ai is None or ai < RIDGE_FLOP_PER_BYTE else "mfma"),
                               "frac_fp32_mfma_peak": tf / PEAK_FP32_MFMA_TFLOPS if tf else None,
                               "frac_of_sustained_mfma": tf / sustained_tf if tf and sustained_tf else None,
                               "gbs": gbs, "frac_hbm": gbs / PEAK_HBM_GBS if gbs else None})
        if args.per_kernel:
            for r in layers_out:
                print("layer %3d %-26s %-28s %8.4f ms  %-44s %s" % (
                    r["layer"], r["desc"], r["call"], r["ms"],
                    ("%6.1f TF/s  %4.1f%% of fp32 MFMA peak" % (r["tflops"], 100 * r["frac_fp32_mfma_peak"])) if r["tflops"] else "",
                    ("%7.0f GB/s %4.1f%% of HBM  [%s]" % (r["gbs"], 100 * r["frac_hbm"], r["bound"])) if r["gbs"] else ""),
                    file=sys.stderr)
    roofline = None
    kernels_out = []
    if kern:
        tot_ms = sum(v[2] for v in kern.values())
        for name, (cnt, fl, ms) in sorted(kern.items(), key=lambda kv: -kv[1][2]):
            kernels_out.append({"kernel": name, "launches_per_step": cnt / len(prof_steps), "avg_ms": ms / cnt,
                                "tflops": fl / (ms * 1e-3) / 1e12 if fl else None, "share": ms / tot_ms})
        if args.per_kernel:
            for k in kernels_out:
                print("%-62s n/step %5.1f avg %9.4f ms  %s  share %5.1f%%" % (
                    k["kernel"], k["launches_per_step"], k["avg_ms"],
                    ("%6.1f TF/s" % k["tflops"]) if k["tflops"] else "           ", 100 * k["share"]), file=sys.stderr)
        dom = kernels_out[0]
        cnt, fl, ms = kern[dom["kernel"]]
        if fl > 0:
            ach = fl / (ms * 1e-3) / 1e12
            roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS,
                        "unit": "TFLOP/s", "frac": ach / PEAK_FP32_MFMA_TFLOPS,
                        "frac_of_sustained": ach / sustained_tf if sustained_tf else None,
                        "traffic": traffic.get(dom["kernel"]), "traffic_source": traffic_note,
                        "launches": cnt, "avg_launch_ms": ms / cnt, "flops_per_launch": fl / cnt,
                        "share_of_step": dom["share"],
                        "timing": "HIP events recorded by the library around each launch (rocprofv3's kernel trace reads "
                                  "about 1 % longer durations for the same launches: profiles/)"}
        else:
            roofline = {"kernel": dom["kernel"], "bound": "hbm", "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": None, "traffic": None, "launches": cnt, "avg_launch_ms": ms / cnt}
        # the SGD update against the HBM roof (12 B/param plain, 20 B/param with momentum)
        for name, (cnt, fl, ms) in kern.items():
            if name.startswith("k_sgd"):
                bpp = 20 if "momentum" in name else 12
                gbs = net.arena_elems * bpp / (ms / cnt * 1e-3) / 1e9
                roofline["sgd_update"] = {"kernel": name, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS,
                                          "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "bytes_per_param": bpp,
                                          "avg_launch_ms": ms / cnt,
                                          "frac_of_measured_copy_stream": gbs / calib["copy"]["best_gbs"] if calib else None}
        if sgd_alone and "sgd_update" not in roofline:
            roofline["sgd_update"] = sgd_alone
        # all contraction kernels together (conv fwd/bwd-data, weight gradient, FC GEMMs)
        cfl = sum(v[1] for v in kern.values()); cms = sum(v[2] for v in kern.values() if v[1] > 0)
        call = cfl / (cms * 1e-3) / 1e12
        roofline["all_contractions"] = {"achieved": call, "frac": call / PEAK_FP32_MFMA_TFLOPS,
                                        "frac_of_sustained": call / sustained_tf if sustained_tf else None,
                                        "unit": "TFLOP/s", "share_of_step": cms / tot_ms}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload (about 15 s of CPU work)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from oracle import net as onet
        n_cpu = int(min(N, max(1, round(15.0 * 35e9 / (flops / N)))))     # the oracle runs at roughly 35 GFLOP/s here
        wl1 = synth.workload(args.config, n_cpu)
        w1 = synth.make_weights(wl1)
        x1 = synth.make_input(wl1)
        lab1 = synth.make_labels(wl1) if wl1.loss else None
        up1 = None if wl1.loss else synth.make_upstream(wl1)
        tim = {}
        c0 = time.perf_counter()
        onet.run_step(wl1.layers, x1, w1, lab1, up1, timings=tim)
        cdt = time.perf_counter() - c0
        cpu = {"value": n_cpu / cdt, "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"a minibatch of {n_cpu} through every layer of {wl.name} (forward, loss, weight gradients, "
                         f"backpropagation; no SGD), {cdt:.1f} s of oracle time",
               "gflops": flops / N * n_cpu / cdt / 1e9}

    tflops = flops / (ms_per_step * 1e-3) / 1e12
    config = {"workload": f"{wl.name}_n{N}", "config_id": args.config, "per_gpu_minibatch": N,
              "passes": "fwd+loss+bwd" + ("+sgd" if wl.sgd else ""), "params": net.n_params,
              "lr": wl.lr, "momentum": wl.momentum}
    if args.config == 3:
        config["lr_note"] = ("the configuration names lr 0.01; from He-normal weights on N(0,1) images that diverges "
                             "within five steps (the run would time NaNs), so the step runs lr 0.001: a scalar operand, "
                             "the work per step is identical")
    out = {
        "metric": "VGG-A conv+FC fwd+bwd images/sec on 1 MI355X; % fp32 MFMA peak per layer" if args.config == 3
                  else f"{wl.name} fwd+bwd images/sec on 1 MI355X",
        "value": N * args.steps / dt, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": config,
        "step_ms": step_ms,
        "images_per_s_median_step": N / (step_ms["median"] * 1e-3),
        "images_per_s_best_step": N / (step_ms["best"] * 1e-3),
        "tflops": tflops,
        "frac_fp32_mfma_peak": tflops / PEAK_FP32_MFMA_TFLOPS,
        "frac_of_sustained_mfma": tflops / sustained_tf if sustained_tf else None,
        "algorithmic_gflop_per_step": flops / 1e9,
        "loss": loss,
        "roofline": roofline,
        "calibration": calib,
        "clocks": clock_report,
        "profiled_steps": prof_steps,
        "cpu_baseline": cpu,
        "kernels": kernels_out,
        "layers": layers_out,
        "context": {"paper_vgg_a_training_images_per_s": 30, "paper_hardware": "2 x 16-core Xeon E5-2698v3 (Section 5.1)"},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
