#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: one step = forward + loss + backward (+ SGD) of a workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]

Default workload (config 3): VGG-A, all conv + FC layers, per-GPU minibatch 64, fp32, forward + softmax
cross-entropy + backward + SGD (lr 0.01, momentum 0.9), synthetic N(0,1) images, He-normal weights -- the
workload BASELINE.json's metric ("VGG-A conv+FC fwd+bwd images/sec on 1 MI355X") is quoted on.
Prints ONE JSON line.  Inputs are resident in HBM before the timed region starts.

`roofline` describes the dominant kernel (largest share of the timed region): achieved = algorithmic
FLOPs of its launches / their summed duration, measured with HIP events that the library records on
its own stream around every kernel launch, inside the timed region, on every 5th timed step
(`--profile-every`, `profiled_steps` in the output): the event records cost ~2 % of a step.
`cpu_baseline` is the CPU oracle (the plain fp64 loop nest, untuned) timed on this machine's host cores on
a bounded sample: a small minibatch (about 15 s of CPU work) through every layer of the same network.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # 256 CUs x 256 FLOP/clk x 2.4 GHz (published dense fp32 matrix peak)
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=None, help="override the per-GPU minibatch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="leave the per-kernel events out of the timed region")
    ap.add_argument("--profile-every", type=int, default=5,
                    help="record the per-kernel HIP events on every P-th step of the timed region (the two event "
                         "records around each launch cost about 0.5 ms per VGG-A step; default: steps 0, 5, ...)")
    ap.add_argument("--separate-sgd", action="store_true",
                    help="store the weight gradients and update in one pass at the end instead of inside their reductions")
    ap.add_argument("--per-kernel", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark: three plain 1 GiB device-to-device copies (libcnn's identity "
                         "re-layout, SW=1), the known-size kernel that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "readings are scaled by")
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
        src = torch.ones((1, n // 4096, 64, 64), dtype=torch.float32, device="cuda")
        for _ in range(3):
            dst = cnn.cnn_pack_act(ctx, src, 1)       # SW = 1: the identity permutation, a plain copy
        torch.cuda.synchronize()
        assert bool((dst.view(-1)[:: 1 << 20] == 1).all())
        print(json.dumps({"calibrate_copy": {"kernel": "k_pack_blocked", "launches": 3, "bytes_read_per_launch": 4 * n,
                                             "bytes_written_per_launch": 4 * n}}))
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    prof_steps = [] if args.no_profile else [i for i in range(args.steps) if i % max(1, args.profile_every) == 0]
    ctx.profile_reset()
    marks = []
    t0 = time.perf_counter()
    for i in range(args.steps):
        ctx.profile(i in prof_steps)         # a host-side flag: no GPU work, no synchronisation
        net.marks = marks if i in prof_steps else None     # which profile entries belong to which call (host list)
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile(False)
    ms_per_step = dt / args.steps * 1e3
    loss = float(net.loss_per_sample.mean().item()) if wl.loss else None
    # a run whose numbers have left the finite range has timed something else (zeros and NaNs also change the clocks)
    finite = all(bool(torch.isfinite(w).all()) for w in net.w) and (loss is None or np.isfinite(loss))
    if not finite:
        print("bench.py: non-finite weights or loss after the timed steps: the measurement is void", file=sys.stderr)
        sys.exit(1)

    # ---- the stand-alone SGD update (the default step folds it into the weight gradients): timed on its own after
    # the timed region, on the same arenas, so that its HBM rate is reported either way
    sgd_alone = None
    if wl.sgd and not args.no_profile:
        n_before = ctx.profile_count()
        ctx.profile(True)
        for _ in range(5):
            net.sgd()
        ctx.profile(False)
        torch.cuda.synchronize()
        ent = ctx.profile_entries()[n_before:]
        ms = sum(e[2] for e in ent) / len(ent)
        bpp = 20 if net.v_arena is not None else 12
        gbs = net.arena_elems * bpp / (ms * 1e-3) / 1e9
        sgd_alone = {"kernel": ent[0][0], "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "bytes_per_param": bpp, "avg_launch_ms": ms, "launches": len(ent),
                     "note": "cnn_sgd_update on the whole parameter arena, outside the timed region"}
        n_sgd_entries = len(ent)
    else:
        n_sgd_entries = 0

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

    # ---- HBM traffic per launch of each kernel, from the committed rocprofv3 --pmc summary of this same command
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "vgg_a_full_n64_hbm_traffic.txt")
    if args.config == 3 and args.batch is None and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch |"):
                _, name, val = [t.strip() for t in line.split("|")]
                traffic[name] = int(val)

    # ---- per-kernel table from the library's own events
    kern = {}
    layers_out = []
    if not args.no_profile:
        entries = ctx.profile_entries()
        entries = entries[:len(entries) - n_sgd_entries]
        for name, fl, ms in entries:
            k = kern.setdefault(name, [0, 0.0, 0.0])
            k[0] += 1; k[1] += fl; k[2] += ms
        # per layer and pass: every kernel a call launched (second-stage reductions, weight transposes included)
        per_call, lo = {}, 0
        for op, layer, hi in marks:
            c = per_call.setdefault((layer, op), [0.0, 0.0])
            for name, fl, ms in entries[lo:hi]:
                c[0] += fl; c[1] += ms
            lo = hi
        for (layer, op), (fl, ms) in sorted(per_call.items(), key=lambda kv: (kv[0][0] < 0, kv[0])):
            ms_step = ms / len(prof_steps)
            desc = "-" if layer < 0 else " ".join(str(t) for t in wl.layers[layer])
            tf = fl / (ms * 1e-3) / 1e12 if fl and ms > 0 else None
            layers_out.append({"layer": layer, "desc": desc, "call": op, "ms": ms_step, "tflops": tf,
                               "frac_fp32_mfma_peak": tf / PEAK_FP32_MFMA_TFLOPS if tf else None})
        if args.per_kernel:
            for r in layers_out:
                print("layer %3d %-26s %-28s %8.4f ms  %s" % (
                    r["layer"], r["desc"], r["call"], r["ms"],
                    ("%6.1f TF/s  %4.1f%% of fp32 MFMA peak" % (r["tflops"], 100 * r["frac_fp32_mfma_peak"])) if r["tflops"] else ""),
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
                        "traffic": traffic.get(dom["kernel"]), "launches": cnt, "avg_launch_ms": ms / cnt, "flops_per_launch": fl / cnt,
                        "share_of_step": dom["share"]}
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
                                          "avg_launch_ms": ms / cnt}
        if sgd_alone and "sgd_update" not in roofline:
            roofline["sgd_update"] = sgd_alone
        # all contraction kernels together (conv fwd/bwd-data, weight gradient, FC GEMMs)
        cfl = sum(v[1] for v in kern.values()); cms = sum(v[2] for v in kern.values() if v[1] > 0)
        roofline["all_contractions"] = {"achieved": cfl / (cms * 1e-3) / 1e12, "frac": cfl / (cms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
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

    out = {
        "metric": "VGG-A conv+FC fwd+bwd images/sec on 1 MI355X; % fp32 MFMA peak per layer" if args.config == 3
                  else f"{wl.name} fwd+bwd images/sec on 1 MI355X",
        "value": N * args.steps / dt, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}_n{N}", "config_id": args.config, "per_gpu_minibatch": N,
                   "passes": "fwd+loss+bwd" + ("+sgd" if wl.sgd else ""), "params": net.n_params,
                   "lr": wl.lr, "momentum": wl.momentum},
        "tflops": flops / (ms_per_step * 1e-3) / 1e12,
        "frac_fp32_mfma_peak": flops / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "algorithmic_gflop_per_step": flops / 1e9,
        "loss": loss,
        "roofline": roofline,
        "profiled_steps": prof_steps,
        "cpu_baseline": cpu,
        "kernels": kernels_out,
        "layers": layers_out,
        "context": {"paper_vgg_a_training_images_per_s": 30, "paper_hardware": "2 x 16-core Xeon E5-2698v3 (Section 5.1)"},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
