"""Per-layer tile table: for every convolution layer of a workload, the tile the library's planner uses, its
bytes-per-FLOP in the traversal form of the paper's cache-blocking model (Section 2.2), and what the exhaustive
block search (run on the GPU through the C ABI) finds under this chip's limits.

    python -m paper_1602_06709_amd.tile_report [--config 3] [--batch 64] [--time]

Limits: accumulators of one workgroup 112 KB (128 features x 224 pixels, the largest tile the convolution kernel
instantiates), staging memory = 160 KB of LDS, 32-wide matrix-core tiles, input features staged 4 at a time.
The chip's own ratio is 8 TB/s / 157.3 TFLOP/s = 0.051 bytes per FLOP: a layer whose whole-layer ratio lies above
it is bound by HBM however it is tiled.
"""
import argparse
import json
import time

import torch

from . import binding as B
from . import synth

ACC_BYTES, LDS_BYTES, SIMD, CHUNK = 112 * 1024, 160 * 1024, 32, 4
CHIP_BF = 8.0e12 / 157.3e12


def conv_layers(wl):
    shp = [tuple(wl.input_shape)] + synth.shapes(wl)
    out = []
    for i, L in enumerate(wl.layers):
        if L[0] == "conv":
            _, c, k, r, s, st, pad = L
            n, _, h, w = shp[i]
            out.append((i, n, c, h, w, k, r, s, st, pad, shp[i + 1][2], shp[i + 1][3]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--time", action="store_true", help="also time the search kernels (candidates per second)")
    args = ap.parse_args()
    wl = synth.workload(args.config, args.batch)
    ctx = B.Context()
    L = B.lib()
    rows = []
    for (i, n, c, h, w, k, r, s, st, pad, p, q) in conv_layers(wl):
        layer = (n, c, k, p, q, r, s, st)
        row = {"layer": i, "shape": f"{c}->{k} {p}x{q} {r}x{s}/{st}", "bf_plane": L.cnn_bf_plane(p, q, r, s, st),
               "bf_layer": L.cnn_bf_layer(n, c, k, p, q, r, s, st)}
        for name, op in (("fwd", B.OP_CONV_FWD), ("bwd", B.OP_CONV_BWD_DATA)):
            info = B.cnn_conv_tile_info(op, n, c, h, w, k, r, s, st, pad)
            row[name] = None if info is None else {"features": info[0][0], "rows": info[0][1], "cols": info[0][2],
                                                   "slices": info[0][4], "lds": info[0][5], "workgroups": info[0][6],
                                                   "bf": info[1]}
        t0 = time.perf_counter()
        blk, bf, cnt = B.cnn_block_search_traversal(ctx, layer, ACC_BYTES, LDS_BYTES, SIMD, CHUNK)
        row["search_traversal"] = {"block": blk, "bf": bf, "feasible": cnt}
        blk, bf, cnt = B.cnn_block_search(ctx, layer, LDS_BYTES, SIMD)
        row["search_single_cache"] = {"block": blk, "bf": bf, "feasible": cnt, "candidates": n * max(1, k // SIMD) * c * p * q * r * s}
        row["search_ms"] = (time.perf_counter() - t0) * 1e3
        rows.append(row)
    print("%-5s %-24s %9s %9s | %-22s %8s | %-22s %8s | %-22s %8s | %8s" % (
        "layer", "shape", "B/F plane", "B/F layer", "fwd tile (f x r x c)", "B/F", "bwd tile", "B/F",
        "search (n,f,c,r,c)", "B/F", "1-cache"))
    for r_ in rows:
        def t(d):
            return ("%dx%dx%d%s" % (d["features"], d["rows"], d["cols"], "" if d["slices"] == 1 else (" runs" if d["slices"] < 0 else " /%d" % d["slices"])),
                    "%.4f" % d["bf"]) if d else ("(other kernel)", "-")
        f, b = t(r_["fwd"]), t(r_["bwd"])
        s_ = r_["search_traversal"]
        print("%-5d %-24s %9.4f %9.5f | %-22s %8s | %-22s %8s | %-22s %8.4f | %8.4f%s" % (
            r_["layer"], r_["shape"], r_["bf_plane"], r_["bf_layer"], f[0], f[1], b[0], b[1], str(s_["block"]), s_["bf"],
            r_["search_single_cache"]["bf"], "   HBM-bound" if r_["bf_layer"] > CHIP_BF else ""))
    print("chip ratio (8 TB/s / 157.3 TFLOP/s): %.4f bytes per FLOP" % CHIP_BF)
    if args.time:
        # the largest space of the table, timed with events on the library's stream
        big = max(rows, key=lambda r_: r_["search_single_cache"]["candidates"])
        i = big["layer"]
        (_, n, c, h, w, k, r, s, st, pad, p, q) = [x for x in conv_layers(wl) if x[0] == i][0]
        layer = (n, c, k, p, q, r, s, st)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.cnn_block_search(ctx, layer, LDS_BYTES, SIMD)
        torch.cuda.synchronize()
        e0.record()
        reps = 5
        for _ in range(reps):
            B.cnn_block_search(ctx, layer, LDS_BYTES, SIMD)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        cand = big["search_single_cache"]["candidates"]
        print(json.dumps({"block_search_timing": {"layer": big["shape"], "minibatch": n, "candidates": cand,
                                                  "feasible": big["search_single_cache"]["feasible"], "ms": ms,
                                                  "candidates_per_s": cand / (ms * 1e-3)}}))
    ctx.close()


if __name__ == "__main__":
    main()
