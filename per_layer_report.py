#!/usr/bin/env python3
"""Per-stage time, algorithmic work and fraction of the fp32 / HBM roofline of one on-line
training step, for every workload, as markdown tables on stdout.

    python3 per_layer_report.py > per_layer.md

A network that runs in resident mode (what bench.py times it in) gets the time line of rank 0 through one image
-- device clock stamps around every phase of the resident kernel, best of five calls of 64 images -- with the
multiply-adds of the phases that have any, and what share of the fp32 peak of ONE compute unit's share of the team
that is.  Every network also gets the stage table of CNN_MODE_PERSISTENT (same stage functions as the one-launch-
per-stage mode, which is what bench.py times the networks in that resident mode cannot take; there the kernel
trace under profiles/ has the per-launch figures): microseconds workgroup 0 spends
on a stage's work items in the last image of a call; best of five calls of 64 images.  Work is
algorithmic: the multiply-adds and compulsory bytes of the stage as the method defines it (the
delta pull is scored against the dense rectangle it multiplies, the weight gradients against
the pooling winners only).  Bound = fp32 peak (157.3 TFLOP/s) when FLOP/B exceeds the machine
balance, else HBM (8 TB/s); a layer whose operands sit in L2 can exceed the HBM line.
"""
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import numpy as np
import torch

from paper_1102_0183_amd import binding, synth
PEAK_F32 = 157.3e12
PEAK_HBM = 8e12
out = []


def trainable_layers(g, wl):
    """The trainable layers in order (a pooling layer folded into its convolution), with their shapes and, for a
    convolutional layer, its number of connections."""
    info = [g.layer_info(l) for l in range(g.num_layers)]
    table = None
    if wl is not None and wl.sparse_conv is not None:
        convs = [l for l in range(1, g.num_layers) if info[l]["kind"] == 1]
        l = convs[wl.sparse_conv]
        table = synth.connection_table(wl, info[l]["maps"], info[l - 1]["maps"])
    layers = []
    for l in range(1, len(info)):
        if info[l]["kind"] == 2:
            layers[-1]["Kp"] = info[l]["K"]; layers[-1]["Hp"] = info[l]["h"]; layers[-1]["Wp"] = info[l]["w"]
            continue
        d = dict(info[l]); d["prev"] = info[l - 1]; d["Kp"] = 1; d["Hp"] = d["h"]; d["Wp"] = d["w"]
        layers.append(d)
    conv_i = 0
    for d in layers:
        if d["kind"] == 1:
            full = d["maps"] * d["prev"]["maps"]
            d["nconn"] = int(table.sum()) if (table is not None and conv_i == wl.sparse_conv) else full
            conv_i += 1
    return info, layers


def resident_phase_rows(g, wl, d_imgs, d_labs, layers, lr):
    """Time line of rank 0 through the last image but one of a call in resident mode: a list of
    {"phase", "at_us", "us", "mflop", "pct_of_team_fp32_peak"} (the last two None for a phase without arithmetic),
    and the time per image rank 0 sees."""
    g.set_mode(binding.MODE_RESIDENT)
    n_conv = sum(1 for d in layers if d["kind"] == 1)
    best = None
    for rep in range(5):
        g.train_many(d_imgs, d_labs, lr); g.synchronize()
        st = g.raw_stamps(128).astype(np.int64)
        if best is None or st[70] - st[0] < best[70] - best[0]:
            best = st
    st = best
    convs = [d for d in layers if d["kind"] == 1]
    fcs = [d for d in layers if d["kind"] == 3]
    fwd = lambda d: (d["nconn"] * d["K"] ** 2 * d["h"] * d["w"]) if d["kind"] == 1 else d["maps"] * d["prev"]["maps"] * d["prev"]["h"] * d["prev"]["w"]
    lab = lambda d: ("%dC%d" % (d["maps"], d["K"])) if d["kind"] == 1 else "%dN" % d["maps"]
    rows = [(1, "image into LDS", 0)]
    for l, d in enumerate(convs):
        rows.append((2 + 2 * l, "FP %s: inputs at hand (adjustments put off from the last image run here)" % lab(d), 0))
        rows.append((3 + 2 * l, "FP %s: multiply-adds, activation, pooling, outputs on their way" % lab(d), 2 * fwd(d)))
    rows += [(30, "FP %s: partial sums over the own columns, on their way" % lab(fcs[0]), 2 * fwd(fcs[0])),
             (31, "FP %s: partial sums of all ranks added" % lab(fcs[0]), 0),
             (32, "FP remaining fully connected layers", 2 * sum(fwd(d) for d in fcs[1:])),
             (33, "output units, error, output delta", 0),
             (34, "BP + AW remaining fully connected layers", 4 * sum(fwd(d) for d in fcs[1:])),
             (35, "BP + AW %s (own columns), deltas of the last conv layer on their way" % lab(fcs[0]), 4 * fwd(fcs[0]))]
    for l in range(n_conv - 1, -1, -1):
        d = convs[l]
        rows.append((40 + 4 * l, "%s: deltas on their way%s" % (lab(d), " (before that: AW of the pull copy of the layer above)" if l + 1 < n_conv else ""), 0))
        rows.append((41 + 4 * l, "AW %s, forward copy / biases" % lab(d), 2 * fwd(d) // max(1, d["Kp"] ** 2) if l == 0 else 0))
        if l >= 1:
            rows.append((42 + 4 * l, "BP through %s: deltas of all maps at hand" % lab(d), 0))
            rows.append((43 + 4 * l, "BP through %s: pull into the own maps below" % lab(d), 2 * fwd(d)))
    rows.append((70, "end of image (AW of the last pull copy before it)", 0))
    t0 = int(st[0])
    ranks = g.resident_ranks()
    res = []
    prev = t0
    for i, what, fl in sorted(rows, key=lambda r: int(st[r[0]])):
        t = int(st[i])
        if t < t0 or t == 0:
            continue
        took = (t - prev) * 0.01
        frac = (fl / (took * 1e-6) / (PEAK_F32 * ranks / 256.0)) if (fl and took > 0) else None
        res.append({"phase": what, "at_us": round((t - t0) * 0.01, 2), "us": round(took, 2),
                    "mflop": round(fl / 1e6, 3) if fl else None,
                    "pct_of_team_fp32_peak": round(100 * frac, 2) if frac else None})
        prev = t
    return res, (int(st[70]) - t0) * 0.01


def resident_phases(name, wl, g, d_imgs, d_labs, layers):
    rows, us = resident_phase_rows(g, wl, d_imgs, d_labs, layers, wl.lr)
    out.append("### %s  `%s`  resident mode, %d ranks%s: %.1f us per image as rank 0 sees it" %
               (name, wl.arch, g.resident_ranks(), ", inputs streamed" if g.resident_streams() else "", us))
    out.append("")
    out.append("| phase of rank 0 | at us | took us | MFLOP (whole team) | % of fp32 peak of the team's compute units |")
    out.append("|---|---|---|---|---|")
    for r in rows:
        out.append("| %s | %.2f | %.2f | %s | %s |" % (r["phase"], r["at_us"], r["us"], ("%.3f" % r["mflop"]) if r["mflop"] else "",
                                                    ("%.2f" % r["pct_of_team_fp32_peak"]) if r["pct_of_team_fp32_peak"] else ""))
    out.append("")


def main():
    for name in ("cfg1", "cfg2b", "cfg3", "cfg4a", "cfg4b", "cfg5"):
        wl = synth.WORKLOADS[name]
        n = 64
        imgs, labs = synth.images(wl, n), synth.labels(wl, n)
        d_imgs = torch.from_numpy(imgs).cuda(); d_labs = torch.from_numpy(labs).cuda()
        g = synth.build_network(binding.Cnn(wl.arch), wl)
        g.set_mode(binding.MODE_PERSISTENT)
        best = None
        for rep in range(5):
            g.train_many(d_imgs, d_labs, wl.lr); g.synchronize()
            st = g.stage_times()
            tot = sum(a + b for a, b in st)
            if best is None or tot < best[0]:
                best = (tot, st)
        st = best[1]
        info, layers = trainable_layers(g, wl)
        if g.mode_supported(binding.MODE_RESIDENT):
            resident_phases(name, wl, g, d_imgs, d_labs, layers)
            g.set_mode(binding.MODE_PERSISTENT)
        lines = [ln for ln in g.plan_text().strip().split("\n")]
        kinds = [(ln.split()[1], int(re.search(r"layer=(\d+)", ln).group(1))) for ln in lines]
        if len(kinds) != len(st):
            print(name, "stage list differs from plan text (%d vs %d): skipped" % (len(kinds), len(st))); g.close(); continue
        out.append("### %s  `%s`  (persistent mode, %d stages, %.1f us/image of stage work + %.1f us of grid barriers)" %
                   (name, wl.arch, len(st), sum(a for a, _ in st), sum(b for _, b in st)))
        out.append("")
        out.append("| stage | layer | us | MFLOP | KB | FLOP/B | bound | % of bound |")
        out.append("|---|---|---|---|---|---|---|---|")
        for (kind, li), (us, _) in zip(kinds, st):
            d = layers[li] if kind != "frontend" else None
            fl = by = 0
            if kind == "frontend":
                nf, h, w = info[0]["maps"], info[0]["h"], info[0]["w"]
                fl = 2 * nf * h * w * 25; by = 4 * (wl.raw_shape[0] * wl.raw_shape[1] * wl.raw_shape[2] + nf * h * w)
                label = "fixed filters"
            else:
                p = d["prev"]
                if d["kind"] == 1:
                    KK = d["K"] ** 2; P = d["h"] * d["w"]; HW = d["Hp"] * d["Wp"]; nin = p["maps"] * p["h"] * p["w"]
                    w_b = 4 * (d["nconn"] * KK + d["maps"])
                    label = "%dC%d" % (d["maps"], d["K"])
                    if kind in ("conv_fwd", "conv_mfma"):
                        fl = 2 * d["nconn"] * KK * P; by = 4 * nin + w_b + 4 * d["maps"] * (P + 2 * HW)
                    elif kind == "conv_epi":
                        fl = d["maps"] * P * 10; by = 4 * d["maps"] * (P + 2 * HW)   # plane sums are the kernel's own traffic, not algorithmic
                    elif kind == "conv_bwd_epi":
                        fl = nin * 4; by = 4 * nin * 2      # plane sums are the kernel's own traffic, not algorithmic
                    elif kind in ("conv_bwd", "conv_bwd_mfma"):
                        fl = 2 * d["nconn"] * KK * P; by = 4 * d["maps"] * HW * 2 + w_b + 4 * nin * 2    # dense count (the kernel multiplies the whole rectangle)
                    elif kind == "conv_wgrad":
                        fl = 2 * d["nconn"] * KK * HW; by = 4 * nin + 4 * d["maps"] * HW * 2 + 2 * w_b  # sparse count: winners only
                else:
                    nin = p["maps"] * p["h"] * p["w"]; nout = d["maps"]
                    w_b = 4 * (nin * nout + nout)
                    label = "%dN" % nout
                    if kind == "fc_fwd":
                        fl = 2 * nin * nout; by = w_b + 4 * (nin + nout)
                    elif kind == "head":
                        fl = 6 * nin * nout; by = 2 * w_b + 4 * (2 * nin + 2 * nout)
                    elif kind == "fc_bwd":
                        fl = 4 * nin * nout; by = 2 * w_b + 4 * (2 * nin + nout)
            t = us * 1e-6
            ai = fl / max(by, 1)
            bound = "FP32" if ai > PEAK_F32 / PEAK_HBM else "HBM"
            frac = (fl / t / PEAK_F32) if bound == "FP32" else (by / t / PEAK_HBM)
            out.append("| %s | %s | %.1f | %.3f | %.1f | %.1f | %s | %.2f |" % (kind, label, us, fl / 1e6, by / 1024, ai, bound, 100 * frac))
        out.append("")
        g.close()
    print("\n".join(out))


if __name__ == "__main__":
    main()
