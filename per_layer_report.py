#!/usr/bin/env python3
"""Per-stage time, algorithmic work and fraction of the fp32 / HBM roofline of one on-line
training step, for every workload, as a markdown table on stdout.

    python3 per_layer_report.py > per_layer.md

Times are the device-side stage timers of CNN_MODE_PERSISTENT (microseconds workgroup 0 spends
on a stage's work items in the last image of a call; best of five calls of 64 images).  Work is
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
for name in ("cfg1", "cfg2b", "cfg3", "cfg4a", "cfg4b", "cfg5"):
    wl = synth.WORKLOADS[name]
    n = 64
    imgs, labs = synth.images(wl, n), synth.labels(wl, n)
    d_imgs = torch.from_numpy(imgs).cuda(); d_labs = torch.from_numpy(labs).cuda()
    g = synth.build_network(binding.Cnn(wl.arch), wl)
    table = None
    if wl.sparse_conv is not None:
        info0 = [g.layer_info(l) for l in range(g.num_layers)]
        convs = [l for l in range(1, g.num_layers) if info0[l]["kind"] == 1]
        l = convs[wl.sparse_conv]
        table = synth.connection_table(wl, info0[l]["maps"], info0[l - 1]["maps"])
    g.set_mode(binding.MODE_PERSISTENT)
    best = None
    for rep in range(5):
        g.train_many(d_imgs, d_labs, wl.lr); g.synchronize()
        st = g.stage_times()
        tot = sum(a + b for a, b in st)
        if best is None or tot < best[0]:
            best = (tot, st)
    st = best[1]
    info = [g.layer_info(l) for l in range(g.num_layers)]
    # trainable layers in order (pool folded into its conv), as the planner numbers them
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
