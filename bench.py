#!/usr/bin/env python3
"""Benchmark of the on-line training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B] [--mode auto|resident|persistent|stages]
                    [--headline cfg2a] [--no-per-config] [--no-extra] [--no-cpu-baseline]

One "step" is one cnn_train_many call: B consecutive images of the headline workload's seeded stream trained
on-line -- forward pass, delta pass, weight gradients and an SGD update after every image.  The stream is
resident in HBM before the timed region starts.  Prints ONE JSON line.

value        = images trained per second over the K timed steps (wall clock, synchronised).
roofline     = the dominant kernel's algorithmic bytes per launch / its mean launch duration, measured with HIP
               events on the launch stream, against the 8 TB/s HBM peak; traffic = HBM bytes per launch from the
               rocprofv3 counter summary under profiles/ (FETCH_SIZE + WRITE_SIZE, scaled by what the counters
               read for a copy of known size), labelled with the file it comes from, or null.
cpu_baseline = the CPU oracle (float32 instantiation, OpenMP over output maps) timed on a prefix of the same
               stream on this machine's host cores.
per_config   = the same for each of the seven benchmark architectures (and, as context, the paper's own NORB and
               CIFAR10 architectures): mode and kernels timed, on-line training and forward-only rates, work per
               image computed from the layer shapes (multiply-adds and compulsory bytes), the fraction of the
               bound that applies, the dependency bound (crossings between compute units x the measured time of
               one, or launches x the measured launch floor), and the oracle's rate on a prefix.
extra        = batched forward pass, on-line deformation, one call per image.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_PEAK_TFLOPS = 157.3      # vector and matrix fp32 alike
HBM_PEAK_GBS = 8000.0
MODE_NAMES = {0: "stages", 1: "persistent", 2: "resident"}
KERNEL_OF_MODE = {"resident": "k_resident", "persistent": "k_persistent", "stages": "per-stage kernels (sum)"}

# the paper's own architectures (Sec. 4.2, 4.3) on synthetic images of the data sets' shapes: context only
# (name, architecture, image shape, classes, what the paper says, fan-in of the tables above the first layer: 0 = full)
PAPER_NETS = [
    ("paper-cifar-100maps", "3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", (3, 32, 32), 10,
     "Table 3, 100 maps per layer: 93 s per epoch (50000 trained + 60000 forward passes, 2011 GPU)", 0),
    ("paper-cifar-200maps", "3x32x32-200C3-MP3-200C3-MP2-200C3-MP2-300N-100N-10N", (3, 32, 32), 10,
     "Table 3, 200 maps per layer: 248 s per epoch", 0),
    ("paper-cifar-300maps", "3x32x32-300C3-MP3-300C3-MP2-300C3-MP2-300N-100N-10N", (3, 32, 32), 10,
     "Table 3, 300 maps per layer: 532 s per epoch", 0),
    ("paper-norb", "2x96x96-300C6S1-MP2-500C4-MP4-500N-5N", (2, 96, 96), 5,
     "Table 2: 1141 s per epoch (set sizes not given in the paper)", 0),
    ("paper-mnist-deep", "1x29x29-20C4-MP2-40C2-60C3-80C3-MP2-100C2-120C3-150N-10N", (1, 29, 29), 10,
     "Table 1, 20M-40M-60M-80M-100M-120M-150N with random partial connectivity: no time given; kernel sizes and the "
     "share of connections kept (here half, in a regular pattern) are not given either", -2),
]


def measured_traffic(kernel, cfg, batch):
    """HBM bytes from a committed rocprofv3 --pmc summary (a text file with lines
    'traffic_bytes_per_launch: N batch: B', one per measured number B of images per call).
    Returns (bytes per launch at this batch or None, bytes per image, the B that figure was measured at,
    file name); all None when there is no file."""
    per_launch, per_image, at, src = None, None, None, None
    for name in ("%s_%s_train_traffic.txt" % (kernel, cfg), "%s_%s_train.txt" % (kernel, cfg)):
        try:
            for line in open(os.path.join(ROOT, "profiles", name)):
                if line.startswith("traffic_bytes_per_launch:"):
                    f = line.split()
                    n, b = int(f[1]), int(f[3])
                    if b == batch:
                        per_launch = n
                    if at is None or b == batch:
                        per_image, at, src = round(n / b), b, "profiles/" + name
        except (OSError, ValueError, IndexError):
            pass
        if src:
            break
    return per_launch, per_image, at, src


def layer_work(info, n_conn):
    """Multiply-adds of one image per trainable layer, from the layer shapes: forward (Sec. 2.2, 2.4), delta pull
    (Sec. 3.3, dense rectangle; none into the network input), weight gradients (Sec. 3.4, dense delta).
    n_conn[i] = connections of the i-th convolutional layer."""
    out = []
    ci = 0
    first = True
    for l in range(1, len(info)):
        a, p = info[l], info[l - 1]
        if a["kind"] == 1:
            fwd = n_conn[ci] * a["K"] * a.get("Kx", a["K"]) * a["h"] * a["w"]
            ci += 1
        elif a["kind"] == 3:
            fwd = a["maps"] * p["maps"] * p["h"] * p["w"]
        else:
            continue
        out.append({"layer": l, "fwd": fwd, "pull": 0 if first else fwd, "wgrad": fwd})
        first = False
    return out


def train_flop(work):
    return 2 * sum(w["fwd"] + w["pull"] + w["wgrad"] for w in work)


def fwd_flop(work):
    return 2 * sum(w["fwd"] for w in work)


def algorithmic_bytes_per_train_image(info, n_weights, image_floats, first_w):
    """Compulsory traffic of one on-line step, fp32: every weight read by the forward pass, read again by the
    delta pass (except the first layer, below which nothing is propagated), and read and written by the update;
    the image read twice (forward, first layer's weight gradients); every layer output written once and read
    once forward and once backward; one delta per pooled position written and read; arg-max bytes."""
    b = 4 * (4 * n_weights - first_w)
    b += 4 * 2 * image_floats
    for l in range(1, len(info)):
        n = info[l]["maps"] * info[l]["h"] * info[l]["w"]
        if info[l]["kind"] == 1:
            b += 4 * n
            pooled = l + 1 < len(info) and info[l + 1]["kind"] == 2
            if not pooled:
                b += 4 * 2 * n + 4 * 2 * n
        elif info[l]["kind"] == 2:
            b += 4 * 3 * n + 2 * n + 4 * 2 * n
        else:
            b += 4 * 3 * n + 4 * 2 * n
    return b


def algorithmic_bytes_per_forward_image(info, n_weights, image_floats):
    b = 4 * n_weights + 4 * image_floats
    for l in range(1, len(info)):
        n = info[l]["maps"] * info[l]["h"] * info[l]["w"]
        b += 4 * n if info[l]["kind"] == 1 else 4 * 2 * n
    return b


def time_steps(torch, fn, steps, warmup):
    """W untimed warm-up steps, then K steps: wall clock bracketed by synchronize on both sides, and HIP events
    around every launch on the launch stream."""
    stream = torch.cuda.current_stream()
    for k in range(warmup):
        fn(k)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record(stream)
        fn(warmup + k)
        ev[k][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) for a, b in ev]


def event_ms(torch, fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=1000, help="images per step (one cnn_train_many call)")
    ap.add_argument("--mode", choices=["auto", "resident", "persistent", "stages"], default="auto",
                    help="auto: resident where the network fits it, else one launch per stage")
    ap.add_argument("--headline", default="cfg2a", help="workload the scored line is measured on")
    ap.add_argument("--grid", type=int, default=0, help="workgroups of the persistent kernel (0 = automatic)")
    ap.add_argument("--ranks", type=int, default=0, help="resident mode: workgroups in the team (0 = automatic)")
    ap.add_argument("--xcd-stride", type=int, default=0, help="resident mode: 8 = team on one XCD, 1 = spread, 0 = automatic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--no-per-config", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--cpu-seconds-per-config", type=float, default=1.5)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (on-line SGD is a strict chain over images); "
                 "--gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch

    from paper_1102_0183_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    nets = []   # every handle made here is closed before the interpreter exits

    def pick_mode(net):
        if args.mode != "auto":
            m = {"resident": binding.MODE_RESIDENT, "persistent": binding.MODE_PERSISTENT,
                 "stages": binding.MODE_STAGES}[args.mode]
            if not net.mode_supported(m):
                m = binding.MODE_STAGES
        else:
            m = binding.MODE_RESIDENT if net.mode_supported(binding.MODE_RESIDENT) else binding.MODE_STAGES
        net.set_mode(m)
        if m == binding.MODE_PERSISTENT and args.grid:
            net.set_grid(args.grid)
        if m == binding.MODE_RESIDENT and (args.ranks or args.xcd_stride):
            net.set_team(args.ranks, args.xcd_stride)
        return MODE_NAMES[m]

    def make_net(workload):
        net = synth.build_network(binding.Cnn(workload.arch), workload)
        nets.append(net)
        return net, pick_mode(net)

    def shapes_of(net):
        info = [net.layer_info(l) for l in range(net.num_layers)]
        # connections of every convolutional layer, from the weight count of the layer (bias + K*Kx per connection)
        n_conn, first_w = [], None
        w_left = net.num_weights
        for l in range(1, len(info)):
            a, p = info[l], info[l - 1]
            if a["kind"] == 3:
                n = a["maps"] * (1 + p["maps"] * p["h"] * p["w"])
                w_left -= n
                first_w = n if first_w is None else first_w
        convs = [l for l in range(1, len(info)) if info[l]["kind"] == 1]
        full = [info[l]["maps"] * info[l - 1]["maps"] for l in convs]
        tabs = getattr(net, "_bench_tables", {})
        for i, l in enumerate(convs):
            n_conn.append(int(tabs[i].sum()) if i in tabs else full[i])
        if convs:
            l = convs[0]
            first_w = info[l]["maps"] + n_conn[0] * info[l]["K"] * info[l]["Kx"]
        return info, n_conn, first_w

    def dependency_bound(net, mode, info, us_per_image, floors):
        """The bound of a chain of dependent stages: how often one image's data must cross between compute units
        (resident mode) or how many kernels are launched per image (stage mode), times what one costs."""
        n_conv = sum(1 for a in info if a["kind"] == 1)
        if mode == "resident":
            ranks = net.resident_ranks() if hasattr(net, "resident_ranks") else 0
            count = 2 * (n_conv - 1) + 1
            if any(q.get("by_cols") for q in binding.resident_plan(net.arch).get("fc", [])):
                count += 2      # a hidden layer held by columns: its partial sums up, the deltas of its inputs down
            key = "crossing_us_%d_ranks" % ranks
            if key not in floors:
                floors[key] = net.measure_crossing(max(2, ranks), 64, 200)
            floor = floors[key]
            kind = "crossings between compute units (pooled maps up, partial sums of the first fully connected " \
                   "layer, deltas down), each an exchange of tagged words among %d ranks" % ranks
        else:
            lines = [ln for ln in net.plan_text().strip().split("\n") if ln.strip()]
            count = sum(1 for ln in lines if "barrier=1" in ln) if mode == "stages" else len(lines)
            if "launch_us" not in floors:
                floors["launch_us"] = net.measure_launch(500)
            floor = floors["launch_us"]
            kind = "kernel launches per image" if mode == "stages" else "grid barriers per image (priced at a launch)"
        us = count * floor
        return {"kind": kind, "count": count, "floor_us_each": round(floor, 3), "us": round(us, 2),
                "share_of_measured": round(us / us_per_image, 3)}

    def oracle_rate(workload, arch, image_shape, n_classes, seconds, tables=None, frontend=None, wts=None, imgs=None, labs=None):
        import oracle
        cores = oracle.set_threads(0)
        ref = oracle.Oracle(arch, 32)
        if workload is not None:
            synth.build_network(ref, workload)
        else:
            for ci, tab in (tables or {}).items():
                ref.set_connection_table(ci, tab)
            rng = np.random.default_rng(7)
            ref.set_weights(((rng.random(ref.num_weights, dtype=np.float32) - np.float32(0.5)) * np.float32(0.1)))
        t0 = time.perf_counter()
        ref.train_many(imgs[:1], labs[:1], 1e-3)
        one = time.perf_counter() - t0
        n = int(max(2, min(len(labs) - 1, seconds / max(one, 1e-6))))
        t0 = time.perf_counter()
        ref.train_many(imgs[1:1 + n], labs[1:1 + n], 1e-3)
        dt = time.perf_counter() - t0
        return {"value": round(n / dt, 2), "unit": "images/s", "cores": cores, "kind": "oracle",
                "sample": "images 1..%d of the same stream, float32 instantiation of the oracle, OpenMP over "
                          "output maps, %.1f s" % (n, dt)}

    floors = {}

    def measure_config(name, arch, workload, n_train, image_shape=None, n_classes=None, note=None, with_cpu=True, fan=0):
        """On-line training and forward-only rates of one architecture in the mode that runs it, with its work per
        image and bounds."""
        if workload is not None:
            net, mode = make_net(workload)
            if workload.sparse_conv is not None:
                convs = [l for l in range(1, net.num_layers) if net.layer_info(l)["kind"] == 1]
                l = convs[workload.sparse_conv]
                net._bench_tables = {workload.sparse_conv: synth.connection_table(
                    workload, net.layer_info(l)["maps"], net.layer_info(l - 1)["maps"])}
            imgs, labs = synth.images(workload, n_train), synth.labels(workload, n_train)
            lr = workload.lr
        else:
            net = binding.Cnn(arch)
            nets.append(net)
            tables = {}
            if fan:
                convs = [l for l in range(1, net.num_layers) if net.layer_info(l)["kind"] == 1]
                for ci in range(1, len(convs)):
                    tables[ci] = synth.regular_table(net.layer_info(convs[ci])["maps"], net.layer_info(convs[ci] - 1)["maps"], fan)
                    net.set_connection_table(ci, tables[ci])
            rng = np.random.default_rng(7)
            net.set_weights(((rng.random(net.num_weights, dtype=np.float32) - np.float32(0.5)) * np.float32(0.1)))
            mode = pick_mode(net)
            imgs = rng.uniform(-1, 1, (n_train,) + tuple(image_shape)).astype(np.float32)
            labs = rng.integers(0, n_classes, n_train).astype(np.int32)
            lr = 1e-3
        d_i, d_l = torch.from_numpy(imgs).to(dev), torch.from_numpy(labs).to(dev)
        info, n_conn, first_w = shapes_of(net)
        work = layer_work(info, n_conn)
        warm = max(8, n_train // 8)
        net.train_many(d_i, d_l, lr, n=warm)
        net.synchronize()
        us_plan_kernel = None
        if mode == "resident" and net.resident_static_id() == 0:
            # no kernel compiled into the library for this network: the one the build step compiled for it and left
            # as a code object (paper_1102_0183_amd/specialize.py), when there is one; else the kernel that reads its plan
            from paper_1102_0183_amd import specialize
            path = specialize.built_code_object(net)
            if path:
                us_plan_kernel = 1e3 * event_ms(torch, lambda: net.train_many(d_i, d_l, lr)) / n_train
                net.load_resident_code(path)
                net.train_many(d_i, d_l, lr, n=warm)
                net.synchronize()
        ms = min(event_ms(torch, lambda: net.train_many(d_i, d_l, lr)) for _ in range(2))
        us_train = 1e3 * ms / n_train
        net.forward_many(d_i, warm)
        net.synchronize()
        ms_f = min(event_ms(torch, lambda: net.forward_many(d_i, n_train)) for _ in range(2))
        assert np.isfinite(net.get_weights()).all(), "training diverged on " + name
        fl, by = train_flop(work), algorithmic_bytes_per_train_image(info, net.num_weights, net.image_size, first_w)
        t_f32, t_hbm = fl / (FP32_PEAK_TFLOPS * 1e12) * 1e6, by / (HBM_PEAK_GBS * 1e9) * 1e6
        bound = "fp32" if t_f32 >= t_hbm else "hbm"
        t_bound = max(t_f32, t_hbm)
        kernels = {"resident": "k_resident (one cooperative launch per call)" +
                               (", compiled for this network and loaded as a code object" if us_plan_kernel else ""),
                   "persistent": "k_persistent (one cooperative launch per call)",
                   "stages": "one launch per stage: " + ", ".join(
                       sorted({ln.split()[1] for ln in net.plan_text().strip().split("\n") if ln.strip()}))}[mode]
        traffic, traffic_image, traffic_at, src = measured_traffic(
            KERNEL_OF_MODE[mode].split()[0] if mode != "stages" else "stage_kernels", name, n_train)
        rec = {
            "name": name, "arch": arch, "mode": mode, "kernels": kernels,
            "train": {"images_per_s": round(1e6 / us_train, 1), "us_per_image": round(us_train, 2), "images": n_train},
            "forward_only": {"images_per_s": round(n_train / (ms_f * 1e-3), 1), "us_per_image": round(1e3 * ms_f / n_train, 2)},
            "weights": net.num_weights,
            "train_mflop_per_image": round(fl / 1e6, 3), "forward_mflop_per_image": round(fwd_flop(work) / 1e6, 3),
            "train_bytes_per_image": by,
            "achieved_tflops": round(fl / (us_train * 1e-6) / 1e12, 4),
            "achieved_gbs": round(by / (us_train * 1e-6) / 1e9, 2),
            "bound": bound, "t_at_fp32_peak_us": round(t_f32, 3), "t_at_hbm_peak_us": round(t_hbm, 3),
            "frac": round(t_bound / us_train, 5),
            "dependency_bound": dependency_bound(net, mode, info, us_train, floors),
            "traffic": traffic, "traffic_bytes_per_image": traffic_image, "traffic_measured_at_images_per_call": traffic_at,
            "traffic_source": src,
        }
        if mode == "resident" and workload is not None:
            import per_layer_report
            _, lay = per_layer_report.trainable_layers(net, workload)
            rows, us0 = per_layer_report.resident_phase_rows(net, workload, d_i.view(-1)[:64 * net.image_size].contiguous(),
                                                             d_l[:64].contiguous(), lay, lr)
            rec["per_layer"] = {"unit": "phases of one image, rank 0 of %d" % net.resident_ranks(),
                                "us_per_image_rank0": round(us0, 2), "phases": rows}
        if us_plan_kernel:
            rec["train_with_the_kernel_reading_its_plan_us_per_image"] = round(us_plan_kernel, 2)
        if note:
            rec["paper_context"] = note
        if with_cpu and not args.no_cpu_baseline:
            rec["cpu_baseline"] = oracle_rate(workload, arch, image_shape, n_classes, args.cpu_seconds_per_config,
                                              tables=None if workload is not None else tables, imgs=imgs, labs=labs)
        net.close()
        nets.remove(net)
        del d_i, d_l
        return rec

    # ---- headline: on-line training of the headline workload's stream
    wl = synth.WORKLOADS[args.headline]
    n_stream = min(wl.n_images, 60000)
    imgs = synth.images(wl, n_stream)
    labs = synth.labels(wl, n_stream)
    d_imgs = torch.from_numpy(imgs).to(dev)
    d_labs = torch.from_numpy(labs).to(dev)
    B = min(args.batch, n_stream)
    per_epoch = n_stream // B

    def train_fn(net):
        sz = net.image_size

        def fn(k):
            o = (k % per_epoch) * B
            net.train_many(d_imgs.view(-1)[o * sz:(o + B) * sz], d_labs[o:o + B], wl.lr, n=B)
        return fn

    def fwd_fn(net):
        sz = net.image_size

        def fn(k):
            o = (k % per_epoch) * B
            net.forward_many(d_imgs.view(-1)[o * sz:(o + B) * sz], B)
        return fn

    net, mode = make_net(wl)
    info, n_conn, first_w = shapes_of(net)
    work = layer_work(info, n_conn)
    wall, kernel_ms = time_steps(torch, train_fn(net), args.steps, args.warmup)
    net.synchronize()
    assert np.isfinite(net.get_weights()).all(), "training diverged"
    value = args.steps * B / wall
    ms_per_step = 1e3 * wall / args.steps
    kern_ms = float(np.mean(kernel_ms))
    bytes_img = algorithmic_bytes_per_train_image(info, net.num_weights, net.image_size, first_w)
    flop_img = train_flop(work)
    achieved = bytes_img * B / (kern_ms * 1e-3) / 1e9
    traffic, _, _, traffic_src = measured_traffic(KERNEL_OF_MODE[mode].split()[0], args.headline, B)
    if traffic is None:
        traffic_src = None
    roofline = {
        "bound": "hbm", "kernel": KERNEL_OF_MODE[mode],
        "achieved": round(achieved, 3), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 6), "traffic": traffic, "traffic_source": traffic_src,
        "algorithmic_bytes_per_image": bytes_img, "images_per_launch": B,
        "launch_ms_mean": round(kern_ms, 4),
        "flop_per_image": flop_img, "achieved_tflops": round(flop_img * B / (kern_ms * 1e-3) / 1e12, 4),
        "us_per_image": round(1e3 * kern_ms / B, 3),
        "dependency_bound": dependency_bound(net, mode, info, 1e3 * kern_ms / B, floors),
    }
    out = {
        "metric": "online-training images/sec", "value": round(value, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %s, %d seeded %dx%dx%d images, %d uniform labels, on-line SGD lr=%g, weights "
                               "U[-0.05,0.05]" % ((args.headline, wl.arch, n_stream) + tuple(wl.raw_shape) + (wl.n_classes, wl.lr)),
                   "images_per_step": B, "mode": mode, "grid": args.grid, "ranks": args.ranks,
                   "xcd_stride": args.xcd_stride},
        "roofline": roofline,
    }
    if mode == "resident":
        # the per-layer share of the roofline in the mode just timed (BASELINE's metric asks for it): the phases of
        # one image as rank 0 of the team sees them (device clock stamps of the resident kernel), each with the
        # team's arithmetic and its share of the fp32 peak of the compute units the team occupies
        import per_layer_report
        _, layers = per_layer_report.trainable_layers(net, wl)
        rows, us_rank0 = per_layer_report.resident_phase_rows(net, wl, d_imgs.view(-1)[:64 * net.image_size].contiguous(),
                                                              d_labs[:64].contiguous(), layers, wl.lr)
        roofline["per_layer"] = {"unit": "phases of one image, rank 0 of %d" % net.resident_ranks(),
                                 "us_per_image_rank0": round(us_rank0, 2), "phases": rows}
    net.close()
    nets.remove(net)

    # ---- every benchmark architecture, each in the mode that runs it
    if not args.no_per_config:
        per = []
        sizes = {"cfg1": 1000, "cfg2a": 4000, "cfg2b": 4000, "cfg3": 1000, "cfg4a": 1000, "cfg4b": 600, "cfg5": 2000}
        for name in ("cfg1", "cfg2a", "cfg2b", "cfg3", "cfg4a", "cfg4b", "cfg5"):
            w_ = synth.WORKLOADS[name]
            per.append(measure_config(name, w_.arch, w_, sizes[name]))
        for name, arch, shape, ncls, note, fan in PAPER_NETS:
            per.append(measure_config(name, arch, None, 200 if "norb" not in name else 60, shape, ncls, note, fan=fan))
        out["per_config"] = per
        out["dependency_floors_us"] = {k: round(v, 3) for k, v in floors.items()}

    # ---- the other measurements the workload names
    if not args.no_extra:
        extra = {}
        k_steps = max(3, min(args.steps, 20))
        for key in ("cfg2a", "cfg2b"):
            w_ = synth.WORKLOADS[key]
            net, _ = make_net(w_)
            fbatch = 4096
            scratch = torch.empty(net.forward_batch_scratch_bytes(fbatch), dtype=torch.uint8, device=dev)
            d_probs = torch.empty(n_stream * net.num_classes, dtype=torch.float32, device=dev)
            src = d_imgs if w_.raw_shape == wl.raw_shape else torch.from_numpy(synth.images(w_, n_stream)).to(dev)
            net.forward_batch(src, n_stream, d_probs, scratch, fbatch)
            net.synchronize()
            best = min(event_ms(torch, lambda: net.forward_batch(src, n_stream, d_probs, scratch, fbatch)) for _ in range(3))
            assert torch.isfinite(d_probs).all()
            inf, nc, _ = shapes_of(net)
            tf = fwd_flop(layer_work(inf, nc)) * n_stream / (best * 1e-3) / 1e12
            extra[key + "_forward_batch_images_per_s"] = round(n_stream / (best * 1e-3), 1)
            extra[key + "_forward_batch_tflops"] = round(tf, 2)
            extra[key + "_forward_batch_fp32_mfma_frac"] = round(tf / FP32_PEAK_TFLOPS, 4)
            del scratch, d_probs
            net.close()
            nets.remove(net)
        for key, fb_o in (("cfg3", 512), ("cfg4a", 512), ("cfg4b", 256), ("cfg5", 1024)):
            wo = synth.WORKLOADS[key]
            net, _ = make_net(wo)
            n_b = 2 * fb_o
            ib = torch.from_numpy(synth.images(wo, n_b)).to(dev)
            scratch = torch.empty(net.forward_batch_scratch_bytes(fb_o), dtype=torch.uint8, device=dev)
            pb = torch.empty(n_b * net.num_classes, dtype=torch.float32, device=dev)
            net.forward_batch(ib, n_b, pb, scratch, fb_o)
            net.synchronize()
            ms = event_ms(torch, lambda: net.forward_batch(ib, n_b, pb, scratch, fb_o))
            inf, nc, _ = shapes_of(net)
            extra[key + "_forward_batch_images_per_s"] = round(n_b / (ms * 1e-3), 1)
            extra[key + "_forward_batch_fp32_mfma_frac"] = round(
                fwd_flop(layer_work(inf, nc)) * n_b / (ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS, 4)
            net.close()
            nets.remove(net)
            del ib, scratch, pb
        # on-line deformation of the training stream (Sec. 4.1): the whole stream in one call, then training with
        # every launch's images deformed just ahead of it on the same stream
        gp = binding.DeformParams(**synth.DEFORM_RECIPE)
        d_src4 = d_imgs.view(n_stream, *wl.raw_shape)
        d_def = torch.empty_like(d_src4)
        binding.deform_images(d_src4, d_def, n_stream, gp, synth.DEFORM_SEED, 0)
        torch.cuda.synchronize()
        best = min(event_ms(torch, lambda r=r: binding.deform_images(d_src4, d_def, n_stream, gp, synth.DEFORM_SEED,
                                                                     (r + 1) * n_stream)) for r in range(5))
        assert torch.isfinite(d_def).all()
        extra["%s_deform_images_per_s" % args.headline] = round(n_stream / (best * 1e-3), 1)
        extra["%s_deform_hbm_frac" % args.headline] = round(
            2 * 4 * int(np.prod(wl.raw_shape)) * n_stream / (best * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        net, _ = make_net(wl)
        buf = torch.empty((B,) + tuple(wl.raw_shape), dtype=torch.float32, device=dev)

        def deformed_step(k):
            o = (k % per_epoch) * B
            binding.deform_images(d_src4[o:o + B], buf, B, gp, synth.DEFORM_SEED, k * B)
            net.train_many(buf.view(-1), d_labs[o:o + B], wl.lr, n=B)
        wall, _ = time_steps(torch, deformed_step, k_steps, 2)
        extra["%s_train_with_deformation_images_per_s" % args.headline] = round(k_steps * B / wall, 1)
        del d_def, buf
        # launch cost: the same images through one cnn_train_step call each
        net.set_weights(synth.weights(wl, net.num_weights))
        sz = net.image_size
        lab_host = labs[:B].tolist()
        nstep = min(B, 500)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(nstep):
            net.train_step(d_imgs.view(-1)[t * sz:(t + 1) * sz], lab_host[t], wl.lr)
        torch.cuda.synchronize()
        extra["%s_train_step_calls_images_per_s" % args.headline] = round(nstep / (time.perf_counter() - t0), 1)
        net.close()
        nets.remove(net)
        # a network the library holds no kernel for: the resident kernel that reads its plan against the one
        # compiled for that network alone and loaded as a code object (paper_1102_0183_amd/specialize.py)
        from paper_1102_0183_amd import specialize
        arch_o = specialize.EXAMPLES["narrow"][0]
        net = binding.Cnn(arch_o)
        nets.append(net)
        rng = np.random.default_rng(7)
        net.set_weights(((rng.random(net.num_weights, dtype=np.float32) - np.float32(0.5)) * np.float32(0.1)))
        net.set_mode(binding.MODE_RESIDENT)
        n_o = 2000
        d_io = torch.from_numpy(rng.uniform(-1, 1, (n_o, net.image_size)).astype(np.float32)).to(dev)
        d_lo = torch.from_numpy(rng.integers(0, net.num_classes, n_o).astype(np.int32)).to(dev)
        net.train_many(d_io, d_lo, 1e-3)
        ms_plan = min(event_ms(torch, lambda: net.train_many(d_io, d_lo, 1e-3)) for _ in range(3))
        specialize.specialize(net)
        net.train_many(d_io, d_lo, 1e-3)
        ms_code = min(event_ms(torch, lambda: net.train_many(d_io, d_lo, 1e-3)) for _ in range(3))
        extra["other_net_arch"] = arch_o
        extra["other_net_kernel_reading_its_plan_us_per_image"] = round(1e3 * ms_plan / n_o, 2)
        extra["other_net_kernel_compiled_for_it_us_per_image"] = round(1e3 * ms_code / n_o, 2)
        net.close()
        nets.remove(net)
        out["extra"] = extra

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores
    if not args.no_cpu_baseline:
        import oracle
        cores = oracle.set_threads(0)
        ref = synth.build_network(oracle.Oracle(wl.arch, 32), wl)
        probe = 200 if wl.name.startswith(("cfg1", "cfg2", "cfg5")) else 4
        t0 = time.perf_counter()
        ref.train_many(imgs[:probe], labs[:probe], wl.lr)
        rate = probe / (time.perf_counter() - t0)
        n = int(max(probe, min(n_stream - probe, rate * args.cpu_seconds)))
        t0 = time.perf_counter()
        ref.train_many(imgs[probe:probe + n], labs[probe:probe + n], wl.lr)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(n / dt, 1), "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": "images %d..%d of the same stream, float32 instantiation of the oracle, "
                      "OpenMP over output maps, %.1f s" % (probe, probe + n, dt)}
        # the same oracle on one thread (the paper's own baseline was one optimised CPU thread)
        oracle.set_threads(1)
        n1 = max(2, min(300, int(rate / max(cores, 1) * 2)))
        t0 = time.perf_counter()
        ref.train_many(imgs[:n1], labs[:n1], wl.lr)
        out["cpu_baseline"]["single_thread_images_per_s"] = round(n1 / (time.perf_counter() - t0), 1)
        oracle.set_threads(0)
    for net in list(nets):
        net.close()
    print(json.dumps(out))
    sys.stdout.flush()


if __name__ == "__main__":
    main()
