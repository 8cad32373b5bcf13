#!/usr/bin/env python3
"""Benchmark of the on-line training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B] [--mode resident|persistent|stages]

One "step" is one cnn_train_many call: B consecutive images of the 60,000-image synthetic
29x29 stream (workload cfg2) trained on-line -- forward, delta pass, weight gradients and an
SGD update after every image -- on the net 1x29x29-20C4-MP2-40C5-MP3-150N-10N.  The stream is
resident in HBM before the timed region starts.  Prints ONE JSON line.

value        = images trained per second over the K timed steps (wall clock, synchronised).
roofline     = the dominant kernel's algorithmic bytes per launch / its mean launch duration,
               measured with HIP events on the launch stream, against the 8 TB/s HBM peak;
               traffic = HBM bytes per launch from the rocprofv3 counter summary under profiles/
               (FETCH_SIZE + WRITE_SIZE, calibrated on a copy of known size), when one is there.
cpu_baseline = the CPU oracle (float32 instantiation, OpenMP over output maps) timed on a
               prefix of the same stream on this machine's host cores.
extra        = the other measurements the workload names (larger net, forward-only passes).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MFMA_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0
KERNEL_OF_MODE = {"resident": "k_resident", "persistent": "k_persistent", "stages": "per-stage kernels (sum)"}


def measured_traffic(mode, batch):
    """HBM bytes per launch of the mode's kernel on the benchmark workload, from the committed
    rocprofv3 --pmc summary (a text file with a line 'traffic_bytes_per_launch: N batch: B')."""
    path = os.path.join(ROOT, "profiles", "%s_cfg2a_train_traffic.txt" % KERNEL_OF_MODE[mode].split()[0])
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                f = line.split()
                if int(f[3]) == batch:
                    return int(f[1])
    except (OSError, ValueError, IndexError):
        pass
    return None


def forward_flops_per_image(info):
    """2 x multiply-accumulates of one forward pass, full connection tables (Sec. 2.2, 2.4)."""
    f = 0
    for l in range(1, len(info)):
        a, p = info[l], info[l - 1]
        if a["kind"] == 1:
            f += 2 * a["maps"] * a["h"] * a["w"] * p["maps"] * a["K"] ** 2
        elif a["kind"] == 3:
            f += 2 * a["maps"] * p["maps"] * p["h"] * p["w"]
    return f


def algorithmic_bytes_per_train_image(info, n_weights, image_floats):
    """Compulsory traffic of one on-line step, fp32: every weight read by the forward pass, read
    again by the delta pass (except the first layer, below which nothing is propagated), and read
    and written by the update; the image read twice (forward, first layer's weight gradients);
    every layer output written once and read once forward and once backward; one delta per
    pooled position written and read; arg-max bytes written and read."""
    first = info[1]
    first_w = first["maps"] * (1 + info[0]["maps"] * first["K"] ** 2) if first["kind"] == 1 else \
        first["maps"] * (1 + info[0]["maps"] * info[0]["h"] * info[0]["w"])
    b = 4 * (4 * n_weights - first_w)
    b += 4 * 2 * image_floats
    for l in range(1, len(info)):
        n = info[l]["maps"] * info[l]["h"] * info[l]["w"]
        if info[l]["kind"] == 1:      # conv: full-resolution output written once
            b += 4 * n
            pooled = l + 1 < len(info) and info[l + 1]["kind"] == 2
            if not pooled:
                b += 4 * 2 * n + 4 * 2 * n      # read fwd + bwd, delta write + read
        elif info[l]["kind"] == 2:    # pool: pooled values w + 2r, arg-max w + r, delta w + r
            b += 4 * 3 * n + 2 * n + 4 * 2 * n
        else:                         # fully connected: output w + 2r, delta w + r
            b += 4 * 3 * n + 4 * 2 * n
    return b


def algorithmic_bytes_per_forward_image(info, n_weights, image_floats):
    b = 4 * n_weights + 4 * image_floats
    for l in range(1, len(info)):
        n = info[l]["maps"] * info[l]["h"] * info[l]["w"]
        b += 4 * n if info[l]["kind"] == 1 else 4 * 2 * n
    return b


def time_steps(torch, fn, steps, warmup):
    """W untimed warm-up steps, then K steps: wall clock bracketed by synchronize on both sides,
    and HIP events around every launch on the launch stream."""
    stream = torch.cuda.current_stream()
    for k in range(warmup):
        fn(k)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record(stream)
        fn(warmup + k)
        ev[k][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [a.elapsed_time(b) for a, b in ev]
    return wall, kernel_ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=1000, help="images per step (one cnn_train_many call)")
    ap.add_argument("--mode", choices=["resident", "persistent", "stages"], default="resident")
    ap.add_argument("--grid", type=int, default=0, help="workgroups of the persistent kernel (0 = automatic)")
    ap.add_argument("--ranks", type=int, default=0, help="resident mode: workgroups in the team (0 = automatic)")
    ap.add_argument("--xcd-stride", type=int, default=0, help="resident mode: 8 = team on one XCD, 1 = spread, 0 = automatic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
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
    wl = synth.WORKLOADS["cfg2a"]
    n_stream = wl.n_images
    imgs = synth.images(wl)
    labs = synth.labels(wl)
    d_imgs = torch.from_numpy(imgs).to(dev)
    d_labs = torch.from_numpy(labs).to(dev)
    B = min(args.batch, n_stream)
    per_epoch = n_stream // B

    def make_net(workload, grid=0):
        net = binding.Cnn(workload.arch)
        net.set_mode({"resident": binding.MODE_RESIDENT, "persistent": binding.MODE_PERSISTENT,
                      "stages": binding.MODE_STAGES}[args.mode])
        if grid:
            net.set_grid(grid)
        if args.mode == "resident" and (args.ranks or args.xcd_stride):
            net.set_team(args.ranks, args.xcd_stride)
        net.set_weights(synth.weights(workload, net.num_weights))
        return net

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

    # ---- headline: on-line training, small cfg2 net
    net = make_net(wl, args.grid)
    info = binding.arch_info(wl.arch)
    wall, kernel_ms = time_steps(torch, train_fn(net), args.steps, args.warmup)
    net.synchronize()
    w_end = net.get_weights()
    assert np.isfinite(w_end).all(), "training diverged"
    value = args.steps * B / wall
    ms_per_step = 1e3 * wall / args.steps
    kern_ms = float(np.mean(kernel_ms))
    bytes_img = algorithmic_bytes_per_train_image(info, net.num_weights, net.image_size)
    achieved = bytes_img * B / (kern_ms * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "kernel": KERNEL_OF_MODE[args.mode],
        "achieved": round(achieved, 3), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 6), "traffic": measured_traffic(args.mode, B),
        "algorithmic_bytes_per_image": bytes_img, "images_per_launch": B,
        "launch_ms_mean": round(kern_ms, 4),
        "flop_per_image": 10.9e6, "achieved_tflops": round(10.9e6 * B / (kern_ms * 1e-3) / 1e12, 4),
        "us_per_image": round(1e3 * kern_ms / B, 3),
    }
    out = {
        "metric": "online-training images/sec", "value": round(value, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "cfg2 small net: %s, 60000 seeded 1x29x29 images U[-1,1], 10 uniform labels, "
                               "on-line SGD lr=0.001, weights U[-0.05,0.05]" % wl.arch,
                   "images_per_step": B, "mode": args.mode, "grid": args.grid, "ranks": args.ranks,
                   "xcd_stride": args.xcd_stride},
        "roofline": roofline,
    }
    net.close()

    # ---- the other measurements the workload names
    if not args.no_extra:
        extra = {}
        k_steps = max(3, min(args.steps, 20))
        net = make_net(wl, args.grid)
        wall, kms = time_steps(torch, fwd_fn(net), k_steps, 2)
        net.synchronize()
        fb = algorithmic_bytes_per_forward_image(info, net.num_weights, net.image_size)
        extra["cfg2a_forward_only_images_per_s"] = round(k_steps * B / wall, 1)
        extra["cfg2a_forward_only_hbm_frac"] = round(fb * B / (np.mean(kms) * 1e-3) / 1e9 / HBM_PEAK_GBS, 6)
        net.close()
        wlb = synth.WORKLOADS["cfg2b"]
        infob = binding.arch_info(wlb.arch)
        net = make_net(wlb, args.grid)
        wall, kms = time_steps(torch, train_fn(net), k_steps, 2)
        net.synchronize()
        tb = algorithmic_bytes_per_train_image(infob, net.num_weights, net.image_size)
        extra["cfg2b_arch"] = wlb.arch
        extra["cfg2b_train_images_per_s"] = round(k_steps * B / wall, 1)
        extra["cfg2b_train_hbm_frac"] = round(tb * B / (np.mean(kms) * 1e-3) / 1e9 / HBM_PEAK_GBS, 6)
        wall, kms = time_steps(torch, fwd_fn(net), k_steps, 2)
        net.synchronize()
        extra["cfg2b_forward_only_images_per_s"] = round(k_steps * B / wall, 1)
        net.close()
        # validation / test passes: the whole stream through the batched forward pass (every layer one
        # matrix product over 4096 images on the matrix cores); timed with events around each call
        for key, w_, inf in (("cfg2a", wl, info), ("cfg2b", wlb, infob)):
            net = make_net(w_, args.grid)
            fbatch = 4096
            scratch = torch.empty(net.forward_batch_scratch_bytes(fbatch), dtype=torch.uint8, device="cuda:0")
            d_probs = torch.empty(n_stream * net.num_classes, dtype=torch.float32, device="cuda:0")
            net.forward_batch(d_imgs, n_stream, d_probs, scratch, fbatch)
            net.synchronize()
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                net.forward_batch(d_imgs, n_stream, d_probs, scratch, fbatch)
                e1.record()
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            assert torch.isfinite(d_probs).all()
            tf = forward_flops_per_image(inf) * n_stream / (best * 1e-3) / 1e12
            extra[key + "_forward_batch_images_per_s"] = round(n_stream / (best * 1e-3), 1)
            extra[key + "_forward_batch_tflops"] = round(tf, 2)
            extra[key + "_forward_batch_fp32_mfma_frac"] = round(tf / FP32_MFMA_PEAK_TFLOPS, 4)
            del scratch, d_probs
            net.close()
        # on-line deformation of the training stream (Sec. 4.1): the whole stream in one call, then training with
        # every launch's images deformed just ahead of it on the same stream
        gp = binding.DeformParams(**synth.DEFORM_RECIPE)
        d_src4 = d_imgs.view(n_stream, *wl.raw_shape)
        d_def = torch.empty_like(d_src4)
        binding.deform_images(d_src4, d_def, n_stream, gp, synth.DEFORM_SEED, 0)
        torch.cuda.synchronize()
        best = None
        for r in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            binding.deform_images(d_src4, d_def, n_stream, gp, synth.DEFORM_SEED, (r + 1) * n_stream)
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        assert torch.isfinite(d_def).all()
        extra["cfg2a_deform_images_per_s"] = round(n_stream / (best * 1e-3), 1)
        extra["cfg2a_deform_hbm_frac"] = round(2 * 4 * int(np.prod(wl.raw_shape)) * n_stream / (best * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        net = make_net(wl, args.grid)
        sz = net.image_size
        buf = torch.empty((B,) + tuple(wl.raw_shape), dtype=torch.float32, device=dev)

        def deformed_step(k):
            o = (k % per_epoch) * B
            binding.deform_images(d_src4[o:o + B], buf, B, gp, synth.DEFORM_SEED, k * B)
            net.train_many(buf.view(-1), d_labs[o:o + B], wl.lr, n=B)
        wall, kms = time_steps(torch, deformed_step, k_steps, 2)
        extra["cfg2a_train_with_deformation_images_per_s"] = round(k_steps * B / wall, 1)
        net.close()
        del d_def, buf
        # the other benchmark networks, each in the mode that runs it fastest: on-line training of 400 seeded
        # images (one launch per stage: wide layers on the matrix cores; cfg5 fits the resident kernel)
        for key, mode_o in (("cfg3", binding.MODE_STAGES), ("cfg4a", binding.MODE_STAGES),
                            ("cfg4b", binding.MODE_STAGES), ("cfg5", binding.MODE_RESIDENT)):
            wo = synth.WORKLOADS[key]
            n_o = 400
            io, lo = synth.images(wo, n_o), synth.labels(wo, n_o)
            d_io, d_lo = torch.from_numpy(io).to(dev), torch.from_numpy(lo).to(dev)
            net = synth.build_network(binding.Cnn(wo.arch), wo)
            net.set_mode(mode_o)
            net.train_many(d_io, d_lo, wo.lr, n=50)
            net.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            net.train_many(d_io, d_lo, wo.lr)
            e1.record()
            e1.synchronize()
            extra[key + "_train_images_per_s"] = round(n_o / (e0.elapsed_time(e1) * 1e-3), 1)
            # forward only: one image at a time in the same mode, and every layer a matrix product over the batch
            net.forward_many(d_io, 50)
            net.synchronize()
            e0.record()
            net.forward_many(d_io, n_o)
            e1.record()
            e1.synchronize()
            extra[key + "_forward_only_images_per_s"] = round(n_o / (e0.elapsed_time(e1) * 1e-3), 1)
            fb_o = {"cfg3": 512, "cfg4a": 512, "cfg4b": 256, "cfg5": 1024}[key]
            n_b = 2 * fb_o
            ib = torch.from_numpy(synth.images(wo, n_b)).to(dev)
            scratch = torch.empty(net.forward_batch_scratch_bytes(fb_o), dtype=torch.uint8, device=dev)
            pb = torch.empty(n_b * net.num_classes, dtype=torch.float32, device=dev)
            net.forward_batch(ib, n_b, pb, scratch, fb_o)
            net.synchronize()
            e0.record()
            net.forward_batch(ib, n_b, pb, scratch, fb_o)
            e1.record()
            e1.synchronize()
            extra[key + "_forward_batch_images_per_s"] = round(n_b / (e0.elapsed_time(e1) * 1e-3), 1)
            net.close()
            del d_io, d_lo, ib, scratch, pb
        # launch cost: the same images through one cnn_train_step call each
        net = make_net(wl, args.grid)
        sz = net.image_size
        lab_host = labs[:B].tolist()
        nstep = min(B, 500)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(nstep):
            net.train_step(d_imgs.view(-1)[t * sz:(t + 1) * sz], lab_host[t], wl.lr)
        torch.cuda.synchronize()
        extra["cfg2a_train_step_calls_images_per_s"] = round(nstep / (time.perf_counter() - t0), 1)
        net.close()
        out["extra"] = extra

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores
    if not args.no_cpu_baseline:
        import oracle
        cores = oracle.set_threads(0)
        ref = oracle.Oracle(wl.arch, 32)
        ref.set_weights(synth.weights(wl, ref.num_weights))
        probe = 200
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
        # the same oracle on one thread (the paper's own baseline was one optimised CPU thread), 300 images
        oracle.set_threads(1)
        t0 = time.perf_counter()
        ref.train_many(imgs[:300], labs[:300], wl.lr)
        out["cpu_baseline"]["single_thread_images_per_s"] = round(300 / (time.perf_counter() - t0), 1)
        oracle.set_threads(0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
