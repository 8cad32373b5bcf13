#!/usr/bin/env python3
"""Small driver to put under rocprofv3: trains a few on-line calls of one synthetic workload.

    python3 probe.py --workload cfg4b --mode stages --images 200 --calls 1
    python3 probe.py --workload cfg2a --mode resident --images 1000 --calls 3 --copy-calibration
    python3 probe.py --workload cfg2a --forward --batch 4096 --images 16384 --calls 3
    python3 probe.py --workload cfg2a --deform --images 60000 --calls 5

--copy-calibration first runs a 256 MiB device-to-device copy three times, so that a counter
collected in the same run (FETCH_SIZE, WRITE_SIZE) can be scaled by what it reads for a
transfer of known size.  Everything the network computes runs in libcnn355.so.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg2a")
    ap.add_argument("--arch", default=None,
                    help="instead of a workload: any architecture, full tables, seeded weights in [-0.05, 0.05], "
                         "images uniform in [-1, 1], rate 0.001")
    ap.add_argument("--fan", type=int, default=0,
                    help="with --arch: output map j of every convolutional layer above the first reads the input maps "
                         "j .. j + fan - 1 (mod M_i); -d: M_i / d of them; 0: full tables")
    ap.add_argument("--code-object", action="store_true",
                    help="resident mode: load the kernel the build step compiled for this network, if there is one")
    ap.add_argument("--mode", choices=["resident", "persistent", "stages"], default="resident")
    ap.add_argument("--images", type=int, default=1000, help="images per cnn_train_many call")
    ap.add_argument("--calls", type=int, default=3)
    ap.add_argument("--forward", action="store_true", help="forward-only calls instead of training")
    ap.add_argument("--batch", type=int, default=0,
                    help="with --forward: cnn_forward_batch with this many images in flight")
    ap.add_argument("--deform", action="store_true",
                    help="instead of the network: cnn_deform_images over --images images of the workload, --calls times")
    ap.add_argument("--copy-calibration", action="store_true")
    args = ap.parse_args()

    import torch

    from paper_1102_0183_amd import binding, synth

    if args.copy_calibration:
        x = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0").normal_()   # 256 MiB
        y = torch.empty_like(x)
        torch.cuda.synchronize()
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
    wl = synth.WORKLOADS[args.workload]
    n = args.images
    if args.arch and not args.deform:
        import numpy as np
        net = binding.Cnn(args.arch)
        if args.fan:
            convs = [l for l in range(1, net.num_layers) if net.layer_info(l)["kind"] == 1]
            for ci in range(1, len(convs)):
                net.set_connection_table(ci, synth.regular_table(net.layer_info(convs[ci])["maps"],
                                                                 net.layer_info(convs[ci] - 1)["maps"], args.fan))
        rng = np.random.default_rng(7)
        net.set_weights(((rng.random(net.num_weights, dtype=np.float32) - np.float32(0.5)) * np.float32(0.1)))
        imgs = rng.uniform(-1, 1, (n * args.calls, net.image_size)).astype(np.float32)
        labs = rng.integers(0, net.num_classes, n * args.calls).astype(np.int32)
        lr, what = 1e-3, args.arch
    elif not args.deform:
        imgs, labs = synth.images(wl, n * args.calls), synth.labels(wl, n * args.calls)
        net = synth.build_network(binding.Cnn(wl.arch), wl)
        lr, what = wl.lr, args.workload
    if args.deform:
        d_src = torch.from_numpy(synth.images(wl, n)).to("cuda:0")
        d_dst = torch.empty_like(d_src)
        gp = binding.DeformParams(**synth.DEFORM_RECIPE)
        for r in range(args.calls):
            binding.deform_images(d_src, d_dst, n, gp, synth.DEFORM_SEED, r * n)
        torch.cuda.synchronize()
        print("probe done: %s, %d calls deforming %d images" % (args.workload, args.calls, n), flush=True)
        return
    d_imgs = torch.from_numpy(imgs).to("cuda:0")
    d_labs = torch.from_numpy(labs).to("cuda:0")
    net.set_mode({"resident": binding.MODE_RESIDENT, "persistent": binding.MODE_PERSISTENT,
                  "stages": binding.MODE_STAGES}[args.mode])
    if args.code_object and args.mode == "resident":
        from paper_1102_0183_amd import specialize
        path = specialize.built_code_object(net)
        if path:
            net.load_resident_code(path)
        print("probe: kernel compiled for this network %s" % ("loaded" if path else "not built"), flush=True)
    sz = net.image_size
    if args.batch:
        scratch = torch.empty(net.forward_batch_scratch_bytes(args.batch), dtype=torch.uint8, device="cuda:0")
        d_probs = torch.empty(n * net.num_classes, dtype=torch.float32, device="cuda:0")
    import time
    per_call = []
    for r in range(args.calls):
        im = d_imgs.view(-1)[r * n * sz:(r + 1) * n * sz]
        net.synchronize()
        t0 = time.perf_counter()
        if args.forward and args.batch:
            net.forward_batch(im, n, d_probs, scratch, args.batch)
        elif args.forward:
            net.forward_many(im, n)
        else:
            net.train_many(im, d_labs[r * n:(r + 1) * n], lr, n=n)
        net.synchronize()
        per_call.append(time.perf_counter() - t0)
    print("probe done: %s, %s mode, %d calls of %d images; best call %.2f us per image (host clock)" %
          (what, args.mode, args.calls, n, min(per_call) / n * 1e6), flush=True)
    net.close()


if __name__ == "__main__":
    main()
