"""Seeded random architectures within the documented limits -- up to three convolutional layers with kernels of 1 to 7
(some with different x and y values), skipping factors 0 to 2, pooling rectangles that tile the map, sparse tables,
up to three fully connected layers -- in every mode that takes them, against the oracle: one step (activations,
deltas, gradients), six lock-step steps, batched call = stepwise calls bit for bit, batched forward pass.
Needs a GPU (marked gpu)."""
import numpy as np
import pytest

import oracle
from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import (TOL_ACT, TOL_W100, build_pair, compare_backward_state, compare_forward_state,
                                  layer_bounds, lockstep_train, rel_err, to_dev)

pytestmark = pytest.mark.gpu


def random_arch(rng, square=False):
    C, H, W = int(rng.integers(1, 4)), int(rng.integers(6, 40)), int(rng.integers(6, 40))
    s = "%dx%dx%d" % (C, H, W)
    h, w, m = H, W, C
    fan = {}
    ci = 0
    for _ in range(int(rng.integers(1 if square else 0, 4))):
        for _try in range(20):
            ky = int(rng.integers(1, min(7, h) + 1))
            kx = ky if (square or rng.random() < 0.6) else int(rng.integers(1, min(7, w) + 1))
            if kx > w:
                continue
            sy = int(rng.integers(0, 3)) if rng.random() < 0.4 else 0
            sx = sy if (square or rng.random() < 0.7) else int(rng.integers(0, 3))
            ho, wo = (h - ky) // (sy + 1) + 1, (w - kx) // (sx + 1) + 1
            if ho >= 1 and wo >= 1:
                break
        else:
            break
        mo = int(rng.integers(1, 13))
        tok = "-%dC%s" % (mo, str(ky) if ky == kx else "%dx%d" % (ky, kx))
        if sy or sx:
            tok += "S%s" % (str(sy) if sy == sx else "%dx%d" % (sy, sx))
        s += tok
        if m > 1 and rng.random() < 0.4:
            fan[ci] = int(rng.integers(1, m + 1))
        ci += 1
        h, w, m = ho, wo, mo
        if rng.random() < 0.7:
            dy = [d for d in range(1, 6) if h % d == 0]
            dx = [d for d in range(1, 6) if w % d == 0]
            py = int(rng.choice([d for d in dy if d in dx] if square else dy))
            px = py if (square or (py in dx and rng.random() < 0.6)) else int(rng.choice(dx))
            s += "-MP%s" % (str(py) if py == px else "%dx%d" % (py, px))
            h, w = h // py, w // px
    for _ in range(int(rng.integers(0, 3))):
        s += "-%dN" % int(rng.integers(2, 40))
    s += "-%dN" % int(rng.integers(2, 12))
    return s, fan


def test_random_architectures_in_every_mode():
    import torch
    rng = np.random.default_rng(2)
    runs = {binding.MODE_STAGES: 0, binding.MODE_PERSISTENT: 0, binding.MODE_RESIDENT: 0}
    for case in range(65):
        arch, fan = random_arch(rng, square=case >= 40)   # the last 25 with equal x and y values: the resident mode's
        o0 = oracle.Oracle(arch)
        convs = [l for l in range(1, o0.num_layers) if o0.layer_info(l)["kind"] == 1]
        tables = {ci: synth.random_table(o0.layer_info(convs[ci])["maps"], o0.layer_info(convs[ci] - 1)["maps"],
                                         f, 100 + case + ci) for ci, f in fan.items()}
        for mode in runs:
            g, o = build_pair(arch=arch, tables=tables, seed=case, wscale=0.3)
            if not g.mode_supported(mode):
                g.close()
                continue
            print("case", case, arch, fan, "mode", mode, flush=True)
            runs[mode] += 1
            g.set_mode(mode)
            r2 = np.random.default_rng(case)
            imgs = r2.uniform(-1, 1, (6, g.image_size)).astype(np.float32)
            labs = r2.integers(0, g.num_classes, size=6).astype(np.int32)
            grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
            grad_o, _ = o.gradients(imgs[0], int(labs[0]))
            compare_forward_state(g, o)
            compare_backward_state(g, o)
            for (a, b) in layer_bounds(o):
                assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (arch, a, b)
            w0 = g.get_weights()
            lockstep_train(g, o, imgs, labs, 0.01)
            w_step = g.get_weights()
            assert rel_err(w_step, o.get_weights()) <= TOL_W100, arch
            g.set_weights(w0)
            g.train_many(to_dev(imgs), to_dev(labs), 0.01)
            np.testing.assert_array_equal(g.get_weights(), w_step)
            if mode == binding.MODE_STAGES:
                n = 6
                d_probs = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
                scratch = torch.empty(g.forward_batch_scratch_bytes(4), dtype=torch.uint8, device="cuda:0")
                g.forward_batch(to_dev(imgs), n, d_probs, scratch, 4)
                g.synchronize()
                want = np.stack([o.forward(imgs[i]) for i in range(n)])
                assert np.abs(d_probs.cpu().numpy().reshape(n, -1) - want).max() / np.abs(want).max() <= 1e-5, arch
            g.close()
    print("runs per mode:", runs, flush=True)
    assert runs[binding.MODE_STAGES] == 65 and runs[binding.MODE_PERSISTENT] == 65 and runs[binding.MODE_RESIDENT] >= 10


def random_deep_arch(rng):
    """Three to six convolutional layers of 2 to 29 maps with small square kernels, a pooling layer behind about a third
    of them, sparse tables on some, one to three hidden fully connected layers of 60 to 129 units."""
    C, H, W = int(rng.integers(1, 4)), int(rng.integers(6, 26)), int(rng.integers(6, 26))
    s = "%dx%dx%d" % (C, H, W)
    h, w, m = H, W, C
    fan = {}
    ci = 0
    for _ in range(int(rng.integers(3, 7))):
        for _try in range(20):
            k = int(rng.integers(1, min(3, h, w) + 1))
            sk = int(rng.integers(0, 3)) if rng.random() < 0.4 else 0
            ho, wo = (h - k) // (sk + 1) + 1, (w - k) // (sk + 1) + 1
            if ho >= 1 and wo >= 1:
                break
        else:
            break
        mo = int(rng.integers(2, 30))
        s += "-%dC%d" % (mo, k) + ("S%d" % sk if sk else "")
        if m > 1 and rng.random() < 0.4:
            fan[ci] = int(rng.integers(1, m + 1))
        ci += 1
        h, w, m = ho, wo, mo
        if rng.random() < 0.35:
            both = [d for d in range(1, 6) if h % d == 0 and w % d == 0]
            p = int(rng.choice(both))
            s += "-MP%d" % p
            h, w = h // p, w // p
    for _ in range(int(rng.integers(1, 4))):
        s += "-%dN" % int(rng.integers(60, 130))
    s += "-%dN" % int(rng.integers(2, 12))
    return s, fan


def test_random_deep_architectures():
    """Deep nets with wide fully connected tails in the launch-per-stage and resident modes: up to six
    convolutional layers in one launch, a second hidden layer held by columns where it is large."""
    import torch
    rng = np.random.default_rng(5)
    n_res = n_cols = n_deep = 0
    for case in range(40):
        arch, fan = random_deep_arch(rng)
        o0 = oracle.Oracle(arch)
        convs = [l for l in range(1, o0.num_layers) if o0.layer_info(l)["kind"] == 1]
        tables = {ci: synth.random_table(o0.layer_info(convs[ci])["maps"], o0.layer_info(convs[ci] - 1)["maps"],
                                         f, 300 + case + ci) for ci, f in fan.items()}
        for mode in (binding.MODE_STAGES, binding.MODE_RESIDENT):
            # (weights wide enough for the signal to reach the top of a deep net of few maps: with the paper's +-0.05 a
            # map of the upper layers varies in its seventh digit only and its pooling winners are ties)
            g, o = build_pair(arch=arch, tables=tables, seed=case, wscale=0.2)
            if not g.mode_supported(mode):
                g.close()
                continue
            print("case", case, arch, fan, "mode", mode, flush=True)
            g.set_mode(mode)
            if mode == binding.MODE_RESIDENT:
                plan = binding.resident_plan(arch)
                n_res += 1
                n_cols += int(any(q["by_cols"] for q in plan["fc"]))
                n_deep += int(plan["numbers"]["n_conv"] >= 5)
            r2 = np.random.default_rng(case)
            imgs = r2.uniform(-1, 1, (6, g.image_size)).astype(np.float32)
            labs = r2.integers(0, g.num_classes, size=6).astype(np.int32)
            grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
            grad_o, _ = o.gradients(imgs[0], int(labs[0]))
            compare_forward_state(g, o)
            compare_backward_state(g, o)
            for (a, b) in layer_bounds(o):
                assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (arch, a, b)
            w0 = g.get_weights()
            lockstep_train(g, o, imgs, labs, 0.01)
            w_step = g.get_weights()
            assert rel_err(w_step, o.get_weights()) <= TOL_W100, arch
            g.set_weights(w0)
            g.train_many(to_dev(imgs), to_dev(labs), 0.01)
            np.testing.assert_array_equal(g.get_weights(), w_step)
            if mode == binding.MODE_STAGES:
                n = 6
                d_probs = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
                scratch = torch.empty(g.forward_batch_scratch_bytes(4), dtype=torch.uint8, device="cuda:0")
                g.forward_batch(to_dev(imgs), n, d_probs, scratch, 4)
                g.synchronize()
                o.set_weights(w_step.astype(np.float64))   # (the pass is checked on the weights it ran with)
                want = np.stack([o.forward(imgs[i]) for i in range(n)])
                assert np.abs(d_probs.cpu().numpy().reshape(n, -1) - want).max() / np.abs(want).max() <= 1e-5, arch
            g.close()
    print("resident runs:", n_res, "with a layer held by columns:", n_cols, "with five or six convolutional layers:", n_deep, flush=True)
    assert n_res >= 30 and n_cols >= 5 and n_deep >= 8
