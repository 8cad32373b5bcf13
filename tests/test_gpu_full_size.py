"""The benchmark workload (both of its networks) at its full size and in the launch configuration bench.py
times: one on-line epoch over the whole 60000-image stream, resident mode, 1000 images per launch.  The
oracle cannot follow 60000 steps in lock-step within a test's time, so it checks sampled
stretches (it continues from the GPU's weights at three points of the stream), and properties
that hold at any size carry the rest.  Needs a GPU (marked gpu)."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import TOL_W100, build_pair, lockstep_train, rel_err, to_dev

pytestmark = pytest.mark.gpu

LAUNCH = 1000


def _epoch(g, d_imgs, d_labs, lr, n, stops=()):
    """Train the stream launch by launch; returns {launch index: weights before that launch}."""
    sz = g.image_size
    snap = {}
    for k in range(n // LAUNCH):
        if k in stops:
            snap[k] = g.get_weights()
        g.train_many(d_imgs.view(-1)[k * LAUNCH * sz:(k + 1) * LAUNCH * sz], d_labs[k * LAUNCH:(k + 1) * LAUNCH],
                     lr, n=LAUNCH)
    g.synchronize()
    return snap


@pytest.mark.parametrize("name,static_id,shares", [("cfg2a", 1, 1), ("cfg2b", 2, 1)])
def test_one_epoch_in_the_benchmark_configuration(name, static_id, shares):
    wl = synth.WORKLOADS[name]
    n = wl.n_images
    assert n == 60000
    imgs, labs = synth.images(wl), synth.labels(wl)
    d_imgs, d_labs = to_dev(imgs), to_dev(labs)
    g, o = build_pair(wl)
    g.set_mode(binding.MODE_RESIDENT)
    assert g.resident_static_id() == static_id  # the kernels bench.py times
    assert g.resident_pull_shares(1) == shares  # (pulls that visit the pooling winners only are not shared)
    stops = (0, 19, 58)
    print("epoch of", n, "images,", LAUNCH, "per launch", flush=True)
    snap = _epoch(g, d_imgs, d_labs, wl.lr, n, stops)
    w_end = g.get_weights()
    w0 = synth.weights(wl, g.num_weights)
    assert np.isfinite(w_end).all() and np.abs(w_end - w0).max() > 1e-3
    # sampled stretches: from the GPU's weights before launch k, 60 images side by side with the oracle
    sz = g.image_size
    for k in stops:
        print("stretch at image", k * LAUNCH, flush=True)
        g2, o2 = build_pair(wl, weights=snap[k])
        g2.set_mode(binding.MODE_RESIDENT)
        lo = k * LAUNCH
        adopted = lockstep_train(g2, o2, imgs[lo:lo + 60], labs[lo:lo + 60], wl.lr)
        wg, wo = g2.get_weights().astype(np.float64), o2.get_weights()
        e, e_upd = rel_err(wg, wo), rel_err(wg - snap[k], wo - snap[k])
        print("  weights rel err %.2e, update rel err %.2e, near-tie winners adopted %d" % (e, e_upd, adopted), flush=True)
        assert e <= TOL_W100 and e_upd <= TOL_W100
        # any size: the same 60 images in one launch land on the bits of the 60 single steps
        g3, _ = build_pair(wl, weights=snap[k])
        g3.set_mode(binding.MODE_RESIDENT)
        g3.train_many(d_imgs.view(-1)[lo * sz:(lo + 60) * sz], d_labs[lo:lo + 60], wl.lr, n=60)
        np.testing.assert_array_equal(g3.get_weights(), g2.get_weights())
        g2.close()
        g3.close()
    # any size: the whole epoch again gives the same bits (no float atomics, no timing dependence),
    # and the accuracy of the trained net on the stream's first images is what the oracle gets
    # from the same weights
    g4, _ = build_pair(wl)
    g4.set_mode(binding.MODE_RESIDENT)
    _epoch(g4, d_imgs, d_labs, wl.lr, n)
    np.testing.assert_array_equal(g4.get_weights(), w_end)
    import torch
    m = 200
    d_probs = torch.empty(m * g.num_classes, dtype=torch.float32, device="cuda:0")
    g.forward_many(d_imgs, m, d_probs)
    g.synchronize()
    o.set_weights(w_end.astype(np.float64))
    want = o.forward_many(imgs[:m], m)
    assert np.abs(d_probs.cpu().numpy().reshape(m, -1) - want).max() <= 1e-5
    g.close()
    g4.close()


def test_batched_forward_over_the_whole_stream():
    """The validation-style pass bench.py times: all 60000 images, 4096 in flight (the last chunk
    ragged), against the oracle on sampled images and against the one-image path on all."""
    import torch
    wl = synth.WORKLOADS["cfg2a"]
    n = wl.n_images
    imgs = synth.images(wl)
    d_imgs = to_dev(imgs)
    g, o = build_pair(wl)
    batch = 4096
    scratch = torch.empty(g.forward_batch_scratch_bytes(batch), dtype=torch.uint8, device="cuda:0")
    d_probs = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
    g.forward_batch(d_imgs, n, d_probs, scratch, batch)
    g.synchronize()
    got = d_probs.cpu().numpy().reshape(n, -1)
    idx = sorted(set(np.linspace(0, n - 1, 40).astype(int).tolist() + [batch - 1, batch, 14 * batch, n - 1]))
    want = np.stack([o.forward(imgs[i]) for i in idx])
    assert np.abs(got[idx] - want).max() / np.abs(want).max() <= 1e-5
    g.set_mode(binding.MODE_RESIDENT)
    d_seq = torch.empty_like(d_probs)
    g.forward_many(d_imgs, n, d_seq)
    g.synchronize()
    assert np.abs(got - d_seq.cpu().numpy().reshape(n, -1)).max() <= 1e-5
    assert np.abs(got.sum(axis=1) - 1.0).max() <= 1e-5
    g.close()
