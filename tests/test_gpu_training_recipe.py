"""The knobs of the paper's training recipe around the on-line step, each against the oracle: edge filters as the
fixed first layer (Sec. 4.3), a learning rate that shrinks after every epoch (Sec. 4.1, 4.3), and training on images
that are deformed anew at every presentation (Sec. 4.1), deformation and training both on the device.
Needs a GPU (marked gpu)."""
import numpy as np
import pytest

from oracle import deform_oracle as DO
from oracle.binding import KIND_POOL
from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import (TOL_ACT, TOL_W100, build_pair, compare_backward_state, compare_forward_state,
                                  layer_bounds, lockstep_train, rel_err, to_dev)

pytestmark = pytest.mark.gpu

SOBEL = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]], dtype=np.float32) / 8
SCHARR = np.array([[-3, 0, 3], [-10, 0, 10], [-3, 0, 3]], dtype=np.float32) / 32


@pytest.mark.parametrize("name,kernel", [("sobel", SOBEL), ("scharr", SCHARR)])
@pytest.mark.parametrize("mode", [binding.MODE_STAGES, binding.MODE_RESIDENT])
def test_edge_filters_as_the_fixed_first_layer(name, kernel, mode):
    """Horizontal and vertical edge maps of every colour channel (3 x 2 maps of 30 x 30 from a 3x32x32 image)
    feed the trainable layers; the filters are never adjusted."""
    print("case", name, "mode", mode, flush=True)
    filt = np.stack([kernel if f % 2 == 0 else kernel.T for f in range(6)]).astype(np.float32)
    src = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)
    g, o = build_pair(arch="6x30x30-8C3-MP2-6C3-MP2-20N-10N", frontend=(filt, src, 3), seed=3, wscale=0.2)
    if not g.mode_supported(mode):
        g.close()
        pytest.skip("mode %d cannot run this network" % mode)
    g.set_mode(mode)
    rng = np.random.default_rng(5)
    imgs = rng.uniform(-1, 1, (10, 3 * 32 * 32)).astype(np.float32)
    labs = rng.integers(0, 10, size=10).astype(np.int32)
    grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
    grad_o, _ = o.gradients(imgs[0], int(labs[0]))
    compare_forward_state(g, o)
    compare_backward_state(g, o)
    for (a, b) in layer_bounds(o):
        assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (a, b)
    lockstep_train(g, o, imgs, labs, 0.01)
    assert rel_err(g.get_weights(), o.get_weights()) <= TOL_W100
    g.close()


@pytest.mark.parametrize("lr0,factor", [(1e-3, 0.993), (1e-3, (3e-5 / 1e-3) ** (1.0 / 500))])
def test_learning_rate_that_shrinks_after_every_epoch(lr0, factor):
    """lr is an argument of every call, so a schedule is the caller's loop: three passes over 40 images with the
    rate multiplied by a constant after each (0.993 in Sec. 4.3; from 1e-3 to 3e-5 over 500 epochs in Sec. 4.1)."""
    wl = synth.WORKLOADS["cfg1"]
    g, o = build_pair(wl)
    g.set_mode(binding.MODE_RESIDENT)
    imgs, labs = synth.images(wl, 40).reshape(40, -1), synth.labels(wl, 40)
    d_imgs, d_labs = to_dev(imgs), to_dev(labs)
    w0 = g.get_weights()
    lr = lr0
    for epoch in range(3):
        lockstep_train(g, o, imgs, labs, lr)
        lr *= factor
    w_step = g.get_weights()
    assert rel_err(w_step, o.get_weights()) <= TOL_W100
    g.set_weights(w0)
    lr = lr0
    for epoch in range(3):
        g.train_many(d_imgs, d_labs, lr)
        lr *= factor
    np.testing.assert_array_equal(g.get_weights(), w_step)
    # a different factor gives different weights: the argument is what is used
    g.set_weights(w0)
    for epoch in range(3):
        g.train_many(d_imgs, d_labs, lr0)
    assert not np.array_equal(g.get_weights(), w_step)
    g.close()


def test_training_on_images_deformed_anew_at_every_presentation():
    """Two epochs over 30 images, every presentation deformed on the device just ahead of the launch that trains on
    it, on one stream with no host in between; the oracle deforms with its own arithmetic and trains on that."""
    import torch
    wl = synth.WORKLOADS["cfg1"]
    g, o = build_pair(wl)
    g.set_mode(binding.MODE_RESIDENT)
    n = 30
    imgs, labs = synth.images(wl, n), synth.labels(wl, n)
    kw = dict(synth.DEFORM_RECIPE)
    gp, op = binding.DeformParams(**kw), DO.DeformParams(**kw)
    d_src, d_labs = to_dev(imgs), to_dev(labs)
    d_buf = torch.empty_like(d_src)
    w0 = g.get_weights()
    seen = []
    for epoch in range(2):
        binding.deform_images(d_src, d_buf, n, gp, synth.DEFORM_SEED, epoch * n)
        g.train_many(d_buf.view(-1), d_labs, wl.lr)
        seen.append(d_buf.cpu().numpy())   # (synchronises; the next epoch overwrites the buffer)
    w_chain = g.get_weights()
    assert not np.array_equal(seen[0], seen[1])
    # the same presentations image by image, the oracle beside it on its own deformed images; where the two sides'
    # pooling winners differ at a near-tie the oracle follows the GPU (see lockstep_train)
    g.set_weights(w0)
    pools = [l for l in range(1, o.num_layers) if o.layer_info(l)["kind"] == KIND_POOL]
    sz = g.image_size
    adopted = 0
    for epoch in range(2):
        want, _ = DO.deform_images(imgs, synth.DEFORM_SEED, epoch * n, op)
        assert rel_err(seen[epoch], want) <= TOL_ACT
        d_seen = to_dev(seen[epoch])
        for t in range(n):
            g.train_step(d_seen.view(-1)[t * sz:(t + 1) * sz], int(labs[t]), wl.lr)
            o.forward(want[t].astype(np.float32))
            for l in pools:
                a, r = o.adopt_argmax_hint(l, g.argmax(l), TOL_ACT)
                assert r == 0
                adopted += a
            o.backward_update(int(labs[t]), wl.lr)
    np.testing.assert_array_equal(g.get_weights(), w_chain)
    e = rel_err(w_chain, o.get_weights())
    print("  weights after 60 deformed presentations: rel err %.2e, near-tie winners adopted: %d" % (e, adopted), flush=True)
    assert e <= TOL_W100
    g.close()
