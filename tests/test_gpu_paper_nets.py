"""The paper's own architectures (Sec. 4.2: the five-hidden-layer NORB net; Sec. 4.3: the
eight-hidden-layer CIFAR10 nets) on seeded synthetic images of the data sets' shapes: one on-line
step and the batched forward pass against the oracle.  Needs a GPU (marked gpu)."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding
from tests.parity_helpers import (TOL_ACT, build_pair, compare_backward_state, compare_forward_state,
                                  layer_bounds, lockstep_train, rel_err, to_dev)

pytestmark = pytest.mark.gpu

# Sec. 4.3: 3x3 kernels, pooling 3 / 2 / 2, two fully connected hidden layers of 300 and 100 neurons,
# the same number of maps in every convolutional layer; Sec. 4.2: 300 maps of 6x6 kernels with
# skipping factor 1, pooling 2, 500 maps of 4x4 kernels, pooling 4, 500 neurons (stereo pair in)
# Sec. 4.1, Table 1: six convolutional layers of 20 to 120 maps with random partial connectivity and 150
# hidden neurons on 29x29 digits; the paper gives neither kernel sizes nor skipping factors for it, so
# these are one choice that ends at 1x1 maps.  Half of the connections above the first layer are kept.
DEEP = "1x29x29-20C4-MP2-40C2-60C3-80C3-MP2-100C2-120C3-150N-10N"

NETS = [
    ("cifar-100", "3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", 10),
    ("cifar-300", "3x32x32-300C3-MP3-300C3-MP2-300C3-MP2-300N-100N-10N", 0),
    ("norb", "2x96x96-300C6S1-MP2-500C4-MP4-500N-5N", 0),
]


@pytest.mark.parametrize("name,arch,n_steps", NETS)
def test_papers_architectures_one_step_and_batched_forward(name, arch, n_steps):
    import torch
    print("case", name, arch, flush=True)
    g, o = build_pair(arch=arch, seed=11, wscale=0.05)
    rng = np.random.default_rng(2011)
    n = 6
    imgs = rng.uniform(-1, 1, (n, g.image_size)).astype(np.float32)
    labs = rng.integers(0, g.num_classes, n).astype(np.int32)
    for mode in (binding.MODE_STAGES, binding.MODE_PERSISTENT):
        g.set_mode(mode)
        grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
        grad_o, loss_o = o.gradients(imgs[0], int(labs[0]))
        compare_forward_state(g, o)
        compare_backward_state(g, o)
        assert abs(g.loss() - loss_o) <= 1e-5 * max(1.0, abs(loss_o))
        for (a, b) in layer_bounds(o):
            assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (mode, a, b)
    # every image through the batched pass, three in flight (two chunks), against the oracle
    d_probs = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
    scratch = torch.empty(g.forward_batch_scratch_bytes(3), dtype=torch.uint8, device="cuda:0")
    g.forward_batch(to_dev(imgs), n, d_probs, scratch, 3)
    g.synchronize()
    want = o.forward_many(imgs, n)
    assert np.abs(d_probs.cpu().numpy().reshape(n, -1) - want).max() / np.abs(want).max() <= 1e-5
    if n_steps:
        w0 = g.get_weights().astype(np.float64)
        more = rng.uniform(-1, 1, (n_steps, g.image_size)).astype(np.float32)
        more_l = rng.integers(0, g.num_classes, n_steps).astype(np.int32)
        lockstep_train(g, o, more, more_l, 0.001)
        wg, wo = g.get_weights().astype(np.float64), o.get_weights()
        assert rel_err(wg, wo) <= 1e-5 and rel_err(wg - w0, wo - w0) <= 1e-4
    g.close()


def test_deep_randomly_connected_net():
    """The deepest net of Sec. 4.1 (Table 1), six convolutional layers with random connection tables:
    one step in every mode, ten lock-step steps in resident mode, and the batched forward pass
    (absent connections are zero columns of its weight matrices)."""
    import torch
    import oracle
    from paper_1102_0183_amd import synth
    o0 = oracle.Oracle(DEEP)
    convs = [l for l in range(1, o0.num_layers) if o0.layer_info(l)["kind"] == 1]
    tables = {ci: synth.random_table(o0.layer_info(convs[ci])["maps"], o0.layer_info(convs[ci] - 1)["maps"],
                                     o0.layer_info(convs[ci] - 1)["maps"] // 2, 400 + ci)
              for ci in range(1, len(convs))}
    g, o = build_pair(arch=DEEP, tables=tables, seed=5, wscale=0.2)
    rng = np.random.default_rng(343)
    n = 10
    imgs = rng.uniform(-1, 1, (n, g.image_size)).astype(np.float32)
    labs = rng.integers(0, g.num_classes, n).astype(np.int32)
    assert g.mode_supported(binding.MODE_RESIDENT)      # (six convolutional layers: the most that mode takes)
    for mode in (binding.MODE_STAGES, binding.MODE_PERSISTENT, binding.MODE_RESIDENT):
        g.set_mode(mode)
        grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
        grad_o, loss_o = o.gradients(imgs[0], int(labs[0]))
        compare_forward_state(g, o)
        compare_backward_state(g, o)
        for (a, b) in layer_bounds(o):
            assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (mode, a, b)
    d_out = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
    scratch = torch.empty(g.forward_batch_scratch_bytes(4), dtype=torch.uint8, device="cuda:0")
    g.forward_batch(to_dev(imgs), n, d_out, scratch, 4)
    g.synchronize()
    want = o.forward_many(imgs, n)
    assert np.abs(d_out.cpu().numpy().reshape(n, -1) - want).max() / np.abs(want).max() <= 1e-5
    # ten on-line steps in lock-step with the oracle, in the mode that runs this net fastest (one launch per call)
    w0 = g.get_weights().astype(np.float64)
    lockstep_train(g, o, imgs, labs, 0.001)
    wg, wo = g.get_weights().astype(np.float64), o.get_weights()
    assert rel_err(wg, wo) <= 1e-5 and rel_err(wg - w0, wo - w0) <= 1e-4
    # ... and the same ten as one call: the same bits
    g.set_weights(w0.astype(np.float32))
    g.train_many(to_dev(imgs), to_dev(labs), 0.001)
    np.testing.assert_array_equal(g.get_weights().astype(np.float64), wg)
    g.close()
