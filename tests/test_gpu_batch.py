"""Batched forward pass (every layer one matrix product over the batch, on the matrix cores)
against the CPU oracle, through the C ABI.  Needs a GPU (marked gpu)."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import build_pair, to_dev

pytestmark = pytest.mark.gpu

# (workload, images, batch, images the oracle checks)
CASES = [
    ("cfg1", 300, 128, 300),      # three chunks, the last one ragged; columns straddle images
    ("cfg1", 5, 64, 5),           # fewer images than one workgroup's columns
    ("cfg2b", 200, 200, 60),
    ("cfg3", 70, 32, 12),
    ("cfg4a", 70, 64, 12),
    ("cfg4b", 40, 16, 3),
    ("cfg5", 150, 100, 40),       # fixed front-end, skipping factor, sparse table
]


def _scratch(g, batch):
    import torch
    return torch.empty(g.forward_batch_scratch_bytes(batch), dtype=torch.uint8, device="cuda:0")


@pytest.mark.parametrize("name,n,batch,n_check", CASES)
def test_batched_forward_matches_the_oracle(name, n, batch, n_check):
    import torch
    wl = synth.WORKLOADS[name]
    print("case", name, "images", n, "batch", batch, flush=True)
    g, o = build_pair(wl)
    imgs = synth.images(wl, n)
    d_imgs = to_dev(imgs)
    d_probs = torch.full((n * g.num_classes,), -1.0, dtype=torch.float32, device="cuda:0")
    g.forward_batch(d_imgs, n, d_probs, _scratch(g, batch), batch)
    g.synchronize()
    got = d_probs.cpu().numpy().reshape(n, -1)
    assert np.all(got >= 0) and np.abs(got.sum(axis=1) - 1.0).max() <= 1e-5
    # the oracle on a sample spread over the chunks (first, last, around the chunk borders)
    idx = sorted(set(np.linspace(0, n - 1, n_check).astype(int).tolist() +
                     [i for i in (batch - 1, batch, n - 1) if 0 <= i < n]))
    want = np.stack([o.forward(imgs[i]) for i in idx])
    e = np.abs(got[idx] - want).max() / np.abs(want).max()
    print("  probabilities, %d images checked by the oracle: rel err %.2e" % (len(idx), e), flush=True)
    assert e <= 1e-5
    # and every image against the one-image path of the same library
    d_seq = torch.empty_like(d_probs)
    g.forward_many(d_imgs, n, d_seq)
    g.synchronize()
    seq = d_seq.cpu().numpy().reshape(n, -1)
    assert np.abs(got - seq).max() <= 1e-5
    g.close()


@pytest.mark.parametrize("arch,fan", [
    ("2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N", {1: 2}),
    ("1x10x12-2C3x5-MP4x2-4N", {}),
    ("3x40x33-9C5x3S1x2-MP2x1-8C2x4-MP1x2-7C3x1S0x1-12N-5N", {1: 4, 2: 3}),
    ("1x30x70-40C7x2-MP8x3-70C2x3S0x1-MP2x1-5N", {}),      # wide enough for several map tiles and k chunks
])
def test_batched_forward_with_different_x_and_y_values(arch, fan):
    """Kernels, skipping factors and pooling rectangles with an x and a y value each (Sec. 2.2, 2.3)."""
    import oracle
    import torch
    print("case", arch, flush=True)
    o0 = oracle.Oracle(arch)
    convs = [l for l in range(1, o0.num_layers) if o0.layer_info(l)["kind"] == 1]
    tables = {ci: synth.random_table(o0.layer_info(convs[ci])["maps"], o0.layer_info(convs[ci] - 1)["maps"], f, 77 + ci)
              for ci, f in fan.items()}
    g, o = build_pair(arch=arch, tables=tables, seed=5, wscale=0.3)
    n, batch = 37, 16
    rng = np.random.default_rng(9)
    imgs = rng.uniform(-1, 1, (n, g.image_size)).astype(np.float32)
    d_probs = torch.full((n * g.num_classes,), -1.0, dtype=torch.float32, device="cuda:0")
    g.forward_batch(to_dev(imgs), n, d_probs, _scratch(g, batch), batch)
    g.synchronize()
    got = d_probs.cpu().numpy().reshape(n, -1)
    want = np.stack([o.forward(imgs[i]) for i in range(n)])
    e = np.abs(got - want).max() / np.abs(want).max()
    print("  probabilities rel err %.2e" % e, flush=True)
    assert e <= 1e-5
    g.close()


def test_batched_forward_sees_trained_weights_and_the_tanh_outputs():
    """The call reads the weights as they stand: after training in resident mode (weights live in
    LDS during a call and are written back at its end) it must see the trained values; with
    scaled-tanh output units it returns the outputs."""
    import torch
    wl = synth.WORKLOADS["cfg1"]
    g, o = build_pair(wl)
    g.set_mode(binding.MODE_RESIDENT)
    g.set_output_units(binding.OUTPUT_TANH_SQERR)
    o.set_output_units(1)
    n = 40
    imgs, labs = synth.images(wl, n), synth.labels(wl, n)
    d_imgs, d_labs = to_dev(imgs), to_dev(labs)
    g.train_many(d_imgs, d_labs, wl.lr)
    d_out = torch.empty(n * g.num_classes, dtype=torch.float32, device="cuda:0")
    g.forward_batch(d_imgs, n, d_out, _scratch(g, 16), 16)
    g.synchronize()
    o.set_weights(g.get_weights().astype(np.float64))
    want = o.forward_many(imgs, n)
    got = d_out.cpu().numpy().reshape(n, -1)
    assert np.abs(got - want).max() / np.abs(want).max() <= 1e-5
    assert np.abs(want.sum(axis=1) - 1.0).max() > 1e-3
    g.close()


def test_batched_forward_argument_errors():
    import torch
    wl = synth.WORKLOADS["cfg1"]
    g, _ = build_pair(wl)
    d_imgs = to_dev(synth.images(wl, 4))
    d_probs = torch.empty(4 * g.num_classes, dtype=torch.float32, device="cuda:0")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.CnnError) as e:
        g.forward_batch(d_imgs, 4, d_probs, small, 4)
    assert e.value.code == binding.E_WORKSPACE
    with pytest.raises(binding.CnnError) as e:
        g.forward_batch(d_imgs, 4, d_probs, _scratch(g, 4), 0)
    assert e.value.code == binding.E_ARG
    g.forward_batch(d_imgs, 0, d_probs[:0], _scratch(g, 4), 4)  # no images: nothing to do
    g.synchronize()
    g.close()


@pytest.mark.parametrize("name,n", [("cfg1", 37), ("cfg2b", 20), ("cfg3", 9), ("cfg4a", 9), ("cfg4b", 5), ("cfg5", 21)])
def test_every_layer_of_the_batched_pass_matches_the_oracle(name, n):
    """The parity tap of the batched pass: the outputs of every trainable layer (pooled maps of a convolutional
    layer, units of a fully connected one, the output layer's sums) for every image of a batch against the
    oracle's, layer by layer, so that an error in one layer cannot hide behind a soft-max that is sure anyway."""
    wl = synth.WORKLOADS[name]
    print("case", name, "images", n, flush=True)
    g, o = build_pair(wl)
    imgs = synth.images(wl, n)
    d_imgs = to_dev(imgs)
    scratch = _scratch(g, n)
    layers = [l for l in range(1, o.num_layers) if o.layer_info(l)["kind"] in (1, 3)]
    want = {k: [] for k in range(len(layers))}
    for i in range(n):
        o.forward(imgs[i])
        for k, l in enumerate(layers):
            pooled = l + 1 < o.num_layers and o.layer_info(l + 1)["kind"] == 2
            a = o.activation(l + 1 if pooled else l)
            want[k].append(np.asarray(a, dtype=np.float64).ravel())
    for k in range(len(layers)):
        got = g.debug_forward_batch_layer(d_imgs, n, k, scratch).astype(np.float64)
        w = np.stack(want[k])
        assert got.shape == w.shape, (k, got.shape, w.shape)
        if k == len(layers) - 1:
            # the tap shows the output layer's sums, the oracle its soft-max: sums minus their log-sum-exp are the
            # logarithms of the probabilities
            m = got.max(axis=1, keepdims=True)
            got = got - (m + np.log(np.exp(got - m).sum(axis=1, keepdims=True)))
            w = np.log(w)
        e = np.abs(got - w).max() / np.abs(w).max()
        print("  trainable layer %d: %d values an image, rel err %.2e" % (k, w.shape[1], e), flush=True)
        assert e <= 1e-5, k
    with pytest.raises(binding.CnnError):
        g.debug_forward_batch_layer(d_imgs, n, len(layers), scratch)
    g.close()
