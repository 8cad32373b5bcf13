"""The batched forward pass for callers that cannot allocate (cnn_forward_batch_static: scratch memory in an
array of the library's own device image) against cnn_forward_batch with caller-owned scratch, through the
C ABI.  Needs a GPU (marked gpu)."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import build_pair, to_dev

pytestmark = pytest.mark.gpu


def _both(g, d_imgs, n, batch):
    """(static-scratch result, caller-scratch result) for the first n images."""
    import torch
    d_a = torch.full((n * g.num_classes,), -1.0, dtype=torch.float32, device="cuda:0")
    d_b = torch.full((n * g.num_classes,), -2.0, dtype=torch.float32, device="cuda:0")
    scratch = torch.empty(g.forward_batch_scratch_bytes(batch), dtype=torch.uint8, device="cuda:0")
    g.forward_batch(d_imgs, n, d_b, scratch, batch)
    g.synchronize()
    g.forward_batch_static(d_imgs, n, d_a, batch)      # (the first call on a device asks for the array's address)
    g.synchronize()
    d_a.fill_(-1.0)
    torch.cuda.synchronize()
    mem, free = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    g.forward_batch_static(d_imgs, n, d_a, batch)
    g.synchronize()
    assert torch.cuda.memory_allocated() == mem and torch.cuda.mem_get_info()[0] >= free   # nothing was allocated
    return d_a.cpu().numpy().reshape(n, -1), d_b.cpu().numpy().reshape(n, -1)


@pytest.mark.parametrize("name,n1,batch1,n2,batch2", [
    ("cfg1", 300, 128, 70, 32),      # ragged last chunk; then fewer images in smaller batches
    ("cfg5", 150, 100, 40, 100),     # fixed front-end, sparse table; then fewer images than one batch
    ("cfg4a", 70, 64, 9, 8),         # wide layers, contraction cut into slices
])
def test_static_scratch_variant_matches_the_caller_scratch_one(name, n1, batch1, n2, batch2):
    """Two calls in a row on one handle, the second on a smaller input (the array then still holds the first
    call's contents beyond what the second writes): both must give the bits of cnn_forward_batch, and the
    oracle's probabilities to 1e-5."""
    wl = synth.WORKLOADS[name]
    print("case", name, flush=True)
    g, o = build_pair(wl)
    imgs = synth.images(wl, n1)
    d_imgs = to_dev(imgs)
    for n, batch in ((n1, batch1), (n2, batch2)):
        assert g.forward_batch_scratch_bytes(batch) <= binding.FORWARD_BATCH_STATIC_SCRATCH_BYTES
        got, want = _both(g, d_imgs, n, batch)
        np.testing.assert_array_equal(got, want)
        idx = sorted({0, n // 2, n - 1})
        ref = np.stack([o.forward(imgs[i]) for i in idx])
        assert np.abs(got[idx] - ref).max() / np.abs(ref).max() <= 1e-5
    g.close()


def test_static_scratch_variant_refuses_what_does_not_fit():
    wl = synth.WORKLOADS["cfg4b"]
    g, _ = build_pair(wl)
    import torch
    batch = 8
    while g.forward_batch_scratch_bytes(batch) <= binding.FORWARD_BATCH_STATIC_SCRATCH_BYTES:
        batch *= 2
    d_imgs = to_dev(synth.images(wl, 2))
    d_probs = torch.zeros(2 * g.num_classes, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.CnnError) as ei:
        g.forward_batch_static(d_imgs, 2, d_probs, batch)
    assert ei.value.code == binding.E_WORKSPACE
    assert str(binding.FORWARD_BATCH_STATIC_SCRATCH_BYTES) in str(ei.value)
    # a batch that fits still runs afterwards
    small = 4
    assert g.forward_batch_scratch_bytes(small) <= binding.FORWARD_BATCH_STATIC_SCRATCH_BYTES
    g.forward_batch_static(d_imgs, 2, d_probs, small)
    g.synchronize()
    p = d_probs.cpu().numpy().reshape(2, -1)
    assert np.abs(p.sum(axis=1) - 1.0).max() <= 1e-5
    g.close()
