"""Stage mode replays a graph of the stage launches of several images (cnn_set_launch_graph): the same kernels in
the same order, so the bits must equal those of launching every stage by itself -- whatever the number of images
(whole graphs plus a rest), for training and forward-only calls, with a fixed front-end, after the stage list
changes, and with a label outside the classes somewhere inside a graph."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import build_pair, to_dev

pytestmark = pytest.mark.gpu


def _run(g, imgs, labs, lr, per_graph):
    import torch
    g.set_launch_graph(per_graph)
    g.train_many(to_dev(imgs), to_dev(labs), lr)
    w = g.get_weights()
    probs = torch.empty(len(labs) * g.num_classes, dtype=torch.float32, device="cuda:0")
    g.forward_many(to_dev(imgs), len(labs), probs)
    g.synchronize()
    return w, probs.cpu().numpy()


@pytest.mark.parametrize("name,n", [("cfg1", 70), ("cfg5", 53), ("cfg4b", 40), ("cfg3", 33)])
def test_graphs_of_stage_launches_give_the_same_bits(name, n):
    wl = synth.WORKLOADS[name]
    print("case", name, n, flush=True)
    g, _ = build_pair(wl)
    g.set_mode(binding.MODE_STAGES)
    imgs, labs = synth.images(wl, n), synth.labels(wl, n)
    w0 = g.get_weights()
    w_plain, p_plain = _run(g, imgs, labs, wl.lr, 0)
    for per_graph in (16, 5, n // 2):   # (whole graphs plus a rest; one graph; two graphs)
        g.set_weights(w0)
        w_graph, p_graph = _run(g, imgs, labs, wl.lr, per_graph)
        assert np.array_equal(w_plain, w_graph), per_graph
        assert np.array_equal(p_plain, p_graph), per_graph
    # the stage list changes: the graph is built again
    g.set_matrix_cores(0)
    g.set_weights(w0)
    w_a, p_a = _run(g, imgs, labs, wl.lr, 16)
    g.set_weights(w0)
    w_b, p_b = _run(g, imgs, labs, wl.lr, 0)
    assert np.array_equal(w_a, w_b) and np.array_equal(p_a, p_b)
    g.close()


def test_a_bad_label_inside_a_graph_is_skipped_and_reported():
    wl = synth.WORKLOADS["cfg1"]
    g, _ = build_pair(wl)
    g.set_mode(binding.MODE_STAGES)
    n = 48
    imgs, labs = synth.images(wl, n), synth.labels(wl, n).copy()
    w0 = g.get_weights()
    keep = np.ones(n, dtype=bool)
    keep[21] = False
    g.train_many(to_dev(imgs[keep]), to_dev(labs[keep]), wl.lr)
    want = g.get_weights()
    g.set_weights(w0)
    labs[21] = 99
    g.train_many(to_dev(imgs), to_dev(labs), wl.lr)
    with pytest.raises(binding.CnnError) as e:
        g.synchronize()
    assert e.value.code == binding.E_ARG
    assert np.array_equal(g.get_weights(), want)
    with pytest.raises(binding.CnnError):
        g.set_launch_graph(-1)
    g.close()
