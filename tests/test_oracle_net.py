"""Pins for the oracle's whole-network forward / backward / update (no GPU)."""
import numpy as np
import pytest

import oracle
from paper_1102_0183_amd import synth
from tests.torch_witness import loss_and_grads

TINY = [
    # (arch, tables {conv_index: fan-in}, frontend?)
    ("1x9x9-3C4-MP2-4C2-5N-3N", {}, False),
    ("2x11x11-3C3S1-4C2-MP2-4N", {1: 2}, False),                 # skip + conv->conv + sparse table
    ("2x12x12-4C5S1-MP2-3C2-3N", {1: 2}, False),                 # (12-5)/2+1 = 4.5 -> floor
    ("3x8x8-4C3-MP3-4C2-6N-5N-4N", {1: 3}, False),               # maps shrink to 1 pixel, two hidden FC
    ("4x8x8-3C3S1-MP1-5N-2N", {}, True),                         # fixed front-end on a 2x12x12 raw image
    ("1x6x6-2C3-3N", {}, False),                                 # no pooling at all
    # kernels, skipping factors and pooling rectangles with different x and y values (Sec. 2.2, 2.3)
    ("2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N", {1: 2}, False),
    ("1x10x12-2C3x5-MP4x2-4N", {}, False),
    ("1x9x9-2C2S0x1-MP2x1-3C2x1S1x0-3N", {}, False),
]


def _build(arch, fan, frontend, seed, out_units=0):
    rng = np.random.default_rng(seed)
    o = oracle.Oracle(arch)
    o.set_output_units(out_units)
    tables = {}
    convs = [l for l in range(1, o.num_layers) if o.layer_info(l)["kind"] == oracle.binding.KIND_CONV]
    for ci, f in fan.items():
        l = convs[ci]
        t = synth.random_table(o.layer_info(l)["maps"], o.layer_info(l - 1)["maps"], f, seed + ci)
        o.set_connection_table(ci, t)
        tables[ci] = t
    fe = None
    if frontend:
        filt = rng.standard_normal((4, 5, 5)).astype(np.float32) * 0.2
        src = np.array([0, 0, 1, 1], dtype=np.int32)
        o.set_fixed_frontend(filt, src, 2)
        fe = (filt.astype(np.float64), src)
    w = rng.uniform(-0.5, 0.5, o.num_weights)
    o.set_weights(w)
    img = rng.uniform(-1, 1, o.image_size).astype(np.float32)
    n_cls = o.layer_info(o.num_layers - 1)["maps"]
    label = int(rng.integers(n_cls))
    return o, w, img, label, tables, fe


def _raw_shape(o, frontend):
    i = o.layer_info(0)
    if frontend:
        return (2, i["h"] + 4, i["w"] + 4)
    return (i["maps"], i["h"], i["w"])


@pytest.mark.parametrize("out_units", [0, 1])
@pytest.mark.parametrize("arch,fan,frontend", TINY)
def test_gradient_vs_central_finite_differences(arch, fan, frontend, out_units):
    """The paper's own check of its CPU version (Sec. 4): analytic gradient against finite
    differences of E, here in double with a relative step; for soft-max + cross-entropy
    outputs and for scaled-tanh + squared-error outputs."""
    o, w, img, label, _, _ = _build(arch, fan, frontend, 1234, out_units)
    g, e = o.gradients(img, label)
    assert e == pytest.approx(o.loss(img, label), rel=1e-14)
    rng = np.random.default_rng(5)
    idx = np.arange(w.size) if w.size <= 400 else rng.choice(w.size, 400, replace=False)
    h = 1e-6
    worst = 0.0
    for t in idx:
        wp = w.copy()
        wp[t] += h
        o.set_weights(wp)
        ep = o.loss(img, label)
        wp[t] -= 2 * h
        o.set_weights(wp)
        em = o.loss(img, label)
        fd = (ep - em) / (2 * h)
        worst = max(worst, abs(fd - g[t]))
    assert worst <= 2e-8 * max(1.0, np.abs(g).max()), worst


@pytest.mark.parametrize("out_units", [0, 1])
@pytest.mark.parametrize("arch,fan,frontend", TINY)
def test_whole_network_vs_autograd_library(arch, fan, frontend, out_units):
    o, w, img, label, tables, fe = _build(arch, fan, frontend, 4321, out_units)
    g, e = o.gradients(img, label)
    p = o.forward(img)
    e2, g2, p2 = loss_and_grads(arch, w, img.reshape(_raw_shape(o, frontend)), label, tables, fe,
                                tanh_outputs=bool(out_units))
    assert e == pytest.approx(e2, rel=1e-12)
    np.testing.assert_allclose(p, p2, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g, g2, rtol=1e-10, atol=1e-12)


def test_benchmark_net_vs_autograd_library():
    wl = synth.WORKLOADS["cfg1"]
    o = oracle.Oracle(wl.arch)
    w = synth.weights(wl, o.num_weights).astype(np.float64)
    o.set_weights(w)
    img = synth.images(wl, 3)[2]
    lab = int(synth.labels(wl, 3)[2])
    g, e = o.gradients(img, lab)
    e2, g2, _ = loss_and_grads(wl.arch, w, img, lab)
    assert e == pytest.approx(e2, rel=1e-12)
    np.testing.assert_allclose(g, g2, rtol=1e-9, atol=1e-13)


def test_sparse_frontend_net_vs_autograd_library():
    """Skipping factor, floor in Eq. 1, 50 % table and the fixed front-end together, at a
    reduced number of maps so that the library witness stays quick."""
    wl = synth.WORKLOADS["cfg5"]
    arch = "4x44x44-6C5S1-MP2-8C3-MP2-10N-5N"
    o = oracle.Oracle(arch)
    t = synth.random_table(8, 6, 3, 99)
    o.set_connection_table(1, t)
    filt, src = synth.contrast_filters(wl)
    o.set_fixed_frontend(filt, src, 2)
    rng = np.random.default_rng(8)
    w = rng.uniform(-0.3, 0.3, o.num_weights)
    o.set_weights(w)
    img = synth.images(wl, 1)[0]
    g, e = o.gradients(img, 3)
    e2, g2, _ = loss_and_grads(arch, w, img, 3, {1: t}, (filt.astype(np.float64), src))
    assert e == pytest.approx(e2, rel=1e-12)
    np.testing.assert_allclose(g, g2, rtol=1e-9, atol=1e-13)


def test_contrast_filters_are_zero_sum_unit_l1():
    filt, src = synth.contrast_filters(synth.WORKLOADS["cfg5"])
    assert filt.shape == (4, 5, 5) and list(src) == [0, 0, 1, 1]
    assert np.abs(filt.sum(axis=(1, 2))).max() < 1e-6
    np.testing.assert_allclose(np.abs(filt).sum(axis=(1, 2)), 1.0, rtol=1e-5)
    assert filt[0, 2, 2] > 0 and filt[1, 2, 2] < 0           # on-centre, off-centre


def test_fixed_frontend_is_linear_and_untouched_by_training():
    o, w, img, label, _, fe = _build("4x8x8-3C3S1-MP1-5N-2N", {}, True, 77)
    o.forward(img)
    a0 = o.activation(0)
    # closed form: correlation of the source channel with the filter, no bias, no tanh
    raw = img.reshape(2, 12, 12).astype(np.float64)
    filt, src = fe
    for f in range(4):
        want = np.zeros((8, 8))
        for y in range(8):
            for x in range(8):
                want[y, x] = (filt[f] * raw[src[f], y:y + 5, x:x + 5]).sum()
        np.testing.assert_allclose(a0[f], want, rtol=1e-12, atol=1e-14)
    o.train_step(img, label, 0.1)
    o.forward(img)
    np.testing.assert_array_equal(o.activation(0), a0)


def test_sgd_step_semantics():
    """Sec. 1 / Sec. 4: plain on-line gradient descent, w <- w - lr * dE/dw after each image."""
    o, w, img, label, _, _ = _build("1x9x9-3C4-MP2-4C2-5N-3N", {}, False, 9)
    g, e = o.gradients(img, label)
    np.testing.assert_array_equal(o.get_weights(), w)       # computing a gradient changes nothing
    o.train_step(img, label, 0.0)
    np.testing.assert_array_equal(o.get_weights(), w)       # lr = 0: bit-unchanged
    e_step = o.train_step(img, label, 0.01)
    assert e_step == pytest.approx(e, rel=1e-14)
    np.testing.assert_allclose(o.get_weights(), w - 0.01 * g, rtol=0, atol=1e-17)
    # presenting the same image again and again lowers its error
    errs = [o.train_step(img, label, 0.01) for _ in range(20)]
    assert all(b < a for a, b in zip(errs, errs[1:]))
    assert errs[0] < e


def test_online_update_uses_the_previous_images_weights():
    """Two on-line steps differ from one step on the sum of two gradients taken at the start."""
    o, w, img, label, _, _ = _build("1x9x9-3C4-MP2-4C2-5N-3N", {}, False, 10)
    rng = np.random.default_rng(3)
    img2 = rng.uniform(-1, 1, img.size).astype(np.float32)
    g1, _ = o.gradients(img, label)
    o.train_step(img, label, 0.05)
    g2_after, _ = o.gradients(img2, 1)
    o.train_step(img2, 1, 0.05)
    np.testing.assert_allclose(o.get_weights(), w - 0.05 * g1 - 0.05 * g2_after, rtol=0, atol=1e-16)
    o.set_weights(w)
    g2_before, _ = o.gradients(img2, 1)
    assert np.abs(g2_before - g2_after).max() > 1e-6


def test_deltas_and_argmax_taps():
    o, w, img, label, _, _ = _build("1x9x9-3C4-MP2-4C2-5N-3N", {}, False, 11)
    o.gradients(img, label)
    p = o.activation(o.num_layers - 1).ravel()
    d_out = o.delta(o.num_layers - 1).ravel()
    onehot = np.eye(3)[label]
    np.testing.assert_allclose(d_out, p - onehot, atol=1e-16)
    # conv layer 1 is pooled 2x2: its delta is non-zero only at the arg-max of each window
    d1 = o.delta(1)
    arg = o.argmax(2)
    a1 = o.activation(1)
    for j in range(3):
        for y in range(3):
            for x in range(3):
                win = d1[j, 2 * y:2 * y + 2, 2 * x:2 * x + 2]
                dy, dx = divmod(int(arg[j, y, x]), 2)
                mask = np.ones((2, 2), bool)
                mask[dy, dx] = False
                assert (win[mask] == 0).all()
                assert a1[j, 2 * y + dy, 2 * x + dx] == o.activation(2)[j, y, x]
    # bias gradient of a conv layer is the sum of its deltas (one bias per map)
    g, _ = o.gradients(img, label)
    np.testing.assert_allclose(g[:3], d1.sum(axis=(1, 2)), rtol=1e-13)


def test_label_out_of_range_is_rejected():
    o = oracle.Oracle("1x6x6-2C3-3N")
    with pytest.raises(oracle.binding.OracleError):
        o.train_step(np.zeros(36, np.float32), 3, 0.1)
    with pytest.raises(oracle.binding.OracleError):
        o.train_step(np.zeros(36, np.float32), -1, 0.1)


def test_float_instantiation_tracks_double():
    wl = synth.WORKLOADS["cfg1"]
    od, of = oracle.Oracle(wl.arch, 64), oracle.Oracle(wl.arch, 32)
    w = synth.weights(wl, od.num_weights)
    od.set_weights(w)
    of.set_weights(w)
    imgs, labs = synth.images(wl, 5), synth.labels(wl, 5)
    od.train_many(imgs, labs, 1e-3)
    of.train_many(imgs, labs, 1e-3)
    d = np.abs(od.get_weights() - of.get_weights()).max()
    assert 0 < d < 1e-6


def test_forward_then_backward_update_equals_train_step():
    o, w, img, label, _, _ = _build("1x9x9-3C4-MP2-4C2-5N-3N", {}, False, 12)
    o2, _, _, _, _, _ = _build("1x9x9-3C4-MP2-4C2-5N-3N", {}, False, 12)
    e1 = o.train_step(img, label, 0.05)
    o2.forward(img)
    e2 = o2.backward_update(label, 0.05)
    assert e1 == e2
    np.testing.assert_array_equal(o.get_weights(), o2.get_weights())


def test_argmax_hints_are_adopted_only_at_near_ties():
    """Hints exist so that a second implementation's valid choice at a near-tie can be
    followed; anything but a near-tie is refused and changes nothing."""
    arch = "1x4x4-1C1-MP2-2N"
    o = oracle.Oracle(arch)
    # weights: conv bias 0, kernel 1 (identity up to the tanh); FC arbitrary
    w = np.zeros(o.num_weights)
    w[1] = 1.0
    w[4:] = np.arange(o.num_weights - 4) * 0.1 - 0.3
    o.set_weights(w)
    img = np.array([[0.50, 0.50 - 1e-9, 0.1, 0.2],
                    [0.10, 0.20, 0.9, 0.3],
                    [0.30, 0.10, 0.4, 0.4],
                    [0.20, 0.25, 0.1, 0.2]], dtype=np.float64).astype(np.float32)
    # float32 rounding makes the first two equal or nearly so; window (1,1) holds an exact tie
    o.forward(img)
    own = o.argmax(2).copy()
    assert own[0, 1, 1] == 0                       # exact tie -> first in row-major order
    pooled = o.activation(2).copy()
    # 1) hint equal to own choice: nothing happens
    assert o.adopt_argmax_hint(2, own, 1e-6) == (0, 0)
    # 2) hint picks the other member of the exact tie: adopted, pooled value unchanged
    hint = own.copy()
    hint[0, 1, 1] = 1
    assert o.adopt_argmax_hint(2, hint, 1e-6) == (1, 0)
    assert o.argmax(2)[0, 1, 1] == 1
    np.testing.assert_allclose(o.activation(2), pooled, atol=1e-12)
    # the delta now goes to the hinted position
    o.backward_update(1, 0.0)
    d = o.delta(1)[0]
    assert d[2, 3] != 0 and d[2, 2] == 0
    # 3) a hint that is not a near-tie is refused and leaves the state alone
    o.forward(img)
    hint = o.argmax(2).copy()
    hint[0, 0, 1] = 0                              # value 0.1 against the maximum 0.9
    assert o.adopt_argmax_hint(2, hint, 1e-6) == (0, 1)
    np.testing.assert_array_equal(o.argmax(2), own)
    # 4) an index outside the rectangle is refused
    hint = own.copy()
    hint[0, 0, 0] = 7
    assert o.adopt_argmax_hint(2, hint, 1e-6) == (0, 1)


def test_tanh_outputs_train_toward_their_targets():
    """Scaled-tanh output units with the squared error: presenting one image again and again
    with a small rate drives E down and every output toward its +-1 target; the soft-max
    default is untouched by the option being set and reset."""
    arch = "1x9x9-3C4-MP2-4C2-5N-3N"
    o, w, img, label, _, _ = _build(arch, {}, False, 77)
    p_softmax = o.forward(img)
    o.set_output_units(1)
    y0 = o.forward(img)
    assert np.all(np.abs(y0) < 1.7159) and abs(y0.sum() - 1.0) > 1e-3   # outputs, not probabilities
    e_first = o.loss(img, label)
    last = e_first
    for _ in range(60):
        e = o.train_step(img, label, 0.02)
        assert e <= last + 1e-12
        last = e
    y = o.forward(img)
    t = -np.ones(3)
    t[label] = 1.0
    assert last < 0.2 * e_first
    assert np.abs(y - t).max() < np.abs(y0 - t).max()
    o.set_output_units(0)
    o.set_weights(w)
    np.testing.assert_array_equal(o.forward(img), p_softmax)
