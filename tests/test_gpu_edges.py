"""Edge cases of the HIP path against the oracle: degenerate and ragged shapes, every kernel
code path (kernel sizes with and without a compiled specialisation, both tilings, skips,
sparse tables, no pooling, conv on conv, 1-pixel maps), and the error paths of the C ABI."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth
from tests.parity_helpers import (TOL_ACT, TOL_W100, build_pair, compare_backward_state, compare_forward_state,
                                  layer_bounds, lockstep_train, rel_err, to_dev)

pytestmark = pytest.mark.gpu
MODES = [binding.MODE_STAGES, binding.MODE_PERSISTENT, binding.MODE_RESIDENT]

# (architecture, {conv_index: fan_in}, front-end K or 0, number of raw channels)
SHAPES = [
    ("1x9x9-3C4-MP2-4C2-5N-3N", {}, 0, 1),
    ("2x11x11-3C3S1-4C2-MP2-4N", {1: 2}, 0, 2),              # skip, conv on conv, sparse table
    ("2x12x12-4C5S1-MP2-3C2-3N", {1: 2}, 0, 2),              # Eq. 1 does not divide: last row/column unread
    ("3x8x8-4C3-MP3-4C2-6N-5N-4N", {1: 3}, 0, 3),            # maps shrink to one pixel; two hidden FC layers
    ("4x8x8-3C3S1-MP1-5N-2N", {}, 5, 2),                     # fixed front-end; pooling rectangle of one
    ("4x12x12-3C3-MP2-5N-2N", {}, 21, 2),                    # 21 x 21 fixed filters (Sec. 4.2) on a 2x32x32 raw image
    ("3x10x10-4C3-MP2-3N", {}, 13, 3),                       # 13 x 13 fixed filters (Sec. 4.3), one per colour channel
    ("1x6x6-2C3-3N", {}, 0, 1),                              # no pooling at all
    ("1x5x5-4N", {}, 0, 1),                                  # no convolution at all: the output layer reads the image
    ("1x5x5-7N-4N", {}, 0, 1),
    ("1x22x6-2N-19N-6N", {}, 2, 1),                          # fully connected layers straight behind a fixed front-end
    ("3x6x6-4N", {}, 3, 2),                                  # ... and the output layer alone behind one
    ("2x10x10-5C1-MP2-3C1S1-6N-2N", {}, 0, 2),               # 1x1 kernels
    ("1x20x20-6C6-MP3-5C3S2-4N", {}, 0, 1),                  # kernel sizes without a compiled specialisation; skip 2
    ("2x23x23-5C7S1-4C2-MP2-3N", {1: 3}, 0, 2),
    ("1x8x600-3C3-MP2-4C2S1-5N", {}, 0, 1),                  # rows wider than one workgroup: two pixels per thread
    ("1x70x70-4C3-MP4-3C4-MP2-6N", {}, 0, 1),                # several row bands per map, ragged last band
    ("3x34x47-7C4S1-8C3-MP2-9C2-MP3-20N-6N", {1: 4, 2: 5}, 0, 3),   # rectangular maps, three conv layers
    ("1x40x40-70C5-MP4-300C3-MP1-10N", {}, 0, 1),            # many maps on few pixels: chunked connection lists
    # kernels, skipping factors and pooling rectangles whose x and y values differ (Sec. 2.2, 2.3)
    ("2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N", {1: 2}, 0, 2),
    ("1x10x12-2C3x5-MP4x2-4N", {}, 0, 1),
    ("1x9x9-2C2S0x1-MP2x1-3C2x1S1x0-3N", {}, 0, 1),
    ("3x40x33-9C5x3S1x2-MP2x1-8C2x4-MP1x2-7C3x1S0x1-12N-5N", {1: 4, 2: 3}, 0, 3),   # three such layers, sparse tables
    ("1x30x70-6C7x2-MP8x3-5N", {}, 0, 1),                    # a kernel size without a compiled loop, a tall pooling rectangle
    # few maps below many above, no pooling above: in resident mode several ranks share the delta pull into one map
    # (9 x 9 kernels: the output layer reads 4 x 4 maps, as it does behind the pooled variants below)
    ("1x28x28-6C5-MP2-100C9-MP1-8N", {}, 0, 1),              # 16 shares a map, full table
    ("1x28x28-6C5-MP2-100C9-MP1-8N", {1: 5}, 0, 1),          # ... sparse table
    ("1x28x28-40C5-MP2-80C9-MP1-8N", {1: 12}, 0, 1),         # 2 shares a map, sparse table
    # pooled layers: in resident mode the delta pull through them visits the pooling winners only, and is not shared
    ("1x28x28-6C5-MP2-100C5-MP2-8N", {}, 0, 1),              # 16 winners a map, 64 connections at a time
    ("1x28x28-40C5-MP2-80C5-MP2-8N", {1: 38}, 0, 1),         # sparse table
    ("1x47x47-6C4-MP2-100C5-MP3-8N", {}, 0, 1),              # 36 winners a map
    ("1x65x65-8C4-MP2-20C5-MP3-6N", {}, 0, 1),               # 81 winners a map: two parts of 41 lanes
    ("1x65x65-8C4-MP2-20C5-MP3-6N", {1: 3}, 0, 1),           # ... sparse table
    ("2x60x60-3C5-MP4-7C4S1-MP3-4C1-MP1-5N", {1: 2}, 0, 2),  # skipping factor 1 under the winners, 1x1 kernels above
    ("1x18x18-3C2-4C2-MP2-5C3-4C2-MP1-3C2S1-4C1-6N-3N", {2: 2, 4: 3}, 0, 1),   # six convolutional layers
]
SHARES = {"1x28x28-6C5-MP2-100C9-MP1-8N": 16, "1x28x28-40C5-MP2-80C9-MP1-8N": 2, "1x28x28-6C5-MP2-100C5-MP2-8N": 1,
          "1x47x47-6C4-MP2-100C5-MP3-8N": 1}

def _pair(arch, fan, fe_k, n_src, seed, wscale=0.3):
    import oracle
    o0 = oracle.Oracle(arch)
    convs = [l for l in range(1, o0.num_layers) if o0.layer_info(l)["kind"] == 1]
    tables = {ci: synth.random_table(o0.layer_info(convs[ci])["maps"], o0.layer_info(convs[ci] - 1)["maps"],
                                     f, 1000 + seed + ci) for ci, f in fan.items()}
    frontend = None
    if fe_k:
        rng = np.random.default_rng(seed)
        c = o0.layer_info(0)["maps"]
        filt = (rng.standard_normal((c, fe_k, fe_k)) * 0.2).astype(np.float32)
        src = rng.integers(0, n_src, size=c).astype(np.int32)
        frontend = (filt, src, n_src)
    return build_pair(arch=arch, tables=tables, frontend=frontend, seed=seed, wscale=wscale)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("arch,fan,fe_k,n_src", SHAPES)
def test_shapes_one_step_and_ten_steps(arch, fan, fe_k, n_src, mode):
    print("case", arch, "mode", mode, flush=True)
    g, o = _pair(arch, fan, fe_k, n_src, 7)
    if not g.mode_supported(mode):
        g.close()
        pytest.skip("mode %d cannot run this network" % mode)
    g.set_mode(mode)
    if mode == binding.MODE_RESIDENT and arch in SHARES:
        assert g.resident_pull_shares(1) == SHARES[arch]
    rng = np.random.default_rng(17)
    n_cls = g.num_classes
    imgs = rng.uniform(-1, 1, (10, g.image_size)).astype(np.float32)
    labs = rng.integers(0, n_cls, size=10).astype(np.int32)
    grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
    grad_o, loss_o = o.gradients(imgs[0], int(labs[0]))
    compare_forward_state(g, o)
    compare_backward_state(g, o)
    assert abs(g.loss() - loss_o) <= 1e-5 * max(1.0, abs(loss_o))
    for (a, b) in layer_bounds(o):
        assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (a, b)
    # ten on-line steps with large weights and a large rate, side by side (near-tie pooling winners
    # follow the GPU, see lockstep_train): the stated bound for trained weights
    w0 = g.get_weights()
    adopted = lockstep_train(g, o, imgs, labs, 0.01)
    w_step = g.get_weights()
    print("  near-tie winners adopted:", adopted, flush=True)
    assert rel_err(w_step, o.get_weights()) <= TOL_W100
    # the batched call lands on the same bits as the image-by-image calls
    g.set_weights(w0)
    g.train_many(to_dev(imgs), to_dev(labs), 0.01)
    np.testing.assert_array_equal(g.get_weights(), w_step)
    g.close()


# Networks whose per-rank share does not fit next to all inputs of every layer: the resident plan streams the
# inputs (chunks of maps through one arena), adjusts every filter above the first layer once and sends it on.
STREAMED = [
    ("3x32x32-100C5-MP2-100C5-MP2-8N", {}, (0, 0)),
    ("3x32x32-100C5-MP2-100C5-MP2-8N", {1: 60}, (50, 1)),      # sparse table, two maps a rank
    ("2x40x40-60C5S1-120C3-MP2-6N", {1: 31}, (50, 1)),         # skipping factor below, ranks with 3 and with 2 maps, sparse
    ("1x40x40-64C5-MP2-64C1-MP2-64C3-9N", {}, (50, 1)),        # three layers, a 1x1 kernel (no compiled filter loop)
    ("1x44x44-90C3-MP2-90C6-MP2-7N", {1: 50}, (0, 0)),         # 6x6 kernel, sparse
]


@pytest.mark.parametrize("arch,fan,team", STREAMED)
def test_streamed_resident_plans(arch, fan, team):
    print("case", arch, fan, team, flush=True)
    # (weights in the paper's range: with hundreds of inputs per unit a wider range saturates whole maps, whose
    # pooling winners are then ties by the hundred -- saturated nets have their own test)
    g, o = _pair(arch, fan, 0, 1, 11, wscale=0.05)
    g.set_mode(binding.MODE_RESIDENT)
    if team != (0, 0):
        g.set_team(*team)
    assert g.resident_streams()
    rng = np.random.default_rng(23)
    imgs = rng.uniform(-1, 1, (10, g.image_size)).astype(np.float32)
    labs = rng.integers(0, g.num_classes, size=10).astype(np.int32)
    grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
    grad_o, loss_o = o.gradients(imgs[0], int(labs[0]))
    compare_forward_state(g, o)
    compare_backward_state(g, o)
    for (a, b) in layer_bounds(o):
        assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (a, b)
    w0 = g.get_weights()
    adopted = lockstep_train(g, o, imgs, labs, 0.01)
    w_step = g.get_weights()
    print("  near-tie winners adopted:", adopted, flush=True)
    assert rel_err(w_step, o.get_weights()) <= TOL_W100
    # the batched call lands on the same bits as the image-by-image calls, and so do two calls of five
    g.set_weights(w0)
    g.train_many(to_dev(imgs), to_dev(labs), 0.01)
    np.testing.assert_array_equal(g.get_weights(), w_step)
    g.set_weights(w0)
    g.train_many(to_dev(imgs[:5]), to_dev(labs[:5]), 0.01)
    g.train_many(to_dev(imgs[5:]), to_dev(labs[5:]), 0.01)
    np.testing.assert_array_equal(g.get_weights(), w_step)
    g.close()


# Networks with a large hidden layer behind the first fully connected one (Sec. 3's CIFAR nets end in 300N-100N-10N):
# the resident plan holds that layer by columns, like the first one.
BY_COLUMNS = [
    ("1x20x20-6C5-MP2-12C4-MP1-120N-90N-7N", (0, 0), 0.1, False),            # ten columns a rank
    ("1x20x20-6C5-MP2-12C4-MP1-120N-90N-7N", (5, 1), 0.1, False),            # 24 columns a rank, ranks with 3 and 2 maps
    ("1x12x12-100C3-MP2-90N-100N-5N", (0, 0), 0.05, False),                  # more ranks than columns
    ("1x16x16-7C3-MP2-100N-83N-11N-4N", (0, 0), 0.1, False),                 # two more layers behind it; ragged columns
    ("3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", (0, 0), 0.05, False),
    ("3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", (50, 1), 0.05, False),
    ("3x32x32-200C3-MP3-200C3-MP2-200C3-MP2-300N-100N-10N", (0, 0), 0.05, True),   # with streamed inputs
    # no such layer, but so many partial sums of the first fully connected layer (ranks x outputs) that each output
    # is added up by one rank and sent round: fewer outputs than ranks, more outputs than ranks
    ("1x12x12-200C3-MP2-90N-5N", (0, 0), 0.05, False),
    ("1x12x12-60C3-MP2-300N-5N", (0, 0), 0.05, False),
]


@pytest.mark.parametrize("arch,team,wscale,streams", BY_COLUMNS)
def test_resident_plans_with_a_hidden_layer_held_by_columns(arch, team, wscale, streams):
    print("case", arch, team, flush=True)
    g, o = _pair(arch, {}, 0, 1, 13, wscale=wscale)
    g.set_mode(binding.MODE_RESIDENT)
    if team != (0, 0):
        g.set_team(*team)
    plan = binding.resident_plan(arch, 0, *team)
    assert bool(g.resident_streams()) == streams
    if len(plan["fc"]) > 2:
        assert plan["fc"][1]["by_cols"] == 1
    else:
        assert plan["numbers"]["fc1_owned"] == 1
    rng = np.random.default_rng(29)
    imgs = rng.uniform(-1, 1, (10, g.image_size)).astype(np.float32)
    labs = rng.integers(0, g.num_classes, size=10).astype(np.int32)
    grad_g = g.debug_gradients(to_dev(imgs[0]), int(labs[0]))
    grad_o, loss_o = o.gradients(imgs[0], int(labs[0]))
    compare_forward_state(g, o)
    compare_backward_state(g, o)
    assert abs(g.loss() - loss_o) <= 1e-5 * max(1.0, abs(loss_o))
    for (a, b) in layer_bounds(o):
        assert rel_err(grad_g[a:b], grad_o[a:b]) <= TOL_ACT, (a, b)
    w0 = g.get_weights()
    adopted = lockstep_train(g, o, imgs, labs, 0.01)
    w_step = g.get_weights()
    print("  near-tie winners adopted:", adopted, flush=True)
    assert rel_err(w_step, o.get_weights()) <= TOL_W100
    # the batched call lands on the same bits as the image-by-image calls, and on those of the launch-per-stage mode
    g.set_weights(w0)
    g.train_many(to_dev(imgs), to_dev(labs), 0.01)
    np.testing.assert_array_equal(g.get_weights(), w_step)
    g.set_weights(w0)
    g.train_many(to_dev(imgs[:5]), to_dev(labs[:5]), 0.01)
    g.train_many(to_dev(imgs[5:]), to_dev(labs[5:]), 0.01)
    np.testing.assert_array_equal(g.get_weights(), w_step)
    g.close()


def test_create_errors():
    import torch
    for arch, code in [("1x29x29-20C4-MP4-10N", binding.E_SHAPE), ("1x29x29-20C4", binding.E_SYNTAX),
                       ("1x200x200-3C3-4N", binding.E_SHAPE)]:       # input map larger than the staging area
        with pytest.raises(binding.CnnError) as e:
            binding.Cnn(arch)
        assert e.value.code == code, arch
        assert str(e.value)
    # workspace too small / misaligned
    L = binding.lib()
    import ctypes as C
    arch = b"1x9x9-3C4-MP2-4C2-5N-3N"
    need = binding.workspace_bytes(arch.decode())
    buf = torch.zeros(need + 512, dtype=torch.uint8, device="cuda:0")
    base = (buf.data_ptr() + 255) // 256 * 256
    h = C.c_void_p()
    assert L.cnn_create(arch, base, need - 1, None, C.addressof(h)) == binding.E_WORKSPACE
    assert L.cnn_create(arch, base + 4, need, None, C.addressof(h)) == binding.E_WORKSPACE
    assert L.cnn_create(arch, None, need, None, C.addressof(h)) == binding.E_WORKSPACE
    assert L.cnn_create(arch, base, need, None, None) == binding.E_ARG
    assert b"workspace" in L.cnn_last_error(None) or L.cnn_last_error(None)


def test_layers_with_different_x_and_y_values_are_refused_by_the_resident_mode():
    import torch
    g = binding.Cnn("1x10x12-2C3x5-MP4x2-4N")
    assert g.mode_supported(binding.MODE_STAGES) and g.mode_supported(binding.MODE_PERSISTENT)
    assert not g.mode_supported(binding.MODE_RESIDENT)
    with pytest.raises(binding.CnnError) as e:
        g.set_mode(binding.MODE_RESIDENT)
    assert e.value.code == binding.E_STATE
    assert g.forward_batch_scratch_bytes(16) > 0   # the batched forward pass takes them
    info = g.layer_info(1)
    assert (info["K"], info["Kx"], info["h"], info["w"]) == (3, 5, 8, 8)
    g.close()
    torch.cuda.synchronize()


def test_argument_errors_and_bad_labels():
    import torch
    g, o = build_pair(arch="1x9x9-3C4-MP2-4C2-5N-3N", seed=3)
    img = torch.zeros(81, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.CnnError) as e:
        g.train_step(img, 3, 0.1)
    assert e.value.code == binding.E_ARG
    with pytest.raises(binding.CnnError):
        g.train_step(img, -1, 0.1)
    with pytest.raises(binding.CnnError):
        g.set_weights(np.zeros(5, np.float32))
    with pytest.raises(binding.CnnError):
        g.set_connection_table(5, np.ones((4, 3), np.uint8))
    with pytest.raises(binding.CnnError):
        g.set_connection_table(1, np.zeros((4, 3), np.uint8))      # an output map without input
    with pytest.raises(binding.CnnError):
        g.argmax(1)                                                # not a pooling layer
    with pytest.raises(binding.CnnError):
        g.delta(2)                                                 # pooling layers hold no delta
    with pytest.raises(binding.CnnError) as e:
        g.set_output_units(7)                                      # neither of the two kinds
    assert e.value.code == binding.E_ARG and g.output_units == binding.OUTPUT_SOFTMAX_XENT
    # a bad label inside a device label array: that image is skipped, the others train, and
    # the next synchronising call reports it
    rng = np.random.default_rng(1)
    imgs = rng.uniform(-1, 1, (4, 81)).astype(np.float32)
    labs = np.array([1, 7, 2, 0], dtype=np.int32)
    for mode in MODES:
        g.set_mode(mode)
        w = (rng.random(g.num_weights, dtype=np.float32) - 0.5).astype(np.float32)
        g.set_weights(w)
        o.set_weights(w.astype(np.float64))
        g.train_many(to_dev(imgs), to_dev(labs), 0.05)
        with pytest.raises(binding.CnnError) as e:
            g.synchronize()
        assert e.value.code == binding.E_ARG
        g.synchronize()                                            # the flag is cleared once reported
        for t in (0, 2, 3):
            o.train_step(imgs[t], int(labs[t]), 0.05)
        assert rel_err(g.get_weights(), o.get_weights()) <= 1e-5
    g.close()


def test_zero_images_is_a_no_op():
    import torch
    g, _ = build_pair(arch="1x9x9-3C4-MP2-4C2-5N-3N", seed=3)
    w = g.get_weights()
    empty = torch.zeros(81, dtype=torch.float32, device="cuda:0")
    labs = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for mode in MODES:
        g.set_mode(mode)
        g.train_many(empty, labs, 0.1, n=0)
        g.forward_many(empty, 0)
    np.testing.assert_array_equal(g.get_weights(), w)
    g.close()


def test_checkpoint_roundtrip():
    """get_weights -> a fresh network -> set_weights gives identical forward bits."""
    import torch
    wl = synth.WORKLOADS["cfg5"]
    g, _ = build_pair(wl)
    imgs, labs = synth.images(wl, 6), synth.labels(wl, 6)
    g.train_many(to_dev(imgs[:5]), to_dev(labs[:5]), 0.01)
    w = g.get_weights()
    p1 = torch.empty(g.num_classes, dtype=torch.float32, device="cuda:0")
    g.forward(to_dev(imgs[5]), p1)
    g.synchronize()
    g2, _ = build_pair(wl, weights=w)
    p2 = torch.empty(g.num_classes, dtype=torch.float32, device="cuda:0")
    g2.forward(to_dev(imgs[5]), p2)
    g2.synchronize()
    assert torch.equal(p1, p2)
    g.close()
    g2.close()


@pytest.mark.parametrize("mode,name,limit", [
    (binding.MODE_PERSISTENT, "cfg1", 0), (binding.MODE_RESIDENT, "cfg1", 0),
    # a few polls allowed: the waits give up at different places from rank to rank, also where the owner of a
    # map waits for the sums of the ranks that share its delta pull (the larger net)
    (binding.MODE_RESIDENT, "cfg2b", 0), (binding.MODE_RESIDENT, "cfg2b", 4), (binding.MODE_RESIDENT, "cfg2b", 40)])
def test_barrier_gives_up_cleanly_when_it_cannot_complete(mode, name, limit):
    """Force the failure path from the host: a spin limit of zero (or a few) polls makes every workgroup
    that has to wait longer (at a grid barrier, or for a tagged word) leave the kernel; the call must
    end, with an error unless nobody had to wait that long, and never hang."""
    wl = synth.WORKLOADS[name]
    print("case", name, "mode", mode, "spin limit", limit, flush=True)
    g, _ = build_pair(wl)
    g.set_mode(mode)
    g.set_spin_limit(limit)
    imgs, labs = synth.images(wl, 2), synth.labels(wl, 2)
    g.train_many(to_dev(imgs), to_dev(labs), 0.001)
    try:
        g.synchronize()
        timed_out = False
    except binding.CnnError as e:
        assert e.code == binding.E_HIP
        timed_out = True
    # with zero polls allowed the only way not to time out is that no workgroup ever waited
    # with no poll allowed some workgroup always has to wait longer than that (every exchange and every
    # grid barrier has a last arrival): the call must have ended with the error
    if limit == 0:
        assert timed_out
    # and the handle is usable again: from the same weights it lands on the bits of an untouched handle
    g.set_spin_limit(1 << 22)
    g.set_weights(synth.weights(wl, g.num_weights))
    g.train_many(to_dev(imgs), to_dev(labs), 0.001)
    g.synchronize()
    g2, _ = build_pair(wl)
    g2.set_mode(mode)
    g2.train_many(to_dev(imgs), to_dev(labs), 0.001)
    np.testing.assert_array_equal(g.get_weights(), g2.get_weights())
    g.close()
    g2.close()
