"""Pins for the oracle's shape inference and architecture grammar (no GPU)."""
import os

import pytest

import oracle
from oracle.binding import OracleError, E_SHAPE, E_SYNTAX, KIND_CONV, KIND_FC, KIND_POOL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_shapes.txt")


def _golden():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_paper_fig2_example():
    """Fig. 2 caption: 29x29, 5x5 kernel, skipping factor 1 -> 13x13."""
    rows = [r for r in _golden() if r[0] == "conv"]
    assert rows
    for _, m, k, s, want in rows:
        assert oracle.conv_out_size(int(m), int(k), int(s)) == int(want)
    # the same through the grammar, end to end
    o = oracle.Oracle("1x29x29-3C5S1-2N")
    i = o.layer_info(1)
    assert (i["h"], i["w"]) == (13, 13)


def test_paper_cifar_chain_ends_at_one_pixel():
    """Sec. 4.3 layer list + Sec. 2.4: the CIFAR10 net shrinks 32x32 to 1 pixel per map."""
    rows = [r for r in _golden() if r[0] == "chain"]
    assert rows
    for r in rows:
        side = int(r[1])
        toks = r[2:]
        arch = "3x%dx%d" % (side, side)
        sizes = []
        for t, s in zip(toks[0::2], toks[1::2]):
            arch += "-MP" + t[2:] if t.startswith("MP") else "-7" + t
            sizes.append(int(s))
        arch += "-10N"
        o = oracle.Oracle(arch)
        got = [o.layer_info(l)["h"] for l in range(1, o.num_layers - 1)]
        assert got == sizes
        assert got[-1] == 1


# layer outputs (maps, h, w) of the seven benchmark architectures, worked out by hand
# from Eq. 1 (floor where it does not divide) and the pooling factor
CHAINS = {
    "1x29x29-20C4-MP2-40C5-MP3-150N-10N":
        [(20, 26, 26), (20, 13, 13), (40, 9, 9), (40, 3, 3), (150, 1, 1), (10, 1, 1)],
    "1x29x29-40C4-MP2-80C5-MP3-300N-10N":
        [(40, 26, 26), (40, 13, 13), (80, 9, 9), (80, 3, 3), (300, 1, 1), (10, 1, 1)],
    "2x48x48-50C5-MP2-128C3-MP4-100N-5N":
        [(50, 44, 44), (50, 22, 22), (128, 20, 20), (128, 5, 5), (100, 1, 1), (5, 1, 1)],
    "3x32x32-100C5-MP2-100C5-MP2-100C4-MP2-300N-10N":
        [(100, 28, 28), (100, 14, 14), (100, 10, 10), (100, 5, 5), (100, 2, 2), (100, 1, 1),
         (300, 1, 1), (10, 1, 1)],
    "3x32x32-300C3-MP2-300C2-MP2-300C4-MP2-300N-10N":
        [(300, 30, 30), (300, 15, 15), (300, 14, 14), (300, 7, 7), (300, 4, 4), (300, 2, 2),
         (300, 1, 1), (10, 1, 1)],
    "4x44x44-40C5S1-MP2-80C3-MP2-100N-5N":
        [(40, 20, 20), (40, 10, 10), (80, 8, 8), (80, 4, 4), (100, 1, 1), (5, 1, 1)],
}
# weights = sum over conv (connections*K*K + maps) + sum over FC (n_in*n_out + n_out)
N_WEIGHTS = {
    "1x29x29-20C4-MP2-40C5-MP3-150N-10N": 76040,
    "1x29x29-40C4-MP2-80C5-MP3-300N-10N": 300070,
    "2x48x48-50C5-MP2-128C3-MP4-100N-5N": 380883,
    "3x32x32-100C5-MP2-100C5-MP2-100C4-MP2-300N-10N": 451110,
    "3x32x32-300C3-MP2-300C2-MP2-300C4-MP2-300N-10N": 2172310,
}


@pytest.mark.parametrize("arch", sorted(CHAINS))
def test_benchmark_architectures(arch):
    o = oracle.Oracle(arch)
    got = []
    for l in range(1, o.num_layers):
        i = o.layer_info(l)
        got.append((i["maps"], i["h"], i["w"]))
    assert got == CHAINS[arch]
    if arch in N_WEIGHTS:
        assert o.num_weights == N_WEIGHTS[arch]


def test_sparse_table_changes_weight_count():
    import numpy as np
    o = oracle.Oracle("4x44x44-40C5S1-MP2-80C3-MP2-100N-5N")
    full = o.num_weights
    t = np.zeros((80, 40), dtype=np.uint8)
    t[:, :20] = 1
    o.set_connection_table(1, t)
    assert full - o.num_weights == 80 * 20 * 9
    # 40*4*25+40 + 80*20*9+80 + 1280*100+100 + 100*5+5
    assert o.num_weights == 147125


def test_floor_when_stride_does_not_divide():
    # (44 - 5) / 2 + 1 = 20.5: the kernel must lie fully inside the image (Sec. 2.2) -> 20
    assert oracle.conv_out_size(44, 5, 1) == 20
    assert oracle.conv_out_size(4, 5, 0) <= 0


def test_sizes_with_different_x_and_y_values():
    # Eq. 1 axis by axis (Sec. 2.2), pooling by Ky and Kx (Sec. 2.3): rows first, then columns
    o = oracle.Oracle("2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N")
    i = o.layer_info(1)
    assert (i["h"], i["w"], i["K"], i["Kx"], i["S"], i["Sx"]) == ((14 - 4) // 2 + 1, (11 - 2) // 1 + 1, 4, 2, 1, 0)
    i = o.layer_info(2)
    assert (i["kind"], i["h"], i["w"], i["K"], i["Kx"]) == (KIND_POOL, 3, 2, 2, 5)
    i = o.layer_info(3)
    assert (i["h"], i["w"], i["K"], i["Kx"]) == (3, 1, 1, 2)
    assert o.num_weights == (3 + 3 * 2 * 8) + (4 + 4 * 3 * 2) + (5 + 5 * 12) + (3 + 3 * 5)
    # one number stands for both directions
    a, b = oracle.Oracle("1x12x12-2C3x3S1x1-MP1x1-3N"), oracle.Oracle("1x12x12-2C3S1-MP1-3N")
    assert [a.layer_info(l) for l in range(a.num_layers)] == [b.layer_info(l) for l in range(b.num_layers)]


def test_kinds():
    o = oracle.Oracle("1x29x29-20C4-MP2-40C5-MP3-150N-10N")
    kinds = [o.layer_info(l)["kind"] for l in range(1, o.num_layers)]
    assert kinds == [KIND_CONV, KIND_POOL, KIND_CONV, KIND_POOL, KIND_FC, KIND_FC]


@pytest.mark.parametrize("arch,code", [
    ("", E_SYNTAX), ("1x29", E_SYNTAX), ("1x29x29", E_SYNTAX), ("1x29x29-20C4", E_SYNTAX),
    ("1x29x29-20C4-MP2", E_SYNTAX), ("1x29x29-20Q4-10N", E_SYNTAX), ("1x29x29-MP2-10N", E_SYNTAX),
    ("1x29x29-10N-20C4-10N", E_SYNTAX), ("1x29x29-20C4-MP2-MP2-10N", E_SYNTAX),
    ("1x29x29-20C4-MP4-10N", E_SHAPE),      # 26 is not a multiple of 4 (Sec. 2.3)
    ("1x4x4-20C5-10N", E_SHAPE),            # kernel larger than the image (Sec. 2.2)
    ("0x4x4-10N", E_SHAPE), ("1x29x29-0C4-10N", E_SHAPE), ("1x29x29-20C4-MP0-10N", E_SHAPE),
    ("1x29x29--10N", E_SYNTAX), ("1x29x29-20C4S-10N", E_SYNTAX), ("1x29x29-20C4-10N-", E_SYNTAX),
    ("1x29x29-20C4x-10N", E_SYNTAX), ("1x29x29-20C4x0-10N", E_SHAPE), ("1x29x29-20C4-MP2x-10N", E_SYNTAX),
    ("1x29x29-20C4-MP2x3-10N", E_SHAPE),    # 26 columns are not a multiple of 3
    ("1x29x29-20C4x30-10N", E_SHAPE),       # kernel wider than the image
])
def test_rejected_architectures(arch, code):
    with pytest.raises(OracleError) as e:
        oracle.Oracle(arch)
    assert e.value.code == code
