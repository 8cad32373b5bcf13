"""Host logic of the resident mode (no GPU): the plan the library derives for an architecture -- team, per-rank
LDS layout, tiles, shared delta pulls -- is checked against rules restated here from what the kernels need:
regions disjoint and inside the LDS, room for the partial sums of every job however its connections are split
over the lanes, room for the zero-bordered delta maps of a pull chunk, shares of a pulled map's entries that tile
the list and fit the pull copy.  Runs on the benchmark networks, on the edge-case shapes and on seeded random ones."""
import numpy as np
import pytest

from paper_1102_0183_amd import binding, synth

CU = 256  # compute units the planner assumes when no device is there


def ceil_div(a, b):
    return -(-a // b)


def split_ways(U, cnt, wg):
    """Ways U units share their (at most cnt) connections over wg lanes: as many as fit, then the fewest that
    need no more passes per lane."""
    if U >= wg or U < 1:
        return 1
    r_max = max(1, min(wg // U, cnt))
    iters = ceil_div(cnt, r_max)
    return ceil_div(cnt, iters)


def job_units(strip, rows, nm, H, W):
    return nm * ceil_div(H, rows) * ceil_div(W, strip) if strip else nm * H * W


def check_plan(p, arch, n_ranks=0, stride=0):
    num, regions = p["numbers"], p["regions"]
    wg, G = num["workgroup"], num["G"]
    # the team
    max_maps = max(c["Mo"] for c in p["conv"])
    want_stride = stride or (8 if (n_ranks or max_maps) <= CU // 8 else 1)
    assert num["stride"] == want_stride
    assert G == max(1, min(n_ranks or max_maps, max_maps, CU // want_stride)), arch
    assert num["n_col_ranks"] == min(G, p["conv"][-1]["Mo"])
    # the partial sums of the first fully connected layer: read by every rank while they are few, else each sum is
    # added up by one rank and sent round
    assert num["fc1_owned"] == (1 if num["n_col_ranks"] * p["fc"][0]["n_out"] > 16384 else 0)
    # regions: disjoint, aligned, inside the LDS
    assert num["lds_floats"] <= num["lds_floats_max"]
    spans = sorted((off, off + n, name) for name, off, n in regions)
    for (a0, a1, an), (b0, b1, bn) in zip(spans, spans[1:]):
        assert a1 <= b0, (arch, an, bn)
    for off, end, name in spans:
        assert off % 4 == 0 and off >= 0 and end <= num["lds_floats"], (arch, name)
    size = {name: n for name, _, n in regions}
    stream = num["stream"]
    if stream:
        # the streamed plan: inputs of the layers above the first, the pull's delta maps and every job's partial
        # sums take turns in one arena
        assert "part" not in size and not any(("conv%d.in" % l) in size for l in range(1, len(p["conv"])))
        size["part"] = size["scratch"]
    # layers
    for l, c in enumerate(p["conv"]):
        KK = c["K"] * c["K"]
        assert c["n_own"] == ceil_div(c["Mo"], G)
        assert c["n_own_below"] == (ceil_div(c["Mi"], G) if l else 0)
        # FP: partial sums of the job, for a rank with the most maps and one with a map fewer
        for nm in {c["n_own"], max(1, c["n_own"] - 1)}:
            U = job_units(c["fwd_strip"], c["fwd_rows"], nm, c["Ho"], c["Wo"])
            R = min(split_ways(U, min(c["max_conn"], c["in_chunk"]), wg), split_ways(U, c["max_conn"], wg))
            assert R * nm * c["Ho"] * c["Wo"] <= size["part"], (arch, l, "fwd")
        assert c["n_own"] * c["Ho"] * c["Wo"] <= size["act"]
        if c["fwd_strip"]:
            assert c["fwd_strip"] in (4, 5, 7) and c["fwd_rows"] in (1, 2) and 2 <= c["K"] <= 5 and c["S"] <= 1
        if l == 0:
            assert c["pull_shares"] == 1
            continue
        # a pooled layer's pull visits the pooling winners only
        HW = c["Hp"] * c["Wp"]
        winners = c["Kp"] >= 2
        # shared pulls
        macs = c["max_back"] * KK * c["Hi"] * c["Wi"]
        shared = 2 * c["Mi"] <= G and macs >= num["share_min_macs"] and not stream and not winners
        H = G // c["Mi"] if shared else 1
        assert c["pull_shares"] == H, (arch, l)
        assert c["back_pitch"] == ceil_div(c["max_back"], H)
        if H > 1:
            assert c["n_own_below"] == 1 and H * c["Mi"] <= G
            for ne in range(c["max_back"] + 1):  # every list length: the shares tile it and fit the pull copy
                cuts = [ne * h // H for h in range(H + 1)]
                assert cuts[0] == 0 and cuts[-1] == ne
                assert all(0 <= b - a <= c["back_pitch"] for a, b in zip(cuts, cuts[1:]))
        pad = 16 + c["Wi"] + c["K"]
        if winners:
            # a connection's winners go to the lanes of one wavefront, at most 64 at a time; as many connections
            # at once as wavefronts have room for, as there are, and as copies of the own input maps fit the arena
            parts = ceil_div(HW, 64)
            lanes = ceil_div(HW, parts)
            assert lanes <= 64
            most = (wg // 64) * (64 // lanes)
            units = c["n_own_below"] * c["back_pitch"] * parts
            copy = c["n_own_below"] * c["Hi"] * c["Wi"]
            assert c["pull_slots"] == min(most, units, size["scratch"] // copy) >= 1, (arch, l)
            assert c["pull_slots"] * copy <= size["scratch"]
        else:
            # the pull: a chunk of zero-bordered delta maps in the scratch area, partial sums of the job
            assert c["pull_slots"] == 0
            border = ((c["Hi"] + c["K"] - 1) * (c["Wi"] + c["K"] - 1)) | 1
            assert 1 <= c["pull_chunk"] <= c["Mo"]
            assert c["pull_chunk"] * border + pad <= size["scratch"], (arch, l)
            max_cnt, plan_cnt = min(c["back_pitch"], c["pull_chunk"]), min(c["back_pitch"], c["Mo"])
            for nm in {c["n_own_below"], max(1, c["n_own_below"] - 1)}:
                U = job_units(c["pull_strip"], c["pull_rows"], nm, c["Hi"], c["Wi"])
                R = min(split_ways(U, max_cnt, wg), split_ways(U, plan_cnt, wg))
                assert R * nm * c["Hi"] * c["Wi"] <= size["part"], (arch, l, "pull")
        assert c["Mo"] * c["Hp"] * c["Wp"] <= size["dall"] == size["yxall"]
        if stream:
            # a chunk of input maps fits the arena, the chunks tile the maps, and the pull walks its maps once
            assert 1 <= c["in_chunk"] <= c["Mi"] and c["in_chunk"] * c["Hi"] * c["Wi"] + pad <= size["scratch"], (arch, l)
            assert winners or job_units(c["pull_strip"], c["pull_rows"], c["n_own_below"], c["Hi"], c["Wi"]) <= wg
        else:
            assert c["in_chunk"] == c["Mi"] and size["conv%d.in" % l] == c["Mi"] * c["Hi"] * c["Wi"]
        # sums over the pooled positions of a weight gradient: split 2^R ways while the weights of either copy fit
        n_w = min(c["n_own"] * c["max_conn"] * KK, c["n_own_below"] * c["back_pitch"] * KK)
        r = c["wgrad_R_log2"]
        assert 0 <= r <= 6 and (r == 0 or ((n_w << r) <= wg and (1 << r) <= c["Hp"] * c["Wp"]))
    # the first fully connected layer is held by columns: those of the own maps of the last conv layer
    last = p["conv"][-1]
    assert p["fc"][0]["n_in"] == last["Mo"] * last["Hp"] * last["Wp"]
    assert size["fc0.w"] == last["n_own"] * last["Hp"] * last["Wp"] * p["fc"][0]["n_out"]
    assert size["part"] >= wg
    # the layers behind it are held whole by every rank, except a hidden second layer of more than 8192 weights:
    # that one by columns rank, rank + G, ... of its matrix
    for f, q in enumerate(p["fc"][1:], 1):
        large = f == 1 and f < len(p["fc"]) - 1 and q["n_in"] * q["n_out"] > 8192
        assert q["by_cols"] == (1 if large else 0), (arch, f)
        if large:
            assert q["n_own"] == ceil_div(q["n_in"], G) and size["fc%d.w" % f] == q["n_own"] * q["n_out"]
        else:
            assert size["fc%d.w" % f] == q["n_in"] * q["n_out"]


@pytest.mark.parametrize("name,static_id", [("cfg1", 1), ("cfg2a", 1), ("cfg2b", 2)])
def test_benchmark_networks_take_the_kernels_compiled_for_them(name, static_id):
    arch = synth.WORKLOADS[name].arch
    p = binding.resident_plan(arch)
    check_plan(p, arch)
    assert p["numbers"]["static_id"] == static_id
    # (the pull through the second layer visits the pooling winners only, which is too little work to share)
    assert p["conv"][1]["pull_shares"] == 1 and p["conv"][1]["pull_slots"] == p["conv"][1]["Mo"]
    for team in ((32, 1), (32, 8), (20, 8)):
        q = binding.resident_plan(arch, 0, *team)
        check_plan(q, arch, *team)
        # (the large net on 20 ranks: four maps a rank, more than its LDS holds next to all inputs: streamed)
        assert q["numbers"]["stream"] == (1 if (name == "cfg2b" and team[0] == 20) else 0)
        assert q["numbers"]["static_id"] == 0 and q["numbers"]["G"] == team[0]


def test_cfg5_with_a_regular_half_table():
    arch = synth.WORKLOADS["cfg5"].arch
    p = binding.resident_plan(arch, fan_in=20)
    check_plan(p, arch)
    assert p["conv"][1]["full_table"] == 0 and p["conv"][1]["max_conn"] == 20 and p["conv"][1]["max_back"] == 40


@pytest.mark.parametrize("name,static_id", [("cfg3", 4), ("cfg4a", 5)])
def test_wide_networks_stream_their_inputs(name, static_id):
    """A rank's share of these nets does not fit next to all input maps of every layer: the plan keeps the
    weights resident and walks the inputs in chunks."""
    arch = synth.WORKLOADS[name].arch
    p = binding.resident_plan(arch)
    check_plan(p, arch)
    assert p["numbers"]["stream"] == 1 and p["numbers"]["static_id"] == static_id
    q = binding.resident_plan(arch, 0, 90, 1)      # another team: the kernel that reads its plan
    assert "unsupported" in q or q["numbers"]["static_id"] == 0
    assert all(c["pull_shares"] == 1 for c in p["conv"])
    assert any(c["in_chunk"] < c["Mi"] for c in p["conv"][1:])


def test_the_widest_network_is_refused():
    """Two maps of 300C4 and their pull copies alone are 19200 weights a rank, next to those of the other layers."""
    p = binding.resident_plan(synth.WORKLOADS["cfg4b"].arch)
    assert "LDS" in p["unsupported"]


def test_other_refusals():
    assert "equal x and y" in binding.resident_plan("1x10x12-2C3x5-MP4x2-4N")["unsupported"]
    assert "at least one convolutional" in binding.resident_plan("1x5x5-7N-4N")["unsupported"]
    assert "at most" in binding.resident_plan("1x40x40-2C2-2C2-2C2-2C2-2C2-2C2-2C2-3N")["unsupported"]
    check_plan(binding.resident_plan("1x16x16-2C2-2C2-2C2-2C2-2C2-2C2-3N"), "1x16x16-2C2-2C2-2C2-2C2-2C2-2C2-3N")   # six layers
    with pytest.raises(binding.CnnError):
        binding.resident_plan("1x5x5-3C9-2N")


@pytest.mark.parametrize("arch,fan", [
    ("1x9x9-3C4-MP2-4C2-5N-3N", 0), ("2x11x11-3C3S1-4C2-MP2-4N", 2), ("3x8x8-4C3-MP3-4C2-6N-5N-4N", 3),
    ("1x6x6-2C3-3N", 0), ("2x10x10-5C1-MP2-3C1S1-6N-2N", 0), ("1x20x20-6C6-MP3-5C3S2-4N", 0),
    ("1x8x600-3C3-MP2-4C2S1-5N", 0), ("1x70x70-4C3-MP4-3C4-MP2-6N", 0), ("3x34x47-7C4S1-8C3-MP2-9C2-MP3-20N-6N", 4),
    ("1x40x40-70C5-MP4-300C3-MP1-10N", 0), ("1x28x28-6C5-MP2-100C5-MP2-8N", 0), ("1x28x28-6C5-MP2-100C5-MP2-8N", 5),
    ("1x28x28-40C5-MP2-80C5-MP2-8N", 38), ("1x28x28-3C5-MP2-250C5-MP2-8N", 0),
    ("1x28x28-6C5-MP2-100C9-MP1-8N", 0), ("1x28x28-6C5-MP2-100C9-MP1-8N", 5), ("1x28x28-40C5-MP2-80C9-MP1-8N", 12),
    ("1x47x47-6C4-MP2-100C5-MP3-8N", 0), ("1x65x65-8C4-MP2-20C5-MP3-6N", 3), ("2x60x60-3C5-MP4-7C4S1-MP3-4C1-MP1-5N", 2),
    # Sec. 4.1's deepest net (Table 1): six convolutional layers, half of the connections above the first
    ("1x29x29-20C4-MP2-40C2-60C3-80C3-MP2-100C2-120C3-150N-10N", 0),
])
def test_edge_shapes(arch, fan):
    p = binding.resident_plan(arch, fan_in=fan)
    if "unsupported" in p:
        pytest.skip(p["unsupported"])
    check_plan(p, arch)
    for team in ((7, 1), (3, 8)):
        q = binding.resident_plan(arch, fan, *team)
        if "unsupported" not in q:
            check_plan(q, arch, *team)


def random_arch(rng, deep=False):
    """1 to 4 convolutional layers of up to 120 maps with square kernels, skips and pooling, then 1 to 3 FC layers.
    deep: up to 6 layers with kernels of at most 3 and less pooling, up to 3 hidden FC layers of up to 300 units."""
    h = w = int(rng.integers(8, 49))
    if rng.random() < 0.3:
        w = int(rng.integers(8, 49))
    s = "%dx%dx%d" % (int(rng.integers(1, 4)), h, w)
    n_conv = 0
    for _ in range(int(rng.integers(3, 7)) if deep else int(rng.integers(1, 5))):
        k = int(rng.integers(1, min(3 if deep else 7, h, w) + 1))
        sk = int(rng.integers(0, 3)) if rng.random() < 0.3 else 0
        ho, wo = (h - k) // (sk + 1) + 1, (w - k) // (sk + 1) + 1
        m = int(rng.choice([2, 5, 12, 20, 40, 64, 100, 120]))
        s += "-%dC%d%s" % (m, k, "S%d" % sk if sk else "")
        n_conv += 1
        h, w = ho, wo
        both = [d for d in range(1, 5) if h % d == 0 and w % d == 0]
        if rng.random() < (0.35 if deep else 0.7):
            d = int(rng.choice(both))
            s += "-MP%d" % d
            h, w = h // d, w // d
        if min(h, w) < 2:
            break
    for _ in range(int(rng.integers(1, 4)) if deep else int(rng.integers(0, 3))):
        s += "-%dN" % int(rng.integers(2, 300 if deep else 200))
    return s + "-%dN" % int(rng.integers(2, 12))


def test_random_architectures():
    rng = np.random.default_rng(5)
    planned = shared = winners = 0
    for _ in range(400):
        arch = random_arch(rng)
        fan = int(rng.integers(1, 40)) if rng.random() < 0.4 else 0
        team = (0, 0) if rng.random() < 0.6 else (int(rng.integers(1, 130)), int(rng.choice([0, 1, 8])))
        p = binding.resident_plan(arch, fan, *team)
        if "unsupported" in p:
            continue
        check_plan(p, arch, *team)
        planned += 1
        shared += any(c["pull_shares"] > 1 for c in p["conv"])
        winners += any(c["pull_slots"] > 0 for c in p["conv"])
    assert planned >= 100 and shared >= 5 and winners >= 20, (planned, shared, winners)


def test_random_deep_architectures():
    rng = np.random.default_rng(6)
    planned = cols = owned = deep = 0
    for _ in range(300):
        arch = random_arch(rng, deep=True)
        fan = int(rng.integers(1, 40)) if rng.random() < 0.4 else 0
        team = (0, 0) if rng.random() < 0.6 else (int(rng.integers(1, 130)), int(rng.choice([0, 1, 8])))
        p = binding.resident_plan(arch, fan, *team)
        if "unsupported" in p:
            continue
        check_plan(p, arch, *team)
        planned += 1
        cols += any(q["by_cols"] for q in p["fc"])
        owned += p["numbers"]["fc1_owned"]
        deep += p["numbers"]["n_conv"] >= 5
    assert planned >= 80 and cols >= 10 and owned >= 5 and deep >= 20, (planned, cols, owned, deep)


@pytest.mark.parametrize("arch,G", [("3x32x32-100C3-MP3-100C3-MP2-100C3-MP2-300N-100N-10N", 100),
                                    ("3x32x32-200C3-MP3-200C3-MP2-200C3-MP2-300N-100N-10N", 200),
                                    ("1x20x20-6C5-MP2-12C4-MP1-120N-90N-7N", 12)])
def test_a_large_hidden_layer_behind_the_first_is_held_by_columns(arch, G):
    """Section 3's CIFAR nets end in 300N-100N-10N: the 30000 weights between the hidden layers do not fit every
    rank's LDS next to its maps, a rank's columns of them do."""
    p = binding.resident_plan(arch)
    check_plan(p, arch)
    assert p["numbers"]["G"] == G and p["fc"][1]["by_cols"] == 1 and p["fc"][2]["by_cols"] == 0
