"""Pins of the deformation oracle (oracle/deform_oracle.py) against things other than itself: the published
SplitMix64 outputs, library routines (scipy.ndimage), closed forms and invariants.  No GPU."""
import math

import numpy as np
import pytest
import scipy.ndimage as ndi

from oracle import deform_oracle as D


def P(**kw):
    return D.DeformParams(**kw)


# ---- generator ---------------------------------------------------------------------------------------

def test_mix64_reproduces_the_published_splitmix64_stream():
    # first three outputs of SplitMix64 seeded with 0 (reference implementation of Steele, Lea, Flood 2014,
    # as distributed with the xoshiro generators): state += GOLDEN, output mix64(state)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state, got = 0, []
    for _ in range(3):
        state = (state + D.GOLDEN) & ((1 << 64) - 1)
        got.append(D.mix64(state))
    assert got == want
    # a draw is that stream's element k + 1 when the key is the seed
    assert D.draw(0, 1) == (want[1] >> 32, want[1] & 0xFFFFFFFF)


def test_unit_is_a_24_bit_fraction_exact_in_float32():
    for b in (0, 1, 255, 256, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 0x12345678):
        u = D.unit(b)
        assert 0.0 <= u < 1.0 and u * (1 << 24) == b >> 8
        assert float(np.float32(u)) == u and float(np.float32(D.sym(b))) == D.sym(b)
    assert D.unit(0xFFFFFFFF) == 1.0 - 2.0 ** -24 and D.sym(0) == -1.0


def test_draws_look_uniform_and_unrelated():
    key = D.image_key(7, 3)
    v = np.array([[D.sym(h), D.sym(l)] for h, l in (D.draw(key, k) for k in range(20000))])
    assert abs(v.mean()) < 0.01 and abs(v.var() - 1.0 / 3.0) < 0.01
    assert abs(np.corrcoef(v[:, 0], v[:, 1])[0, 1]) < 0.03           # the two halves of a draw
    assert abs(np.corrcoef(v[:-1, 0], v[1:, 0])[0, 1]) < 0.03        # consecutive draws
    other = np.array([D.sym(D.draw(D.image_key(7, 4), k)[0]) for k in range(20000)])
    assert abs(np.corrcoef(v[:, 0], other)[0, 1]) < 0.03             # consecutive images
    other = np.array([D.sym(D.draw(D.image_key(8, 3), k)[0]) for k in range(20000)])
    assert abs(np.corrcoef(v[:, 0], other)[0, 1]) < 0.03             # consecutive seeds


# ---- the affine part ---------------------------------------------------------------------------------

def test_each_range_governs_its_own_parameter():
    H, W = 20, 30
    neutral = dict(tx=0.0, ty=0.0, theta=0.0, shear=0.0, sx=1.0, sy=1.0)
    cases = {"max_translation": ("tx", "ty"), "max_rotation": ("theta",), "max_shear": ("shear",), "max_scaling": ("sx", "sy")}
    for field, moved in cases.items():
        seen = {m: [] for m in moved}
        for t in range(200):
            q = D.image_parameters(5, t, P(**{field: 0.1}), H, W)
            for name, val in q.items():
                if name in moved:
                    seen[name].append(val - neutral[name])
                else:
                    assert val == neutral[name]
        bound = {"tx": 0.1 * W, "ty": 0.1 * H, "theta": math.radians(0.1), "shear": 0.1, "sx": 0.1, "sy": 0.1}
        for name, vals in seen.items():
            vals = np.array(vals)
            assert np.all(np.abs(vals) <= bound[name])
            assert vals.min() < -0.7 * bound[name] and vals.max() > 0.7 * bound[name]  # both signs, most of the range
        if len(moved) == 2:
            assert abs(np.corrcoef(seen[moved[0]], seen[moved[1]])[0, 1]) < 0.25  # drawn independently


def test_affine_matrix_closed_forms():
    np.testing.assert_allclose(D.affine_matrix(0.0, 0.0, 1.0, 1.0), np.eye(2), atol=0)
    np.testing.assert_allclose(D.affine_matrix(math.pi / 2, 0.0, 1.0, 1.0), [[0, -1], [1, 0]], atol=1e-15)
    np.testing.assert_allclose(D.affine_matrix(0.0, 0.5, 1.0, 1.0), [[1, 0.5], [0, 1]], atol=0)
    np.testing.assert_allclose(D.affine_matrix(0.0, 0.0, 2.0, 3.0), [[2, 0], [0, 3]], atol=0)
    # rotation . shear . scaling, worked by hand: [[0,-1],[1,0]] [[1,.5],[0,1]] = [[0,-1],[1,.5]]; times diag(2,3)
    np.testing.assert_allclose(D.affine_matrix(math.pi / 2, 0.5, 2.0, 3.0), [[0, -3], [2, 1.5]], atol=1e-15)
    A = D.affine_matrix(0.3, 0.0, 1.0, 1.0)
    np.testing.assert_allclose(A @ A.T, np.eye(2), atol=1e-15)
    assert abs(np.linalg.det(D.affine_matrix(0.3, 0.7, 1.2, 0.9)) - 1.2 * 0.9) < 1e-15


def test_source_coordinates_translation_and_quarter_turn():
    H, W = 5, 7
    rng = np.random.default_rng(1)
    src = rng.uniform(-1, 1, (2, H, W))
    Z = np.zeros((H, W))
    ys, xs = D.source_coordinates(H, W, np.eye(2), 2.0, -1.0, Z, Z)
    out = D.bilinear(src, ys, xs, 9.0)
    for y in range(H):
        for x in range(W):
            inside = 0 <= y - 1 < H and 0 <= x + 2 < W
            np.testing.assert_array_equal(out[:, y, x], src[:, y - 1, x + 2] if inside else [9.0, 9.0])
    # a quarter turn about the centre of an odd square: source of (y, x) is (cy + (x - cx), cx - (y - cy))
    n = 5
    sq = rng.uniform(-1, 1, (1, n, n))
    Zs = np.zeros((n, n))
    ys, xs = D.source_coordinates(n, n, D.affine_matrix(math.pi / 2, 0, 1, 1), 0.0, 0.0, Zs, Zs)
    out = D.bilinear(sq, ys, xs, 0.0)
    for y in range(n):
        for x in range(n):
            assert abs(out[0, y, x] - sq[0, x, n - 1 - y]) < 1e-14
    # the elastic displacement is added as it is
    Dx, Dy = rng.uniform(-1, 1, (H, W)), rng.uniform(-1, 1, (H, W))
    ys2, xs2 = D.source_coordinates(H, W, np.eye(2), 0.0, 0.0, Dx, Dy)
    yy, xx = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    np.testing.assert_allclose(xs2 - xx, Dx, atol=1e-15)
    np.testing.assert_allclose(ys2 - yy, Dy, atol=1e-15)


# ---- interpolation and smoothing against library routines ----------------------------------------------

@pytest.mark.parametrize("fill", [0.0, -1.0, 2.5])
def test_bilinear_equals_scipy_map_coordinates(fill):
    rng = np.random.default_rng(3)
    src = rng.uniform(-1, 1, (3, 9, 11))
    ys = rng.uniform(-3, 12, (40, 50))
    xs = rng.uniform(-3, 14, (40, 50))
    got = D.bilinear(src, ys, xs, fill)
    for c in range(3):
        want = ndi.map_coordinates(src[c], [ys, xs], order=1, mode="grid-constant", cval=fill)
        np.testing.assert_allclose(got[c], want, atol=1e-13)


@pytest.mark.parametrize("sigma", [0.8, 2.0, 5.5])
def test_smooth_equals_scipy_gaussian_filter(sigma):
    rng = np.random.default_rng(4)
    f = rng.uniform(-1, 1, (17, 23))
    R = int(math.ceil(3 * sigma))
    want = ndi.gaussian_filter(f, sigma, mode="constant", cval=0.0, radius=R)
    np.testing.assert_allclose(D.smooth(f, sigma), want, atol=1e-14)


def test_gaussian_taps_and_impulse_response():
    for sigma in (0.5, 1.0, 4.0, 6.0):
        g = D.gaussian_taps(sigma)
        R = int(math.ceil(3 * sigma))
        assert len(g) == 2 * R + 1 and abs(g.sum() - 1.0) < 1e-15
        np.testing.assert_allclose(g, g[::-1], atol=0)
        assert abs(g[R + 1] / g[R] - math.exp(-1.0 / (2 * sigma * sigma))) < 1e-14
    g = D.gaussian_taps(1.0)
    f = np.zeros((11, 13))
    f[5, 6] = 1.0
    s = D.smooth(f, 1.0)
    np.testing.assert_allclose(s[2:9, 3:10], np.outer(g, g), atol=1e-16)
    assert abs(s.sum() - 1.0) < 1e-14


# ---- the whole deformation ---------------------------------------------------------------------------

def ramp(C, H, W, a, b, c):
    y, x = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    return np.stack([a * x + b * y + c + k for k in range(C)])


def test_no_deformation_is_the_identity():
    rng = np.random.default_rng(5)
    src = rng.uniform(-1, 1, (2, 12, 9))
    out, disp = D.deform_image(src, 1, 0, P(fill=7.0))
    np.testing.assert_array_equal(out, src)
    np.testing.assert_array_equal(disp, np.zeros((2, 12, 9)))
    out, disp = D.deform_image(src, 1, 0, P(sigma=3.0, alpha=0.0, fill=7.0))
    np.testing.assert_array_equal(out, src)


def test_constant_image_stays_constant():
    src = np.full((3, 16, 16), 0.25)
    out, _ = D.deform_image(src, 9, 4, P(max_translation=0.1, max_rotation=20, max_scaling=0.2, max_shear=0.2,
                                         sigma=2.0, alpha=6.0, fill=0.25))
    np.testing.assert_allclose(out, src, atol=1e-15)


def test_image_and_displacement_agree_on_a_ramp():
    # bilinear interpolation reproduces a linear function exactly, so wherever all four neighbours are inside
    # the output is the ramp at the source point: out - src = a dx + b dy
    C, H, W, a, b = 2, 21, 25, 0.03, -0.02
    src = ramp(C, H, W, a, b, 0.1)
    prm = P(max_translation=0.05, max_rotation=10, max_scaling=0.1, max_shear=0.1, sigma=2.0, alpha=3.0, fill=1e9)
    for t in range(5):
        out, disp = D.deform_image(src, 11, t, prm)
        ok = out[0] < 1e6
        assert ok.sum() > 0.5 * H * W
        for c in range(C):
            np.testing.assert_allclose((out[c] - src[c])[ok], (a * disp[0] + b * disp[1])[ok], atol=1e-12)


def centred(H, W):
    y, x = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    return x - (W - 1) / 2.0, y - (H - 1) / 2.0


def test_each_ingredient_moves_pixels_the_way_its_name_says():
    H, W = 15, 19
    src = np.zeros((1, H, W))
    u, v = centred(H, W)
    for t in range(6):
        q = D.image_parameters(2, t, P(max_translation=0.05, max_rotation=15, max_scaling=0.15, max_shear=0.2), H, W)
        _, d = D.deform_image(src, 2, t, P(max_translation=0.05))
        assert np.ptp(d[0]) < 1e-12 and np.ptp(d[1]) < 1e-12
        assert abs(d[0, 0, 0]) <= 0.05 * W and abs(d[1, 0, 0]) <= 0.05 * H
        np.testing.assert_allclose([d[0, 0, 0], d[1, 0, 0]], [q["tx"], q["ty"]], atol=1e-12)
        _, d = D.deform_image(src, 2, t, P(max_shear=0.2))
        np.testing.assert_allclose(d[0], q["shear"] * v, atol=1e-12)   # horizontal: x moves in proportion to y
        np.testing.assert_allclose(d[1], 0.0, atol=1e-12)
        _, d = D.deform_image(src, 2, t, P(max_scaling=0.15))
        np.testing.assert_allclose(d[0], (q["sx"] - 1) * u, atol=1e-12)
        np.testing.assert_allclose(d[1], (q["sy"] - 1) * v, atol=1e-12)
        _, d = D.deform_image(src, 2, t, P(max_rotation=15))
        np.testing.assert_allclose(np.hypot(u + d[0], v + d[1]), np.hypot(u, v), atol=1e-12)  # radii kept
        ang = np.arctan2(v + d[1], u + d[0]) - np.arctan2(v, u)
        far = np.hypot(u, v) > 1
        np.testing.assert_allclose(np.mod(ang[far] - q["theta"] + math.pi, 2 * math.pi) - math.pi, 0.0, atol=1e-12)
        assert abs(q["theta"]) <= math.radians(15)


def test_elastic_field_has_the_predicted_spread_and_ignores_the_affine_ranges():
    H = W = 21
    sigma, alpha = 1.5, 4.0
    src = np.zeros((1, H, W))
    g = D.gaussian_taps(sigma)
    want_var = alpha * alpha * (1.0 / 3.0) * float(np.sum(np.outer(g, g) ** 2))
    centre = np.array([D.deform_image(src, 3, t, P(sigma=sigma, alpha=alpha))[1][:, H // 2, W // 2] for t in range(400)])
    assert abs(centre.mean()) < 0.15 * math.sqrt(want_var)
    assert abs(centre[:, 0].var() / want_var - 1.0) < 0.2 and abs(centre[:, 1].var() / want_var - 1.0) < 0.2
    assert abs(np.corrcoef(centre[:, 0], centre[:, 1])[0, 1]) < 0.15
    # the elastic part is the same whatever the affine ranges are
    _, only = D.deform_image(src, 3, 7, P(sigma=sigma, alpha=alpha))
    _, shift = D.deform_image(src, 3, 7, P(sigma=sigma, alpha=alpha, max_translation=0.05))
    q = D.image_parameters(3, 7, P(max_translation=0.05), H, W)
    np.testing.assert_allclose(shift[0] - only[0], q["tx"], atol=1e-12)
    np.testing.assert_allclose(shift[1] - only[1], q["ty"], atol=1e-12)
    # neighbours move together (smooth), far pixels do not
    field = np.array([D.deform_image(src, 3, t, P(sigma=sigma, alpha=alpha))[1][0] for t in range(200)])
    assert np.corrcoef(field[:, 10, 10], field[:, 10, 11])[0, 1] > 0.7
    assert abs(np.corrcoef(field[:, 10, 3], field[:, 10, 17])[0, 1]) < 0.25


def test_batches_are_presentations_in_order():
    rng = np.random.default_rng(6)
    src = rng.uniform(-1, 1, (4, 1, 8, 8))
    prm = P(max_translation=0.05, max_rotation=10, sigma=1.0, alpha=1.0, fill=-1.0)
    out, disp = D.deform_images(src, 21, 100, prm)
    for k in range(4):
        o, d = D.deform_image(src[k], 21, 100 + k, prm)
        np.testing.assert_array_equal(out[k], o)
        np.testing.assert_array_equal(disp[k], d)
    out2, _ = D.deform_images(src, 21, 100, prm, src_index=[3, 3, 0])
    np.testing.assert_array_equal(out2[1], D.deform_image(src[3], 21, 101, prm)[0])
    np.testing.assert_array_equal(out2[2], D.deform_image(src[0], 21, 102, prm)[0])
    assert not np.array_equal(out2[0], out2[1])  # the same source presented twice is deformed anew
