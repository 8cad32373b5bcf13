"""On-line deformation of training images (cnn_deform_images) against the CPU oracle, through the C ABI.
Needs a GPU (marked gpu).  Bar: the random draws are integers and must agree exactly, which shows in the
displacements; displacements and images within 1e-5 of the oracle's largest value (fp32 against float64: a
source position is off by about 1e-6 pixel -- its affine part is worked out in double, the elastic part and the
interpolation in fp32 -- and neighbouring pixels differ by at most 2)."""
import numpy as np
import pytest

from oracle import deform_oracle as DO
from paper_1102_0183_amd import binding, synth

pytestmark = pytest.mark.gpu

SEED = synth.DEFORM_SEED
TOL = 1e-5

ALL = dict(synth.DEFORM_RECIPE)
CASES = [
    # C, H, W, images, parameters
    (1, 29, 29, 40, ALL),                                                        # the benchmark stream's shape
    (2, 48, 48, 6, dict(ALL, sigma=8.0, alpha=60.0, fill=0.0)),                  # a stereo pair shares one deformation
    (3, 32, 32, 10, dict(max_translation=0.05, fill=0.0)),                       # translation alone (Sec. 4.2, 4.3)
    (3, 7, 5, 20, dict(ALL, sigma=1.0, alpha=2.0)),                              # ragged, smaller than a wavefront
    (1, 1, 1, 5, dict(ALL, sigma=0.5, alpha=1.0, fill=0.5)),                     # a single pixel
    (1, 96, 96, 2, dict(max_rotation=30.0, sigma=16.0, alpha=300.0, fill=2.0)),  # largest map, widest Gaussian
    (1, 20, 31, 12, dict(sigma=2.0, alpha=8.0, fill=0.0)),                       # elastic part alone
    (2, 16, 16, 12, dict(max_rotation=180.0, max_scaling=0.9, max_shear=1.0, max_translation=0.5, fill=3.0)),  # far outside
]


def params(**kw):
    return binding.DeformParams(**kw), DO.DeformParams(**kw)


def run(src, n, gp, seed, first, index=None, want_disp=True):
    import torch
    d_src = torch.from_numpy(src).to("cuda:0")
    d_dst = torch.full((n,) + src.shape[1:], 77.0, dtype=torch.float32, device="cuda:0")
    d_disp = torch.full((n, 2) + src.shape[2:], 77.0, dtype=torch.float32, device="cuda:0") if want_disp else None
    d_idx = None if index is None else torch.tensor(index, dtype=torch.int32, device="cuda:0")
    binding.deform_images(d_src, d_dst, n, gp, seed, first, d_idx, d_disp)
    torch.cuda.synchronize()
    return d_dst.cpu().numpy(), (d_disp.cpu().numpy() if want_disp else None)


def rel(got, want):
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


@pytest.mark.parametrize("C,H,W,n,kw", CASES)
def test_deformed_images_match_the_oracle(C, H, W, n, kw):
    print("case", C, H, W, "images", n, kw, flush=True)
    rng = np.random.default_rng(SEED + C * 1000 + H)
    src = rng.uniform(-1, 1, (n, C, H, W)).astype(np.float32)
    gp, op = params(**kw)
    got, disp = run(src, n, gp, SEED, 1000)
    want, want_disp = DO.deform_images(src, SEED, 1000, op)
    e_d = float(np.abs(disp - want_disp).max() / max(np.abs(want_disp).max(), 1.0))
    e_i = rel(got, want)
    print("  displacement err %.2e (largest %.2f pixels), image err %.2e" % (e_d, np.abs(want_disp).max(), e_i), flush=True)
    assert e_d <= TOL and e_i <= TOL


def test_no_ranges_is_a_bit_exact_copy_and_the_draws_do_not_depend_on_the_call():
    import torch
    rng = np.random.default_rng(SEED)
    src = rng.uniform(-1, 1, (50, 2, 13, 17)).astype(np.float32)
    gp, _ = params(fill=9.0)
    got, disp = run(src, 50, gp, SEED, 0)
    assert np.array_equal(got, src) and not disp.any()
    # presentations 20..29 alone are the same bits as inside a call over 0..49
    gp, _ = params(**ALL)
    whole, wd = run(src, 50, gp, SEED, 7)
    part, pd = run(src[20:30].copy(), 10, gp, SEED, 27)
    assert np.array_equal(part, whole[20:30]) and np.array_equal(pd, wd[20:30])
    again, _ = run(src, 50, gp, SEED, 7)
    assert np.array_equal(again, whole)
    other, _ = run(src, 50, gp, SEED + 1, 7)
    assert not np.array_equal(other, whole)
    # a bilinear sample is a convex combination of source pixels and the fill value
    assert whole.min() >= min(src.min(), -1.0) - 1e-6 and whole.max() <= max(src.max(), -1.0) + 1e-6
    torch.cuda.synchronize()


def test_index_list_presentation_numbers_beyond_32_bits_and_a_long_call():
    rng = np.random.default_rng(SEED + 1)
    src = rng.uniform(-1, 1, (6, 1, 8, 8)).astype(np.float32)
    kw = dict(ALL, sigma=1.0, alpha=2.0, fill=0.25)
    gp, op = params(**kw)
    # the same source presented twice is deformed anew; an entry that names no image gives the fill value
    idx = [5, 5, 0, 6, -1, 3]
    got, _ = run(src, 6, gp, SEED, 3, index=idx)
    want, _ = DO.deform_images(src, SEED, 3, op, src_index=[5, 5, 0, 0, 0, 3])
    for k in (0, 1, 2, 5):
        assert rel(got[k], want[k]) <= TOL
    assert np.all(got[3] == np.float32(0.25)) and np.all(got[4] == np.float32(0.25))
    assert not np.array_equal(got[0], got[1])
    # presentation numbers are 64-bit and wrap like the oracle's
    first = (1 << 64) - 3
    got, disp = run(src, 6, gp, SEED, first)
    want = np.stack([DO.deform_image(src[k], SEED, (first + k) % (1 << 64), op)[0] for k in range(6)])
    assert rel(got, want) <= TOL
    # more images than workgroups in the launch: every workgroup takes several
    n = 20000
    big = rng.uniform(-1, 1, (n, 1, 8, 8)).astype(np.float32)
    got, disp = run(big, n, gp, SEED, 0)
    for k in (0, 1, 8191, 8192, 8193, 16384, n - 1):
        w, wd = DO.deform_image(big[k], SEED, k, op)
        assert rel(got[k], w) <= TOL and np.abs(disp[k] - wd).max() <= TOL * max(np.abs(wd).max(), 1.0)


def test_random_shapes_and_ranges_within_the_documented_limits():
    """40 seeded draws of map shape (up to 96 x 96), number of maps, every range (rotations up to 90 degrees,
    translations up to 30 % of the side, sigma up to 16) and seed: the bar must hold for all of them (the affine
    part of a source position is worked out in double for that: displacements reach tens of pixels here)."""
    rng = np.random.default_rng(SEED + 5)
    worst = 0.0
    for case in range(40):
        while True:
            H, W = int(rng.integers(1, 97)), int(rng.integers(1, 97))
            if H * (W | 1) <= 9312:
                break
        C, n = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        sigma = float(rng.choice([0.0, 0.3, 1.0, 2.5, 6.0, 11.0, 16.0]))
        if H * W > 3000:
            sigma = min(sigma, 6.0)   # (keeps the oracle's two-dimensional convolution short)
        kw = dict(max_translation=float(rng.uniform(0, 0.3)), max_rotation=float(rng.uniform(0, 90)),
                  max_scaling=float(rng.uniform(0, 0.5)), max_shear=float(rng.uniform(0, 0.5)), sigma=sigma,
                  alpha=float(rng.uniform(0, 40)), fill=float(rng.uniform(-2, 2)))
        print("case", case, C, H, W, n, kw, flush=True)
        src = rng.uniform(-1, 1, (n, C, H, W)).astype(np.float32)
        seed, first = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 40))
        gp, op = params(**kw)
        got, disp = run(src, n, gp, seed, first)
        want, want_disp = DO.deform_images(src, seed, first, op)
        e_i = rel(got, want)
        e_d = float(np.abs(disp - want_disp).max() / max(np.abs(want_disp).max(), 1.0))
        worst = max(worst, e_i, e_d)
        assert e_i <= TOL and e_d <= TOL, (case, e_i, e_d)
    print("  worst error %.2e" % worst, flush=True)


def test_bad_arguments_are_refused():
    import torch
    src = torch.zeros((4, 1, 8, 8), dtype=torch.float32, device="cuda:0")
    dst = torch.zeros((8, 1, 8, 8), dtype=torch.float32, device="cuda:0")
    ok = binding.DeformParams(sigma=1.0, alpha=1.0)
    binding.deform_images(src, dst, 0, None, 1, 0)  # nothing to do: not an error
    for bad, code in ((dict(sigma=17.0, alpha=1.0), binding.E_ARG), (dict(max_rotation=-1.0), binding.E_ARG),
                      (dict(max_scaling=1.0), binding.E_ARG), (dict(fill=float("nan")), binding.E_ARG),
                      (dict(alpha=float("inf"), sigma=1.0), binding.E_ARG)):
        with pytest.raises(binding.CnnError) as e:
            binding.deform_images(src, dst, 4, binding.DeformParams(**bad), 1, 0)
        assert e.value.code == code, bad
    with pytest.raises(binding.CnnError) as e:
        binding.deform_images(src, dst, 4, None, 1, 0)
    assert e.value.code == binding.E_ARG
    with pytest.raises(binding.CnnError) as e:   # more outputs than sources without an index list
        binding.deform_images(src, dst, 8, ok, 1, 0)
    assert e.value.code == binding.E_ARG
    with pytest.raises(binding.CnnError) as e:
        binding.deform_images(src, src, 4, ok, 1, 0)
    assert e.value.code == binding.E_ARG
    wide = torch.zeros((1, 1, 97, 96), dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.CnnError) as e:
        binding.deform_images(wide, torch.zeros_like(wide), 1, ok, 1, 0)
    assert e.value.code == binding.E_SHAPE
    torch.cuda.synchronize()


def test_the_whole_training_stream_in_the_benchmark_configuration():
    """60000 images of 1x29x29 deformed in one call, as bench.py times it: the oracle on a sample; the rest by
    properties that hold at any size (same bits when the stream is cut into calls of 1000, bounds)."""
    import torch
    n, C, H, W = 60000, 1, 29, 29
    rng = np.random.default_rng(SEED + 2)
    src = rng.uniform(-1, 1, (n, C, H, W)).astype(np.float32)
    gp, op = params(**ALL)
    d_src = torch.from_numpy(src).to("cuda:0")
    d_dst = torch.empty_like(d_src)
    binding.deform_images(d_src, d_dst, n, gp, SEED, 120000)
    torch.cuda.synchronize()
    got = d_dst.cpu().numpy()
    for k in (0, 1, 255, 8191, 8192, 30000, 59998, n - 1) + tuple(int(x) for x in rng.integers(0, n, 16)):
        w, _ = DO.deform_image(src[k], SEED, 120000 + k, op)
        assert rel(got[k], w) <= TOL, k
    d_cut = torch.empty_like(d_src)
    for k0 in range(0, n, 1000):
        binding.deform_images(d_src[k0:k0 + 1000], d_cut[k0:k0 + 1000], 1000, gp, SEED, 120000 + k0)
    torch.cuda.synchronize()
    assert torch.equal(d_cut, d_dst)
    assert got.min() >= -1.0 - 1e-6 and got.max() <= 1.0 + 1e-6
    moved = np.abs(got - src).reshape(n, -1).max(axis=1)
    assert (moved > 0.05).all()   # every presentation was deformed
