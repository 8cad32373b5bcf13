"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers: images, labels, initial weights, connection
tables and the fixed contrast filters.  It holds none of the network's
arithmetic, so both the GPU path and the CPU oracle can be fed from it without
sharing any of the method's code.

Stand-ins (the datasets themselves are never needed):
  29x29 single map  ~ the padded digit images of Sec. 4.1 (size as in Fig. 2)
  2x48x48 stereo    ~ the two-map stereo input of Sec. 4.2
  3x32x32 colour    ~ the three-map input of Sec. 4.3
Weights follow Sec. 4: uniform in [-0.05, 0.05] (biases included).
The generator is NumPy's PCG64 (`default_rng(seed)`), fixed and portable.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

SEED0 = 11020183


@dataclass(frozen=True)
class Workload:
    name: str
    arch: str
    raw_shape: Tuple[int, int, int]      # shape of one image as handed to the network
    n_images: int
    n_classes: int
    pixels: str                          # "u11": U[-1,1];  "u01c": U[0,1] minus per-channel mean
    seeds: Tuple[int, ...]               # offsets from SEED0: images, labels, weights[, table, filters]
    lr: float = 1e-3
    sparse_conv: Optional[int] = None    # index of the conv layer that gets a random table
    fan_in: Optional[int] = None
    frontend: bool = False
    note: str = ""
    extra: dict = field(default_factory=dict)


WORKLOADS = {
    "cfg1": Workload("cfg1", "1x29x29-20C4-MP2-40C5-MP3-150N-10N", (1, 29, 29), 1000, 10, "u11",
                     (10, 11, 12)),
    "cfg2a": Workload("cfg2a", "1x29x29-20C4-MP2-40C5-MP3-150N-10N", (1, 29, 29), 60000, 10, "u11",
                      (20, 21, 22)),
    "cfg2b": Workload("cfg2b", "1x29x29-40C4-MP2-80C5-MP3-300N-10N", (1, 29, 29), 60000, 10, "u11",
                      (20, 21, 22)),
    "cfg3": Workload("cfg3", "2x48x48-50C5-MP2-128C3-MP4-100N-5N", (2, 48, 48), 20000, 5, "u11",
                     (30, 31, 32)),
    "cfg4a": Workload("cfg4a", "3x32x32-100C5-MP2-100C5-MP2-100C4-MP2-300N-10N", (3, 32, 32), 10000,
                      10, "u01c", (40, 41, 42)),
    "cfg4b": Workload("cfg4b", "3x32x32-300C3-MP2-300C2-MP2-300C4-MP2-300N-10N", (3, 32, 32), 10000,
                      10, "u01c", (40, 41, 42)),
    "cfg5": Workload("cfg5", "4x44x44-40C5S1-MP2-80C3-MP2-100N-5N", (2, 48, 48), 20000, 5, "u11",
                     (50, 51, 52, 53, 54), sparse_conv=1, fan_in=20, frontend=True),
}


# Ranges of the on-line deformation the measurements and full-size tests use (Sec. 4.1 names the ingredients and
# gives no ranges): up to 5 % translation (Sec. 4.2), 15 degrees, 15 % scaling, 0.15 shear, an elastic field of
# std about one pixel (sigma 6, alpha 36); -1 outside the image.  Seed of the draws: SEED0 + 60.
DEFORM_RECIPE = dict(max_translation=0.05, max_rotation=15.0, max_scaling=0.15, max_shear=0.15, sigma=6.0, alpha=36.0,
                     fill=-1.0)
DEFORM_SEED = SEED0 + 60


def images(wl: Workload, n: Optional[int] = None) -> np.ndarray:
    """First n images of the workload's stream, float32 [n, C, H, W].

    The stream is drawn image by image, so a prefix of a longer stream equals the
    shorter stream.  For "u01c" the per-channel mean subtracted is that of the
    distribution's own first 1000 images (a fixed constant of the recipe), so a
    prefix does not depend on how many images are asked for.
    """
    n = wl.n_images if n is None else int(n)
    rng = np.random.default_rng(SEED0 + wl.seeds[0])
    c, h, w = wl.raw_shape
    if wl.pixels == "u11":
        x = rng.random((n, c, h, w), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    elif wl.pixels == "u01c":
        x = rng.random((n, c, h, w), dtype=np.float32)
        ref = np.random.default_rng(SEED0 + wl.seeds[0]).random((min(1000, wl.n_images), c, h, w),
                                                                dtype=np.float32)
        mean = ref.mean(axis=(0, 2, 3), dtype=np.float64).astype(np.float32)
        x = x - mean[None, :, None, None]
    else:
        raise ValueError(wl.pixels)
    return np.ascontiguousarray(x, dtype=np.float32)


def labels(wl: Workload, n: Optional[int] = None) -> np.ndarray:
    n = wl.n_images if n is None else int(n)
    rng = np.random.default_rng(SEED0 + wl.seeds[1])
    return rng.integers(0, wl.n_classes, size=n, dtype=np.int32)


def weights(wl: Workload, n_weights: int) -> np.ndarray:
    """Initial weights and biases, uniform in [-0.05, 0.05] (Sec. 4), float32."""
    rng = np.random.default_rng(SEED0 + wl.seeds[2])
    return ((rng.random(n_weights, dtype=np.float32) - np.float32(0.5)) * np.float32(0.1)).astype(
        np.float32)


def random_table(m_out: int, m_in: int, fan_in: int, seed: int) -> np.ndarray:
    """Random sparse connection table [m_out, m_in] of 0/1 with a fixed fan-in.

    The paper drops connections "in a random way" without giving a distribution
    (Sec. 4.1); this recipe picks `fan_in` distinct input maps per output map.
    """
    rng = np.random.default_rng(seed)
    t = np.zeros((m_out, m_in), dtype=np.uint8)
    for j in range(m_out):
        t[j, rng.choice(m_in, size=fan_in, replace=False)] = 1
    return t


def regular_table(m_out: int, m_in: int, fan_in: int) -> np.ndarray:
    """Connection table [m_out, m_in] in which output map j reads the input maps j, j + 1, ..., j + fan_in - 1
    (mod m_in); fan_in = -d stands for m_in / d of them.  Every output map reads as many maps and every input map
    feeds (nearly) as many, so the table's sizes, which the resident plan depends on, follow from the three numbers."""
    if fan_in < 0:
        fan_in = max(1, m_in // -fan_in)
    t = np.zeros((m_out, m_in), dtype=np.uint8)
    for j in range(m_out):
        for k in range(min(fan_in, m_in)):
            t[j, (j + k) % m_in] = 1
    return t


def connection_table(wl: Workload, m_out: int, m_in: int) -> Optional[np.ndarray]:
    if wl.sparse_conv is None:
        return None
    return random_table(m_out, m_in, wl.fan_in, SEED0 + wl.seeds[3])


def contrast_filters(wl: Workload, k: int = 5):
    """Four fixed centre-minus-surround filters (contrast extraction, Sec. 2.1, Sec. 4.2).

    Filter f reads raw channel f // 2; even f is on-centre, odd f is the same
    shape negated (off-centre).  Each is a difference of two Gaussians
    (sigma_c ~ U[0.6, 1.0], sigma_s = 2 sigma_c), made zero-sum and scaled to unit
    L1 norm.  Returns (filters [4, k, k] float32, src_channel [4] int32).
    """
    rng = np.random.default_rng(SEED0 + wl.seeds[4])
    r = np.arange(k, dtype=np.float64) - (k - 1) / 2.0
    yy, xx = np.meshgrid(r, r, indexing="ij")
    d2 = yy * yy + xx * xx
    filt = np.zeros((4, k, k), dtype=np.float64)
    for f in range(4):
        sc = rng.uniform(0.6, 1.0)
        ss = 2.0 * sc
        g = np.exp(-d2 / (2 * sc * sc)) / (sc * sc) - np.exp(-d2 / (2 * ss * ss)) / (ss * ss)
        g -= g.mean()
        g /= np.abs(g).sum()
        filt[f] = g if f % 2 == 0 else -g
    return filt.astype(np.float32), np.array([0, 0, 1, 1], dtype=np.int32)


def build_network(net, wl: Workload):
    """Give a freshly created network (the GPU library's or the oracle's: same method names) the
    workload's connection table, fixed front-end and seeded weights.  Returns the network."""
    if wl.sparse_conv is not None:
        convs = [l for l in range(1, net.num_layers) if net.layer_info(l)["kind"] == 1]
        l = convs[wl.sparse_conv]
        net.set_connection_table(wl.sparse_conv, connection_table(wl, net.layer_info(l)["maps"],
                                                                  net.layer_info(l - 1)["maps"]))
    if wl.frontend:
        filt, src = contrast_filters(wl)
        net.set_fixed_frontend(filt, src, wl.raw_shape[0])
    net.set_weights(weights(wl, net.num_weights))
    return net
