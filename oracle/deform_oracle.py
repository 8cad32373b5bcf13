"""CPU oracle of the on-line deformation of training images.  Test infrastructure only: the product
never imports this file; nothing here is shared with the HIP path.

What is computed (Sec. 4.1: the training images are deformed anew at every presentation by a combination
of affine maps -- translation, rotation, scaling, horizontal shearing -- and elastic deformations after
Simard et al. 2003; Sec. 4.2 and 4.3: random translations of at most 5 % of the image side).  The paper
names the ingredients and gives no formula, range or order; the reading taken here, in float64:

  for the image presented as number t of the stream (all its maps share one deformation):
    key       = mix64(seed + GOLDEN * (t + 1))                    counter-based generator: every draw is
    draw(k)   = mix64(key + GOLDEN * (k + 1)),  k = 0, 1, ...      a function of (seed, t, k) alone
    unit(b)   = (b >> 8) / 2**24   for a 32-bit half b of a draw   24 bits: exact in float32 as well
    sym(b)    = 2 * unit(b) - 1                                    in [-1, 1)
    draw 0: tx = sym(hi) * max_translation * W,  ty = sym(lo) * max_translation * H    (pixels)
    draw 1: theta = sym(hi) * max_rotation (degrees),  shear = sym(lo) * max_shear
    draw 2: sx = 1 + sym(hi) * max_scaling,  sy = 1 + sym(lo) * max_scaling
    draw 3 + y*W + x: rx[y,x] = sym(hi), ry[y,x] = sym(lo)         the two random displacement fields
    g[i] = exp(-i^2 / (2 sigma^2)), i = -R..R, R = ceil(3 sigma), divided by their sum
    Dx = alpha * (g (x) g) * rx,  Dy likewise                      'same' size, rx = 0 outside the image
    A  = Rot(theta) . [[1, shear], [0, 1]] . diag(sx, sy)          about the image centre ((W-1)/2, (H-1)/2)
    source of output pixel (y, x), u = x - cx, v = y - cy:
       xs = cx + A00 u + A01 v + tx + Dx[y,x],   ys = cy + A10 u + A11 v + ty + Dy[y,x]
    out[c,y,x] = bilinear interpolation of map c at (ys, xs); a neighbour outside the map counts as `fill`

mix64 is the output function of SplitMix64 (Steele, Lea, Flood 2014), GOLDEN = 0x9E3779B97F4A7C15.
"""
import math
from dataclasses import dataclass

import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
_MASK = (1 << 64) - 1


@dataclass
class DeformParams:
    max_translation: float = 0.0  # fraction of the image side
    max_rotation: float = 0.0     # degrees
    max_scaling: float = 0.0      # fraction: factors in [1 - m, 1 + m), x and y drawn independently
    max_shear: float = 0.0        # horizontal shear coefficient: x += shear * y
    sigma: float = 0.0            # std of the Gaussian that smooths the random fields, pixels; 0: no elastic part
    alpha: float = 0.0            # amplitude of the elastic part, pixels
    fill: float = 0.0             # value of everything outside the source image


def mix64(z):
    """Output function of SplitMix64 on Python ints (any size in, 64 bits out)."""
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def image_key(seed, t):
    return mix64(seed + GOLDEN * (t + 1))


def draw(key, k):
    """(hi, lo) 32-bit halves of draw number k under a key."""
    d = mix64(key + GOLDEN * (k + 1))
    return d >> 32, d & 0xFFFFFFFF


def unit(bits32):
    return (bits32 >> 8) / float(1 << 24)


def sym(bits32):
    return 2.0 * unit(bits32) - 1.0


def image_parameters(seed, t, P, H, W):
    """The six numbers of the affine part for presentation t: tx, ty (pixels), theta (radians), shear, sx, sy."""
    key = image_key(seed, t)
    h0, l0 = draw(key, 0)
    h1, l1 = draw(key, 1)
    h2, l2 = draw(key, 2)
    return dict(tx=sym(h0) * P.max_translation * W, ty=sym(l0) * P.max_translation * H,
                theta=math.radians(sym(h1) * P.max_rotation), shear=sym(l1) * P.max_shear,
                sx=1.0 + sym(h2) * P.max_scaling, sy=1.0 + sym(l2) * P.max_scaling)


def noise_fields(seed, t, H, W):
    key = image_key(seed, t)
    rx = np.zeros((H, W))
    ry = np.zeros((H, W))
    for y in range(H):
        for x in range(W):
            hi, lo = draw(key, 3 + y * W + x)
            rx[y, x] = sym(hi)
            ry[y, x] = sym(lo)
    return rx, ry


def gaussian_taps(sigma):
    R = int(math.ceil(3.0 * sigma))
    i = np.arange(-R, R + 1, dtype=np.float64)
    g = np.exp(-(i * i) / (2.0 * sigma * sigma))
    return g / g.sum()


def smooth(field, sigma):
    """Two-dimensional convolution with g (x) g, same size, zeros outside the field."""
    g = gaussian_taps(sigma)
    R = (len(g) - 1) // 2
    H, W = field.shape
    padded = np.zeros((H + 2 * R, W + 2 * R))
    padded[R:R + H, R:R + W] = field
    out = np.zeros((H, W))
    for j in range(-R, R + 1):
        for i in range(-R, R + 1):
            out += g[j + R] * g[i + R] * padded[R + j:R + j + H, R + i:R + i + W]
    return out


def affine_matrix(theta, shear, sx, sy):
    c, s = math.cos(theta), math.sin(theta)
    rot = np.array([[c, -s], [s, c]])
    sh = np.array([[1.0, shear], [0.0, 1.0]])
    sc = np.array([[sx, 0.0], [0.0, sy]])
    return rot @ sh @ sc


def source_coordinates(H, W, A, tx, ty, Dx, Dy):
    cy, cx = (H - 1) / 2.0, (W - 1) / 2.0
    y, x = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    u, v = x - cx, y - cy
    xs = cx + A[0, 0] * u + A[0, 1] * v + tx + Dx
    ys = cy + A[1, 0] * u + A[1, 1] * v + ty + Dy
    return ys, xs


def bilinear(src, ys, xs, fill):
    """src [C][H][W]; ys, xs [Ho][Wo] -> [C][Ho][Wo]."""
    C, H, W = src.shape
    y0 = np.floor(ys).astype(np.int64)
    x0 = np.floor(xs).astype(np.int64)
    fy, fx = ys - y0, xs - x0

    def at(yy, xx):
        inside = (yy >= 0) & (yy < H) & (xx >= 0) & (xx < W)
        vals = src[:, np.clip(yy, 0, H - 1), np.clip(xx, 0, W - 1)]
        return np.where(inside[None], vals, fill)

    return ((1 - fy) * (1 - fx))[None] * at(y0, x0) + ((1 - fy) * fx)[None] * at(y0, x0 + 1) \
        + (fy * (1 - fx))[None] * at(y0 + 1, x0) + (fy * fx)[None] * at(y0 + 1, x0 + 1)


def deform_image(src, seed, t, P):
    """src [C][H][W] float64 -> (deformed [C][H][W], displacement [2][H][W] = (xs - x, ys - y))."""
    src = np.asarray(src, dtype=np.float64)
    C, H, W = src.shape
    q = image_parameters(seed, t, P, H, W)
    if P.sigma > 0.0 and P.alpha != 0.0:
        rx, ry = noise_fields(seed, t, H, W)
        Dx, Dy = P.alpha * smooth(rx, P.sigma), P.alpha * smooth(ry, P.sigma)
    else:
        Dx = Dy = np.zeros((H, W))
    A = affine_matrix(q["theta"], q["shear"], q["sx"], q["sy"])
    ys, xs = source_coordinates(H, W, A, q["tx"], q["ty"], Dx, Dy)
    y, x = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    return bilinear(src, ys, xs, P.fill), np.stack([xs - x, ys - y])


def deform_images(src, seed, first_index, P, src_index=None):
    """src [N][C][H][W]; output k is source image src_index[k] (k itself without an index list),
    deformed as presentation first_index + k."""
    src = np.asarray(src, dtype=np.float64)
    n = src.shape[0] if src_index is None else len(src_index)
    out = np.zeros((n,) + src.shape[1:])
    disp = np.zeros((n, 2) + src.shape[2:])
    for k in range(n):
        out[k], disp[k] = deform_image(src[k if src_index is None else src_index[k]], seed, first_index + k, P)
    return out, disp
