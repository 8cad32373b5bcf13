// On-line deformation of training images (Sec. 4.1: affine maps -- translation, rotation, scaling,
// horizontal shearing -- combined with elastic deformations after Simard et al. 2003; Sec. 4.2, 4.3:
// random translations), one workgroup per image.  It depends on no weight, so it runs fully parallel
// over a batch of presentations ahead of the on-line training chain, on the same stream.
//
// Every random number is a function of (seed, presentation number, draw number) alone: mix64, the output
// function of SplitMix64 (Steele, Lea, Flood 2014), applied to key + GOLDEN * (draw + 1), where the key
// of a presentation is mix64(seed + GOLDEN * (presentation + 1)).  A draw's two 32-bit halves give two
// numbers of 24 bits each, so the same values exist exactly in float and in double.
#include <hip/hip_runtime.h>

// device pointers of the job descriptor are global-address-space pointers in this translation unit
#define CNN_GLOBAL __attribute__((address_space(1)))
#include "cnn355_dev.h"

namespace cnn355 {

namespace {

constexpr int DT = 256;  // threads per workgroup
constexpr unsigned long long GOLDEN = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// 32 random bits -> [-1, 1) in steps of 2^-23
__device__ __forceinline__ float sym(unsigned int bits) { return (float)(bits >> 8) * (2.0f / 16777216.0f) - 1.0f; }

constexpr int SW = 4;    // outputs of one lane along the line being smoothed

// One pass of the separable Gaussian over both fields: the lane's SW outputs out[k], k = at .. at + SW - 1,
// of the line starting at `ax` / `ay` (elements `step` apart, `len` of them; outside counts as zero).  The loop
// runs over the source elements that reach any of the outputs; the tap that links source j to output k is
// tp[j - k]: as j advances the SW taps in use slide by one, so an iteration reads one tap and one element of
// each field for 2 * SW multiply-adds.  tp points at the centre tap; R + SW zeros lie on either side of the taps.
__device__ __forceinline__ void blur_strip(const float* ax, const float* ay, int at, int len, int step, const float* tp,
                                           int R, float (&ox)[SW], float (&oy)[SW]) {
  const int jlo = max(0, at - R), jhi = min(len - 1, at + SW - 1 + R);
  float t[SW];
#pragma unroll
  for (int o = 0; o < SW; ++o) {
    ox[o] = 0.f;
    oy[o] = 0.f;
    t[o] = tp[jlo - 1 - (at + o)];  // the taps of the element before the first
  }
  for (int j = jlo; j <= jhi; ++j) {
#pragma unroll
    for (int o = SW - 1; o > 0; --o) t[o] = t[o - 1];  // tp[j - (at + o)] = what output o - 1 used one element ago
    t[0] = tp[j - at];
    const float vx = ax[j * step], vy = ay[j * step];
#pragma unroll
    for (int o = 0; o < SW; ++o) {
      ox[o] = fmaf(t[o], vx, ox[o]);
      oy[o] = fmaf(t[o], vy, oy[o]);
    }
  }
}

__global__ void __launch_bounds__(DT) k_deform(const DeformJob J) {
  extern __shared__ float lds[];
  const int H = J.H, W = J.W, HW = H * W, R = J.R;
  const int Wp = W | 1;       // odd row pitch: lanes on consecutive rows fall on different LDS banks
  float* rx = lds;            // [H][Wp] random fields, then the smoothed ones
  float* ry = lds + H * Wp;
  float* hx = lds + 2 * H * Wp;   // after the pass along rows
  float* hy = lds + 3 * H * Wp;
  float* taps = lds + 4 * H * Wp; // [R + SW zeros][2R + 1 taps][R + SW zeros]
  const float* tp = taps + 2 * R + SW;  // the centre tap
  const int tid = threadIdx.x;
  const bool elastic = R >= 0;
  if (elastic) {
    for (int i = tid; i < 4 * R + 2 * SW + 1; i += DT) {
      const int q = i - (R + SW);
      taps[i] = q >= 0 && q <= 2 * R ? J.taps[q] : 0.f;
    }
  }
  const float cx = 0.5f * (float)(W - 1), cy = 0.5f * (float)(H - 1);
  for (long long k = blockIdx.x; k < J.n; k += gridDim.x) {
    const unsigned long long key = mix64(J.seed + GOLDEN * (J.first_index + (unsigned long long)k + 1ull));
    // ---- the affine part: displacement = (A - I) (u, v) + (tx, ty), A = Rot . Shear . Scale
    const unsigned long long d0 = mix64(key + GOLDEN * 1ull), d1 = mix64(key + GOLDEN * 2ull), d2 = mix64(key + GOLDEN * 3ull);
    // (in double: the products reach tens of pixels on large maps, where a float keeps 1e-5 of a pixel at best)
    const double tx = sym((unsigned int)(d0 >> 32)) * J.max_tx, ty = sym((unsigned int)d0) * J.max_ty;
    const double theta = sym((unsigned int)(d1 >> 32)) * J.max_rot, sh = sym((unsigned int)d1) * J.max_shear;
    const double sx = 1.0 + sym((unsigned int)(d2 >> 32)) * J.max_scale, sy = 1.0 + sym((unsigned int)d2) * J.max_scale;
    double sn, cs;
    sincos(theta, &sn, &cs);
    const double a00 = cs * sx - 1.0, a01 = (cs * sh - sn) * sy, a10 = sn * sx, a11 = (sn * sh + cs) * sy - 1.0;
    // ---- the elastic part: two random fields, smoothed along rows, then along columns
    if (elastic) {
      __syncthreads();  // the previous image's fields have been read
      unsigned long long ctr = key + GOLDEN * (unsigned long long)(tid + 4);
      for (int p = tid; p < HW; p += DT, ctr += GOLDEN * (unsigned long long)DT) {
        const unsigned long long d = mix64(ctr);
        const int y = p / W, x = p - y * W;
        rx[y * Wp + x] = sym((unsigned int)(d >> 32));
        ry[y * Wp + x] = sym((unsigned int)d);
      }
      __syncthreads();
      const int nsx = (W + SW - 1) / SW, nsy = (H + SW - 1) / SW;
      for (int it = tid; it < H * nsx; it += DT) {  // along rows; consecutive lanes take consecutive rows
        const int s = it / H, y = it - s * H, x0 = s * SW;
        float ox[SW], oy[SW];
        blur_strip(rx + y * Wp, ry + y * Wp, x0, W, 1, tp, R, ox, oy);
#pragma unroll
        for (int o = 0; o < SW; ++o)
          if (x0 + o < W) {
            hx[y * Wp + x0 + o] = ox[o];
            hy[y * Wp + x0 + o] = oy[o];
          }
      }
      __syncthreads();
      for (int it = tid; it < W * nsy; it += DT) {  // along columns; consecutive lanes take consecutive columns
        const int s = it / W, x = it - s * W, y0 = s * SW;
        float ox[SW], oy[SW];
        blur_strip(hx + x, hy + x, y0, H, Wp, tp, R, ox, oy);
#pragma unroll
        for (int o = 0; o < SW; ++o)
          if (y0 + o < H) {
            rx[(y0 + o) * Wp + x] = ox[o];
            ry[(y0 + o) * Wp + x] = oy[o];
          }
      }
      __syncthreads();
    }
    // ---- sample the source
    long long s = J.src_index ? (long long)J.src_index[k] : k;
    const bool known = s >= 0 && s < J.n_src;  // an index that names no source image gives an image of `fill`
    if (!known) s = 0;
    const CNN_GLOBAL float* src = J.src + s * J.C * HW;
    CNN_GLOBAL float* dst = J.dst + k * J.C * HW;
    for (int p = tid; p < HW; p += DT) {
      const int y = p / W, x = p - y * W;
      const double u = (double)x - (double)cx, v = (double)y - (double)cy;
      double dx = fma(a00, u, fma(a01, v, tx)), dy = fma(a10, u, fma(a11, v, ty));
      if (elastic) {
        dx += (double)(J.alpha * rx[y * Wp + x]);
        dy += (double)(J.alpha * ry[y * Wp + x]);
      }
      if (J.disp) {
        J.disp[(k * 2) * HW + p] = (float)dx;
        J.disp[(k * 2 + 1) * HW + p] = (float)dy;
      }
      // far outside in any direction reads the fill value only; the clamp keeps the integers small
      const double fdx = floor(fmin(fmax(dx, -(double)(W + 2)), (double)(W + 2)));
      const double fdy = floor(fmin(fmax(dy, -(double)(H + 2)), (double)(H + 2)));
      const float fx = fminf(fmaxf((float)(dx - fdx), 0.f), 1.f), fy = fminf(fmaxf((float)(dy - fdy), 0.f), 1.f);
      const int x0 = x + (int)fdx, y0 = y + (int)fdy;
      const bool in_x0 = x0 >= 0 && x0 < W, in_x1 = x0 + 1 >= 0 && x0 + 1 < W;
      const bool in_y0 = y0 >= 0 && y0 < H, in_y1 = y0 + 1 >= 0 && y0 + 1 < H;
      const int xa = min(max(x0, 0), W - 1), xb = min(max(x0 + 1, 0), W - 1);
      const int ya = min(max(y0, 0), H - 1), yb = min(max(y0 + 1, 0), H - 1);
      const float w00 = (1.f - fy) * (1.f - fx), w01 = (1.f - fy) * fx, w10 = fy * (1.f - fx), w11 = fy * fx;
      for (int c = 0; c < J.C; ++c) {
        const CNN_GLOBAL float* m = src + (long long)c * HW;
        const float v00 = in_y0 && in_x0 ? m[ya * W + xa] : J.fill;
        const float v01 = in_y0 && in_x1 ? m[ya * W + xb] : J.fill;
        const float v10 = in_y1 && in_x0 ? m[yb * W + xa] : J.fill;
        const float v11 = in_y1 && in_x1 ? m[yb * W + xb] : J.fill;
        dst[(long long)c * HW + p] = known ? fmaf(w00, v00, fmaf(w01, v01, fmaf(w10, v10, w11 * v11))) : J.fill;
      }
    }
  }
}

}  // namespace

size_t deform_lds_bytes(const DeformJob& J) {
  return J.R >= 0 ? ((size_t)4 * J.H * (J.W | 1) + 4 * J.R + 2 * SW + 1) * sizeof(float) : 0;
}

hipError_t launch_deform(hipStream_t stream, const DeformJob& J) {
  if (J.n <= 0) return hipSuccess;
  const size_t lds = deform_lds_bytes(J);
  hipError_t e = hipFuncSetAttribute((const void*)k_deform, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  const unsigned int grid = (unsigned int)(J.n < 8192 ? J.n : 8192);
  hipLaunchKernelGGL(k_deform, dim3(grid), dim3(DT), lds, stream, J);
  return hipGetLastError();
}

}  // namespace cnn355
