// Batched forward propagation (Sec. 3.2 for many images at once): validation and test passes
// change no weight (Sec. 4), so their images are independent and every layer becomes one dense
// matrix product over the whole batch,
//     sums[j][n] = sum_k  Wt[k][j] * X[k][n],     n = (image b, output pixel p),  k = (input map i, ky, kx),
// which is what the matrix cores are for.  X is never formed: its element is
// in[b][i][(y (S+1) + ky)][(x (S+1) + kx)], read from the images staged in LDS at offset
// koff(k) + pbase(n).  A fully connected layer is the same product with 1 x 1 maps and K = 1.
// fp32 operands and fp32 accumulation (v_mfma_f32_32x32x2_f32): the results stay within the
// tolerance of the one-image path.
#include <hip/hip_runtime.h>

#include <cstdint>

#define CNN_GLOBAL __attribute__((address_space(1)))
#include "cnn355_dev.h"

namespace cnn355 {

typedef const CNN_GLOBAL float* cgf;
typedef CNN_GLOBAL float* gf;
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

constexpr int BT = 256;        // threads of a GEMM workgroup: four wavefronts, 32 columns each
constexpr int BCOLS = 128;     // columns (image, pixel) of a workgroup

// scaled tanh 1.7159 tanh(0.6666 a) (Sec. 4) as A (1 - 2 / (e^{2 B a} + 1)) on the hardware
// exponential and reciprocal: absolute error about 3e-7; below |B a| = 0.3 the odd series of tanh up to x^9
// (5e-8 of the result there), so that small activations keep their digits
__device__ __forceinline__ float b_act(float a) {
  const float z = __builtin_amdgcn_exp2f((2.0f * 0.6666f * 1.44269504088896340736f) * a);
  const float big = 1.7159f - (2.0f * 1.7159f) * __builtin_amdgcn_rcpf(z + 1.0f);
  const float x = 0.6666f * a, x2 = x * x;
  float p = fmaf(x2, 62.0f / 2835.0f, -17.0f / 315.0f);
  p = fmaf(x2, p, 2.0f / 15.0f);
  p = fmaf(x2, p, -1.0f / 3.0f);
  const float small = 1.7159f * fmaf(x, x2 * p, x);
  return fabsf(x) < 0.3f ? small : big;
}

constexpr int PRE_IN = 16;     // floats per thread a prefetched chunk may hold: staged images ...
constexpr int PRE_W = 48;      // ... and rows of Wt

// Workgroup (x, y): columns [128 x, 128 x + 128) and map tiles [MT y, MT y + MT) of TR maps each.  TR = 32:
// v_mfma_f32_32x32x2_f32, a wavefront's 32 columns are one tile wide, a lane takes the even or the odd k.  TR = 16:
// v_mfma_f32_16x16x4_f32, the 32 columns are two tiles of 16, a lane takes one k in four; it is chosen where 16-row
// tiles pad fewer maps (40 maps: 48 rows instead of 64).
// Every wavefront owns 32 columns and all MT map tiles, so one operand fetched from the staged
// images feeds MT matrix instructions.  The k range is walked in chunks of IC input maps: the
// chunk's maps of every image the columns touch, and the chunk's rows of Wt, are staged in LDS.
// With g.prefetch the next chunk is fetched into registers while the matrix cores work on the
// present one (global latency hidden behind arithmetic); the host sets it only when a chunk
// fits the register budget (PRE_IN, PRE_W floats per thread).
template <int MT, int TR>
__global__ void __launch_bounds__(BT) k_batch_gemm(BatchGemm g) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  constexpr int KS = TR == 32 ? 2 : 4;             // k values one instruction takes, one per group of 64 / KS lanes
  constexpr int CT = 32 / TR;                      // column tiles of a wavefront
  constexpr int AV = TR == 32 ? 16 : 4;            // accumulator floats per lane and tile
  const int lrow = lane & (TR - 1), lk = lane / TR;
  const int HiWi = g.Hi * g.Wi, KK = g.K * g.Kx;
  const int slot_sz = g.IC * HiWi;
  const int KC = g.IC * KK;                        // k per full chunk
  constexpr int WROW = MT * TR;
  float* lds_in = lds;                              // [n_img_max][IC][Hi*Wi]
  float* lds_w = lds + ((g.n_img_max * slot_sz + 3) & ~3);  // [KC + 1][MT * 32]; the row behind the last is zero
  // byte offset of k inside a staged image, the k of every residue mod KS apart so that a lane (which takes the
  // k of its own residue) finds the four it needs next to each other: [KS][KH], KH a multiple of 4
  const int KH = (((KC + KS - 1) / KS) + 3) & ~3;
  int* koff = (int*)(lds_w + (KC + 1) * WROW);

  // (columns are counted in 32 bits: the host keeps batch * P below 2^31)
  const int N = (int)g.N;
  const int n0 = blockIdx.x * BCOLS;
  const int mt0 = blockIdx.y * MT;                 // first tile (of TR maps) of the workgroup
  const int b_lo = n0 / g.P;
  const int n_last = min(n0 + BCOLS, N) - 1;
  const int n_img = n_last / g.P - b_lo + 1;

  for (int x = tid; x < KS * KH; x += BT) {
    const int par = x / KH, h = x - par * KH;
    const int k = min(KS * h + par, KC - 1);
    const int c = k / KK, t = k - c * KK;
    const int ky = t / g.Kx, kx = t - ky * g.Kx;
    koff[x] = (c * HiWi + ky * g.Wi + kx) * 4;
  }
  // the lane's column in each of the wavefront's column tiles
  bool col_ok[CT];
  int cb[CT], cp[CT], pbase[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int n = n0 + wave * 32 + ct * TR + lrow;
    col_ok[ct] = n < N;
    cb[ct] = 0; cp[ct] = 0; pbase[ct] = 0;
    if (col_ok[ct]) {
      cb[ct] = n / g.P;
      cp[ct] = n - cb[ct] * g.P;
      const int y = cp[ct] / g.Wo, x = cp[ct] - y * g.Wo;
      pbase[ct] = (cb[ct] - b_lo) * slot_sz + y * (g.Kp * g.stride) * g.Wi + x * (g.Kpx * g.stride_x);
    }
  }
  typedef float accv __attribute__((ext_vector_type(AV)));
  accv acc[MT][CT], best[MT][CT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int v = 0; v < AV; ++v) { acc[m][ct][v] = 0.f; best[m][ct][v] = -INFINITY; }

  // Element e of a chunk's staged images is float x of image slot s, e = s * cnt + x, where
  // cnt = n_ic * Hi * Wi is the run of contiguous floats the chunk takes from one image; a thread
  // walks e = tid, tid + BT, ... and keeps (s, x) by carrying instead of dividing.  Element e of
  // the chunk's weights is Wt[ic0 * KK + e / WROW][mt0 * 32 + e % WROW], WROW a power of two.
  struct Walk {
    int s, x, cnt, sh;   // sh >= 0: cnt == 1 << sh
    __device__ __forceinline__ Walk(int tid, int cnt_) : cnt(cnt_) {
      sh = (cnt_ & (cnt_ - 1)) == 0 ? __ffs(cnt_) - 1 : -1;
      s = sh >= 0 ? tid >> sh : tid / cnt_;
      x = tid - s * cnt_;
    }
    __device__ __forceinline__ void step() {
      x += BT;
      if (sh >= 0) { s += x >> sh; x &= cnt - 1; }
      else while (x >= cnt) { x -= cnt; ++s; }
    }
  };
  // addresses as a uniform base plus a 32-bit offset per lane (the host keeps every array the
  // kernel indexes this way below 2^31 floats)
  const cgf in0 = g.in + (long long)b_lo * g.in_stride;
  const unsigned in_stride32 = (unsigned)g.in_stride;
  auto in_ptr = [&](int ic0, const Walk& w, bool ok) -> cgf {
    return in0 + ic0 * HiWi + (ok ? (unsigned)w.s * in_stride32 + (unsigned)w.x : 0u);
  };
  // four weights at a time: rows of Wt and of the staged copy start on 128-byte boundaries
  auto w_val = [&](int ic0, int kc, int e4) -> v4f {
    const int kr = e4 / (WROW / 4), c = (e4 - kr * (WROW / 4)) * 4;
    if (kr >= kc) return v4f{0.f, 0.f, 0.f, 0.f};
    return *(const CNN_GLOBAL v4f*)(g.wt + ((long long)ic0 * KK * g.MoPad + mt0 * TR) + (unsigned)(kr * g.MoPad + c));
  };
  // straight to LDS, eight loads in flight per thread (first chunk, and every chunk without prefetch)
  auto stage_now = [&](int ic0) {
    const int n_ic = min(g.IC, g.Mi - ic0);
    const int cnt = n_ic * HiWi, tot = n_img * cnt;
    Walk w(tid, cnt);
    for (int e0 = 0; e0 < tot; e0 += 8 * BT) {
      float v[8];
      int d[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool ok = e0 + u * BT + tid < tot;
        v[u] = *in_ptr(ic0, w, ok);
        d[u] = ok ? w.s * slot_sz + w.x : -1;
        w.step();
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (d[u] >= 0) lds_in[d[u]] = v[u];
    }
    const int kc = n_ic * KK, wtot = (kc + 1) * (WROW / 4);
    for (int e0 = 0; e0 < wtot; e0 += 4 * BT) {
      v4f v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = w_val(ic0, kc, min(e0 + u * BT + tid, wtot - 1));
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (e0 + u * BT + tid < wtot) ((v4f*)lds_w)[e0 + u * BT + tid] = v[u];
    }
  };
  float ri[PRE_IN];
  v4f rw[PRE_W / 4];
  auto fetch = [&](int ic0) {
    const int n_ic = min(g.IC, g.Mi - ic0);
    const int cnt = n_ic * HiWi, tot = n_img * cnt;
    Walk w(tid, cnt);
#pragma unroll
    for (int u = 0; u < PRE_IN; ++u) {
      ri[u] = *in_ptr(ic0, w, u * BT + tid < tot);
      w.step();
    }
    const int kc = n_ic * KK, wtot = (kc + 1) * (WROW / 4);
#pragma unroll
    for (int u = 0; u < PRE_W / 4; ++u)
      rw[u] = (u * BT < wtot) ? w_val(ic0, kc, min(u * BT + tid, wtot - 1)) : v4f{0.f, 0.f, 0.f, 0.f};
  };
  auto put = [&](int ic0) {
    const int n_ic = min(g.IC, g.Mi - ic0);
    const int cnt = n_ic * HiWi, tot = n_img * cnt;
    Walk w(tid, cnt);
#pragma unroll
    for (int u = 0; u < PRE_IN; ++u) {
      if (u * BT + tid < tot) lds_in[w.s * slot_sz + w.x] = ri[u];
      w.step();
    }
    const int wtot = (n_ic * KK + 1) * (WROW / 4);
#pragma unroll
    for (int u = 0; u < PRE_W / 4; ++u)
      if (u * BT + tid < wtot) ((v4f*)lds_w)[u * BT + tid] = rw[u];
  };

  // slice blockIdx.z of the k range: chunks [z * cps, (z + 1) * cps)
  const int ic_first = blockIdx.z * g.chunks_per_slice * g.IC;
  const int ic_end = min(g.Mi, ic_first + g.chunks_per_slice * g.IC);
  for (int ic0 = ic_first; ic0 < ic_end; ic0 += g.IC) {
    const int n_ic = min(g.IC, g.Mi - ic0);
    const int kc = n_ic * KK;
    if (ic0 == ic_first || !g.prefetch) stage_now(ic0);
    else put(ic0);
    __syncthreads();
    if (g.prefetch && ic0 + g.IC < ic_end) fetch(ic0 + g.IC);
    // Members of the pooling window, one after the other (one member, the pixel itself, without
    // pooling; with it the host has made the k range a single chunk, so a member's sums are
    // complete when its loop ends).
    for (int d = 0; d < g.Kp * g.Kpx; ++d) {
      const int dy = d / g.Kpx, dx = d - dy * g.Kpx;
      const int pd = dy * g.stride * g.Wi + dx * g.stride_x;
      // KS k per instruction (lanes 0 .. 64/KS - 1 the first, and so on); the operands of four instructions per
      // tile are fetched together.  Whole groups of 4 KS k first, without any clamping; then the tail, where k
      // beyond the chunk meets the zero row of Wt.
      const char* in_b[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) in_b[ct] = (const char*)lds_in + (pbase[ct] + pd) * 4;
#define CNN355_MAC(a, bv)                                                                                            \
  _Pragma("unroll") for (int u = 0; u < 4; ++u)                                                                      \
  _Pragma("unroll") for (int m = 0; m < MT; ++m)                                                                     \
  _Pragma("unroll") for (int ct = 0; ct < CT; ++ct) {                                                                \
    if constexpr (TR == 32) acc[m][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][m], bv[u][ct], acc[m][ct], 0, 0, 0); \
    else acc[m][ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][m], bv[u][ct], acc[m][ct], 0, 0, 0);                  \
  }
      constexpr int KG = 4 * KS;
      const int kcg = kc - kc % KG;
      for (int kk = 0; kk < kcg; kk += KG) {
        const int4 ko = *(const int4*)(koff + lk * KH + kk / KS);
        const float* wr = lds_w + (kk + lk) * WROW + lrow;
        float a[4][MT], bv[4][CT];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int m = 0; m < MT; ++m) a[u][m] = wr[KS * u * WROW + m * TR];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          bv[0][ct] = *(const float*)(in_b[ct] + ko.x);
          bv[1][ct] = *(const float*)(in_b[ct] + ko.y);
          bv[2][ct] = *(const float*)(in_b[ct] + ko.z);
          bv[3][ct] = *(const float*)(in_b[ct] + ko.w);
        }
        CNN355_MAC(a, bv)
      }
      if (kcg < kc) {
        float a[4][MT], bv[4][CT];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = kcg + KS * u + lk;
          const int kr = min(k, kc);               // row kc is the zero row
          const int ko = koff[lk * KH + min(k / KS, KH - 1)];
#pragma unroll
          for (int m = 0; m < MT; ++m) a[u][m] = lds_w[kr * WROW + m * TR + lrow];
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) bv[u][ct] = *(const float*)(in_b[ct] + ko);
        }
        CNN355_MAC(a, bv)
      }
#undef CNN355_MAC
      if (g.Kp * g.Kpx > 1) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < AV; ++v) {
              best[m][ct][v] = fmaxf(best[m][ct][v], acc[m][ct][v]);
              acc[m][ct][v] = 0.f;
            }
      }
    }
    __syncthreads();
  }
  // element v of a lane, 32-row tiles: row (v / 4) * 8 + (lane / 32) * 4 + v % 4 of the tile, column lane % 32;
  // 16-row tiles: row (lane / 16) * 4 + v, column lane % 16
  gf dst = g.out + (long long)blockIdx.z * g.slice_stride;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    if (!col_ok[ct]) continue;
    const unsigned o0 = (unsigned)cb[ct] * (unsigned)g.out_stride + (unsigned)cp[ct];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int v = 0; v < AV; ++v) {
        const int j = (mt0 + m) * TR + (TR == 32 ? (v >> 2) * 8 + lk * 4 + (v & 3) : lk * 4 + v);
        if (j < g.Mo) {
          float sv = (g.Kp * g.Kpx > 1) ? best[m][ct][v] : acc[m][ct][v];
          if (g.fuse) sv += g.bias[j];
          if (g.fuse == 1) sv = b_act(sv);
          dst[o0 + (unsigned)j * (unsigned)g.P] = sv;
        }
      }
  }
}

// bias + scaled tanh + max-pooling (Sec. 2.2, 2.3) of the raw sums of a whole batch; the sums may
// come as several planes (slices of the k range), added here in a fixed order.  The activation
// function is increasing, so the maximum is taken first: one tanh per window.  act 0: none (the
// output layer's sums go on to the output units).
__global__ void __launch_bounds__(256) k_batch_pool(BatchPool q) {
  const long long x = (long long)blockIdx.x * 256 + threadIdx.x;
  if (x >= q.total) return;
  const int HpWp = q.Hp * q.Wp;
  const long long bj = x / HpWp;
  const int w = (int)(x - bj * HpWp);
  const int j = (int)(bj % q.Mo);
  const int py = w / q.Wp, px = w - py * q.Wp;
  cgf src = q.sums + bj * ((long long)q.Ho * q.Wo) + (py * q.Kp) * q.Wo + px * q.Kpx;
  float best = -INFINITY;
  for (int dy = 0; dy < q.Kp; ++dy)
    for (int dx = 0; dx < q.Kpx; ++dx) {
      float v = 0.f;
      for (int sl = 0; sl < q.n_slices; ++sl) v += src[(long long)sl * q.slice_stride + dy * q.Wo + dx];
      best = fmaxf(best, v);
    }
  best += q.bias[j];
  q.out[x] = q.act ? b_act(best) : best;
}

// Output units of a whole batch: soft-max of the output layer's sums (bias included), or the
// scaled tanh for the variant with tanh output neurons.  One thread per image.
__global__ void __launch_bounds__(256) k_batch_outputs(cgf logits, gf probs, long long n_images, int n_classes,
                                                       int out_units) {
  const long long b = (long long)blockIdx.x * 256 + threadIdx.x;
  if (b >= n_images) return;
  cgf a = logits + b * n_classes;
  gf o = probs + b * n_classes;
  if (out_units == 1) {
    for (int k = 0; k < n_classes; ++k) o[k] = b_act(a[k]);
    return;
  }
  float mx = a[0];
  for (int k = 1; k < n_classes; ++k) mx = fmaxf(mx, a[k]);
  float z = 0.f;
  for (int k = 0; k < n_classes; ++k) z += expf(a[k] - mx);
  for (int k = 0; k < n_classes; ++k) o[k] = expf(a[k] - mx) / z;
}

// Wt[k][j] of one layer from the canonical weights: k = (input map, ky, kx), j = output map;
// absent connections and the padding maps stay zero (the buffer is cleared first).
__global__ void __launch_bounds__(256) k_batch_pack(BatchPack q) {
  const long long x = (long long)blockIdx.x * 256 + threadIdx.x;
  if (x >= q.total) return;
  if (q.is_fc) {  // W[n_out][n_in]
    const int j = (int)(x / q.n_in), m = (int)(x - (long long)j * q.n_in);
    q.wt[(long long)m * q.MoPad + j] = q.w[x];
    return;
  }
  const int KK = q.K * q.Kx;
  const long long slot = x / KK;
  const int t = (int)(x - slot * KK);
  int j, i;
  if (q.full_table) {
    j = (int)(slot / q.Mi);
    i = (int)(slot - (long long)j * q.Mi);
  } else {
    // row j with csr_ptr[j] <= slot < csr_ptr[j + 1]
    int lo = 0, hi = q.Mo;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (q.csr_ptr[mid] <= slot) lo = mid; else hi = mid;
    }
    j = lo;
    i = q.csr_idx[slot];
  }
  q.wt[((long long)i * KK + t) * q.MoPad + j] = q.w[x];
}

__global__ void __launch_bounds__(256) k_batch_zero(gf p, long long n) {
  const long long x = (long long)blockIdx.x * 256 + threadIdx.x;
  if (x < n) p[x] = 0.f;
}

template <int MT, int TR>
hipError_t launch_gemm_mt(hipStream_t stream, const BatchGemm& g, size_t lds_bytes) {
  hipError_t e = hipFuncSetAttribute((const void*)k_batch_gemm<MT, TR>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  const unsigned gx = (unsigned)((g.N + BCOLS - 1) / BCOLS);
  const unsigned gy = (unsigned)((g.MoPad / TR + MT - 1) / MT);
  hipLaunchKernelGGL((k_batch_gemm<MT, TR>), dim3(gx, gy, (unsigned)g.KS), dim3(BT), lds_bytes, stream, g);
  return hipGetLastError();
}

}  // namespace

size_t batch_gemm_lds_bytes(const BatchGemm& g) {
  const int KC = g.IC * g.K * g.Kx;
  const size_t KS = g.TR == 32 ? 2 : 4;
  const size_t KH = ((((size_t)KC + KS - 1) / KS) + 3) & ~(size_t)3;
  return ((((size_t)g.n_img_max * g.IC * g.Hi * g.Wi + 3) & ~(size_t)3) + (size_t)(KC + 1) * g.MT * g.TR + KS * KH) * sizeof(float);
}

hipError_t launch_batch_gemm(hipStream_t stream, const BatchGemm& g) {
  if (g.N <= 0) return hipSuccess;
  const size_t lds_bytes = batch_gemm_lds_bytes(g);
  if (g.TR == 32) {
    switch (g.MT) {
      case 1: return launch_gemm_mt<1, 32>(stream, g, lds_bytes);
      case 2: return launch_gemm_mt<2, 32>(stream, g, lds_bytes);
      case 4: return launch_gemm_mt<4, 32>(stream, g, lds_bytes);
      default: return hipErrorInvalidValue;
    }
  }
  if (g.TR != 16) return hipErrorInvalidValue;
  switch (g.MT) {
    case 2: return launch_gemm_mt<2, 16>(stream, g, lds_bytes);
    case 3: return launch_gemm_mt<3, 16>(stream, g, lds_bytes);
    case 4: return launch_gemm_mt<4, 16>(stream, g, lds_bytes);
    case 5: return launch_gemm_mt<5, 16>(stream, g, lds_bytes);
    case 6: return launch_gemm_mt<6, 16>(stream, g, lds_bytes);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_batch_pool(hipStream_t stream, const BatchPool& q) {
  if (q.total <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_batch_pool, dim3((unsigned)((q.total + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

hipError_t launch_batch_outputs(hipStream_t stream, const float* logits, float* probs, long long n_images,
                                int n_classes, int out_units) {
  if (n_images <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_batch_outputs, dim3((unsigned)((n_images + 255) / 256)), dim3(256), 0, stream, (cgf)logits,
                     (gf)probs, n_images, n_classes, out_units);
  return hipGetLastError();
}

hipError_t launch_batch_pack(hipStream_t stream, const BatchPack& q, long long wt_floats) {
  hipLaunchKernelGGL(k_batch_zero, dim3((unsigned)((wt_floats + 255) / 256)), dim3(256), 0, stream, q.wt, wt_floats);
  hipLaunchKernelGGL(k_batch_pack, dim3((unsigned)((q.total + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

}  // namespace cnn355
