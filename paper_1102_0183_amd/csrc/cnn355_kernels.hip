// gfx950 kernels for on-line back-propagation training of the CNN variant of Ciresan et al.
// (IDSIA TR 01-11).  Every stage of the per-image step is a device function that processes
// one independent work item with one 256-thread workgroup (four 64-lane wavefronts), staging
// its operands through LDS.  The same functions run either as one kernel launch per stage or
// inside one persistent kernel whose stages are separated by grid barriers.
//
// Notation follows the paper: layer n has M maps; a K x K kernel moves over the valid region
// with skipping factor S (stride S+1) (Sec. 2.2); FP / BP / AW are the forward, delta and
// weight-adjusting phases of Sec. 3.2 - 3.4.
#include <hip/hip_runtime.h>

#if defined(__HIP_DEVICE_COMPILE__)
#define CNN_GLOBAL __attribute__((address_space(1)))
#endif
#include "cnn355_dev.h"

namespace cnn355 {

typedef CNN_GLOBAL float gfloat;  // a float in device (global) memory

// Scaled hyperbolic tangent of Sec. 4, constants as printed.
#define ACT_A 1.7159f
#define ACT_B 0.6666f
__device__ __forceinline__ float act_f(float a) { return ACT_A * tanhf(ACT_B * a); }
// Its derivative A B (1 - tanh^2(B a)) = 4 A B z / (1 + z)^2 with z = e^{-2B|a|}, from the sum a the unit
// received (the forward pass stores it wherever a delta can arrive: at the pooling winners and at the hidden
// fully connected units).  Written in terms of the output, A B - (B/A) y^2, the two terms cancel to 1e-3 of
// themselves at a saturated unit and fp32 keeps only 1e-4 of the result; here nothing cancels.
__device__ __forceinline__ float dact_pre_f(float a) {
  const float z = expf(-2.0f * ACT_B * fabsf(a));
  const float r = 1.0f / (1.0f + z);
  return (4.0f * ACT_A * ACT_B) * z * r * r;
}

// Optional fine-grained timestamps inside work items (development aid; compiled out unless
// CNN355_STAMPS is defined): workgroup 0 records 100 MHz ticks at numbered points.
#ifdef CNN355_STAMPS
__device__ unsigned long long g_dbg[64];
#define DBG(i) do { if (blockIdx.x == 0 && threadIdx.x == 0) g_dbg[i] = wall_clock64(); } while (0)
#else
#define DBG(i) do { } while (0)
#endif

struct Ctx {
  const gfloat* image;
  gfloat* probs_out;
  gfloat* grad_out;
  int label;
  int train;  // this image is trained on (0 for forward-only calls and for rejected labels)
  float lr;
};

// Sum of n_terms partial sums for each of n_out outputs, parts[k * n_out + o]: up to 64 lanes share an output
// (lane g adds the terms g, g + G, ... in that order, the G sums are then added across the lanes in a fixed
// pattern) instead of one lane walking a chain of n_terms dependent LDS reads.  The totals pass through
// res[n_out]; lane o < n_out returns output o.  Every lane of the workgroup must call it.
__device__ __forceinline__ float sum_terms(const float* parts, int n_terms, int n_out, float* res) {
  const int tid = threadIdx.x;
  int gl2 = 0;
  while (gl2 < 6 && (n_out << (gl2 + 1)) <= WG && (2 << gl2) <= n_terms) ++gl2;
  const int G = 1 << gl2, o = tid >> gl2, g = tid & (G - 1);
  float s = 0.f;
  if (o < n_out)
    for (int k = g; k < n_terms; k += G) s += parts[k * n_out + o];
  for (int off = G >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (o < n_out && g == 0) res[o] = s;
  __syncthreads();
  return tid < n_out ? res[tid] : 0.f;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// floor / ceiling of a quotient with positive divisor and possibly negative numerator
__device__ __forceinline__ int floor_div(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }
__device__ __forceinline__ int ceil_div(int a, int b) { return -floor_div(-a, b); }

// Copy n maps of map_sz floats each into LDS (dst[c * map_sz + o] = base[off_of(c) + o]).  Lane groups
// of 2^tw_log2 threads take one map each; every thread issues up to U independent,
// unconditional global loads before it waits, so the copy costs a few memory latencies instead
// of one per map (indices past the end are clamped to the last map and not stored).
template <int U, class OffOf>
__device__ __forceinline__ void stage_maps_u(float* dst, const gfloat* base, int n, int map_sz,
                                             int tw_log2, OffOf off_of) {
  const int tid = threadIdx.x;
  const int tw = 1 << tw_log2;
  const int tc = tid >> tw_log2, to = tid & (tw - 1), tcn = WG >> tw_log2;
  for (int c0 = tc; c0 < n; c0 += tcn * U) {
    int off[U];  // element offset of each map from `base` (32 bits: keeps the register count low)
#pragma unroll
    for (int u = 0; u < U; ++u) off[u] = off_of(min(c0 + u * tcn, n - 1));
    if (map_sz <= tw) {  // one step
      if (to < map_sz) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = base[off[u] + to];
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (c0 + u * tcn < n) dst[(c0 + u * tcn) * map_sz + to] = v[u];
      }
      continue;
    }
    // a map larger than the lanes that walk it: V steps of the walk at a time, so that U x V loads are in
    // flight before the first wait instead of U
    constexpr int V = U >= 8 ? 1 : (U == 4 ? 2 : 4);
    for (int o = to; o < map_sz; o += tw * V) {
      float v[V][U];
#pragma unroll
      for (int s = 0; s < V; ++s)
#pragma unroll
        for (int u = 0; u < U; ++u) v[s][u] = base[off[u] + min(o + s * tw, map_sz - 1)];
#pragma unroll
      for (int s = 0; s < V; ++s)
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (c0 + u * tcn < n && o + s * tw < map_sz) dst[(c0 + u * tcn) * map_sz + o + s * tw] = v[s][u];
    }
  }
}
// off_of(c) = element offset of map c from `base`
template <class OffOf>
__device__ __forceinline__ void stage_maps(float* dst, const gfloat* base, int n, int map_sz,
                                           int tw_log2, OffOf off_of) {
  const int tcn = WG >> tw_log2;
  if (n <= tcn) stage_maps_u<1>(dst, base, n, map_sz, tw_log2, off_of);
  else if (n <= 2 * tcn) stage_maps_u<2>(dst, base, n, map_sz, tw_log2, off_of);
  else if (n <= 4 * tcn) stage_maps_u<4>(dst, base, n, map_sz, tw_log2, off_of);
  else stage_maps_u<8>(dst, base, n, map_sz, tw_log2, off_of);
}

// First batch of a flat global -> LDS copy, split in two so that other loads can be issued
// between the two halves: prefetch_flat puts up to U elements per thread in flight (indices past
// the end are clamped), commit_flat stores them; copy_flat_rest handles what lies beyond U * WG.
template <int U, class T, class P>
__device__ __forceinline__ void prefetch_flat(T (&v)[U], P src, int n) {
#pragma unroll
  for (int u = 0; u < U; ++u) v[u] = src[min((int)threadIdx.x + u * WG, n - 1)];
}
template <int U, class T, class D>
__device__ __forceinline__ void commit_flat(const T (&v)[U], D* dst, int n) {
#pragma unroll
  for (int u = 0; u < U; ++u)
    if ((int)threadIdx.x + u * WG < n) dst[threadIdx.x + u * WG] = v[u];
}
template <int U, class D, class P>
__device__ __forceinline__ void copy_flat_rest(D* dst, P src, int n) {
  for (int base = U * WG; base < n; base += U * WG) {
    D v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = src[min(base + (int)threadIdx.x + u * WG, n - 1)];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + (int)threadIdx.x + u * WG < n) dst[base + threadIdx.x + u * WG] = v[u];
  }
}

// ------------------------------------------------------------------------------------------
// Fixed image-processing layer (Sec. 2.1): filter f correlated with raw channel src[f];
// no bias, no non-linearity, never trained.  One thread per output pixel.
// ------------------------------------------------------------------------------------------
__device__ void frontend_item(const FrontendDev& fe, int item, const gfloat* image) {
  const int idx = item * WG + threadIdx.x;
  const int hw = fe.H * fe.W;
  if (idx >= fe.n_filters * hw) return;
  const int f = idx / hw;
  const int rem = idx - f * hw;
  const int y = rem / fe.W, x = rem - y * fe.W;
  const gfloat* src = image + ((size_t)fe.src[f] * fe.Hr + y) * fe.Wr + x;
  const gfloat* flt = fe.filters + (size_t)f * fe.K * fe.K;
  float s = 0.f;
  for (int ky = 0; ky < fe.K; ++ky)
    for (int kx = 0; kx < fe.K; ++kx) s = fmaf(flt[ky * fe.K + kx], src[ky * fe.Wr + kx], s);
  fe.out[idx] = s;
}

// ------------------------------------------------------------------------------------------
// FP of a convolutional layer (Sec. 2.2, Sec. 3.2) fused with the max-pooling layer that
// follows it (Sec. 2.3).  Work item = (output map j, band of conv rows).  The connected input
// maps (rows under the band only) and their filters are staged through LDS chunk by chunk;
// every thread owns TT output pixels, or, when the band has fewer than 256 pixels, the
// connected maps are split R ways over the spare lanes and the partial sums are combined
// through LDS.  Epilogue: bias, scaled tanh, store, then the pooled maximum with the index of
// the first maximum in row-major order.
// ------------------------------------------------------------------------------------------
// multiply-accumulate over the maps c = c_first, c_first + R, ... of one staged chunk; the only
// part of the forward stage that is compiled once per kernel size (KT = 0: any size)
template <int KT, int TT>
__device__ __forceinline__ void conv_fwd_mac(const float* lds_in, const float* lds_w, int c_first,
                                             int n, int R, int map_sz, int Wi, int Krt, int Kxrt,
                                             const int (&base)[TT], float (&acc)[TT]) {
  const int K = KT ? KT : Krt, Kx = KT ? KT : Kxrt;  // KT: a square kernel of that size
  const int KK = K * Kx;
  for (int c = c_first; c < n; c += R) {
    const float* ip = lds_in + c * map_sz;
    const float* wp = lds_w + c * KK;
#pragma unroll
    for (int ky = 0; ky < K; ++ky) {
#pragma unroll
      for (int kx = 0; kx < Kx; ++kx) {
        const float wv = wp[ky * Kx + kx];
        const int off = ky * Wi + kx;
#pragma unroll
        for (int t = 0; t < TT; ++t) acc[t] = fmaf(wv, ip[base[t] + off], acc[t]);
      }
    }
  }
}

template <int TT>
__device__ void conv_fwd_item(const LayerDev& L, const Stage& st, int item,
                              const gfloat* in, float* lds) {
  const int tid = threadIdx.x;
  const int K = L.K, Kx = L.Kx;
  const int KK = K * Kx;
  const int Wi = L.Wi, Wo = L.Wo, Ho = L.Ho;
  const int stride = L.S + 1, stride_x = L.Sx + 1;
  // st.rows_per_wg (> 1) output maps per work item, one after the other: they read the same input maps (full
  // table, one chunk), which are staged once
  const int mp = max(st.rows_per_wg, 1);
  const int jg = item / st.n_tiles;
  const int tile = item - jg * st.n_tiles;
  const int y0 = tile * st.tile_rows;
  const int rows = min(st.tile_rows, Ho - y0);
  const int P = rows * Wo;
  const int map_sz = ((rows - 1) * stride + K) * Wi;
  const int in_map = L.Hi * Wi;
  const gfloat* in0 = in + (size_t)y0 * stride * Wi;

  float* lds_in = lds;
  float* lds_w = lds + LDS_IN;
  float* lds_part = lds + LDS_IN + LDS_AUX + LDS_AUX2;
  float* lds_out = lds_part + WG;
  float* lds_pre = lds_w;  // the sums the tile's units received: kept (once the filters are done with) for the
                           // derivative at the pooling winners
  const int Kp = L.Kp, Kpx = L.Kpx;
  const bool pooled = Kp > 1 || Kpx > 1;

  DBG(0);
  for (int jj = 0; jj < mp; ++jj) {
  const int j = jg * mp + jj;
  if (j >= L.Mo) break;
  const float b = L.bias[j];  // issued first, used last
  int c_begin = j * L.Mi, n_conn = L.Mi;
  if (!L.full_table) {
    c_begin = L.csr_ptr[j];
    n_conn = L.csr_ptr[j + 1] - c_begin;
  }
  DBG(1);

  int R = 1, r = 0, p0 = tid;
  if (TT == 1) {
    R = max(1, min(WG / P, min(st.chunk, n_conn)));  // P <= WG here; no more ways than one chunk has connections
    r = tid / P;
    p0 = tid - r * P;
  }
  float acc[TT];
  int base[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int p = p0 + t * WG;
    const bool ok = (r < R) && (p < P);
    const int y = p / Wo, x = p - y * Wo;
    base[t] = ok ? (y * stride * Wi + x * stride_x) : 0;  // idle lanes read a valid address, result unused
    acc[t] = 0.f;
  }

  for (int c0 = 0; c0 < n_conn; c0 += st.chunk) {
    const int n = min(st.chunk, n_conn - c0);
    const gfloat* wsrc = L.w + (size_t)(c_begin + c0) * KK;
    float wv[4];
    prefetch_flat(wv, wsrc, n * KK);  // filters in flight together with the input maps
    if (jj > 0) {
      // (the maps the first output map of this item staged are the ones this one reads)
    } else if (L.full_table)  // uniform: input map of slot c is c itself
      stage_maps(lds_in, in0, n, map_sz, st.tw_log2, [&](int c) { return (c0 + c) * in_map; });
    else
      stage_maps(lds_in, in0, n, map_sz, st.tw_log2,
                 [&](int c) { return L.csr_idx[c_begin + c0 + c] * in_map; });
    DBG(2);
    commit_flat(wv, lds_w, n * KK);
    copy_flat_rest<4>(lds_w, wsrc, n * KK);
    __syncthreads();
    DBG(3);
    {
      const int c_first = min(r, R - 1);  // lanes beyond the R splits repeat split R-1, unused
      switch (K == Kx ? K : 0) {  // compiled sizes are square; any other kernel takes the run-time loop
        case 2: conv_fwd_mac<2, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
        case 3: conv_fwd_mac<3, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
        case 4: conv_fwd_mac<4, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
        case 5: conv_fwd_mac<5, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
        case 6: conv_fwd_mac<6, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
        default: conv_fwd_mac<0, TT>(lds_in, lds_w, c_first, n, R, map_sz, Wi, K, Kx, base, acc); break;
      }
    }
    __syncthreads();
    DBG(4);
  }

  if (TT == 1 && R > 1) {
    if (r < R) lds_part[tid] = acc[0];  // tid == r * P + p0
    __syncthreads();
    acc[0] = sum_terms(lds_part, R, P, lds_out);
  }
  DBG(5);
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int p = tid + t * WG;
    if (p < P && (TT > 1 || r == 0)) {
      const float sum = acc[t] + b;
      const float a = act_f(sum);
      L.act[((size_t)j * Ho + y0) * Wo + p] = a;
      lds_out[p] = a;
      lds_pre[p] = sum;
      if (!pooled) L.dact[((size_t)j * Ho + y0) * Wo + p] = dact_pre_f(sum);
    }
  }
  __syncthreads();
  DBG(6);
  if (pooled) {
    const int Wp = L.Wp;
    const int nq = (rows / Kp) * Wp;
    for (int q = tid; q < nq; q += WG) {
      const int py = q / Wp, px = q - py * Wp;
      const float* win = lds_out + py * Kp * Wo + px * Kpx;
      float best = win[0];
      int wy = 0, wx = 0;
      for (int dy = 0; dy < Kp; ++dy)
        for (int dx = 0; dx < Kpx; ++dx) {
          const float v = win[dy * Wo + dx];
          if (v > best) { best = v; wy = dy; wx = dx; }
        }
      const size_t o = ((size_t)j * L.Hp + (y0 / Kp + py)) * Wp + px;
      L.out[o] = best;
      L.dact[o] = dact_pre_f(lds_pre[(py * Kp + wy) * Wo + px * Kpx + wx]);
      L.arg[o] = (uint8_t)(wy * Kpx + wx);
      L.argyx[o] = ((y0 + py * Kp + wy) << 16) | (px * Kpx + wx);
    }
    __syncthreads();
  }
  }
  DBG(7);
}

// ------------------------------------------------------------------------------------------
// FP of a wide, fully connected-table convolutional layer as an implicit GEMM on the matrix
// cores (fp32 MFMA).  C[j][p] = sum_k W[j][k] X[k][p] with k = (input map i, tap ky, kx) and
// p = output pixel: W is the layer's filter block as it lies in memory (row j holds Mi*K*K
// contiguous floats), X is never formed: X[k][p] = in_i[(y(S+1)+ky) Wi + x(S+1)+kx] is the
// sum of an offset that depends on k only and one that depends on p only.
// Work item = (tile of 32 output maps, slice of the input maps).  The slice's input maps and
// the 32 x (maps*K*K) block of filters are staged through LDS chunk by chunk; each wavefront
// owns one (or several) tiles of 32 pixels, and when there are fewer pixel tiles than
// wavefronts the spare ones split the chunk's k range.  v_mfma_f32_32x32x2_f32: lane l feeds
// A[l%32][l/32] and B[l/32][l%32], two k per instruction, 16 accumulators per lane.
// The partial sums of every (slice, k split) go to their own plane of mm_part; ST_CONV_EPI
// adds the planes in a fixed order (no atomics: results do not depend on timing).
// ------------------------------------------------------------------------------------------
typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int MM_TPW = 4;  // pixel tiles one wavefront can carry (64 accumulators)

// BWD = false: FP, rows = output maps, contraction over (input map, tap), staged maps = the
// layer's inputs.  BWD = true: the delta pull of Sec. 3.3 as FP's mirror image (skipping factor 0
// only): rows = input maps i, contraction over (output map j, tap), staged maps = the deltas of
// the output maps put at their winners' places inside (Hi+K-1) x (Wi+K-1) zeros, so that
//   g_i[r][c] = sum_j sum_{ky,kx} D_j[r + K-1-ky][c + K-1-kx] w_{j,i}[ky][kx]
// has the same operand pattern in[koff(k) + pbase(p)] as FP; the weights are used as they lie
// (the tap order is turned round in koff instead).  One plane of partial sums per work item.
template <bool BWD>
__device__ void conv_mfma_item(const LayerDev& L, const Stage& st, int item, const gfloat* in, float* lds) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int lrow = lane & 31, lk = lane >> 5;
  const int KS = st.n_tiles;
  const int jt = item / KS, ks = item - jt * KS;
  const int j0 = jt * 32;
  const int K = L.K, KK = K * K;
  // rows of the product, maps contracted over, size and row pitch of a staged map, output pixels
  const int Mo = BWD ? L.Mi : L.Mo, Mi = BWD ? L.Mo : L.Mi;
  const int Wi = BWD ? L.Wi + K - 1 : L.Wi, HiWi = BWD ? (L.Hi + K - 1) * (L.Wi + K - 1) : L.Hi * L.Wi;
  const int Wo = BWD ? L.Wi : L.Wo, P = BWD ? L.Hi * L.Wi : L.Ho * L.Wo, stride = BWD ? 1 : L.S + 1;
  const int per = (Mi + KS - 1) / KS;
  const int i_lo = ks * per, i_hi = min(Mi, i_lo + per);
  const int IC = st.chunk;
  const int WP = IC * KK + 1 + ((IC * KK) & 1);   // odd row pitch: the 32 rows of a column lie in 32 banks
  const int NT = (P + 31) >> 5;
  constexpr int WAVES = WG / 64;
  const int NTw = min(NT, WAVES);
  const int KW = (NT >= WAVES) ? 1 : WAVES / NT;
  const int kw = (NT >= WAVES) ? 0 : wave / NT;
  const int tw = (NT >= WAVES) ? wave : wave - kw * NT;
  const bool wave_on = kw < KW;

  float* lds_in = lds;                         // [IC][Hi*Wi]
  float* lds_w = lds + IC * HiWi;              // [32][WP]
  int* koff = (int*)(lds_w + 32 * WP);         // [IC*KK] offset of k inside the staged maps

  for (int x = tid; x < IC * KK; x += WG) {
    const int c = x / KK, t = x - c * KK;
    const int ky = t / K, kx = t - ky * K;
    koff[x] = BWD ? c * HiWi + (K - 1 - ky) * Wi + (K - 1 - kx) : c * HiWi + ky * Wi + kx;
  }
  int pbase[MM_TPW];
#pragma unroll
  for (int t = 0; t < MM_TPW; ++t) {
    const int p = (tw + t * NTw) * 32 + lrow;
    const int y = p / Wo, x = p - y * Wo;
    pbase[t] = (p < P) ? (y * Wi + x) * stride : 0;
  }
  v16f acc[MM_TPW];
#pragma unroll
  for (int t = 0; t < MM_TPW; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  const int n_my_tiles = wave_on ? ((NT - tw + NTw - 1) / NTw) : 0;   // 1 unless there are more than 16 pixel tiles

  for (int ic0 = i_lo; ic0 < i_hi; ic0 += IC) {
    const int n_ic = min(IC, i_hi - ic0);
    const int kc = n_ic * KK;
    if constexpr (!BWD) {  // stage the chunk, eight loads in flight per lane: the inputs (one contiguous block) ...
      const gfloat* src = in + (size_t)ic0 * HiWi;
      const int n_in = n_ic * HiWi;
      for (int x0 = 0; x0 < n_in; x0 += 8 * WG) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[min(x0 + u * WG + tid, n_in - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (x0 + u * WG + tid < n_in) lds_in[x0 + u * WG + tid] = v[u];
      }
      // ... and the 32 filter rows (one contiguous run of kc floats each; 32 lanes per row)
      const int r = tid >> 5, xl = tid & 31;
      const bool row_ok = j0 + r < Mo;
      const gfloat* wr = L.w + ((size_t)min(j0 + r, Mo - 1) * Mi + ic0) * KK;
      for (int x0 = 0; x0 < kc; x0 += 8 * 32) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = wr[min(x0 + u * 32 + xl, kc - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (x0 + u * 32 + xl < kc) lds_w[r * WP + x0 + u * 32 + xl] = row_ok ? v[u] : 0.f;
      }
    } else {
      // the filters w_{j,i} of the chunk's output maps j and the 32 input maps i of this tile: for
      // one j they are 32 * KK consecutive floats (i runs fastest after the tap)
      const int n_rows = min(32, Mo - j0);
      const int run = n_rows * KK, tot = n_ic * run;
      for (int x0 = 0; x0 < tot; x0 += 8 * WG) {
        float v[8];
        int d[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int x = min(x0 + u * WG + tid, tot - 1);
          const int jj = x / run, rem = x - jj * run;
          const int r = rem / KK, t = rem - r * KK;
          v[u] = L.w[((size_t)(ic0 + jj) * Mo + j0) * KK + rem];
          d[u] = r * WP + jj * KK + t;
        }
        if (x0 == 0) {  // the zero fill overlaps the first batch of loads
          for (int x = tid; x < n_ic * HiWi; x += WG) lds_in[x] = 0.f;
          if (n_rows < 32)
            for (int x = tid; x < (32 - n_rows) * WP; x += WG) lds_w[n_rows * WP + x] = 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (x0 + u * WG + tid < tot) lds_w[d[u]] = v[u];
      }
      __syncthreads();
      // the chunk's deltas, each to its winner's place inside the zeros
      const int HW = L.Hp * L.Wp, ntot = n_ic * HW;
      for (int x0 = 0; x0 < ntot; x0 += 4 * WG) {
        float dv[4];
        int yx[4], cc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int x = min(x0 + u * WG + tid, ntot - 1);
          cc[u] = x / HW;
          const size_t o = (size_t)(ic0 + cc[u]) * HW + (x - cc[u] * HW);
          yx[u] = L.argyx[o];
          dv[u] = L.delta[o];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (x0 + u * WG + tid < ntot)
            lds_in[cc[u] * HiWi + ((yx[u] >> 16) + K - 1) * Wi + (yx[u] & 0xffff) + K - 1] = dv[u];
      }
    }
    __syncthreads();
    if (wave_on) {
      // this wavefront's share of the chunk's k range (even bounds: two k per instruction);
      // four instructions' operands are fetched from LDS together
      const int kper = (((kc + KW - 1) / KW) + 1) & ~1;
      const int k_lo = kw * kper, k_hi = min(kc, k_lo + kper);
      for (int kk = k_lo; kk < k_hi; kk += 8) {
        float a[4];
        int ko[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = kk + 2 * u + lk;
          a[u] = (k < k_hi) ? lds_w[lrow * WP + min(k, kc - 1)] : 0.f;
          ko[u] = koff[min(k, kc - 1)];
        }
#pragma unroll
        for (int t = 0; t < MM_TPW; ++t)
          if (t < n_my_tiles) {
            float b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) b[u] = lds_in[ko[u] + pbase[t]];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc[t], 0, 0, 0);
          }
      }
    }
    __syncthreads();
  }
  // the k splits inside the workgroup are added here (through LDS, in a fixed order), so that one
  // work item leaves one plane of partial sums
  gfloat* plane = L.mm_part + (size_t)ks * Mo * P;
  if (KW > 1) {
    float* red = lds;  // [KW][NT][32 rows][32 pixels]
    if (wave_on) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        red[((kw * NT + tw) * 32 + (v >> 2) * 8 + lk * 4 + (v & 3)) * 32 + lrow] = acc[0][v];
    }
    __syncthreads();
    for (int x = tid; x < NT * 1024; x += WG) {
      const int t = x >> 10, row = (x >> 5) & 31, col = x & 31;
      float sum = 0.f;
      for (int q = 0; q < KW; ++q) sum += red[((q * NT + t) * 32 + row) * 32 + col];
      const int p = t * 32 + col, j = j0 + row;
      if (p < P && j < Mo) plane[(size_t)j * P + p] = sum;
    }
    __syncthreads();
  } else if (wave_on) {
#pragma unroll
    for (int t = 0; t < MM_TPW; ++t)
      if (t < n_my_tiles) {
        const int p = (tw + t * NTw) * 32 + lrow;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int j = j0 + (v >> 2) * 8 + lk * 4 + (v & 3);
          if (p < P && j < Mo) plane[(size_t)j * P + p] = acc[t][v];
        }
      }
  }
}

// Second half of the matrix-core forward pass.  Work item = output map j: add the planes of
// partial sums (lane groups share the planes, eight loads in flight per lane, fixed order), bias,
// scaled tanh, store; then the pooled maximum with the index of the first maximum in row-major
// order, exactly as the one-stage forward kernel does.
__device__ void conv_epi_item(const LayerDev& L, const Stage& st, int item, float* lds) {
  const int tid = threadIdx.x;
  const int Wo = L.Wo, Ho = L.Ho, P = Ho * Wo, Mo = L.Mo;
  const int n_planes = st.rows_per_wg;
  // st.chunk maps per work item, side by side in the lanes (one map when it has more pixels than half the lanes)
  const int mp = st.chunk;
  const int lpm = WG / mp;                // lanes of one map
  float* lds_out = lds;                   // [mp][P]
  float* lds_part = lds + MAX_TILE_PIX;   // [mp][G][P] partial sums of the plane groups
  float* lds_pre = lds_part + WG;         // [mp][P] the sums the maps' units received, for the derivative at the winners
  const bool pooled = L.Kp > 1;
  const int slot = (P >= WG) ? 0 : tid / lpm, lt = (P >= WG) ? tid : tid - slot * lpm;
  const int j = item * mp + slot;
  const bool mine = slot < mp && j < Mo;
  const float b = mine ? L.bias[j] : 0.f;
  // G lane groups of P lanes each take every G-th block of 8 planes
  const int G = (P >= WG) ? 1 : min(lpm / P, (n_planes + 7) / 8);
  const int grp = (P >= WG) ? 0 : lt / P;
  for (int p0 = 0; p0 < P; p0 += WG) {
    const int p = (P >= WG) ? p0 + tid : lt - grp * P;
    const bool on = mine && grp < G && p < P;
    float s = 0.f;
    if (on)
      for (int s0 = grp * 8; s0 < n_planes; s0 += G * 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = L.mm_part[((size_t)min(s0 + u, n_planes - 1) * Mo + j) * P + p];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (s0 + u < n_planes) ? v[u] : 0.f;
      }
    if (G > 1) {
      if (on) lds_part[slot * lpm + grp * P + p] = s;
      __syncthreads();
      if (mine && lt < P) {
        s = 0.f;
        for (int q = 0; q < G; ++q) s += lds_part[slot * lpm + q * P + lt];
      }
    }
    if ((G > 1) ? (mine && lt < P) : on) {
      const int pp = (G > 1) ? lt : p;
      const float a = act_f(s + b);
      L.act[(size_t)j * P + pp] = a;
      lds_out[slot * P + pp] = a;
      lds_pre[slot * P + pp] = s + b;
      if (!pooled) L.dact[(size_t)j * P + pp] = dact_pre_f(s + b);
    }
  }
  __syncthreads();
  const int Kp = L.Kp;
  if (pooled) {
    const int Wp = L.Wp;
    const int nq = L.Hp * Wp;
    for (int x = tid; x < mp * nq; x += WG) {
      const int sl = x / nq, q = x - sl * nq;
      const int jj = item * mp + sl;
      if (jj >= Mo) break;
      const int py = q / Wp, px = q - py * Wp;
      const float* win = lds_out + sl * P + py * Kp * Wo + px * Kp;
      float best = win[0];
      int wy = 0, wx = 0;
      for (int dy = 0; dy < Kp; ++dy)
        for (int dx = 0; dx < Kp; ++dx) {
          const float v = win[dy * Wo + dx];
          if (v > best) { best = v; wy = dy; wx = dx; }
        }
      const size_t o = (size_t)jj * nq + q;
      L.out[o] = best;
      L.dact[o] = dact_pre_f(lds_pre[sl * P + (py * Kp + wy) * Wo + px * Kp + wx]);
      L.arg[o] = (uint8_t)(wy * Kp + wx);
      L.argyx[o] = ((py * Kp + wy) << 16) | (px * Kp + wx);
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Hidden fully connected layer forward (Sec. 2.4) + scaled tanh.  Work item = rows_per_wg
// neurons; the lanes of a neuron stride over its inputs, then reduce by wave shuffles and LDS.
// ------------------------------------------------------------------------------------------
__device__ void fc_fwd_item(const LayerDev& L, const Stage& st, int item,
                            const gfloat* v, float* lds) {
  const int tid = threadIdx.x;
  const int rpw = st.rows_per_wg;
  const int lpr = WG / rpw;  // lanes per neuron: 64 .. 1024
  const int row = item * rpw + tid / lpr;
  const int lane = tid & (lpr - 1);
  const int n_in = L.n_in;
  const float bias = (tid < rpw && item * rpw + tid < L.n_out) ? L.bias[item * rpw + tid] : 0.f;
  float s = 0.f;
  if (row < L.n_out) {
    const gfloat* wr = L.w + (size_t)row * n_in;
#pragma unroll 8
    for (int m = lane; m < n_in; m += lpr) s = fmaf(wr[m], v[m], s);
  }
  s = wave_sum(s);
  float* part = lds + LDS_IN + LDS_AUX + LDS_AUX2;
  if ((tid & 63) == 0) part[tid >> 6] = s;
  __syncthreads();
  if (tid < rpw) {
    const int wpr = lpr >> 6;  // waves per neuron
    float t = 0.f;
    for (int k = 0; k < wpr; ++k) t += part[tid * wpr + k];
    const int rr = item * rpw + tid;
    if (rr < L.n_out) {
      L.act[rr] = act_f(t + bias);
      L.dact[rr] = dact_pre_f(t + bias);
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Output layer (Sec. 2.4): logits, soft-max, cross-entropy error and output delta
// delta_k = p_k - [k == label]; when training, the same workgroup then pulls the deltas of the
// layer below (g_m = sum_k W[k][m] delta_k with W still at its old value, times the activation
// derivative, Sec. 3.3) and adjusts W and the bias (Sec. 3.4) in the same pass over W.
// One work item.
// ------------------------------------------------------------------------------------------
__device__ void head_item(const LayerDev& L, const LayerDev* Lp, const gfloat* v,
                          const Ctx& ctx, StatusDev* status, float* lds) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int N = L.n_out, n_in = L.n_in;
  float* lds_W = lds;                 // copy of W when it fits (N * n_in <= LDS_IN)
  float* logit = lds + LDS_IN;
  float* dl = lds + LDS_IN + LDS_AUX;
  const bool cached = N * n_in <= LDS_IN;
  DBG(10);
#ifdef CNN355_STAMPS
  {  // probe: one load of fresh data (written by the previous stage), one of old data, timed alone
    float probe = v[tid % n_in];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    DBG(30);
    float probe2 = L.w[tid];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    DBG(31);
    float probe3 = v[(tid + 64) % n_in];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    DBG(32);
    float probe4 = L.w[tid + 700];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    DBG(33);
    if (probe + probe2 + probe3 + probe4 == 123.456f) lds[0] = probe;
  }
#endif
  {
    // lane groups of 2^lpl lanes per output neuron, as many neurons side by side as fit
    int lpl = 6;
    while (lpl > 0 && (WG >> lpl) < N) --lpl;
    const int lpr = 1 << lpl, rows_pp = WG >> lpl;
    const int sub = tid & (lpr - 1);
    for (int k0 = 0; k0 < N; k0 += rows_pp) {
      const int k = k0 + (tid >> lpl);
      const float bk = (sub == 0 && k < N) ? L.bias[k] : 0.f;
      float s = 0.f;
      if (k < N) {
        const gfloat* wr = L.w + (size_t)k * n_in;
        if (cached) {
#pragma unroll 8
          for (int m = sub; m < n_in; m += lpr) {
            const float w = wr[m];
            lds_W[k * n_in + m] = w;
            s = fmaf(w, v[m], s);
          }
        } else {
#pragma unroll 8
          for (int m = sub; m < n_in; m += lpr) s = fmaf(wr[m], v[m], s);
        }
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1)
        if (off < lpr) s += __shfl_xor(s, off, 64);
      if (sub == 0 && k < N) logit[k] = s + bk;
    }
  }
  __syncthreads();
  DBG(11);
  if (wave == 0 && L.out_units == 1) {
    // scaled-tanh output neurons (Sec. 4), squared error against targets +1 (the image's class) / -1
    float e = 0.f;
    for (int k = lane; k < N; k += 64) {
      const float y = act_f(logit[k]);
      const float t = (k == ctx.label) ? 1.f : -1.f;
      L.act[k] = y;
      if (ctx.probs_out) ctx.probs_out[k] = y;
      const float d = (y - t) * dact_pre_f(logit[k]);
      dl[k] = d;
      e = fmaf(y - t, y - t, e);
      if (ctx.train) L.delta[k] = d;
    }
    e = wave_sum(e);
    if (ctx.train && lane == 0) status->loss = 0.5f * e;
  } else if (wave == 0) {
    float mx = -INFINITY;
    for (int k = lane; k < N; k += 64) mx = fmaxf(mx, logit[k]);
    mx = wave_max(mx);
    // the label's delta p - 1 = -(sum of the other classes' exponentials) / z: summed apart from the label's
    // own term, so that a confident net (p -> 1) loses no digits of it
    float zo = 0.f;
    for (int k = lane; k < N; k += 64) zo += (k == ctx.label) ? 0.f : expf(logit[k] - mx);
    zo = wave_sum(zo);
    const bool has_label = ctx.label >= 0 && ctx.label < N;
    const float z = zo + (has_label ? expf(logit[has_label ? ctx.label : 0] - mx) : 0.f);
    for (int k = lane; k < N; k += 64) {
      const float p = expf(logit[k] - mx) / z;
      L.act[k] = p;
      if (ctx.probs_out) ctx.probs_out[k] = p;
      const float d = (k == ctx.label) ? -zo / z : p;
      dl[k] = d;
      if (ctx.train) {
        L.delta[k] = d;
        if (k == ctx.label) status->loss = -logf(p);
      }
    }
  }
  __syncthreads();
  DBG(12);
  if (!ctx.train) return;
  const float lr = ctx.lr;
  gfloat* g_out = ctx.grad_out;
  for (int m = tid; m < n_in; m += WG) {
    const float vm = v[m];
    float g = 0.f;
    if (cached) {
#pragma unroll 4
      for (int k = 0; k < N; ++k) {
        const float w = lds_W[k * n_in + m];
        const float d = dl[k];
        g = fmaf(w, d, g);
        if (g_out) g_out[L.w_canon + (size_t)k * n_in + m] = d * vm;
        else L.w[(size_t)k * n_in + m] = w - lr * (d * vm);
      }
    } else {
#pragma unroll 8
      for (int k = 0; k < N; ++k) {
        gfloat* wp = L.w + (size_t)k * n_in + m;
        const float w = *wp;
        const float d = dl[k];
        g = fmaf(w, d, g);
        if (g_out) g_out[L.w_canon + (size_t)k * n_in + m] = d * vm;
        else *wp = w - lr * (d * vm);
      }
    }
    if (Lp) Lp->delta[m] = g * Lp->dact[m];
  }
  DBG(13);
  for (int k = tid; k < N; k += WG) {
    if (g_out) g_out[L.b_canon + k] = dl[k];
    else L.bias[k] -= lr * dl[k];
  }
  __syncthreads();
  DBG(14);
}

// ------------------------------------------------------------------------------------------
// Hidden fully connected layer backward: pull deltas for the layer below through W (old
// values), multiply by the activation derivative (Sec. 3.3), and adjust W in the same pass
// (Sec. 3.4: dE/dW[k][m] = delta_k v_m).  Work item = tile of CM input columns; the 256/CM lane
// groups split the rows of W and combine through LDS.
// ------------------------------------------------------------------------------------------
__device__ void fc_bwd_item(const LayerDev& L, const LayerDev* Lp, const Stage& st, int item,
                            const gfloat* v, const Ctx& ctx, float* lds) {
  const int tid = threadIdx.x;
  const int cml = st.cm_log2, CM = 1 << cml, KS = WG >> cml;
  const int ks = tid >> cml, cm = tid & (CM - 1);
  const int m = item * CM + cm;
  const int N = L.n_out, n_in = L.n_in;
  float* dl = lds + LDS_IN;
  float* part = lds + LDS_IN + LDS_AUX + LDS_AUX2;
  // every global load this item needs is issued before the first wait: this column's first FB
  // weights (rows ks, ks + KS, ...), its input, and the layer's deltas
  constexpr int FB = 4;
  const int mc = min(m, n_in - 1);
  float wv[FB];
#pragma unroll
  for (int u = 0; u < FB; ++u) wv[u] = L.w[(size_t)min(ks + u * KS, N - 1) * n_in + mc];
  const float vm = v[mc];
  for (int k = tid; k < N; k += WG) dl[k] = L.delta[k];
  __syncthreads();
  const float lr = ctx.lr;
  gfloat* g_out = ctx.grad_out;
  float g = 0.f;
  if (m < n_in) {
#pragma unroll
    for (int u = 0; u < FB; ++u) {
      const int k = ks + u * KS;
      if (k < N) {
        const float d = dl[k];
        g = fmaf(wv[u], d, g);
        if (g_out) g_out[L.w_canon + (size_t)k * n_in + m] = d * vm;
        else L.w[(size_t)k * n_in + m] = wv[u] - lr * (d * vm);
      }
    }
    // the rows beyond, FB2 at a time: all their loads first, then the arithmetic and the stores (a store to one
    // row of W and a load from another cannot be told apart by the compiler, which would run them one by one)
    constexpr int FB2 = 8;
    if (N <= (FB + 2) * KS) {  // (a row or two: nothing to batch)
      for (int k = ks + FB * KS; k < N; k += KS) {
        gfloat* wp = L.w + (size_t)k * n_in + m;
        const float w = *wp;
        const float d = dl[k];
        g = fmaf(w, d, g);
        if (g_out) g_out[L.w_canon + (size_t)k * n_in + m] = d * vm;
        else *wp = w - lr * (d * vm);
      }
    } else
    for (int k0 = ks + FB * KS; k0 < N; k0 += FB2 * KS) {
      float wn[FB2];
#pragma unroll
      for (int u = 0; u < FB2; ++u) wn[u] = (k0 + u * KS < N) ? L.w[(size_t)(k0 + u * KS) * n_in + m] : 0.f;
#pragma unroll
      for (int u = 0; u < FB2; ++u) {
        const int k = k0 + u * KS;
        if (k < N) {
          const float d = dl[k];
          g = fmaf(wn[u], d, g);
          if (g_out) g_out[L.w_canon + (size_t)k * n_in + m] = d * vm;
          else L.w[(size_t)k * n_in + m] = wn[u] - lr * (d * vm);
        }
      }
    }
  }
  part[tid] = g;
  __syncthreads();
  if (ks == 0 && m < n_in && Lp) {
    float s = 0.f;
    for (int kk = 0; kk < KS; ++kk) s += part[kk * CM + cm];
    Lp->delta[m] = s * Lp->dact[m];
  }
  if (item == 0) {
    for (int k = tid; k < N; k += WG) {
      if (g_out) g_out[L.b_canon + k] = dl[k];
      else L.bias[k] -= lr * dl[k];
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------
// BP through a convolutional layer in pull form (Sec. 3.3).  Neuron (r, c) of input map i
// collects, over every output map j that reads map i, the deltas of the output neurons whose
// K x K receptive field covers it:
//   max(ceil((r-K+1)/(S+1)), 0) <= y <= min(floor(r/(S+1)), Ho-1)   (and the same in x),
// each times w_{j,i}[r - y(S+1)][c - x(S+1)] (old value).  After max-pooling only the winner of
// each rectangle carries a delta: the staged chunk of delta maps is rebuilt at full resolution
// in LDS (zero-fill, then scatter the winners), so the inner loop is the plain rectangle of the
// paper with no data-dependent addressing.  Epilogue: times the activation derivative of the
// layer below.  Work item = (input map i, tile of PT input pixels); the 256/PT lane groups
// split the output maps and combine through LDS.
// ------------------------------------------------------------------------------------------
template <int KT>
__device__ __forceinline__ float conv_bwd_mac(const float* lds_d, const float* lds_w, int c_first, int n,
                                              int R, int HWd, const int (&yo)[5], const int (&xo)[5],
                                              float acc) {
  for (int c = c_first; c < n; c += R) {
    const float* dp = lds_d + c * HWd;
    const float* wp = lds_w + c * (KT * KT);
#pragma unroll
    for (int ky = 0; ky < KT; ++ky)
#pragma unroll
      for (int kx = 0; kx < KT; ++kx) acc = fmaf(dp[yo[ky] + xo[kx]], wp[ky * KT + kx], acc);
  }
  return acc;
}

__device__ void conv_bwd_item(const LayerDev& L, const LayerDev& Lp, const Stage& st, int item,
                              float* lds) {
  const int tid = threadIdx.x;
  const int K = L.K, Kx = L.Kx;
  const int KK = K * Kx;
  const int stride = L.S + 1, stride_x = L.Sx + 1;
  const int Wi = L.Wi, Pin = L.Hi * L.Wi;
  const int Ho = L.Ho, Wo = L.Wo, HW = L.Hp * L.Wp;
  // the staged delta maps carry one extra row and one extra column of zeros: a kernel tap that
  // has no output neuron (border, or a skipped position) reads a zero instead of branching
  const int Wd = Wo + 1, HWd = (Ho + 1) * Wd;
  const int i = item / st.n_tiles;
  const int tile = item - i * st.n_tiles;
  const int ptl = st.tw_log2;              // log2 of the pixel tile
  const int PT = 1 << ptl, R = WG >> ptl;
  const int r = tid >> ptl;
  const int p = tile * PT + (tid & (PT - 1));
  const bool active = p < Pin;
  const int pr = p / Wi, pc = p - pr * Wi;

  float* lds_d = lds;                       // [chunk][(Ho+1)*(Wo+1)] deltas at full resolution
  float* lds_w = lds + LDS_IN;              // [chunk][K*K]
  float* lds_part = lds + LDS_IN + LDS_AUX + LDS_AUX2;

  // tap ky of the kernel reaches output row (pr - ky) / (S+1) when that is a whole, existing
  // row (the inequalities of Sec. 3.3 solved tap by tap); otherwise the zero row
  auto row_off = [&](int ky) {
    const int ry = pr - ky;
    const int y = ry / stride;
    const bool ok = active && ry >= 0 && ry - y * stride == 0 && y < Ho;
    return (ok ? y : Ho) * Wd;
  };
  auto col_off = [&](int kx) {
    const int rx = pc - kx;
    const int x = rx / stride_x;
    const bool ok = active && rx >= 0 && rx - x * stride_x == 0 && x < Wo;
    return ok ? x : Wo;
  };
  int yo[5], xo[5];
#pragma unroll
  for (int k = 0; k < 5; ++k) { yo[k] = row_off(k); xo[k] = col_off(k); }

  int j_begin = 0, nj = L.Mo;
  if (!L.full_table) {
    j_begin = L.csc_ptr[i];
    nj = L.csc_ptr[i + 1] - j_begin;
  }
  float acc = 0.f;
  constexpr int BU = 4;  // loads in flight per thread and array
  for (int j0 = 0; j0 < nj; j0 += st.chunk) {
    const int n = min(st.chunk, nj - j0);
    // filters of the chunk, gathered: entry c of the chunk uses weight slot (j, i)
    for (int base = 0; base < n * KK; base += BU * WG) {
      float wv[BU];
#pragma unroll
      for (int u = 0; u < BU; ++u) {
        const int idx = min(base + tid + u * WG, n * KK - 1);
        const int c = idx / KK, t = idx - c * KK;
        const int slot = L.full_table ? ((j0 + c) * L.Mi + i) : L.csc_slot[j_begin + j0 + c];
        wv[u] = L.w[(size_t)slot * KK + t];
      }
      if (base == 0)  // the zero fill overlaps the first batch of loads
        for (int idx = tid; idx < n * HWd; idx += WG) lds_d[idx] = 0.f;
#pragma unroll
      for (int u = 0; u < BU; ++u)
        if (base + tid + u * WG < n * KK) lds_w[base + tid + u * WG] = wv[u];
    }
    __syncthreads();
    // winners' deltas scattered to their place in the zeroed full-resolution maps
    for (int base = 0; base < n * HW; base += BU * WG) {
      float dv[BU];
      int yxv[BU], cv[BU];
#pragma unroll
      for (int u = 0; u < BU; ++u) {
        const int idx = min(base + tid + u * WG, n * HW - 1);
        const int c = idx / HW, q = idx - c * HW;
        const int j = L.full_table ? (j0 + c) : L.csc_j[j_begin + j0 + c];
        cv[u] = c;
        yxv[u] = L.argyx[(size_t)j * HW + q];
        dv[u] = L.delta[(size_t)j * HW + q];
      }
#pragma unroll
      for (int u = 0; u < BU; ++u)
        if (base + tid + u * WG < n * HW)
          lds_d[cv[u] * HWd + (yxv[u] >> 16) * Wd + (yxv[u] & 0xffff)] = dv[u];
    }
    __syncthreads();
    switch (K == Kx ? K : 0) {  // compiled sizes are square; any other kernel takes the run-time loop
      case 1: acc = conv_bwd_mac<1>(lds_d, lds_w, r, n, R, HWd, yo, xo, acc); break;
      case 2: acc = conv_bwd_mac<2>(lds_d, lds_w, r, n, R, HWd, yo, xo, acc); break;
      case 3: acc = conv_bwd_mac<3>(lds_d, lds_w, r, n, R, HWd, yo, xo, acc); break;
      case 4: acc = conv_bwd_mac<4>(lds_d, lds_w, r, n, R, HWd, yo, xo, acc); break;
      case 5: acc = conv_bwd_mac<5>(lds_d, lds_w, r, n, R, HWd, yo, xo, acc); break;
      default:
        for (int c = r; c < n; c += R) {
          const float* dp = lds_d + c * HWd;
          const float* wp = lds_w + c * KK;
          for (int ky = 0; ky < K; ++ky) {
            const int ro = row_off(ky);
            for (int kx = 0; kx < Kx; ++kx) acc = fmaf(dp[ro + col_off(kx)], wp[ky * Kx + kx], acc);
          }
        }
        break;
    }
    __syncthreads();
  }
  if (R > 1) {
    lds_part[tid] = acc;  // tid == r * PT + (p - tile * PT)
    __syncthreads();
    acc = sum_terms(lds_part, R, PT, lds_part + WG);
  }
  if (r == 0 && active) {
    const size_t o = (size_t)i * Pin + p;
    Lp.delta[o] = acc * Lp.dact[o];
  }
}

// ------------------------------------------------------------------------------------------
// AW of a convolutional layer (Sec. 3.4): dE/dw_{j,i}[ky][kx] = sum over output neurons of
// delta_j[y][x] * in_i[y(S+1)+ky][x(S+1)+kx], dE/db_j = sum delta_j, then w <- w - lr dE/dw in
// place.  Only the winners of the pooling rectangles carry a delta, so the sum runs over the
// pooled positions.  Work item = (output map j, chunk of its connections): the chunk's input
// maps, delta_j and the winner coordinates are staged in LDS; a thread owns one weight, or,
// when the chunk has fewer than 256 weights, the pooled positions are split R ways.
// ------------------------------------------------------------------------------------------
__device__ void conv_wgrad_item(const LayerDev& L, const Stage& st, int item,
                                const gfloat* in, const Ctx& ctx, float* lds) {
  const int tid = threadIdx.x;
  const int K = L.K, Kx = L.Kx;
  const int KK = K * Kx;
  const int stride = L.S + 1, stride_x = L.Sx + 1;
  const int Wi = L.Wi, Min = L.Hi * L.Wi, HW = L.Hp * L.Wp;
  const int j = item / st.n_tiles;
  const int kc = item - j * st.n_tiles;
  int c_begin = j * L.Mi, n_conn = L.Mi;
  if (!L.full_table) {
    c_begin = L.csr_ptr[j];
    n_conn = L.csr_ptr[j + 1] - c_begin;
  }
  const int c0 = kc * st.chunk;
  if (c0 >= n_conn) return;  // uniform over the workgroup
  const int n = min(st.chunk, n_conn - c0);

  float* lds_in = lds;
  float* lds_dp = lds + LDS_IN;
  int* lds_yx = (int*)(lds + LDS_IN + LDS_AUX);
  float* lds_part = lds + LDS_IN + LDS_AUX + LDS_AUX2;

  const int NW = n * KK;
  gfloat* wbase = L.w + (size_t)(c_begin + c0) * KK;
  constexpr int WU = 4;
  float w_old[WU];  // the weights this thread will adjust: in flight from the start
  prefetch_flat(w_old, wbase, NW);
  const float b_old = L.bias[j];
  {
    float dv[2];
    int yv[2];
    prefetch_flat(dv, L.delta + (size_t)j * HW, HW);
    prefetch_flat(yv, L.argyx + (size_t)j * HW, HW);
    if (L.full_table)
      stage_maps(lds_in, in, n, Min, st.tw_log2, [&](int c) { return (c0 + c) * Min; });
    else
      stage_maps(lds_in, in, n, Min, st.tw_log2, [&](int c) { return L.csr_idx[c_begin + c0 + c] * Min; });
    commit_flat(dv, lds_dp, HW);
    commit_flat(yv, lds_yx, HW);
    copy_flat_rest<2>(lds_dp, L.delta + (size_t)j * HW, HW);
    copy_flat_rest<2>(lds_yx, L.argyx + (size_t)j * HW, HW);
  }
  __syncthreads();

  int R = 1, rr = 0, wi0 = tid;
  if (NW < WG) {
    R = min(WG / NW, HW);
    rr = tid / NW;
    wi0 = tid - rr * NW;
  }
  const float lr = ctx.lr;
  gfloat* g_out = ctx.grad_out;
  const long long canon = L.w_canon + (long long)(c_begin + c0) * KK;
  // gradient of weight wi of the chunk, summed over the pooled positions q = q0, q0 + qs, ...
  auto grad_of = [&](int wi, int q0, int qs) {
    const int c = wi / KK, t = wi - c * KK;
    const int ky = t / Kx, kx = t - ky * Kx;
    const float* ip = lds_in + c * Min + ky * Wi + kx;
    float s = 0.f;
#pragma unroll 4
    for (int q = q0; q < HW; q += qs) {
      const int yx = lds_yx[q];
      s = fmaf(lds_dp[q], ip[(yx >> 16) * stride * Wi + (yx & 0xffff) * stride_x], s);
    }
    return s;
  };
  if (R == 1) {
#pragma unroll
    for (int u = 0; u < WU; ++u) {
      const int wi = tid + u * WG;
      if (wi < NW) {
        const float g = grad_of(wi, 0, 1);
        if (g_out) g_out[canon + wi] = g;
        else wbase[wi] = w_old[u] - lr * g;
      }
    }
    for (int wi = tid + WU * WG; wi < NW; wi += WG) {
      const float g = grad_of(wi, 0, 1);
      if (g_out) g_out[canon + wi] = g;
      else wbase[wi] -= lr * g;
    }
  } else {
    if (rr < R) lds_part[tid] = grad_of(wi0, rr, R);  // tid == rr * NW + wi0
    __syncthreads();
    const float g = sum_terms(lds_part, R, NW, lds_part + WG);
    if (tid < NW) {
      if (g_out) g_out[canon + tid] = g;
      else wbase[tid] = w_old[0] - lr * g;
    }
  }
  if (kc == 0 && tid < 64) {
    float s = 0.f;
    for (int q = tid; q < HW; q += 64) s += lds_dp[q];
    s = wave_sum(s);
    if (tid == 0) {
      if (g_out) g_out[L.b_canon + j] = s;
      else L.bias[j] = b_old - lr * s;
    }
  }
  __syncthreads();
}

// Weight gradients of a wide layer with a full table on the matrix cores (Sec. 3.4), and the
// adjustment that follows them.  With the deltas written out over the whole output map (zero
// except at the pooling winners) the sum over output neurons is a plain matrix product,
//   dE/dw_{j,i}[ky][kx] = sum_p delta_j[p] * in_i[pos(p) + (ky, kx)],
// rows = output maps j, columns = (input map i, tap), contraction over the output pixels p --
// the forward product with pixels and taps in each other's place, so the operand pattern
// in[koff(p) + cbase(column)] is the same.  It multiplies Kp^2 times more zeros than the vector
// kernel skips, which the matrix cores do faster than that kernel follows each map's winners.
// Work item = (tile of 32 output maps, chunk of IC input maps): it holds the whole contraction,
// so every weight is read and written by exactly one work item.  Bias: the items of chunk 0.
__device__ void conv_wgrad_mfma_item(const LayerDev& L, const Stage& st, int item, const gfloat* in,
                                     const Ctx& ctx, float* lds) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int lrow = lane & 31, lk = lane >> 5;
  const int NC = st.n_tiles;                 // chunks of input maps
  const int jt = item / NC, ks = item - jt * NC;
  const int j0 = jt * 32;
  const int K = L.K, KK = K * K, Mi = L.Mi, Mo = L.Mo, Wi = L.Wi, HiWi = L.Hi * L.Wi;
  const int Wo = L.Wo, P = L.Ho * L.Wo, HW = L.Hp * L.Wp, stride = L.S + 1;
  const int IC = st.chunk;
  const int ic0 = ks * IC, n_ic = min(IC, Mi - ic0);
  const int ncol = n_ic * KK;                // columns of this item
  const int WP = P + 1 + (P & 1);            // odd row pitch of the delta rows
  const int NT = (ncol + 31) >> 5;           // column tiles
  constexpr int WAVES = WG / 64;
  const int NTw = min(NT, WAVES);
  const int KW = (NT >= WAVES) ? 1 : WAVES / NT;
  const int kw = (NT >= WAVES) ? 0 : wave / NT;
  const int tw = (NT >= WAVES) ? wave : wave - kw * NT;
  const bool wave_on = kw < KW;

  float* lds_in = lds;                        // [IC][Hi*Wi]
  float* lds_d = lds + IC * HiWi;             // [32][WP] deltas over the whole output map
  int* koff = (int*)(lds_d + 32 * WP);        // [P] place of output pixel p's field in an input map

  for (int x = tid; x < P; x += WG) {
    const int y = x / Wo, xx = x - y * Wo;
    koff[x] = (y * Wi + xx) * stride;
  }
  for (int x = tid; x < 32 * WP; x += WG) lds_d[x] = 0.f;
  {  // the chunk's input maps: one contiguous block
    const gfloat* src = in + (size_t)ic0 * HiWi;
    const int n_in = n_ic * HiWi;
    for (int x0 = 0; x0 < n_in; x0 += 8 * WG) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = src[min(x0 + u * WG + tid, n_in - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (x0 + u * WG + tid < n_in) lds_in[x0 + u * WG + tid] = v[u];
    }
  }
  __syncthreads();
  {  // the tile's deltas, each to its winner's place
    const int n_rows = min(32, Mo - j0), ntot = n_rows * HW;
    for (int x0 = 0; x0 < ntot; x0 += 4 * WG) {
      float dv[4];
      int yx[4], rr[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int x = min(x0 + u * WG + tid, ntot - 1);
        rr[u] = x / HW;
        const size_t o = (size_t)(j0 + rr[u]) * HW + (x - rr[u] * HW);
        yx[u] = L.argyx[o];
        dv[u] = L.delta[o];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (x0 + u * WG + tid < ntot) lds_d[rr[u] * WP + (yx[u] >> 16) * Wo + (yx[u] & 0xffff)] = dv[u];
    }
  }
  int cbase[MM_TPW];
#pragma unroll
  for (int t = 0; t < MM_TPW; ++t) {
    const int n = (tw + t * NTw) * 32 + lrow;
    const int c = n / KK, tt = n - c * KK;
    const int ky = tt / K, kx = tt - ky * K;
    cbase[t] = (n < ncol) ? c * HiWi + ky * Wi + kx : 0;
  }
  v16f acc[MM_TPW];
#pragma unroll
  for (int t = 0; t < MM_TPW; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  const int n_my_tiles = wave_on ? ((NT - tw + NTw - 1) / NTw) : 0;
  __syncthreads();
  if (wave_on) {
    const int kper = (((P + KW - 1) / KW) + 1) & ~1;
    const int k_lo = kw * kper, k_hi = min(P, k_lo + kper);
    for (int kk = k_lo; kk < k_hi; kk += 8) {
      float a[4];
      int ko[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int k = kk + 2 * u + lk;
        a[u] = (k < k_hi) ? lds_d[lrow * WP + min(k, P - 1)] : 0.f;
        ko[u] = koff[min(k, P - 1)];
      }
#pragma unroll
      for (int t = 0; t < MM_TPW; ++t)
        if (t < n_my_tiles) {
          float b[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) b[u] = lds_in[ko[u] + cbase[t]];
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc[t], 0, 0, 0);
        }
    }
  }
  // bias gradients of the tile (the work items of chunk 0): sum of a delta row
  const float lr = ctx.lr;
  gfloat* g_out = ctx.grad_out;
  if (ks == 0) {
    for (int r = wave; r < 32; r += WAVES) {
      float sb = 0.f;
      for (int q = lane; q < P; q += 64) sb += lds_d[r * WP + q];
      sb = wave_sum(sb);
      if (lane == 0 && j0 + r < Mo) {
        if (g_out) g_out[L.b_canon + j0 + r] = sb;
        else L.bias[j0 + r] -= lr * sb;
      }
    }
  }
  __syncthreads();
  // weight (j, ic0 * KK + n) of the full table lies at ((j * Mi + ic0) * KK + n)
  auto apply = [&](int j, int n, float g) {
    const size_t o = ((size_t)j * Mi + ic0) * KK + n;
    if (g_out) g_out[L.w_canon + o] = g;
    else L.w[o] -= lr * g;
  };
  if (KW > 1) {
    float* red = lds;  // [KW][NT][32 rows][32 columns]; the staged maps are no longer needed
    if (wave_on) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        red[((kw * NT + tw) * 32 + (v >> 2) * 8 + lk * 4 + (v & 3)) * 32 + lrow] = acc[0][v];
    }
    __syncthreads();
    for (int x = tid; x < NT * 1024; x += WG) {
      const int t = x >> 10, row = (x >> 5) & 31, col = x & 31;
      float sum = 0.f;
      for (int q = 0; q < KW; ++q) sum += red[((q * NT + t) * 32 + row) * 32 + col];
      const int n = t * 32 + col, j = j0 + row;
      if (n < ncol && j < Mo) apply(j, n, sum);
    }
    __syncthreads();
  } else if (wave_on) {
#pragma unroll
    for (int t = 0; t < MM_TPW; ++t)
      if (t < n_my_tiles) {
        const int n = (tw + t * NTw) * 32 + lrow;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int j = j0 + (v >> 2) * 8 + lk * 4 + (v & 3);
          if (n < ncol && j < Mo) apply(j, n, acc[t][v]);
        }
      }
  }
}

// Second half of the matrix-core delta pull: the planes of partial sums of input map i added in a
// fixed order, times the derivative of the activation function at the output of the layer below
// (Sec. 3.3): delta of that layer at its pooled positions.  One work item per input map.
__device__ void conv_bwd_epi_item(const LayerDev& L, const LayerDev& Lp, const Stage& st, int item) {
  const int tid = threadIdx.x;
  const int P = L.Hi * L.Wi, Mi = L.Mi;
  const int n_planes = st.rows_per_wg;
  // st.chunk input maps per work item: their pixels are laid side by side over the lanes
  const int i0 = item * st.chunk;
  const int n = min(st.chunk, Mi - i0) * P;
  for (int x = tid; x < n; x += WG) {
    const size_t o = (size_t)i0 * P + x;   // (map i0 + x / P, pixel x % P: consecutive maps are consecutive in memory)
    float s = 0.f;
    for (int s0 = 0; s0 < n_planes; s0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = L.mm_part[(size_t)min(s0 + u, n_planes - 1) * Mi * P + o];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += (s0 + u < n_planes) ? v[u] : 0.f;
    }
    Lp.delta[o] = s * Lp.dact[o];
  }
}

// ------------------------------------------------------------------------------------------
// Dispatch of one work item of one stage.  KIND is a compile-time constant in the per-stage
// kernels (so each holds only its own code) and comes from a switch in the persistent kernel.
// ------------------------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ void run_item(const ProgramDev& P, const Stage& st, int item,
                                         const Ctx& ctx, StatusDev* status, float* lds) {
  const LayerDev& L = P.layers[st.layer];
  const gfloat* in = L.in_is_image ? ctx.image : L.in;
  // the trainable layer below, if any (behind a fixed front-end the first layer reads a stored input
  // but has no layer below it: nothing to pull deltas into)
  const LayerDev* below = (L.in_is_image || st.layer == 0) ? nullptr : &P.layers[st.layer - 1];
  if constexpr (KIND == ST_FRONTEND) {
    frontend_item(P.fe, item, ctx.image);
  } else if constexpr (KIND == ST_CONV_FWD) {
    if (st.pix_per_thread == 1) conv_fwd_item<1>(L, st, item, in, lds);
    else conv_fwd_item<2>(L, st, item, in, lds);
  } else if constexpr (KIND == ST_FC_FWD) {
    fc_fwd_item(L, st, item, in, lds);
  } else if constexpr (KIND == ST_HEAD) {
    head_item(L, below, in, ctx, status, lds);
  } else if constexpr (KIND == ST_FC_BWD) {
    fc_bwd_item(L, below, st, item, in, ctx, lds);
  } else if constexpr (KIND == ST_CONV_BWD) {
    conv_bwd_item(L, P.layers[st.layer - 1], st, item, lds);
  } else if constexpr (KIND == ST_CONV_WGRAD) {
    conv_wgrad_item(L, st, item, in, ctx, lds);
  } else if constexpr (KIND == ST_CONV_FWD_MFMA) {
    conv_mfma_item<false>(L, st, item, in, lds);
  } else if constexpr (KIND == ST_CONV_EPI) {
    conv_epi_item(L, st, item, lds);
  } else if constexpr (KIND == ST_CONV_BWD_MFMA) {
    conv_mfma_item<true>(L, st, item, in, lds);
  } else if constexpr (KIND == ST_CONV_BWD_EPI) {
    conv_bwd_epi_item(L, P.layers[st.layer - 1], st, item);
  } else if constexpr (KIND == ST_CONV_WGRAD_MFMA) {
    conv_wgrad_mfma_item(L, st, item, in, ctx, lds);
  }
}

// MM: the forward matrix-core stage kinds are compiled in (64 accumulators per lane push other
// stages' registers out to scratch memory, so plans without such stages get a kernel without
// them).  The matrix-core pull is not compiled into the persistent kernel at all: with it the
// register allocation of every stage suffers (measured: all stages 1.5 x slower); the host plans
// it for the stage-launch mode only.
// (Forced inline: as a called function it would get the program and stage descriptors in vector registers and
// every stage would fetch its operands' addresses with per-lane loads -- measured, all stages 2 x slower.)
template <bool MM>
__device__ __forceinline__ void run_stage_items(const ProgramDev& P, const Stage& st, int first, int step,
                                const Ctx& ctx, StatusDev* status, float* lds) {
  if constexpr (MM) {
    switch (st.kind) {
#define RUN_KIND(KIND) \
      case KIND: for (int item = first; item < st.n_items; item += step) run_item<KIND>(P, st, item, ctx, status, lds); return;
      RUN_KIND(ST_CONV_FWD_MFMA)
      RUN_KIND(ST_CONV_EPI)
#undef RUN_KIND
      default: break;
    }
  }
  switch (st.kind) {
#define RUN_KIND(KIND) \
    case KIND: for (int item = first; item < st.n_items; item += step) run_item<KIND>(P, st, item, ctx, status, lds); break;
    RUN_KIND(ST_FRONTEND)
    RUN_KIND(ST_CONV_FWD)
    RUN_KIND(ST_FC_FWD)
    RUN_KIND(ST_HEAD)
    RUN_KIND(ST_FC_BWD)
    RUN_KIND(ST_CONV_BWD)
    RUN_KIND(ST_CONV_WGRAD)
#undef RUN_KIND
    default: break;
  }
}

__device__ __forceinline__ Ctx make_ctx(const ProgramDev& P, const RunArgs& a, long long t,
                                        StatusDev* status) {
  Ctx c;
  if (a.call) {   // a node of a replayed graph: the call's arguments lie in device memory
    const CNN_GLOBAL CallArgs& q = *a.call;
    const long long tq = q.t0 + a.t_local;
    c.image = q.images + tq * q.image_stride;
    c.probs_out = q.probs_out ? q.probs_out + tq * P.n_classes : nullptr;
    c.grad_out = nullptr;
    c.label = q.labels[tq];
    c.lr = q.lr;
    c.train = q.train;
  } else {
  c.image = a.images + t * a.image_stride;
  c.probs_out = a.probs_out ? a.probs_out + t * P.n_classes : nullptr;
  c.grad_out = a.grad_out;
  c.label = a.labels ? a.labels[t] : a.label_imm;
  c.lr = a.lr;
  c.train = a.train;
  }
  if (a.train && (c.label < 0 || c.label >= P.n_classes)) {
    // a label outside the classes: the image is skipped and the host is told
    c.train = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) status->bad_label = 1u;
  }
  return c;
}

// ---- one launch per stage: grid = n_items of the stage -------------------------------------
#define STAGE_KERNEL(name, KIND)                                                             \
  __global__ void __launch_bounds__(WG) name(const ProgramDev* __restrict__ P, int s,        \
                                             StatusDev* status, RunArgs a) {                 \
    __shared__ float lds[LDS_FLOATS];                                                        \
    const Ctx ctx = make_ctx(*P, a, 0, status);                                              \
    const Stage& st = P->stages[s];                                                          \
    if (st.train_only && !ctx.train) return;                                                 \
    run_item<KIND>(*P, st, blockIdx.x, ctx, status, lds);                                    \
  }
STAGE_KERNEL(k_frontend, ST_FRONTEND)
STAGE_KERNEL(k_conv_fwd, ST_CONV_FWD)
STAGE_KERNEL(k_fc_fwd, ST_FC_FWD)
STAGE_KERNEL(k_head, ST_HEAD)
STAGE_KERNEL(k_fc_bwd, ST_FC_BWD)
STAGE_KERNEL(k_conv_bwd, ST_CONV_BWD)
STAGE_KERNEL(k_conv_wgrad, ST_CONV_WGRAD)
STAGE_KERNEL(k_conv_fwd_mfma, ST_CONV_FWD_MFMA)
STAGE_KERNEL(k_conv_epi, ST_CONV_EPI)
STAGE_KERNEL(k_conv_bwd_mfma, ST_CONV_BWD_MFMA)
STAGE_KERNEL(k_conv_bwd_epi, ST_CONV_BWD_EPI)
STAGE_KERNEL(k_conv_wgrad_mfma, ST_CONV_WGRAD_MFMA)

// Two consecutive stages that the plan declares independent (no barrier between them: a layer's weight
// adjustment next to the stage that follows its pull) in one launch: the first stage's items, then the second's.
// A launch costs some 4 us however little it does, so a step of 10 to 13 stages gains what a launch costs.
template <int KA, int KB>
__global__ void __launch_bounds__(WG) k_pair(const ProgramDev* __restrict__ P, int s, StatusDev* status, RunArgs a) {
  __shared__ float lds[LDS_FLOATS];
  const Ctx ctx = make_ctx(*P, a, 0, status);
  const Stage& sa = P->stages[s];
  const int n_a = sa.n_items;
  if ((int)blockIdx.x < n_a) {
    if (sa.train_only && !ctx.train) return;
    run_item<KA>(*P, sa, blockIdx.x, ctx, status, lds);
  } else {
    const Stage& sb = P->stages[s + 1];
    if (sb.train_only && !ctx.train) return;
    run_item<KB>(*P, sb, (int)blockIdx.x - n_a, ctx, status, lds);
  }
}

// Fixed image-processing layer for a whole batch at once (it depends on no weight, so it need not
// sit inside the on-line chain): image t of `images` -> out[t], one workgroup per WG output pixels.
// (plain pointer types in the signature: the host and the device pass must agree on its mangled name)
__global__ void __launch_bounds__(WG) k_frontend_batch(const ProgramDev* __restrict__ P, const float* images,
                                                       long long image_stride, int items_per_image, float* out) {
  const int t = blockIdx.x / items_per_image;
  const int item = blockIdx.x - t * items_per_image;
  FrontendDev fe = P->fe;
  fe.out = (gfloat*)out + (size_t)t * fe.n_filters * fe.H * fe.W;
  frontend_item(fe, item, (const gfloat*)images + (size_t)t * image_stride);
}

__global__ void k_reset_status(StatusDev* status, int clear_label_flag) {
  const int t = threadIdx.x;
  if (blockIdx.x != 0) return;
  if (t == 0) {
    status->barrier_count = 0u;
    status->abort_flag = 0u;
    status->top_count = 0u;
    if (clear_label_flag) status->bad_label = 0u;
  }
  for (int i = t; i < 16 * 32; i += blockDim.x) {
    status->xcd_members[i] = 0u;
    status->xcd_count[i] = 0u;
    status->xcd_go[i] = 0u;
  }
}

// ---- persistent kernel: all stages of all images in one cooperative launch ------------------
__device__ __forceinline__ unsigned int ld_agent(unsigned int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded wait until *p has reached `target` (wrap-safe).  A wait that exceeds spin_limit polls,
// or that sees the abort flag, raises the flag and fails, so that every wave terminates
// whatever happens to the other workgroups.
__device__ __forceinline__ bool wait_reached(StatusDev* status, unsigned int* p, unsigned int target,
                                             unsigned int spin_limit) {
  unsigned int spins = 0;
  while ((int)(ld_agent(p) - target) < 0) {
    __builtin_amdgcn_s_sleep(1);
    ++spins;
    if (spins > spin_limit || ((spins & 255u) == 0u && ld_agent(&status->abort_flag))) {
      __hip_atomic_store(&status->abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return false;
    }
  }
  return true;
}

// Grid barrier, kind 0: one monotone arrival counter.  Thread 0 of every workgroup releases its
// workgroup's writes (device-scope fence: L2 write-back), adds one, polls until the counter
// reaches barrier_number * gridDim.x, then acquires (device-scope fence: L2 + L1 invalidate).
__device__ bool grid_barrier(StatusDev* status, unsigned int target, unsigned int spin_limit,
                             int* s_ok) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    __hip_atomic_fetch_add(&status->barrier_count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool ok = wait_reached(status, &status->barrier_count, target, spin_limit);
    __threadfence();
    *s_ok = ok ? 1 : 0;
  }
  __syncthreads();
  return *s_ok != 0;
}

// Which XCD (accelerator die) this wave runs on: hardware register XCC_ID, bits 3:0.
__device__ __forceinline__ unsigned int xcc_id() {
  return __builtin_amdgcn_s_getreg(((4 - 1) << 11) | (0 << 6) | 20) & 0xfu;
}

struct BarCtx {
  unsigned int xcd, n_local, n_xcd;
};

// Grid barrier, kind 1: two levels, built for a part whose eight XCDs each have a private L2.
// A device-scope release writes back a whole L2; when every workgroup issues one they queue up
// 32 deep per L2, which is where most of the time of kind 0 goes.  Here each workgroup first
// makes sure its own stores have landed in its XCD's L2 (every wave waits for its outstanding
// memory operations) and arrives on its XCD's counter.  The last arrival of an XCD alone
// performs the device-scope release, arrives on the cross-XCD counter, waits for all XCDs and
// releases its XCD.  Every workgroup still performs its own device-scope acquire afterwards
// (measured: dropping only the CU's L1 lines in the followers leaves stale data behind).
__device__ bool xcd_barrier(StatusDev* status, unsigned int epoch, const BarCtx& bc,
                            unsigned int spin_limit, int* s_ok) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's stores are in L2
  __syncthreads();
  if (threadIdx.x == 0) {
    bool ok;
    const unsigned int arrived = __hip_atomic_fetch_add(&status->xcd_count[bc.xcd * 32], 1u,
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (arrived + 1u == epoch * bc.n_local) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __hip_atomic_fetch_add(&status->top_count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = wait_reached(status, &status->top_count, epoch * bc.n_xcd, spin_limit);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(&status->xcd_go[bc.xcd * 32], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      ok = wait_reached(status, &status->xcd_go[bc.xcd * 32], epoch, spin_limit);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    *s_ok = ok ? 1 : 0;
  }
  __syncthreads();
  return *s_ok != 0;
}

template <bool MM>
__global__ void __launch_bounds__(WG) k_persistent(const ProgramDev* __restrict__ P,
                                                   StatusDev* status, RunArgs a) {
  __shared__ float lds[LDS_FLOATS];
  __shared__ int s_ok;
  __shared__ BarCtx s_bc;
  unsigned int n_barriers = 0;
  const int G = gridDim.x;
  const bool two_level = a.barrier_kind == 1;
  if (two_level) {
    // roll call: how many workgroups of this launch sit on each XCD
    if (threadIdx.x == 0) {
      s_bc.xcd = xcc_id();
      __hip_atomic_fetch_add(&status->xcd_members[s_bc.xcd * 32], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    ++n_barriers;
    if (!grid_barrier(status, n_barriers * (unsigned int)G, a.spin_limit, &s_ok)) return;
    if (threadIdx.x == 0) {
      s_bc.n_local = ld_agent(&status->xcd_members[s_bc.xcd * 32]);
      unsigned int nx = 0;
      for (int x = 0; x < 16; ++x) nx += ld_agent(&status->xcd_members[x * 32]) ? 1u : 0u;
      s_bc.n_xcd = nx;
    }
    __syncthreads();
  }
  const BarCtx bc = s_bc;
  unsigned int epoch = 0;
  for (long long t = 0; t < a.n_images; ++t) {
    const Ctx ctx = make_ctx(*P, a, t, status);
    const bool stamp = (t == a.n_images - 1) && blockIdx.x == 0 && threadIdx.x == 0;
    if (stamp) status->stamps[0] = wall_clock64();
    for (int s = 0; s < P->n_stages; ++s) {
      const Stage& st = P->stages[s];
      if (st.train_only && !ctx.train) continue;
      run_stage_items<MM>(*P, st, blockIdx.x, G, ctx, status, lds);
      if (stamp) status->stamps[1 + 2 * s] = wall_clock64();
      if (st.barrier_after) {
        bool ok;
        if (two_level) {
          ++epoch;
          ok = xcd_barrier(status, epoch, bc, a.spin_limit, &s_ok);
        } else {
          ++n_barriers;
          ok = grid_barrier(status, n_barriers * (unsigned int)G, a.spin_limit, &s_ok);
        }
        if (!ok) return;
      }
      if (stamp) status->stamps[2 + 2 * s] = wall_clock64();
    }
  }
}

// ---- host-side launchers (called from the C ABI translation unit) ---------------------------
hipError_t launch_stage(int kind, int n_items, hipStream_t stream, const ProgramDev* d_prog, int s,
                        StatusDev* d_status, const RunArgs& a) {
  if (n_items <= 0) return hipSuccess;
  dim3 grid(n_items), block(WG);
  switch (kind) {
    case ST_FRONTEND: hipLaunchKernelGGL(k_frontend, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_FWD: hipLaunchKernelGGL(k_conv_fwd, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_FC_FWD: hipLaunchKernelGGL(k_fc_fwd, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_HEAD: hipLaunchKernelGGL(k_head, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_FC_BWD: hipLaunchKernelGGL(k_fc_bwd, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_BWD: hipLaunchKernelGGL(k_conv_bwd, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_WGRAD: hipLaunchKernelGGL(k_conv_wgrad, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_FWD_MFMA: hipLaunchKernelGGL(k_conv_fwd_mfma, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_EPI: hipLaunchKernelGGL(k_conv_epi, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_BWD_MFMA: hipLaunchKernelGGL(k_conv_bwd_mfma, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_BWD_EPI: hipLaunchKernelGGL(k_conv_bwd_epi, grid, block, 0, stream, d_prog, s, d_status, a); break;
    case ST_CONV_WGRAD_MFMA: hipLaunchKernelGGL(k_conv_wgrad_mfma, grid, block, 0, stream, d_prog, s, d_status, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---- the stage launches of several images as one graph ----------------------------------------------------
// A launch costs about 2.5 us however little the kernel does, a kernel node of a graph about 1.5: the nets that
// run one launch per stage (10 - 14 per image) replay a graph of the launches of a few images instead.  The
// kernels of a node are the ones above; what changes from one replay to the next -- the images, labels, outputs
// and rate of the call, and how far into it the graph starts -- lies in device memory (CallArgs).
__global__ void k_call_set(CallArgs* d, CallArgs v) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *(CNN_GLOBAL CallArgs*)d = v;
}
__global__ void k_call_advance(CallArgs* d, int images) {
  if (threadIdx.x == 0 && blockIdx.x == 0) ((CNN_GLOBAL CallArgs*)d)->t0 += images;
}
hipError_t launch_call_set(hipStream_t stream, CallArgs* d_call, const CallArgs& v) {
  hipLaunchKernelGGL(k_call_set, dim3(1), dim3(64), 0, stream, d_call, v);
  return hipGetLastError();
}
const void* call_advance_kernel() { return (const void*)k_call_advance; }
// the kernel of a stage kind, and of two kinds in one launch (null: none compiled)
const void* stage_kernel(int kind) {
  switch (kind) {
    case ST_FRONTEND: return (const void*)k_frontend;
    case ST_CONV_FWD: return (const void*)k_conv_fwd;
    case ST_FC_FWD: return (const void*)k_fc_fwd;
    case ST_HEAD: return (const void*)k_head;
    case ST_FC_BWD: return (const void*)k_fc_bwd;
    case ST_CONV_BWD: return (const void*)k_conv_bwd;
    case ST_CONV_WGRAD: return (const void*)k_conv_wgrad;
    case ST_CONV_FWD_MFMA: return (const void*)k_conv_fwd_mfma;
    case ST_CONV_EPI: return (const void*)k_conv_epi;
    case ST_CONV_BWD_MFMA: return (const void*)k_conv_bwd_mfma;
    case ST_CONV_BWD_EPI: return (const void*)k_conv_bwd_epi;
    case ST_CONV_WGRAD_MFMA: return (const void*)k_conv_wgrad_mfma;
    default: return nullptr;
  }
}
const void* stage_pair_kernel(int kind_a, int kind_b) {
#define PAIR(KA, KB) if (kind_a == KA && kind_b == KB) return (const void*)k_pair<KA, KB>;
  PAIR(ST_CONV_WGRAD, ST_CONV_BWD_EPI)
  PAIR(ST_CONV_WGRAD_MFMA, ST_CONV_BWD_EPI)
  PAIR(ST_CONV_WGRAD, ST_CONV_WGRAD)
  PAIR(ST_CONV_WGRAD, ST_CONV_BWD)
#undef PAIR
  return nullptr;
}

// Stages s and s + 1 of kinds kind_a and kind_b in one launch; *done = false when no kernel is compiled for the pair
// (the caller then launches them one after the other).
hipError_t launch_stage_pair(int kind_a, int n_a, int kind_b, int n_b, hipStream_t stream, const ProgramDev* d_prog,
                             int s, StatusDev* d_status, const RunArgs& a, bool* done) {
  *done = false;
  if (n_a <= 0 || n_b <= 0) return hipSuccess;
  dim3 grid(n_a + n_b), block(WG);
#define PAIR(KA, KB)                                                                              \
  if (kind_a == KA && kind_b == KB) {                                                             \
    hipLaunchKernelGGL((k_pair<KA, KB>), grid, block, 0, stream, d_prog, s, d_status, a);         \
    *done = true;                                                                                 \
    return hipGetLastError();                                                                     \
  }
  PAIR(ST_CONV_WGRAD, ST_CONV_BWD_EPI)
  PAIR(ST_CONV_WGRAD_MFMA, ST_CONV_BWD_EPI)
  PAIR(ST_CONV_WGRAD, ST_CONV_WGRAD)
  PAIR(ST_CONV_WGRAD, ST_CONV_BWD)
#undef PAIR
  return hipSuccess;
}

hipError_t launch_frontend_batch(hipStream_t stream, const ProgramDev* d_prog, const float* d_images,
                                 long long image_stride, int n_images, int items_per_image, float* d_out) {
  if (n_images <= 0 || items_per_image <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_frontend_batch, dim3((unsigned)n_images * items_per_image), dim3(WG), 0, stream, d_prog,
                     d_images, image_stride, items_per_image, d_out);
  return hipGetLastError();
}

hipError_t launch_reset_status(hipStream_t stream, StatusDev* d_status, int clear_label_flag) {
  hipLaunchKernelGGL(k_reset_status, dim3(1), dim3(256), 0, stream, d_status, clear_label_flag);
  return hipGetLastError();
}

// with_matrix_stages: the plan holds forward matrix-core stages (the kernel without them is leaner)
hipError_t launch_persistent(int grid, bool with_matrix_stages, hipStream_t stream, const ProgramDev* d_prog,
                             StatusDev* d_status, const RunArgs& a) {
  RunArgs args = a;
  void* params[] = {(void*)&d_prog, (void*)&d_status, (void*)&args};
  const void* k = with_matrix_stages ? (const void*)k_persistent<true> : (const void*)k_persistent<false>;
  return hipLaunchCooperativeKernel(k, dim3(grid), dim3(WG), params, 0, stream);
}

void read_dbg(unsigned long long* out) {
#ifdef CNN355_STAMPS
  (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_dbg), sizeof(g_dbg));
#else
  for (int i = 0; i < 64; ++i) out[i] = 0;
#endif
}

int persistent_max_blocks_per_cu() {
  int n = 0;
  int m = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)k_persistent<true>, WG, 0) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&m, (const void*)k_persistent<false>, WG, 0) != hipSuccess) return 0;
  return n < m ? n : m;
}

}  // namespace cnn355
