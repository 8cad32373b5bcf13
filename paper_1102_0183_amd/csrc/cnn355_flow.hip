// Resident mode: on-line back-propagation (Sec. 1, Sec. 3.2 - 3.4 of Ciresan et al., IDSIA TR
// 01-11) as one kernel per call in which every workgroup ("rank") owns whole maps and keeps
// their weights in LDS from the first image of the call to the last.
//
// On-line training is a chain: image t+1 needs every weight adjusted by image t, and inside an
// image every layer waits for the one below (FP) or above (BP).  At one image at a time the
// arithmetic is microseconds of work for a few compute units, so what limits the rate is how
// often data crosses between compute units and how long each crossing takes.  This kernel is
// laid out to cross as rarely as the method allows:
//   * rank r owns output maps r, r+G, ... of every convolutional layer.  It holds the filters of
//     those maps (row j of the connection table; what FP and AW of the paper need) and, for its
//     maps of the layer below, a second copy of the filters that read them (column i of the
//     table; what the pull-form BP of Sec. 3.3 needs).  Both copies are adjusted by their
//     holder from the same deltas and inputs in the same order, so they stay identical bit for
//     bit and no weight ever travels;
//   * the first fully connected layer is owned by columns (the inputs a rank produced itself):
//     ranks exchange partial sums going forward and nothing going back; the small layers
//     behind it are computed by every rank redundantly;
//   * what does travel (pooled outputs, partial sums, deltas at the pooling winners) goes
//     through global memory as 64-bit words {value, tag} stored and polled with device-scope
//     atomics.  The tag is the number of the image, so a reader needs neither barrier nor
//     fence: it polls until the tag matches.  Buffers are double-buffered by the parity of the
//     tag; the all-to-all exchange of partial sums in every image keeps any rank from running
//     two images ahead of another, so a buffer is never overwritten before it has been read.
// Three such crossings per image for a network with two convolutional layers, against seven
// grid-wide barriers in the stage-by-stage schedule.
#include <hip/hip_runtime.h>

#if defined(__HIP_DEVICE_COMPILE__)
#define CNN_GLOBAL __attribute__((address_space(1)))
#endif
#include "cnn355_dev.h"

namespace cnn355 {

typedef CNN_GLOBAL float gfloat;
typedef CNN_GLOBAL tagged_t gtagged;

#define ACT_A 1.7159f
#define ACT_B 0.6666f
__device__ __forceinline__ float f_act(float a) { return ACT_A * tanhf(ACT_B * a); }
__device__ __forceinline__ float f_dact(float y) {
  return (float)(1.7159 * 0.6666) - (float)(0.6666 / 1.7159) * y * y;
}
__device__ __forceinline__ float f_wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float f_wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

__device__ __forceinline__ int n_mine(int M, int rank, int G) { return rank < M ? (M - rank + G - 1) / G : 0; }

// ---- tagged words ---------------------------------------------------------------------------
__device__ __forceinline__ void put_f(gtagged* p, float v, unsigned int tag) {
  const tagged_t w = ((tagged_t)tag << 32) | (tagged_t)__float_as_uint(v);
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void put_i(gtagged* p, int v, unsigned int tag) {
  const tagged_t w = ((tagged_t)tag << 32) | (tagged_t)(unsigned int)v;
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct Rt {  // what every phase needs
  const ProgramDev* P;
  const FlowDev* F;
  StatusDev* status;
  float* lds;
  int* s_fail;
  int rank;
  unsigned int spin_limit;
};

// Copy n tagged words into LDS (their 32-bit payloads), each lane polling its own words until
// they carry `tag`.  Every wait is bounded: a lane that polls more than spin_limit times, or
// that sees the abort flag, raises the flag; the caller then leaves the kernel.  Returns false
// (to every thread of the workgroup) in that case.  Ends with a workgroup barrier.
__device__ bool gather(const Rt& rt, unsigned int* dst, const gtagged* src, int n, unsigned int tag) {
  constexpr int U = 4;
  const int tid = threadIdx.x;
  for (int base = 0; base < n; base += U * WG) {
    tagged_t w[U];
    unsigned int spins = 0;
    while (true) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        w[u] = __hip_atomic_load(src + min(base + tid + u * WG, n - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      bool done = true;
#pragma unroll
      for (int u = 0; u < U; ++u) done = done && ((unsigned int)(w[u] >> 32) == tag);
      if (done) break;
      ++spins;
      if (spins > rt.spin_limit ||
          ((spins & 63u) == 0u && __hip_atomic_load(&rt.status->abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
        __hip_atomic_store(&rt.status->abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *rt.s_fail = 1;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + tid + u * WG < n) dst[base + tid + u * WG] = (unsigned int)w[u];
  }
  __syncthreads();
  return *rt.s_fail == 0;
}

// ---- weights: global (canonical order) <-> LDS -------------------------------------------------
__device__ void flow_load(const Rt& rt) {
  const ProgramDev& P = *rt.P;
  const FlowDev& F = *rt.F;
  float* lds = rt.lds;
  const int tid = threadIdx.x, G = F.G, rank = rt.rank;
  for (int l = 0; l < F.n_conv; ++l) {
    const LayerDev& L = P.layers[l];
    const FlowConv& C = F.conv[l];
    const int KK = L.K * L.K;
    const int nm = n_mine(L.Mo, rank, G);
    float* wf = lds + C.o_wf;
    float* bf = lds + C.o_bf;
    int* cidx = (int*)(lds + C.o_cidx);
    int* ncf = (int*)(lds + C.o_ncf);
    for (int a = 0; a < nm; ++a) {
      const int j = rank + a * G;
      int cb = j * L.Mi, nc = L.Mi;
      if (!L.full_table) { cb = L.csr_ptr[j]; nc = L.csr_ptr[j + 1] - cb; }
      for (int x = tid; x < L.max_conn * KK; x += WG)
        wf[a * L.max_conn * KK + x] = (x < nc * KK) ? L.w[(size_t)cb * KK + x] : 0.f;
      for (int c = tid; c < L.max_conn; c += WG)
        cidx[a * L.max_conn + c] = (c < nc) ? (L.full_table ? c : L.csr_idx[cb + c]) : 0;
      if (tid == 0) { bf[a] = L.bias[j]; ncf[a] = nc; }
    }
    if (l >= 1) {
      const int nb = n_mine(L.Mi, rank, G);
      float* wb = lds + C.o_wb;
      int* bj = (int*)(lds + C.o_bj);
      int* ncb = (int*)(lds + C.o_ncb);
      for (int a = 0; a < nb; ++a) {
        const int i = rank + a * G;
        int eb = 0, ne = L.Mo;
        if (!L.full_table) { eb = L.csc_ptr[i]; ne = L.csc_ptr[i + 1] - eb; }
        for (int x = tid; x < C.max_back * KK; x += WG) {
          const int e = x / KK, t = x - e * KK;
          float v = 0.f;
          if (e < ne) {
            const int slot = L.full_table ? (e * L.Mi + i) : L.csc_slot[eb + e];
            v = L.w[(size_t)slot * KK + t];
          }
          wb[a * C.max_back * KK + x] = v;
        }
        for (int e = tid; e < C.max_back; e += WG)
          bj[a * C.max_back + e] = (e < ne) ? (L.full_table ? e : L.csc_j[eb + e]) : 0;
        if (tid == 0) ncb[a] = ne;
      }
    }
  }
  {  // first fully connected layer: the columns fed by the own maps of the last convolutional layer
    const LayerDev& Lc = P.layers[F.n_conv - 1];
    const LayerDev& L = P.layers[F.n_conv];
    const int HW = Lc.Hp * Lc.Wp, n1 = L.n_out;
    const int nm = n_mine(Lc.Mo, rank, G);
    float* wc = lds + F.fc[0].o_w;
    for (int x = tid; x < nm * HW * n1; x += WG) {
      const int c = x / n1, k = x - c * n1;
      const int a = c / HW, q = c - a * HW;
      wc[x] = L.w[(size_t)k * L.n_in + (size_t)(rank + a * G) * HW + q];
    }
    for (int k = tid; k < n1; k += WG) lds[F.fc[0].o_b + k] = L.bias[k];
  }
  for (int f = 1; f < F.n_fc; ++f) {
    const LayerDev& L = P.layers[F.n_conv + f];
    for (int x = tid; x < L.n_out * L.n_in; x += WG) lds[F.fc[f].o_w + x] = L.w[x];
    for (int k = tid; k < L.n_out; k += WG) lds[F.fc[f].o_b + k] = L.bias[k];
  }
  __syncthreads();
}

__device__ void flow_store(const Rt& rt) {
  const ProgramDev& P = *rt.P;
  const FlowDev& F = *rt.F;
  float* lds = rt.lds;
  const int tid = threadIdx.x, G = F.G, rank = rt.rank;
  __syncthreads();
  for (int l = 0; l < F.n_conv; ++l) {
    const LayerDev& L = P.layers[l];
    const FlowConv& C = F.conv[l];
    const int KK = L.K * L.K;
    const int nm = n_mine(L.Mo, rank, G);
    const int* ncf = (const int*)(lds + C.o_ncf);
    for (int a = 0; a < nm; ++a) {
      const int j = rank + a * G;
      const int nc = ncf[a];
      const int cb = L.full_table ? j * L.Mi : L.csr_ptr[j];
      for (int x = tid; x < nc * KK; x += WG) L.w[(size_t)cb * KK + x] = lds[C.o_wf + a * L.max_conn * KK + x];
      if (tid == 0) L.bias[j] = lds[C.o_bf + a];
    }
  }
  {
    const LayerDev& Lc = P.layers[F.n_conv - 1];
    const LayerDev& L = P.layers[F.n_conv];
    const int HW = Lc.Hp * Lc.Wp, n1 = L.n_out;
    const int nm = n_mine(Lc.Mo, rank, G);
    for (int x = tid; x < nm * HW * n1; x += WG) {
      const int c = x / n1, k = x - c * n1;
      const int a = c / HW, q = c - a * HW;
      L.w[(size_t)k * L.n_in + (size_t)(rank + a * G) * HW + q] = lds[F.fc[0].o_w + x];
    }
    if (rank == 0)
      for (int k = tid; k < n1; k += WG) L.bias[k] = lds[F.fc[0].o_b + k];
  }
  if (rank == 0)
    for (int f = 1; f < F.n_fc; ++f) {
      const LayerDev& L = P.layers[F.n_conv + f];
      for (int x = tid; x < L.n_out * L.n_in; x += WG) L.w[x] = lds[F.fc[f].o_w + x];
      for (int k = tid; k < L.n_out; k += WG) L.bias[k] = lds[F.fc[f].o_b + k];
    }
}

// ---- FP of one own map (Sec. 2.2, Sec. 3.2): inputs, filters and index list all in LDS ------------
template <int KT>
__device__ __forceinline__ float conv_acc(const float* in, const float* wf, const int* cidx, int c0, int cstep,
                                          int nc, int HiWi, int Wi, int Krt, int base) {
  const int K = KT ? KT : Krt;
  const int KK = K * K;
  float acc = 0.f;
  for (int c = c0; c < nc; c += cstep) {
    const float* ip = in + cidx[c] * HiWi + base;
    const float* wp = wf + c * KK;
#pragma unroll
    for (int ky = 0; ky < K; ++ky)
#pragma unroll
      for (int kx = 0; kx < K; ++kx) acc = fmaf(wp[ky * K + kx], ip[ky * Wi + kx], acc);
  }
  return acc;
}
__device__ __forceinline__ float conv_acc_k(int K, const float* in, const float* wf, const int* cidx, int c0,
                                            int cstep, int nc, int HiWi, int Wi, int base) {
  switch (K) {
    case 2: return conv_acc<2>(in, wf, cidx, c0, cstep, nc, HiWi, Wi, K, base);
    case 3: return conv_acc<3>(in, wf, cidx, c0, cstep, nc, HiWi, Wi, K, base);
    case 4: return conv_acc<4>(in, wf, cidx, c0, cstep, nc, HiWi, Wi, K, base);
    case 5: return conv_acc<5>(in, wf, cidx, c0, cstep, nc, HiWi, Wi, K, base);
    default: return conv_acc<0>(in, wf, cidx, c0, cstep, nc, HiWi, Wi, K, base);
  }
}

// act[p] = A tanh(B (bias + sum over connections and taps)) for every pixel p of the map.  Maps
// with at most WG/2 pixels split the connections over the spare lanes and add the partial sums
// in a fixed order.
__device__ void flow_conv_fwd_map(const LayerDev& L, const float* in, const float* wf, const int* cidx, int nc,
                                  float bias, float* act, float* part) {
  const int tid = threadIdx.x;
  const int Wo = L.Wo, Wi = L.Wi, HiWi = L.Hi * L.Wi, stride = L.S + 1;
  const int Pn = L.Ho * Wo;
  if (2 * Pn <= WG) {
    const int R = WG / Pn;
    const int r = tid / Pn, p = tid - r * Pn;
    float acc = 0.f;
    if (r < R) {
      const int y = p / Wo, x = p - y * Wo;
      acc = conv_acc_k(L.K, in, wf, cidx, r, R, nc, HiWi, Wi, (y * Wi + x) * stride);
    }
    part[tid] = acc;
    __syncthreads();
    if (tid < Pn) {
      float s = 0.f;
      for (int rr = 0; rr < R; ++rr) s += part[rr * Pn + tid];
      act[tid] = f_act(s + bias);
    }
  } else {
    for (int p = tid; p < Pn; p += WG) {
      const int y = p / Wo, x = p - y * Wo;
      const float acc = conv_acc_k(L.K, in, wf, cidx, 0, 1, nc, HiWi, Wi, (y * Wi + x) * stride);
      act[p] = f_act(acc + bias);
    }
  }
  __syncthreads();
}

// Max-pooling of one own map (Sec. 2.3): value and position of the first maximum in row-major
// order; the pooled value is what the next layer reads, so it is published at once.
__device__ void flow_pool_map(const LayerDev& L, const FlowConv& C, float* lds, int a, int j, const float* act,
                              unsigned int tag, bool taps) {
  const int tid = threadIdx.x;
  const int Kp = L.Kp, Wo = L.Wo, Wp = L.Wp, HW = L.Hp * L.Wp;
  float* pool = lds + C.o_pool + a * HW;
  int* yx = (int*)(lds + C.o_yx) + a * HW;
  gtagged* xo = C.x_out ? C.x_out + (size_t)(tag & 1u) * L.Mo * HW + (size_t)j * HW : nullptr;
  for (int q = tid; q < HW; q += WG) {
    const int py = q / Wp, px = q - py * Wp;
    const float* win = act + py * Kp * Wo + px * Kp;
    float best = win[0];
    int wy = 0, wx = 0;
    for (int dy = 0; dy < Kp; ++dy)
      for (int dx = 0; dx < Kp; ++dx) {
        const float v = win[dy * Wo + dx];
        if (v > best) { best = v; wy = dy; wx = dx; }
      }
    const int code = ((py * Kp + wy) << 16) | (px * Kp + wx);
    pool[q] = best;
    yx[q] = code;
    if (xo) put_f(xo + q, best, tag);
    if (taps) {
      const size_t o = (size_t)j * HW + q;
      if (Kp > 1) L.out[o] = best;
      L.arg[o] = (uint8_t)(wy * Kp + wx);
      L.argyx[o] = code;
    }
  }
  if (taps)
    for (int p = tid; p < L.Ho * Wo; p += WG) L.act[(size_t)j * L.Ho * Wo + p] = act[p];
  __syncthreads();
}

// ---- AW of a set of filters held in LDS (Sec. 3.4) ------------------------------------------------
// dE/dw = sum over the pooled positions q of delta[q] * in[(y_q (S+1) + ky) Wi + x_q (S+1) + kx]
// (only the winner of a pooling rectangle carries a delta), then w <- w - lr dE/dw.  The same
// routine adjusts the forward copy and the pull copy of a layer's filters; R (fixed per layer) and
// the order of the sum are the same for both, which keeps the copies identical bit for bit.
struct WgradInfo {
  bool ok;
  const float* d;   // deltas of the output map, [HW]
  const int* yx;    // winner coordinates, [HW]
  const float* in;  // input map, already advanced to tap (ky, kx)
  long long canon;  // position of the weight in the canonical vector
};
template <class Info>
__device__ __forceinline__ void flow_wgrad(float* w, int n_w, int HW, int stride, int Wi, int Rl2, float lr,
                                           gfloat* g_out, Info info) {
  const int R = 1 << Rl2;
  const int tid = threadIdx.x;
  const int total = n_w << Rl2;
  for (int u0 = 0; u0 < total; u0 += WG) {
    const int u = u0 + tid;
    const int wi = u >> Rl2, rr = u & (R - 1);
    float s = 0.f;
    WgradInfo I;
    I.ok = false;
    I.canon = 0;
    if (wi < n_w) {
      I = info(wi);
      if (I.ok)
        for (int q = rr; q < HW; q += R) {
          const int yx = I.yx[q];
          s = fmaf(I.d[q], I.in[((yx >> 16) * Wi + (yx & 0xffff)) * stride], s);
        }
    }
    for (int off = R >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (I.ok && rr == 0) {
      if (g_out) g_out[I.canon] = s;
      else w[wi] = fmaf(-lr, s, w[wi]);
    }
  }
}

// ---- BP through a convolutional layer, pull form (Sec. 3.3), for one own input map -------------------
template <int KT>
__device__ __forceinline__ float pull_acc(const float* dd, const float* wb, int c0, int cstep, int n, int HWd,
                                          const int (&yo)[5], const int (&xo)[5], float acc) {
  for (int c = c0; c < n; c += cstep) {
    const float* dp = dd + c * HWd;
    const float* wp = wb + c * (KT * KT);
#pragma unroll
    for (int ky = 0; ky < KT; ++ky)
#pragma unroll
      for (int kx = 0; kx < KT; ++kx) acc = fmaf(dp[yo[ky] + xo[kx]], wp[ky * KT + kx], acc);
  }
  return acc;
}

// Neuron (r, c) of input map i collects, over every output map j that reads map i, the deltas of
// the output neurons whose receptive field covers it (the four inequalities of Sec. 3.3), each
// times its weight (old value).  The deltas of a chunk of output maps are rebuilt at full
// resolution in LDS with one extra row and column of zeros (only pooling winners are non-zero),
// so a tap that has no output neuron reads a zero and the inner loop has no branches.
// out[p] = pulled sum * f'(y[p]).
__device__ void flow_pull_map(const Rt& rt, const LayerDev& L, const FlowConv& C, int a, int ne, const float* dall,
                              const int* yxall, const float* ybelow, float* out) {
  const FlowDev& F = *rt.F;
  float* lds = rt.lds;
  const int tid = threadIdx.x;
  const int K = L.K, KK = K * K, stride = L.S + 1;
  const int Wi = L.Wi, Pin = L.Hi * L.Wi;
  const int Ho = L.Ho, Wo = L.Wo, HW = L.Hp * L.Wp;
  const int Wd = Wo + 1, HWd = (Ho + 1) * Wd;
  float* dd = lds + F.o_scratch;
  float* part = lds + F.o_part;
  const float* wb = lds + C.o_wb + a * C.max_back * KK;
  const int* bj = (const int*)(lds + C.o_bj) + a * C.max_back;
  const bool split = 2 * Pin <= WG;
  const int R = split ? WG / Pin : 1;
  const int PB = split ? Pin : WG;
  for (int p0 = 0; p0 < Pin; p0 += PB) {
    const int r = split ? tid / Pin : 0;
    const int p = split ? tid - r * Pin : p0 + tid;
    const bool on = r < R && p < Pin;
    const int pr = p / Wi, pc = p - pr * Wi;
    auto row_off = [&](int ky) {
      const int ry = pr - ky;
      const int y = ry / stride;
      const bool ok = on && ry >= 0 && ry - y * stride == 0 && y < Ho;
      return (ok ? y : Ho) * Wd;
    };
    auto col_off = [&](int kx) {
      const int rx = pc - kx;
      const int x = rx / stride;
      const bool ok = on && rx >= 0 && rx - x * stride == 0 && x < Wo;
      return ok ? x : Wo;
    };
    int yo[5], xo[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) { yo[k] = row_off(k); xo[k] = col_off(k); }
    float acc = 0.f;
    for (int e0 = 0; e0 < ne; e0 += C.pull_chunk) {
      const int n = min(C.pull_chunk, ne - e0);
      for (int idx = tid; idx < n * HWd; idx += WG) dd[idx] = 0.f;
      __syncthreads();
      for (int idx = tid; idx < n * HW; idx += WG) {
        const int c = idx / HW, q = idx - c * HW;
        const int j = bj[e0 + c];
        const int yx = yxall[j * HW + q];
        dd[c * HWd + (yx >> 16) * Wd + (yx & 0xffff)] = dall[j * HW + q];
      }
      __syncthreads();
      const float* wbc = wb + e0 * KK;
      const int c0 = min(r, R - 1);
      switch (K) {
        case 1: acc = pull_acc<1>(dd, wbc, c0, R, n, HWd, yo, xo, acc); break;
        case 2: acc = pull_acc<2>(dd, wbc, c0, R, n, HWd, yo, xo, acc); break;
        case 3: acc = pull_acc<3>(dd, wbc, c0, R, n, HWd, yo, xo, acc); break;
        case 4: acc = pull_acc<4>(dd, wbc, c0, R, n, HWd, yo, xo, acc); break;
        case 5: acc = pull_acc<5>(dd, wbc, c0, R, n, HWd, yo, xo, acc); break;
        default:
          for (int c = c0; c < n; c += R) {
            const float* dp = dd + c * HWd;
            const float* wp = wbc + c * KK;
            for (int ky = 0; ky < K; ++ky) {
              const int ro = row_off(ky);
              for (int kx = 0; kx < K; ++kx) acc = fmaf(dp[ro + col_off(kx)], wp[ky * K + kx], acc);
            }
          }
          break;
      }
      __syncthreads();
    }
    if (split) {
      part[tid] = (r < R) ? acc : 0.f;
      __syncthreads();
      if (tid < Pin) {
        float s = 0.f;
        for (int rr = 0; rr < R; ++rr) s += part[rr * Pin + tid];
        out[tid] = s * f_dact(ybelow[tid]);
      }
      __syncthreads();
    } else if (on) {
      out[p] = acc * f_dact(ybelow[p]);
    }
  }
  __syncthreads();
}

// y[k] = b[k] + sum_m W[k][m] v[m], all in LDS; lane groups of a power of two per row.
__device__ void flow_matvec(const float* W, const float* b, const float* v, float* y, int n_out, int n_in) {
  const int tid = threadIdx.x;
  int lpl = 6;
  while (lpl > 0 && (WG >> lpl) < n_out) --lpl;
  const int lpr = 1 << lpl, rows_pp = WG >> lpl;
  const int sub = tid & (lpr - 1);
  for (int k0 = 0; k0 < n_out; k0 += rows_pp) {
    const int k = k0 + (tid >> lpl);
    float s = 0.f;
    if (k < n_out) {
      const float* wr = W + k * n_in;
      for (int m = sub; m < n_in; m += lpr) s = fmaf(wr[m], v[m], s);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
      if (off < lpr) s += __shfl_xor(s, off, 64);
    if (sub == 0 && k < n_out) y[k] = s + b[k];
  }
  __syncthreads();
}

#define STAMP(i)                                                                              \
  do {                                                                                        \
    if (stamp) rt.status->stamps[i] = wall_clock64();                                         \
  } while (0)

__global__ void __launch_bounds__(WG) k_resident(const ProgramDev* __restrict__ Pp, const FlowDev* __restrict__ Fp,
                                                 StatusDev* status, RunArgs a) {
  extern __shared__ float lds[];
  __shared__ int s_fail;
  const FlowDev& F = *Fp;
  const ProgramDev& P = *Pp;
  if (blockIdx.x % F.stride != 0) return;
  const int rank = blockIdx.x / F.stride;
  if (rank >= F.G) return;
  const int tid = threadIdx.x, G = F.G;
  if (tid == 0) s_fail = 0;
  Rt rt;
  rt.P = Pp; rt.F = Fp; rt.status = status; rt.lds = lds; rt.s_fail = &s_fail; rt.rank = rank;
  rt.spin_limit = a.spin_limit;
  flow_load(rt);

  const int n_conv = F.n_conv, n_fc = F.n_fc;
  const LayerDev& Lc = P.layers[n_conv - 1];       // last convolutional layer
  const LayerDev& L1 = P.layers[n_conv];           // first fully connected layer
  const int HWc = Lc.Hp * Lc.Wp;
  const int ncols = n_mine(Lc.Mo, rank, G) * HWc;  // own columns of the first fully connected layer
  const int n1 = L1.n_out;
  float* part = lds + F.o_part;
  float* act = lds + F.o_act;
  gfloat* g_out = a.grad_out;
  const float lr = a.lr;

  for (long long t = 0; t < a.n_images; ++t) {
    const unsigned int tag = a.epoch_base + (unsigned int)t + 1u;
    const unsigned int par = tag & 1u;
    const bool taps = (t == a.n_images - 1);
    const bool stamp = taps && rank == 0 && tid == 0;
    int label = a.labels ? a.labels[t] : a.label_imm;
    bool train = a.train != 0;
    if (train && (label < 0 || label >= P.n_classes)) {
      train = false;
      if (rank == 0 && tid == 0) status->bad_label = 1u;
    }
    STAMP(0);
    {  // the image
      const gfloat* img = a.images + t * a.image_stride;
      const LayerDev& L = P.layers[0];
      const int n = L.Mi * L.Hi * L.Wi;
      float* in = lds + F.conv[0].o_in;
      for (int x = tid; x < n; x += WG) in[x] = img[x];
      __syncthreads();
    }
    STAMP(1);
    // ---- FP, convolutional layers ----
    for (int l = 0; l < n_conv; ++l) {
      const LayerDev& L = P.layers[l];
      const FlowConv& C = F.conv[l];
      const int KK = L.K * L.K;
      if (l >= 1) {
        const int nw = L.Mi * L.Hi * L.Wi;
        if (!gather(rt, (unsigned int*)(lds + C.o_in), F.conv[l - 1].x_out + (size_t)par * nw, nw, tag)) return;
      }
      STAMP(2 + 2 * l);
      const int nm = n_mine(L.Mo, rank, G);
      for (int am = 0; am < nm; ++am) {
        flow_conv_fwd_map(L, lds + C.o_in, lds + C.o_wf + am * L.max_conn * KK,
                          (const int*)(lds + C.o_cidx) + am * L.max_conn, ((const int*)(lds + C.o_ncf))[am],
                          lds[C.o_bf + am], act, part);
        flow_pool_map(L, C, lds, am, rank + am * G, act, tag, taps);
      }
      STAMP(3 + 2 * l);
    }
    // ---- FP, first fully connected layer: partial sums over the own columns, exchanged ----
    {
      const float* wc = lds + F.fc[0].o_w;
      const float* vcol = lds + F.conv[n_conv - 1].o_pool;
      if (rank < F.n_col_ranks) {
        gtagged* xp = F.xp + ((size_t)par * F.n_col_ranks + rank) * n1;
        for (int k = tid; k < n1; k += WG) {
          float s = 0.f;
          for (int c = 0; c < ncols; ++c) s = fmaf(wc[c * n1 + k], vcol[c], s);
          put_f(xp + k, s, tag);
        }
      }
      STAMP(30);
      float* stage = lds + F.o_scratch;
      if (!gather(rt, (unsigned int*)stage, F.xp + (size_t)par * F.n_col_ranks * n1, F.n_col_ranks * n1, tag)) return;
      STAMP(31);
      float* y = lds + F.fc[0].o_act;
      const float* b = lds + F.fc[0].o_b;
      for (int k = tid; k < n1; k += WG) {
        float s = b[k];
        for (int r = 0; r < F.n_col_ranks; ++r) s += stage[r * n1 + k];
        y[k] = L1.is_output ? s : f_act(s);
      }
      __syncthreads();
    }
    // ---- FP, remaining fully connected layers: every rank computes all of them ----
    for (int f = 1; f < n_fc; ++f) {
      const LayerDev& L = P.layers[n_conv + f];
      float* y = lds + F.fc[f].o_act;
      flow_matvec(lds + F.fc[f].o_w, lds + F.fc[f].o_b, lds + F.fc[f - 1].o_act, y, L.n_out, L.n_in);
      if (!L.is_output) {
        for (int k = tid; k < L.n_out; k += WG) y[k] = f_act(y[k]);
        __syncthreads();
      }
    }
    STAMP(32);
    {  // soft-max, cross-entropy error, output delta  delta_k = p_k - [k == label]
      const LayerDev& L = P.layers[n_conv + n_fc - 1];
      float* y = lds + F.fc[n_fc - 1].o_act;
      float* d = lds + F.fc[n_fc - 1].o_delta;
      const int N = L.n_out;
      if (tid < 64) {
        float mx = -INFINITY;
        for (int k = tid; k < N; k += 64) mx = fmaxf(mx, y[k]);
        mx = f_wave_max(mx);
        float z = 0.f;
        for (int k = tid; k < N; k += 64) z += expf(y[k] - mx);
        z = f_wave_sum(z);
        for (int k = tid; k < N; k += 64) {
          const float p = expf(y[k] - mx) / z;
          y[k] = p;
          d[k] = p - (k == label ? 1.f : 0.f);
          if (rank == 0) {
            if (a.probs_out) a.probs_out[t * P.n_classes + k] = p;
            if (train && k == label) status->loss = -logf(p);
          }
        }
      }
      __syncthreads();
    }
    if (taps && rank == 0)
      for (int f = 0; f < n_fc; ++f) {
        const LayerDev& L = P.layers[n_conv + f];
        for (int k = tid; k < L.n_out; k += WG) L.act[k] = lds[F.fc[f].o_act + k];
      }
    STAMP(33);
    if (!train) continue;

    // ---- BP + AW, fully connected layers behind the first (every rank, same arithmetic) ----
    for (int f = n_fc - 1; f >= 1; --f) {
      const LayerDev& L = P.layers[n_conv + f];
      float* W = lds + F.fc[f].o_w;
      float* b = lds + F.fc[f].o_b;
      const float* d = lds + F.fc[f].o_delta;
      const float* v = lds + F.fc[f - 1].o_act;
      float* dprev = lds + F.fc[f - 1].o_delta;
      const int n_in = L.n_in, n_out = L.n_out;
      for (int m = tid; m < n_in; m += WG) {
        const float vm = v[m];
        float g = 0.f;
        for (int k = 0; k < n_out; ++k) {
          const float w = W[k * n_in + m];
          const float dk = d[k];
          g = fmaf(w, dk, g);
          if (g_out) { if (rank == 0) g_out[L.w_canon + (long long)k * n_in + m] = dk * vm; }
          else W[k * n_in + m] = fmaf(-lr, dk * vm, w);
        }
        dprev[m] = g * f_dact(vm);
      }
      for (int k = tid; k < n_out; k += WG) {
        if (g_out) { if (rank == 0) g_out[L.b_canon + k] = d[k]; }
        else b[k] = fmaf(-lr, d[k], b[k]);
        if (taps && rank == 0) L.delta[k] = d[k];
      }
      __syncthreads();
    }
    STAMP(34);
    {  // ---- BP + AW, first fully connected layer: own columns ----
      float* wc = lds + F.fc[0].o_w;
      float* b = lds + F.fc[0].o_b;
      const float* d = lds + F.fc[0].o_delta;
      const float* vcol = lds + F.conv[n_conv - 1].o_pool;
      float* dconv = lds + F.conv[n_conv - 1].o_delta;
      const int wave = tid >> 6, lane = tid & 63;
      for (int c = wave; c < ncols; c += WG / 64) {
        float s = 0.f;
        for (int k = lane; k < n1; k += 64) s = fmaf(wc[c * n1 + k], d[k], s);
        s = f_wave_sum(s);
        if (lane == 0) dconv[c] = s * f_dact(vcol[c]);
      }
      __syncthreads();
      for (int x = tid; x < ncols * n1; x += WG) {
        const int c = x / n1, k = x - c * n1;
        const float g = d[k] * vcol[c];
        if (g_out) {
          const int am = c / HWc, q = c - am * HWc;
          g_out[L1.w_canon + (long long)k * L1.n_in + (long long)(rank + am * G) * HWc + q] = g;
        } else {
          wc[x] = fmaf(-lr, g, wc[x]);
        }
      }
      for (int k = tid; k < n1; k += WG) {
        if (g_out) { if (rank == 0) g_out[L1.b_canon + k] = d[k]; }
        else b[k] = fmaf(-lr, d[k], b[k]);
        if (taps && rank == 0) L1.delta[k] = d[k];
      }
      __syncthreads();
    }
    STAMP(35);
    // ---- BP + AW, convolutional layers, top down ----
    for (int l = n_conv - 1; l >= 0; --l) {
      const LayerDev& L = P.layers[l];
      const FlowConv& C = F.conv[l];
      const int K = L.K, KK = K * K, HW = L.Hp * L.Wp, stride = L.S + 1, Wi = L.Wi, HiWi = L.Hi * L.Wi;
      const int nm = n_mine(L.Mo, rank, G);
      const float* dl = lds + C.o_delta;
      const int* yx = (const int*)(lds + C.o_yx);
      if (l >= 1 || taps) {
        for (int x = tid; x < nm * HW; x += WG) {
          const int am = x / HW, q = x - am * HW;
          const size_t o = (size_t)(rank + am * G) * HW + q;
          if (l >= 1) {
            put_f(C.x_delta + (size_t)par * L.Mo * HW + o, dl[x], tag);
            put_i(C.x_yx + (size_t)par * L.Mo * HW + o, yx[x], tag);
          }
          if (taps) L.delta[o] = dl[x];
        }
      }
      STAMP(40 + 4 * l);
      {  // forward copy of the own maps' filters, and their biases
        const int* cidx = (const int*)(lds + C.o_cidx);
        const int* ncf = (const int*)(lds + C.o_ncf);
        const float* in = lds + C.o_in;
        const int per_map = L.max_conn * KK;
        flow_wgrad(lds + C.o_wf, nm * per_map, HW, stride, Wi, C.wgrad_R_log2, lr, g_out, [&](int wi) {
          const int am = wi / per_map, rem = wi - am * per_map;
          const int c = rem / KK, tt = rem - c * KK;
          const int ky = tt / K, kx = tt - ky * K;
          WgradInfo I;
          I.ok = c < ncf[am];
          I.d = dl + am * HW;
          I.yx = yx + am * HW;
          I.in = in + cidx[am * L.max_conn + c] * HiWi + ky * Wi + kx;
          const int j = rank + am * G;
          I.canon = L.w_canon + (long long)((L.full_table ? j * L.Mi : L.csr_ptr[j]) + c) * KK + tt;
          return I;
        });
        const int wave = tid >> 6, lane = tid & 63;
        for (int am = wave; am < nm; am += WG / 64) {
          float s = 0.f;
          for (int q = lane; q < HW; q += 64) s += dl[am * HW + q];
          s = f_wave_sum(s);
          if (lane == 0) {
            if (g_out) g_out[L.b_canon + rank + am * G] = s;
            else lds[C.o_bf + am] = fmaf(-lr, s, lds[C.o_bf + am]);
          }
        }
        __syncthreads();
      }
      STAMP(41 + 4 * l);
      if (l >= 1) {
        const LayerDev& Lb = P.layers[l - 1];
        const FlowConv& Cb = F.conv[l - 1];
        const int nb = n_mine(L.Mi, rank, G);
        if (nb > 0) {
          float* dall = lds + F.o_dall;
          int* yxall = (int*)(lds + F.o_yxall);
          if (!gather(rt, (unsigned int*)dall, C.x_delta + (size_t)par * L.Mo * HW, L.Mo * HW, tag)) return;
          if (!gather(rt, (unsigned int*)yxall, C.x_yx + (size_t)par * L.Mo * HW, L.Mo * HW, tag)) return;
          STAMP(42 + 4 * l);
          const int* ncb = (const int*)(lds + C.o_ncb);
          for (int ab = 0; ab < nb; ++ab)
            flow_pull_map(rt, L, C, ab, ncb[ab], dall, yxall, lds + Cb.o_pool + ab * HiWi, lds + Cb.o_delta + ab * HiWi);
          STAMP(43 + 4 * l);
          // pull copy of the filters that read the own maps of the layer below
          const int* bj = (const int*)(lds + C.o_bj);
          const float* in = lds + C.o_in;
          const int per_map = C.max_back * KK;
          flow_wgrad(lds + C.o_wb, nb * per_map, HW, stride, Wi, C.wgrad_R_log2, lr, (gfloat*)nullptr, [&](int wi) {
            const int ab = wi / per_map, rem = wi - ab * per_map;
            const int e = rem / KK, tt = rem - e * KK;
            const int ky = tt / K, kx = tt - ky * K;
            const int j = bj[ab * C.max_back + e];
            WgradInfo I;
            I.ok = e < ncb[ab] && !g_out;
            I.d = dall + j * HW;
            I.yx = yxall + j * HW;
            I.in = in + (rank + ab * G) * HiWi + ky * Wi + kx;
            I.canon = 0;
            return I;
          });
          __syncthreads();
        }
        (void)Lb;
      }
    }
    STAMP(60);
  }
  if (!g_out && a.train) flow_store(rt);
}

hipError_t launch_resident(int grid, size_t lds_bytes, hipStream_t stream, const ProgramDev* d_prog,
                           const FlowDev* d_flow, StatusDev* d_status, const RunArgs& a) {
  hipError_t e = hipFuncSetAttribute((const void*)k_resident, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  RunArgs args = a;
  void* params[] = {(void*)&d_prog, (void*)&d_flow, (void*)&d_status, (void*)&args};
  return hipLaunchCooperativeKernel((const void*)k_resident, dim3(grid), dim3(WG), params, (unsigned int)lds_bytes, stream);
}

}  // namespace cnn355
