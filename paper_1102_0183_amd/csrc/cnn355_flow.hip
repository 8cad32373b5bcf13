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
//
// Inside a rank the two heavy loops (FP of a map, and the delta pull, which is FP's mirror image:
// a correlation of the zero-padded delta maps with the filters rotated by 180 degrees) keep a strip
// of output pixels in registers, so that one LDS read of an input or a weight feeds several
// multiply-adds; with one pixel per lane the loop is bound by LDS bandwidth, not by the ALUs.
#include <hip/hip_runtime.h>

#if defined(__HIP_DEVICE_COMPILE__)
#define CNN_GLOBAL __attribute__((address_space(1)))
#endif
#include "cnn355_dev.h"
#include "cnn355_flowspec.h"

namespace cnn355 {

typedef CNN_GLOBAL float gfloat;
typedef CNN_GLOBAL tagged_t gtagged;

#define ACT_A 1.7159f
#define ACT_B 0.6666f
// Scaled hyperbolic tangent of Sec. 4, constants as printed, as 1 - 2 / (e^{2Ba} + 1) on the hardware
// exponential and reciprocal: absolute error about 3e-7 (the library tanhf costs thirty times as
// many cycles on the critical path of every layer); saturates correctly at both ends.  This one is for the
// units of the convolutional layers (the series below, applied to them too, was measured to cost 1.3 % of the
// time per image of the benchmark net).
__device__ __forceinline__ float f_act(float a) {
  const float z = __builtin_amdgcn_exp2f((2.0f * ACT_B * 1.44269504088896340736f) * a);
  return fmaf(-2.0f * ACT_A, __builtin_amdgcn_rcpf(z + 1.0f), ACT_A);
}
// The same for the units of the fully connected layers (one per lane, once per image: what it costs does not
// show): below |Ba| = 0.3 the odd series of tanh up to x^9 (next term 1382/155925 x^11: 5e-8 of the result at
// 0.3), so that a small output keeps its digits.
__device__ __forceinline__ float f_act_fc(float a) {
  const float big = f_act(a);
  const float x = ACT_B * a, x2 = x * x;
  float p = fmaf(x2, 62.0f / 2835.0f, -17.0f / 315.0f);
  p = fmaf(x2, p, 2.0f / 15.0f);
  p = fmaf(x2, p, -1.0f / 3.0f);
  const float small = ACT_A * fmaf(x, x2 * p, x);
  return fabsf(x) < 0.3f ? small : big;
}
// Its derivative A B (1 - tanh^2(B a)) = 4 A B z / (1 + z)^2 with z = e^{-2B|a|}, taken from the sum a the
// unit received: no difference of nearly equal numbers anywhere, so a saturated unit keeps the relative
// accuracy of its z (written in terms of the output, A B - (B/A) y^2, the two terms cancel to 1e-3 of
// themselves there and fp32 keeps only 1e-4 of the result).
__device__ __forceinline__ float f_dact_pre(float a) {
  const float z = __builtin_amdgcn_exp2f(-(2.0f * ACT_B * 1.44269504088896340736f) * fabsf(a));
  const float r = __builtin_amdgcn_rcpf(z + 1.0f);
  return (4.0f * ACT_A * ACT_B) * z * r * r;
}
// Cross-lane moves inside a row of 16 lanes through the data-parallel primitives of the ALU (a few
// cycles each), instead of the LDS crossbar a general shuffle goes through (an LDS latency each).
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
#define DPP_XOR1 0xB1         // quad_perm [1,0,3,2]
#define DPP_XOR2 0x4E         // quad_perm [2,3,0,1]
#define DPP_HALF_MIRROR 0x141 // lane i <-> 7 - i of every 8
#define DPP_MIRROR 0x140      // lane i <-> 15 - i of every 16
__device__ __forceinline__ float lane_f(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// Sum over the aligned group of 2^gl2 lanes (gl2 <= 6) each lane belongs to; every lane of the group
// gets the same bits (each step adds two values that are equal across the halves it joins).
__device__ __forceinline__ float group_sum(float v, int gl2) {
  if (gl2 >= 1) v += dpp_mov<DPP_XOR1>(v);
  if (gl2 >= 2) v += dpp_mov<DPP_XOR2>(v);
  if (gl2 >= 3) v += dpp_mov<DPP_HALF_MIRROR>(v);
  if (gl2 >= 4) v += dpp_mov<DPP_MIRROR>(v);
  if (gl2 >= 5) v += __shfl_xor(v, 16, 64);
  if (gl2 >= 6) v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ __forceinline__ float f_wave_sum(float v) {
  v += dpp_mov<DPP_XOR1>(v);
  v += dpp_mov<DPP_XOR2>(v);
  v += dpp_mov<DPP_HALF_MIRROR>(v);
  v += dpp_mov<DPP_MIRROR>(v);
  return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}
__device__ __forceinline__ float f_wave_max(float v) {
  v = fmaxf(v, dpp_mov<DPP_XOR1>(v));
  v = fmaxf(v, dpp_mov<DPP_XOR2>(v));
  v = fmaxf(v, dpp_mov<DPP_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_mov<DPP_MIRROR>(v));
  return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}

// sum of part[p], part[p + pitch], ... (n terms) in that order, the LDS reads issued eight at a time
__device__ __forceinline__ float sum_strided(const float* part, int n, int pitch, int p) {
  float s = 0.f;
  for (int r0 = 0; r0 < n; r0 += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[min(r0 + u, n - 1) * pitch + p];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (r0 + u < n) ? v[u] : 0.f;
  }
  return s;
}

// The same sums for tot outputs p, fn(p, sum) called once per output.  With many terms and few
// outputs eight lanes share an output -- lane g adds the terms g, g + 8, ... in that order, the
// eight are then added across the lanes in a fixed pattern -- instead of one lane walking a long
// chain of dependent LDS reads.
template <class Fn>
__device__ __forceinline__ void reduce_partials(const float* part, int n, int tot, Fn fn) {
  const int tid = threadIdx.x;
  int gl2 = 0;                                  // log2 of the lanes that share an output: up to 8
  if (n >= 16)
    while (gl2 < 3 && (tot << (gl2 + 1)) <= WG) ++gl2;
  if (gl2 > 0) {
    const int G = 1 << gl2;
    const int p = tid >> gl2, g = tid & (G - 1);
    float s = 0.f;
    if (p < tot)
      for (int r0 = g; r0 < n; r0 += 4 * G) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = part[min(r0 + u * G, n - 1) * tot + p];
#pragma unroll
        for (int u = 0; u < 4; ++u) s += (r0 + u * G < n) ? v[u] : 0.f;
      }
    s = group_sum(s, gl2);
    if (p < tot && g == 0) fn(p, s);
  } else {
    for (int p = tid; p < tot; p += WG) fn(p, sum_strided(part, n, tot, p));
  }
}

__device__ __forceinline__ int n_mine(int M, int rank, int G) { return rank < M ? (M - rank + G - 1) / G : 0; }
// Input maps of a layer with Mi of them whose delta pull a rank works on: its own maps i = rank, rank + G, ...
// (all entries of each), or, when the pull is shared (H > 1 shares per map), the one map rank % Mi, share rank / Mi.
__device__ __forceinline__ int n_pull_maps(int Mi, int rank, int G, int H) {
  return H > 1 ? (rank < H * Mi ? 1 : 0) : n_mine(Mi, rank, G);
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// x / d for 0 <= x < 2^20 and 1 <= d < 2^20 by a float multiplication with the hardware
// reciprocal (1 ulp): (x + 0.5) / d lies at least 0.5 / d away from the next integer, the
// product is off by less than x / d * 2^-21, which is smaller
// (a divisor the compiler knows -- the kernels instantiated for a fixed network -- is divided by directly)
struct FDiv {
  int d;
  float inv;
  __device__ __forceinline__ explicit FDiv(int d_) : d(d_), inv(__builtin_amdgcn_rcpf((float)d_)) {}
  __device__ __forceinline__ int div(int x) const {
    return __builtin_constant_p(d) ? x / d : (int)(((float)x + 0.5f) * inv);
  }
};

// ---- tagged words ---------------------------------------------------------------------------
__device__ __forceinline__ void put_f(gtagged* p, float v, unsigned int tag) {
  const tagged_t w = ((tagged_t)tag << 32) | (tagged_t)__float_as_uint(v);
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void put_i(gtagged* p, int v, unsigned int tag) {
  const tagged_t w = ((tagged_t)tag << 32) | (tagged_t)(unsigned int)v;
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A copy of the plan and of the pointers in LDS: reading them from global memory in every phase of
// every image costs a memory round trip each time the scalar cache has dropped them.  A kernel
// instantiated for a fixed network (ID > 0) takes the plan from StaticSpec<ID> instead, as literals.
struct JobDyn {  // the part of a correlation job that depends on the rank
  int n_maps, U, R, passes;
};
struct Shared {
  FlowPtrs ptrs;
  JobDyn fwd[FLOW_MAX_CONV];   // FP of the own maps of every convolutional layer
  JobDyn pull[FLOW_MAX_CONV];  // delta pull through layer l into the own maps of layer l-1 (l >= 1)
  int fail;
};

static_assert(sizeof(Shared) + sizeof(float) * FLOW_LDS_FLOATS_MAX <= 160 * 1024, "LDS of one gfx950 compute unit");

#ifdef CNN355_STAMPS
#define DSTAMP(i) do { if (rt.dbg) rt.status->stamps[i] = wall_clock64(); } while (0)
#else
#define DSTAMP(i) do { } while (0)
#endif

struct Rt {  // what every phase needs
  bool dbg;
  const FlowSpec* spec;  // the plan (the kernel argument)
  Shared* sh;
  StatusDev* status;
  float* lds;
  int rank;
  unsigned int spin_limit;
};

// The plan: literals in a kernel instantiated for a fixed network, the kernel's by-value argument otherwise
// (read with scalar loads, uniform by construction).  (A
// function-local constexpr copy, not a reference to the class-scope constant: a device-side
// global may be initialised from outside the module, so the compiler would not fold its contents.)
#define DECL_SPEC(Z, rt_)                                                    \
  constexpr FlowSpec Z##_lit = StaticSpec<(ID ? ID : 1)>::value;             \
  const FlowSpec& Z = ID ? Z##_lit : *(rt_).spec
// a value every lane holds alike, made known to the compiler as such (nothing to do for a literal)
template <int ID>
__device__ __forceinline__ int uni_of(int v) {
  if constexpr (ID == 0) return __builtin_amdgcn_readfirstlane(v);
  else return v;
}

// Loops over layers.  In a kernel instantiated for a fixed network they are unrolled by the
// compiler front end itself (the layer index is a template constant in every copy), so that
// every size and offset taken from the plan folds; otherwise they are ordinary loops.  The body
// returns false to stop (a wait gave up).
template <int V>
struct IC { static constexpr int value = V; };
__device__ __forceinline__ constexpr int lv(int x) { return x; }
template <int V>
__device__ __forceinline__ constexpr int lv(IC<V>) { return V; }

template <int I, int MAXN, class F>
__device__ __forceinline__ bool for_up_static(int n, F& f) {
  if constexpr (I < MAXN) {
    if (I < n && !f(IC<I>{})) return false;
    return for_up_static<I + 1, MAXN>(n, f);
  } else {
    return true;
  }
}
template <int I, int LO, class F>
__device__ __forceinline__ bool for_down_static(int n, F& f) {
  if constexpr (I >= LO) {
    if (I < n && !f(IC<I>{})) return false;
    return for_down_static<I - 1, LO>(n, f);
  } else {
    return true;
  }
}
// l = LO .. n-1
template <int ID, int LO, int MAXN, class F>
__device__ __forceinline__ bool for_up(int n, F f) {
  if constexpr (ID == 0) {
    for (int l = LO; l < n; ++l)
      if (!f(l)) return false;
    return true;
  } else {
    return for_up_static<LO, MAXN>(n, f);
  }
}
// l = n-1 .. LO
template <int ID, int LO, int MAXN, class F>
__device__ __forceinline__ bool for_down(int n, F f) {
  if constexpr (ID == 0) {
    for (int l = n - 1; l >= LO; --l)
      if (!f(l)) return false;
    return true;
  } else {
    return for_down_static<MAXN - 1, LO>(n, f);
  }
}

// Bounded polling: returns false when this lane has polled too often or another workgroup has
// raised the abort flag; the flag is raised so that every workgroup leaves.
__device__ __forceinline__ bool poll_again(const Rt& rt, unsigned int& spins) {
  ++spins;
  if (spins > rt.spin_limit ||
      ((spins & 63u) == 0u && __hip_atomic_load(&rt.status->abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
    __hip_atomic_store(&rt.status->abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    rt.sh->fail = 1;
    return false;
  }
  __builtin_amdgcn_s_sleep(1);
  return true;
}

// Fetch U tagged words (addr(u) gives their places) until every one carries `tag`: all are loaded
// together, again and again.  False: gave up.
template <int U, class Addr>
__device__ __forceinline__ bool fetch_tagged(const Rt& rt, tagged_t (&w)[U], unsigned int tag, Addr addr) {
  unsigned int spins = 0;
  while (true) {
#pragma unroll
    for (int u = 0; u < U; ++u) w[u] = __hip_atomic_load(addr(u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool done = true;
#pragma unroll
    for (int u = 0; u < U; ++u) done = done && ((unsigned int)(w[u] >> 32) == tag);
    if (done) return true;
    if (!poll_again(rt, spins)) return false;
  }
}

// Copy n tagged words into LDS (their 32-bit payloads), each lane waiting for its own words to
// carry `tag`.  Ends with a workgroup barrier; returns false (to every thread of the workgroup)
// when a wait gave up: the caller then leaves the kernel.
__device__ __forceinline__ bool gather(const Rt& rt, unsigned int* dst, const gtagged* src, int n, unsigned int tag) {
  constexpr int U = 4;
  const int tid = threadIdx.x;
  for (int base = 0; base < n; base += U * WG) {
    tagged_t w[U];
    if (!fetch_tagged<U>(rt, w, tag, [&](int u) { return src + min(base + tid + u * WG, n - 1); })) break;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + tid + u * WG < n) dst[base + tid + u * WG] = (unsigned int)w[u];
  }
  __syncthreads();
  return rt.sh->fail == 0;
}

// The same for two arrays of n words each, fetched together (one round trip instead of two).
__device__ __forceinline__ bool gather2(const Rt& rt, unsigned int* dst_a, const gtagged* src_a, unsigned int* dst_b,
                                        const gtagged* src_b, int n, unsigned int tag) {
  constexpr int U = 2;
  const int tid = threadIdx.x;
  for (int base = 0; base < n; base += U * WG) {
    tagged_t w[2 * U];
    if (!fetch_tagged<2 * U>(rt, w, tag, [&](int u) {
          return ((u & 1) ? src_b : src_a) + min(base + tid + (u >> 1) * WG, n - 1);
        }))
      break;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + tid + u * WG < n) {
        dst_a[base + tid + u * WG] = (unsigned int)w[2 * u];
        dst_b[base + tid + u * WG] = (unsigned int)w[2 * u + 1];
      }
  }
  __syncthreads();
  return rt.sh->fail == 0;
}

// ---- bulk exchange (streamed plans) -----------------------------------------------------------------
// The pooled maps a wide layer hands to the next are too many words to poll one by one, twice over.  In a
// streamed plan they travel as plain floats, written through to device scope, plus one flag word per map that
// its owner sets to the image's tag once the stores have completed; a reader polls the flags of the maps it is
// about to fetch and then loads their floats 128 bits at a time, past the caches.  Layout inside the layer's
// exchange area of 2 N tagged words (N = Mo Hp Wp): floats [2][N], then flags [2][Mo].
typedef unsigned int u4v __attribute__((ext_vector_type(4)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef CNN_GLOBAL unsigned int guint;
__device__ __forceinline__ gfloat* bulk_data(gtagged* x, int N, unsigned int par) { return (gfloat*)x + (size_t)par * N; }
__device__ __forceinline__ guint* bulk_flags(gtagged* x, int N, int Mo, unsigned int par) {
  return (guint*)((gfloat*)x + 2 * (size_t)N) + (size_t)par * Mo;
}
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// n floats at `data` (whose n_flags maps' flags must carry `tag`) -> dst (16-byte aligned LDS, may be written up to
// 3 floats past n).  Ends with a workgroup barrier; false: a wait gave up.
__device__ __forceinline__ bool gather_bulk(const Rt& rt, float* dst, const gfloat* data, int n, const guint* flags,
                                            int n_flags, unsigned int tag) {
  const int tid = threadIdx.x;
  for (int m = tid; m < n_flags; m += WG) {
    unsigned int spins = 0;
    while (__hip_atomic_load(flags + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tag)
      if (!poll_again(rt, spins)) break;
  }
  __syncthreads();
  if (rt.sh->fail) return false;
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)data, 0, n * 4, 0x00020000);
  constexpr int U = 4;
  for (int base = tid * 4; base < n; base += U * WG * 4) {
    u4v v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)   // (a load past n floats returns zeros: the buffer descriptor bounds it)
      v[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, (base + u * WG * 4) * 4, 0, 16 /* device scope */);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + u * WG * 4 < n) *(u4v*)(dst + base + u * WG * 4) = v[u];
  }
  __syncthreads();
  return true;
}

// The same in three steps, so that a chunk can be on its way while the one before it is worked on: wait for the
// flags (ends with a workgroup barrier), issue the loads into registers (at most BULK_PF x 128 bits a lane: chunks
// of up to BULK_PF * 4 * WG floats), store the registers to LDS.
constexpr int BULK_PF = 4;
__device__ __forceinline__ bool bulk_wait(const Rt& rt, const guint* flags, int n_flags, unsigned int tag) {
  for (int m = threadIdx.x; m < n_flags; m += WG) {
    unsigned int spins = 0;
    while (__hip_atomic_load(flags + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tag)
      if (!poll_again(rt, spins)) break;
  }
  __syncthreads();
  return rt.sh->fail == 0;
}
__device__ __forceinline__ void bulk_issue(u4v (&v)[BULK_PF], const gfloat* data, int n) {
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)data, 0, n * 4, 0x00020000);
#pragma unroll
  for (int u = 0; u < BULK_PF; ++u)   // (a load past n floats returns zeros: the buffer descriptor bounds it)
    v[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, (threadIdx.x * 4 + u * WG * 4) * 4, 0, 16 /* device scope */);
}
__device__ __forceinline__ void bulk_commit(const u4v (&v)[BULK_PF], float* dst, int n) {
#pragma unroll
  for (int u = 0; u < BULK_PF; ++u)
    if ((int)threadIdx.x * 4 + u * WG * 4 < n) *(u4v*)(dst + threadIdx.x * 4 + u * WG * 4) = v[u];
}

// ---- weights: global (canonical order) <-> LDS -------------------------------------------------
template <int ID>
__device__ __forceinline__ void flow_load(const Rt& rt) {
  DECL_SPEC(Z, rt);
  const FlowPtrs& Q = rt.sh->ptrs;
  float* lds = rt.lds;
  const int tid = threadIdx.x, G = Z.G, rank = rt.rank;
  for (int x = tid; x < Z.scratch_floats; x += WG) lds[Z.o_scratch + x] = 0.f;  // stays zero between uses
  for_up<ID, 0, FLOW_MAX_CONV>(Z.n_conv, [&](auto lc) {
    const int l = lv(lc);
    const ConvSpec& C = Z.conv[l];
    const FlowConvPtrs& P = Q.conv[l];
    const int KK = C.K * C.K;
    const int nm = n_mine(C.Mo, rank, G);
    float* wf = lds + C.o_wf;
    float* bf = lds + C.o_bf;
    int* cidx = (int*)(lds + C.o_cidx);
    int* ncf = (int*)(lds + C.o_ncf);
    for (int a = 0; a < nm; ++a) {
      const int j = rank + a * G;
      int cb = j * C.Mi, nc = C.Mi;
      if (!C.full_table) { cb = P.csr_ptr[j]; nc = P.csr_ptr[j + 1] - cb; }
      for (int x = tid; x < C.max_conn * KK; x += WG)
        wf[a * C.max_conn * KK + x] = (x < nc * KK) ? P.w[(size_t)cb * KK + x] : 0.f;
      for (int c = tid; c < C.max_conn; c += WG)
        cidx[a * C.max_conn + c] = (c < nc) ? (C.full_table ? c : P.csr_idx[cb + c]) : 0;
      if (tid == 0) { bf[a] = P.bias[j]; ncf[a] = nc; }
    }
    if (l >= 1) {
      // pull copy: the filters that read the own maps of the layer below, each rotated by 180
      // degrees (tap t stored at K*K-1-t), entries in ascending order of the output map
      const int H = C.pull_shares, BP = C.back_pitch;
      const int nb = n_pull_maps(C.Mi, rank, G, H);
      float* wb = lds + C.o_wb;
      int* bj = (int*)(lds + C.o_bj);
      int* ncb = (int*)(lds + C.o_ncb);
      for (int a = 0; a < nb; ++a) {
        const int i = H > 1 ? rank % C.Mi : rank + a * G;
        int eb = 0, ne = C.Mo;
        if (!C.full_table) { eb = P.csc_ptr[i]; ne = P.csc_ptr[i + 1] - eb; }
        if (H > 1) {  // this rank's share of the map's entries
          const int h = rank / C.Mi;
          const int lo = (int)((long long)ne * h / H), hi = (int)((long long)ne * (h + 1) / H);
          eb += lo;
          ne = hi - lo;
        }
        const int e0 = C.full_table ? eb : 0;  // (full table: entry e is output map e, eb counts from 0)
        for (int x = tid; x < BP * KK; x += WG) {
          const int e = x / KK, t = x - e * KK;
          float v = 0.f;
          if (e < ne) {
            const int slot = C.full_table ? ((e0 + e) * C.Mi + i) : P.csc_slot[eb + e];
            v = P.w[(size_t)slot * KK + (KK - 1 - t)];
          }
          wb[a * BP * KK + x] = v;
        }
        for (int e = tid; e < BP; e += WG)
          bj[a * BP + e] = (e < ne) ? (C.full_table ? e0 + e : P.csc_j[eb + e]) : 0;
        if (tid == 0) ncb[a] = ne;
      }
    }
    return true;
  });
  {  // first fully connected layer: the columns fed by the own maps of the last convolutional layer
    const ConvSpec& Cc = Z.conv[Z.n_conv - 1];
    const FcSpec& L = Z.fc[0];
    const int HW = Cc.Hp * Cc.Wp, n1 = L.n_out;
    const int nm = n_mine(Cc.Mo, rank, G);
    float* wc = lds + L.o_w;
    for (int x = tid; x < nm * HW * n1; x += WG) {
      const int c = x / n1, k = x - c * n1;
      const int a = c / HW, q = c - a * HW;
      wc[x] = Q.fc[0].w[(size_t)k * L.n_in + (size_t)(rank + a * G) * HW + q];
    }
    for (int k = tid; k < n1; k += WG) lds[L.o_b + k] = Q.fc[0].bias[k];
  }
  for_up<ID, 1, FLOW_MAX_FC>(Z.n_fc, [&](auto fc_) {
    const int f = lv(fc_);
    const FcSpec& L = Z.fc[f];
    if (L.by_cols) {  // the columns rank, rank + G, ... of the weight matrix, column after column
      const int nq = n_mine(L.n_in, rank, G) * L.n_out;
      for (int x = tid; x < nq; x += WG) {
        const int c = x / L.n_out, k = x - c * L.n_out;
        lds[L.o_w + x] = Q.fc[f].w[(size_t)k * L.n_in + rank + c * G];
      }
    } else {
      for (int x = tid; x < L.n_out * L.n_in; x += WG) lds[L.o_w + x] = Q.fc[f].w[x];
    }
    for (int k = tid; k < L.n_out; k += WG) lds[L.o_b + k] = Q.fc[f].bias[k];
    return true;
  });
  __syncthreads();
}

template <int ID>
__device__ __forceinline__ void flow_store(const Rt& rt) {
  DECL_SPEC(Z, rt);
  const FlowPtrs& Q = rt.sh->ptrs;
  float* lds = rt.lds;
  const int tid = threadIdx.x, G = Z.G, rank = rt.rank;
  __syncthreads();
  for_up<ID, 0, FLOW_MAX_CONV>(Z.n_conv, [&](auto lc) {
    const int l = lv(lc);
    const ConvSpec& C = Z.conv[l];
    const FlowConvPtrs& P = Q.conv[l];
    const int KK = C.K * C.K;
    const int nm = n_mine(C.Mo, rank, G);
    const int* ncf = (const int*)(lds + C.o_ncf);
    for (int a = 0; a < nm; ++a) {
      const int j = rank + a * G;
      const int nc = ncf[a];
      const int cb = C.full_table ? j * C.Mi : P.csr_ptr[j];
      for (int x = tid; x < nc * KK; x += WG) P.w[(size_t)cb * KK + x] = lds[C.o_wf + a * C.max_conn * KK + x];
      if (tid == 0) P.bias[j] = lds[C.o_bf + a];
    }
    return true;
  });
  {
    const ConvSpec& Cc = Z.conv[Z.n_conv - 1];
    const FcSpec& L = Z.fc[0];
    const int HW = Cc.Hp * Cc.Wp, n1 = L.n_out;
    const int nm = n_mine(Cc.Mo, rank, G);
    for (int x = tid; x < nm * HW * n1; x += WG) {
      const int c = x / n1, k = x - c * n1;
      const int a = c / HW, q = c - a * HW;
      Q.fc[0].w[(size_t)k * L.n_in + (size_t)(rank + a * G) * HW + q] = lds[L.o_w + x];
    }
    if (rank == 0)
      for (int k = tid; k < n1; k += WG) Q.fc[0].bias[k] = lds[L.o_b + k];
  }
  for_up<ID, 1, FLOW_MAX_FC>(Z.n_fc, [&](auto fc_) {
    const int f = lv(fc_);
    const FcSpec& L = Z.fc[f];
    if (L.by_cols) {
      const int nq = n_mine(L.n_in, rank, G) * L.n_out;
      for (int x = tid; x < nq; x += WG) {
        const int c = x / L.n_out, k = x - c * L.n_out;
        Q.fc[f].w[(size_t)k * L.n_in + rank + c * G] = lds[L.o_w + x];
      }
    } else if (rank == 0) {
      for (int x = tid; x < L.n_out * L.n_in; x += WG) Q.fc[f].w[x] = lds[L.o_w + x];
    }
    if (rank == 0)
      for (int k = tid; k < L.n_out; k += WG) Q.fc[f].bias[k] = lds[L.o_b + k];
    return true;
  });
}

// ---- the two multiply-accumulate loops -------------------------------------------------------------
// One output pixel: sum over the connections c0, c0 + cstep, ... < nc and the K x K taps.  Map
// of connection c is idx[c] - idx_off.  Any K (KT = 0: run-time size).
template <int KT>
__device__ __forceinline__ float pixel_mac(const float* in, const float* w, const int* idx, int idx_off, int c0,
                                           int cstep, int nc, int map_sz, int Wi, int Krt, int base) {
  const int K = KT ? KT : Krt;
  const int KK = K * K;
  float acc = 0.f;
  for (int c = c0; c < nc; c += cstep) {
    const float* ip = in + (idx[c] - idx_off) * map_sz + base;
    const float* wp = w + c * KK;
#pragma unroll
    for (int ky = 0; ky < K; ++ky)
#pragma unroll
      for (int kx = 0; kx < K; ++kx) acc = fmaf(wp[ky * K + kx], ip[ky * Wi + kx], acc);
  }
  return acc;
}
__device__ __forceinline__ float pixel_mac_k(int K, const float* in, const float* w, const int* idx, int idx_off,
                                             int c0, int cstep, int nc, int map_sz, int Wi, int base) {
  switch (K) {
    case 1: return pixel_mac<1>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
    case 2: return pixel_mac<2>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
    case 3: return pixel_mac<3>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
    case 4: return pixel_mac<4>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
    case 5: return pixel_mac<5>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
    default: return pixel_mac<0>(in, w, idx, idx_off, c0, cstep, nc, map_sz, Wi, K, base);
  }
}

// A tile of TH rows x SW consecutive output pixels, input stride ST.  Per connection the K*K weights
// are read once; every input row of (SW-1)ST+K floats is read once and feeds the (up to K) kernel rows
// and (up to TH) output rows it meets: ((TH-1)ST+K)((SW-1)ST+K) + K*K LDS reads for TH*SW*K*K multiply-adds.
// CLIP: only the input rows iy in [iy_lo, iy_hi) are read; the others are known to hold zeros.
template <int K, int SW, int TH, bool CLIP, int ST>
__device__ __forceinline__ void strip_mac(const float* in, const float* w, const int* idx, int idx_off, int c0,
                                          int cstep, int nc, int map_sz, int Wi, int base, int iy_lo, int iy_hi,
                                          float (&acc)[TH * SW]) {
  for (int c = c0; c < nc; c += cstep) {
    const float* ip = in + (idx[c] - idx_off) * map_sz + base;
    const float* wp = w + c * (K * K);
    float wk[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) wk[t] = wp[t];
#pragma unroll
    for (int iy = 0; iy < (TH - 1) * ST + K; ++iy) {
      if (CLIP && (iy < iy_lo || iy >= iy_hi)) continue;
      float row[(SW - 1) * ST + K];
#pragma unroll
      for (int i = 0; i < (SW - 1) * ST + K; ++i) row[i] = ip[iy * Wi + i];
#pragma unroll
      for (int ty = 0; ty < TH; ++ty) {
        const int ky = iy - ty * ST;
        if (ky >= 0 && ky < K) {
#pragma unroll
          for (int s = 0; s < SW; ++s)
#pragma unroll
            for (int kx = 0; kx < K; ++kx)
              acc[ty * SW + s] = fmaf(wk[ky * K + kx], row[s * ST + kx], acc[ty * SW + s]);
        }
      }
    }
  }
}

// A correlation job: n_maps output maps of Ho x Wo, each the sum over its connection list of
// K x K correlations (unit stride for the strip form) of input maps of map_sz floats and row
// pitch Wi.  Lanes take (map, row, strip of SW pixels) units, or (map, pixel) units when SW = 1,
// and share the connections R ways when there are fewer units than lanes; partial sums go to
// part[(r * n_maps + map) * Ho*Wo + pixel].  A job is the same for every image of a call: the
// part of it that depends on the rank (how many maps, hence units and ways) is worked out once,
// and (LDS permitting) every lane's share of it is decoded once and kept in a table, because
// working it out again per image -- integer divisions, a dozen descriptor reads -- costs more
// than the multiply-accumulates of a small layer.
struct JobStat {  // the part of a job the plan fixes
  int in, w, idx, cnt;  // LDS offsets (floats): inputs [..][map_sz], weights [n_maps][w_pitch][K*K],
                        // input map of every connection [n_maps][w_pitch], connections per map [n_maps]
  int w_pitch, Ho, Wo, K, stride, map_sz, Wi, max_cnt;
  int plan_cnt;         // the connection count the planner sized the partial sums for (>= max_cnt)
  int variant;          // (stride - 1) * 128 + (TH - 1) * 64 + SW * 8 + K for a job in tiles of TH rows x SW pixels, 0: one pixel per
                        // lane (any K, any stride)
  int table;            // LDS offset of the lane table [3][WG] (int), or -1
  int band_lo, band_hi; // rows [band_lo, band_hi) of an input map that can hold non-zeros; outside lie the zero
                        // borders of the pull's delta maps (FP: the whole map)
  int ways_side_by_side; // lanes that share a unit are neighbours, so that a wavefront's lanes skip the same rows
                        // (they then read different maps and filters at once: map_sz and K * K must be odd
                        // to spread those reads over the LDS banks)
};
__device__ __forceinline__ JobStat fwd_job(const FlowSpec& Z, int l) {
  const ConvSpec& C = Z.conv[l];
  JobStat S;
  S.in = C.o_in; S.w = C.o_wf; S.idx = C.o_cidx; S.cnt = C.o_ncf;
  S.w_pitch = C.max_conn; S.Ho = C.Ho; S.Wo = C.Wo; S.K = C.K; S.stride = C.S + 1;
  S.map_sz = C.Hi * C.Wi; S.Wi = C.Wi; S.max_cnt = min(C.max_conn, C.in_chunk); S.plan_cnt = C.max_conn;
  S.variant = C.fwd_strip ? C.S * 128 + (C.fwd_rows - 1) * 64 + C.fwd_strip * 8 + C.K : 0;
  S.table = C.o_tab_fwd;
  S.band_lo = 0; S.band_hi = C.Hi; S.ways_side_by_side = 0;
  return S;
}
__device__ __forceinline__ JobStat pull_job(const FlowSpec& Z, int l) {
  const ConvSpec& C = Z.conv[l];
  JobStat S;
  S.in = Z.o_scratch; S.w = C.o_wb; S.idx = C.o_bj; S.cnt = C.o_ncb;
  S.w_pitch = C.back_pitch; S.Ho = C.Hi; S.Wo = C.Wi; S.K = C.K; S.stride = 1;
  S.Wi = C.Wi + C.K - 1; S.map_sz = (int)flow_border_map(C.Hi, C.Wi, C.K);
  S.max_cnt = min(C.back_pitch, C.pull_chunk);
  S.plan_cnt = min(C.back_pitch, C.Mo);
  S.variant = C.pull_strip ? (C.pull_rows - 1) * 64 + C.pull_strip * 8 + C.K : 0;
  S.table = C.o_tab_pull;
  S.band_lo = C.K - 1; S.band_hi = C.K - 1 + (C.Ho - 1) * (C.S + 1) + 1; S.ways_side_by_side = C.K & 1;
  return S;
}

struct Lane {
  int r, am, pix, base, ncols, nrows;
  bool on;
};

__device__ __forceinline__ JobDyn job_dyn(const JobStat& S, int n_maps) {
  const int SW = (S.variant >> 3) & 7, TH = ((S.variant >> 6) & 1) + 1;
  JobDyn D;
  D.n_maps = n_maps;
  D.U = SW ? n_maps * ((S.Ho + TH - 1) / TH) * ((S.Wo + SW - 1) / SW) : n_maps * S.Ho * S.Wo;
  // the ways one chunk of connections can be shared, but never more than the planner laid out
  // partial sums for (it counted the whole list; a shorter chunk can divide into more ways)
  D.R = min(flow_split_ways(D.U, S.max_cnt), flow_split_ways(D.U, S.plan_cnt));
  D.passes = (D.U * D.R + WG - 1) / WG;
  return D;
}

// the share of lane `tid` in pass `pass`
__device__ __forceinline__ Lane lane_decode(const JobStat& S, const JobDyn& D, int pass) {
  const int SW = (S.variant >> 3) & 7, TH = ((S.variant >> 6) & 1) + 1;
  Lane ln;
  const int u = pass * WG + (int)threadIdx.x;
  ln.on = u < D.U * D.R;
  int v;
  if (S.ways_side_by_side) {
    const FDiv dR(D.R);
    v = dR.div(u);
    ln.r = u - v * D.R;
  } else {
    const FDiv dU(D.U);
    ln.r = dU.div(u);
    v = u - ln.r * D.U;
  }
  ln.nrows = 1;
  if (SW) {
    const int NS = (S.Wo + SW - 1) / SW, NG = (S.Ho + TH - 1) / TH;
    const FDiv dNS(NS), dNG(NG);
    const int row = dNS.div(v), s = v - row * NS;
    ln.am = dNG.div(row);
    const int y = (row - ln.am * NG) * TH, x0 = s * SW;
    ln.pix = y * S.Wo + x0;
    ln.ncols = min(SW, S.Wo - x0);
    ln.nrows = min(TH, S.Ho - y);
    ln.base = (y * S.Wi + x0) * S.stride;
  } else {
    const int Pn = S.Ho * S.Wo;
    const FDiv dP(Pn), dW(S.Wo);
    ln.am = dP.div(v);
    ln.pix = v - ln.am * Pn;
    const int y = dW.div(ln.pix), x = ln.pix - y * S.Wo;
    ln.ncols = 1;
    ln.base = (y * S.Wi + x) * S.stride;
  }
  if (!ln.on) { ln.r = 0; ln.am = 0; ln.pix = 0; ln.base = 0; ln.ncols = 0; ln.nrows = 0; }
  return ln;
}
__device__ __forceinline__ void lane_save(const Lane& ln, int* tab) {
  const int tid = threadIdx.x;
  tab[tid] = ln.base;
  tab[WG + tid] = ln.pix;
  tab[2 * WG + tid] = ln.r | (ln.am << 10) | (ln.ncols << 20) | (ln.nrows << 24) | ((ln.on ? 1 : 0) << 28);
}
__device__ __forceinline__ Lane lane_load(const int* tab) {
  const int tid = threadIdx.x;
  Lane ln;
  ln.base = tab[tid];
  ln.pix = tab[WG + tid];
  const int m = tab[2 * WG + tid];
  ln.r = m & 1023;
  ln.am = (m >> 10) & 1023;
  ln.ncols = (m >> 20) & 15;
  ln.nrows = (m >> 24) & 15;
  ln.on = (m >> 28) != 0;
  return ln;
}
__device__ __forceinline__ Lane lane_get(const JobStat& S, const JobDyn& D, const float* lds, int pass) {
  if (S.table >= 0 && D.passes == 1) return lane_load((const int*)(lds + S.table));
  return lane_decode(S, D, pass);
}

// call f(K, SW, TH, ST) with the job's compile-time kernel size, tile and input stride (K = 0: any size, one
// pixel per lane, any stride).  STRIDE2: the caller has jobs with a skipping factor of 1 (FP only; tiles of one row)
template <bool STRIDE2, class Fn>
__device__ __forceinline__ void job_dispatch(int variant, Fn f) {
  switch (variant) {
#define JOB_CASE(SW, K)                                                  \
  case SW * 8 + K: f(IC<K>{}, IC<SW>{}, IC<1>{}, IC<1>{}); break;        \
  case 64 + SW * 8 + K: f(IC<K>{}, IC<SW>{}, IC<2>{}, IC<1>{}); break;
    JOB_CASE(4, 2) JOB_CASE(4, 3) JOB_CASE(4, 4) JOB_CASE(4, 5)
    JOB_CASE(5, 2) JOB_CASE(5, 3) JOB_CASE(5, 4) JOB_CASE(5, 5)
    JOB_CASE(7, 2) JOB_CASE(7, 3) JOB_CASE(7, 4) JOB_CASE(7, 5)
#undef JOB_CASE
    default:
      if constexpr (STRIDE2) {
        switch (variant) {
#define JOB_CASE(SW, K) \
  case 128 + SW * 8 + K: f(IC<K>{}, IC<SW>{}, IC<1>{}, IC<2>{}); return;
          JOB_CASE(4, 2) JOB_CASE(4, 3) JOB_CASE(4, 4) JOB_CASE(4, 5)
          JOB_CASE(5, 2) JOB_CASE(5, 3) JOB_CASE(5, 4) JOB_CASE(5, 5)
#undef JOB_CASE
          default: break;
        }
      }
      f(IC<0>{}, IC<1>{}, IC<1>{}, IC<1>{});
      break;
  }
}

// acc[] += the lane's share of connections [e_lo, e_hi) of its map (maps numbered from idx_off)
template <int K, int SW, int TH, bool CLIP, int ST>
__device__ __forceinline__ void job_mac(const JobStat& S, int R, const float* lds, const Lane& ln, int e_lo, int e_hi,
                                        int idx_off, float (&acc)[TH * SW]) {
  const float* w = lds + S.w + (ln.am * S.w_pitch) * (S.K * S.K);
  const int* idx = (const int*)(lds + S.idx) + ln.am * S.w_pitch;
  if constexpr (K == 0)
    acc[0] += pixel_mac_k(S.K, lds + S.in, w, idx, idx_off, e_lo + ln.r, R, e_hi, S.map_sz, S.Wi, ln.base);
  else if constexpr (CLIP) {
    const int y = ln.pix / S.Wo;  // first output row of the tile = first input row it reads
    strip_mac<K, SW, TH, true, ST>(lds + S.in, w, idx, idx_off, e_lo + ln.r, R, e_hi, S.map_sz, S.Wi, ln.base,
                               S.band_lo - y, S.band_hi - y, acc);
  } else
    strip_mac<K, SW, TH, false, ST>(lds + S.in, w, idx, idx_off, e_lo + ln.r, R, e_hi, S.map_sz, S.Wi, ln.base, 0, 0, acc);
}

// ---- FP of the own maps of one layer (Sec. 2.2, Sec. 3.2) ------------------------------------------
// src: the exchange area of the layer below when the plan streams this layer's inputs (they are then fetched
// chunk by chunk of in_chunk maps into the arena); else null: the inputs are in LDS already.  False: a wait gave up.
template <int ID>
__device__ __forceinline__ bool flow_conv_fwd(const Rt& rt, int l, gtagged* src, unsigned int tag) {
  DECL_SPEC(Z, rt);
  const ConvSpec& C = Z.conv[l];
  float* lds = rt.lds;
  const JobStat S = fwd_job(Z, l);
  const JobDyn D = rt.sh->fwd[l];
  const int nm = D.n_maps;
  float* part = lds + Z.o_part;
  float* act = lds + Z.o_act;
  const float* bf = lds + C.o_bf;
  const int* cnt = (const int*)(lds + S.cnt);
  const int Pn = S.Ho * S.Wo, tot = nm * Pn;
  const bool stream = Z.stream != 0 && src != nullptr;
  bool ok = true;
  job_dispatch<true>(S.variant, [&](auto k_, auto sw_, auto th_, auto st_) {
    constexpr int K = decltype(k_)::value, SW = decltype(sw_)::value, TH = decltype(th_)::value, ST = decltype(st_)::value;
    for (int pass = 0; pass < D.passes && ok; ++pass) {
      const Lane ln = lane_get(S, D, lds, pass);
      float acc[TH * SW];
#pragma unroll
      for (int i = 0; i < TH * SW; ++i) acc[i] = 0.f;
      if (stream) {
        const int Mi = C.Mi, chunk = C.in_chunk, full = C.full_table;
        int e_next = 0;
        if (l == 1) DSTAMP(100);
        // chunks that fit the prefetch registers travel while the chunk before them is multiplied
        const bool ahead = chunk * S.map_sz <= BULK_PF * 4 * WG && Mi > chunk;
        const gfloat* data = bulk_data(src, Mi * S.map_sz, tag & 1u);
        u4v pf[BULK_PF];
        if (ahead) {
          if (pass > 0) __syncthreads();
          if (!bulk_wait(rt, bulk_flags(src, Mi * S.map_sz, Mi, tag & 1u), Mi, tag)) { ok = false; break; }
          bulk_issue(pf, data, min(chunk, Mi) * S.map_sz);
        }
        for (int i0 = 0; i0 < Mi; i0 += chunk) {
          const int n = min(chunk, Mi - i0);
          if (ahead) {
            if (i0 > 0) __syncthreads();  // the chunk before has been read by everybody
            bulk_commit(pf, lds + S.in, n * S.map_sz);
            __syncthreads();
            if (i0 + chunk < Mi) bulk_issue(pf, data + (size_t)(i0 + chunk) * S.map_sz, min(chunk, Mi - i0 - chunk) * S.map_sz);
          } else {
          if (i0 > 0 || pass > 0) __syncthreads();  // the chunk before has been read by everybody
          if (!gather_bulk(rt, lds + S.in, data + (size_t)i0 * S.map_sz, n * S.map_sz,
                           bulk_flags(src, Mi * S.map_sz, Mi, tag & 1u) + i0, n, tag)) { ok = false; break; }
          }
          if (l == 1 && i0 / chunk < 4) DSTAMP(101 + 2 * (i0 / chunk));
          if (ln.on) {
            // connections of the lane's map whose input map lies in [i0, i0 + n): the list is sorted
            int e_lo = i0, e_hi = i0 + n;
            if (!full) {
              const int* ci = (const int*)(lds + S.idx) + ln.am * S.w_pitch;
              e_lo = e_next;
              int lo = e_lo, hi = cnt[ln.am];
              while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (ci[mid] < i0 + n) lo = mid + 1; else hi = mid;
              }
              e_hi = lo;
              e_next = e_hi;
            }
            job_mac<K, SW, TH, false, ST>(S, D.R, lds, ln, e_lo, e_hi, i0, acc);
          }
          if (l == 1 && i0 / chunk < 4) DSTAMP(102 + 2 * (i0 / chunk));
        }
      } else if (ln.on) {
        job_mac<K, SW, TH, false, ST>(S, D.R, lds, ln, 0, cnt[ln.am], 0, acc);
      }
      if (Z.stream != 0 && D.R > 1) __syncthreads();  // the partial sums go where the last chunk of maps lies
      if (ln.on && ok) {
        if (D.R == 1) {  // unsplit: the finished sums (the activation function is applied where they are pooled)
          const float b = bf[ln.am];
          float* dst = act + ln.am * Pn + ln.pix;
#pragma unroll
          for (int ty = 0; ty < TH; ++ty)
#pragma unroll
            for (int i = 0; i < SW; ++i)
              if (ty < ln.nrows && i < ln.ncols) dst[ty * S.Wo + i] = acc[ty * SW + i] + b;
        } else {
          float* dst = part + (ln.r * nm + ln.am) * Pn + ln.pix;
#pragma unroll
          for (int ty = 0; ty < TH; ++ty)
#pragma unroll
            for (int i = 0; i < SW; ++i)
              if (ty < ln.nrows && i < ln.ncols) dst[ty * S.Wo + i] = acc[ty * SW + i];
        }
      }
    }
  });
  __syncthreads();
  if (l == 1) DSTAMP(110);
  if (!ok || rt.sh->fail) return false;
  if (D.R > 1) {
    const FDiv dP(Pn);
    reduce_partials(part, D.R, tot, [&](int p, float s) { act[p] = s + bf[dP.div(p)]; });
    __syncthreads();
  }
  if (l == 1) DSTAMP(111);
  return true;
}

// Max-pooling of the own maps (Sec. 2.3): value and position of the first maximum in row-major
// order; the pooled value is what the next layer reads, so it is published at once.
template <int ID>
__device__ __forceinline__ void flow_pool(const Rt& rt, int l, int nm, unsigned int tag, bool taps) {
  DECL_SPEC(Z, rt);
  const ConvSpec& C = Z.conv[l];
  const FlowConvPtrs& P = rt.sh->ptrs.conv[l];
  float* lds = rt.lds;
  const int tid = threadIdx.x, G = Z.G, rank = rt.rank;
  const int Kp = C.Kp, Wo = C.Wo, Wp = C.Wp, HW = C.Hp * C.Wp, Pn = C.Ho * C.Wo;
  const float* act = lds + Z.o_act;   // the sums the own maps' units received (bias included)
  float* pool = lds + C.o_pool;
  float* dact = lds + C.o_dact;
  int* yx = (int*)(lds + C.o_yx);
  const bool bulk = Z.stream != 0 && C.has_x_out;   // (the next layer streams its inputs)
  gtagged* xo = (C.has_x_out && !bulk) ? P.x_out + (size_t)(tag & 1u) * C.Mo * HW : nullptr;
  gfloat* xb = bulk ? bulk_data(P.x_out, C.Mo * HW, tag & 1u) : nullptr;
  const FDiv dHW(HW), dWp(Wp);
  // the outputs of the own maps, every lane its share (the partial sums' area is free by now and at least as
  // large): the maximum below is taken over them -- they are what the parity taps show -- and the winner's
  // derivative from the sum it received
  float* yout = lds + Z.o_part;
  for (int x = tid; x < nm * Pn; x += WG) yout[x] = f_act(act[x]);
  __syncthreads();
  for (int x = tid; x < nm * HW; x += WG) {
    const int am = dHW.div(x), q = x - am * HW;
    const int py = dWp.div(q), px = q - py * Wp;
    const int w0 = am * Pn + py * Kp * Wo + px * Kp;
    const float* win = yout + w0;
    float best = win[0];
    int wy = 0, wx = 0;
#pragma unroll 4
    for (int dy = 0; dy < Kp; ++dy)
#pragma unroll 4
      for (int dx = 0; dx < Kp; ++dx) {
        const float v = win[dy * Wo + dx];
        if (v > best) { best = v; wy = dy; wx = dx; }
      }
    const int code = ((py * Kp + wy) << 16) | (px * Kp + wx);
    pool[x] = best;
    dact[x] = f_dact_pre(act[w0 + wy * Wo + wx]);
    yx[x] = code;
    const size_t o = (size_t)(rank + am * G) * HW + q;
    if (xo) put_f(xo + o, best, tag);
    if (xb) __hip_atomic_store(xb + o, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (taps) {
      if (Kp > 1) P.out[o] = best;
      P.arg[o] = (uint8_t)(wy * Kp + wx);
      P.argyx[o] = code;
    }
  }
  if (taps) {
    const FDiv dP(Pn);
    for (int x = tid; x < nm * Pn; x += WG) {
      const int am = dP.div(x), p = x - am * Pn;
      P.act[(size_t)(rank + am * G) * Pn + p] = yout[x];
    }
  }
  if (bulk) stores_done();
  __syncthreads();
  if (bulk) {  // every lane's stores have completed: the maps' flags go up
    guint* fl = bulk_flags(P.x_out, C.Mo * HW, C.Mo, tag & 1u);
    for (int am = tid; am < nm; am += WG) __hip_atomic_store(fl + rank + am * G, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
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
        for (int q0 = rr; q0 < HW; q0 += 4 * R) {
          int yx[4];
          float dv[4], iv[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int q = min(q0 + u * R, HW - 1);
            yx[u] = I.yx[q];
            dv[u] = I.d[q];
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) iv[u] = I.in[((yx[u] >> 16) * Wi + (yx[u] & 0xffff)) * stride];
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (q0 + u * R < HW) s = fmaf(dv[u], iv[u], s);
        }
    }
    s = group_sum(s, Rl2);
    if (I.ok && rr == 0) {
      if (g_out) g_out[I.canon] = s;
      else w[wi] = fmaf(-lr, s, w[wi]);
    }
  }
}

// AW of the pull copy in a streamed plan (Sec. 3.4), where it is the only place a filter above the first layer
// is adjusted: a lane takes a whole K x K filter -- entry e of an own input map, i.e. the connection to output
// map bj[e] -- and a share of that map's pooling winners, so that a winner's delta and coordinates are read once
// for K*K multiply-adds (flow_wgrad reads them once per multiply-add); the shares are then added across the
// 2^gl2 neighbouring lanes that split the winners.  The adjusted filter goes to its place in the rotated copy
// and, tap order turned back, on its way to the rank that holds the forward copy (x_w, table order).
template <int K>
__device__ __forceinline__ void flow_wgrad_entries(float* wb, const int* bj, const int* ncb, int nb, int pitch,
                                                   const float* dall, const int* yxall, int HW, const float* own_in,
                                                   int HiWi, int Wi, int stride, float lr, int Mi, int Mo, int rank, int G,
                                                   bool full, const CNN_GLOBAL int* csc_ptr, const CNN_GLOBAL int* csc_slot,
                                                   gtagged* xw, unsigned int tag, const Rt& rt) {
  constexpr int KK = K * K;
  const int tid = threadIdx.x;
  int gl2 = 0;  // winners of a map are split over 2^gl2 lanes
  while (gl2 < 3 && ((nb * pitch) << (gl2 + 1)) <= WG && (2 << gl2) <= HW) ++gl2;
  const int Gq = 1 << gl2;
  const int total = (nb * pitch) << gl2;
  for (int u0 = 0; u0 < total; u0 += WG) {
    const int u = u0 + tid;
    const int ei = u >> gl2, g = u & (Gq - 1);
    const int ab = ei / pitch, e = ei - ab * pitch;
    const bool on = u < total && e < ncb[min(ab, nb - 1)];
    float acc[KK];
#pragma unroll
    for (int t = 0; t < KK; ++t) acc[t] = 0.f;
    int j = 0;
    if (on) {
      j = bj[ab * pitch + e];
      const float* d = dall + j * HW;
      const int* yx = yxall + j * HW;
      const float* in = own_in + ab * HiWi;
      for (int q = g; q < HW; q += Gq) {
        const int c = yx[q];
        const float dv = d[q];
        const float* p = in + ((c >> 16) * Wi + (c & 0xffff)) * stride;
#pragma unroll
        for (int ky = 0; ky < K; ++ky)
#pragma unroll
          for (int kx = 0; kx < K; ++kx) acc[ky * K + kx] = fmaf(dv, p[ky * Wi + kx], acc[ky * K + kx]);
      }
    }
    DSTAMP(112);
#pragma unroll
    for (int t = 0; t < KK; ++t) acc[t] = group_sum(acc[t], gl2);
    DSTAMP(113);
    if (on) {  // every lane of the group holds all K*K sums: lane g stores the taps g, g + Gq, ...
      const int i = rank + ab * G;
      // where the filter goes: with a sparse table, as tagged words to its place in table order; the filters of a
      // full table are sent afterwards, all of an input map in one run (ship_rows)
      const size_t at = full ? 0 : (size_t)csc_slot[csc_ptr[i] + e] * KK;
      float* w = wb + (ab * pitch + e) * KK;
      float wv[KK];   // (all of the filter read at once: one LDS latency instead of one per tap)
#pragma unroll
      for (int t = 0; t < KK; ++t) wv[t] = w[KK - 1 - t];   // natural tap t lies at KK-1-t of the rotated copy
#pragma unroll
      for (int t = 0; t < KK; ++t) wv[t] = fmaf(-lr, acc[t], wv[t]);
#pragma unroll
      for (int t = 0; t < KK; ++t)
        if ((t & (Gq - 1)) == g) {
          w[KK - 1 - t] = wv[t];
          if (!full) put_f(xw + at + t, wv[t], tag);
        }
    }
    DSTAMP(114);
  }
}

// ---- BP through a pooled convolutional layer: only the pooling winners carry a delta ------------------
// Under max-pooling of Kp x Kp one output neuron in Kp^2 has a non-zero delta (Sec. 2.3: the others did not
// reach the layer above), so the sums of Sec. 3.3 have K^2 HW non-zero terms per connection instead of K^2
// times the map.  They are formed term by term: a lane takes a winner p of one connection (an entry of an own
// input map's list), its delta and coordinates, and adds delta * w[ky][kx] at the K^2 input neurons of that
// winner's receptive field.  The lanes that share a connection hold different winners, i.e. different receptive
// fields' corners, so at one tap they add at different places; the taps follow one another in program order and
// LDS serves a wavefront's instructions in order, so every place receives its terms in a fixed order and the
// result does not depend on timing.  A term costs two LDS accesses here, against a third of one and Kp^2 times the
// terms in the correlation over whole maps; measured, it pays from 2 x 2 pooling on.  Connections worked on at the same time (a slot: UW lanes of a wavefront)
// add into copies of their own of the rank's input maps; the copies are added up afterwards (reduce_partials),
// in the order of the slots.  Every copy: [n_maps][Hi * Wi].
template <int ID>
__device__ __forceinline__ void pull_winners(const Rt& rt, int l, const float* dall, const int* yxall, float* copies,
                                             int slots, int nb) {
  DECL_SPEC(Z, rt);
  const ConvSpec& C = Z.conv[l];
  float* lds = rt.lds;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = uni_of<ID>(C.K), KK = K * K, HW = uni_of<ID>(C.Hp) * uni_of<ID>(C.Wp), stride = uni_of<ID>(C.S) + 1;
  const int Wi = uni_of<ID>(C.Wi), HiWi = uni_of<ID>(C.Hi) * Wi, pitch = uni_of<ID>(C.back_pitch);
  const int parts = (HW + 63) >> 6, UW = (HW + parts - 1) / parts, UPW = 64 / UW;
  const int tot = nb * HiWi;
  for (int x = tid; x < slots * tot; x += WG) copies[x] = 0.f;
  __syncthreads();
  const FDiv dUW(UW), dP(parts), dPitch(pitch);
  const int su = dUW.div(lane), pl = lane - su * UW;
  const int slot = wave * UPW + su;
  const int* cnt = (const int*)(lds + C.o_ncb);
  const int* bj = (const int*)(lds + C.o_bj);
  const float* wb = lds + C.o_wb;
  const int n_units = nb * pitch * parts;
  if (su < UPW && slot < slots) {
    float* mine = copies + slot * tot;
    for (int u = slot; u < n_units; u += slots) {
      const int ue = dP.div(u), part = u - ue * parts;
      const int am = dPitch.div(ue), e = ue - am * pitch;
      const int p = part * UW + pl;
      if (e < cnt[am] && p < HW) {
        const int j = bj[am * pitch + e];
        const float d = dall[j * HW + p];
        const int yx = yxall[j * HW + p];
        float* o = mine + am * HiWi + ((yx >> 16) * stride) * Wi + (yx & 0xffff) * stride;
        const float* w = wb + (am * pitch + e) * KK + (KK - 1);   // (the copy is rotated: tap t lies at K*K-1-t)
        // (read, add, write, with the compiler kept from moving the next tap's read above this tap's write:
        // another lane of the unit may have written that place.  LDS atomic float adds would say the same in one
        // instruction and take 30 x as long on this hardware: measured.)
        auto taps = [&](auto k_) __attribute__((always_inline)) {
          constexpr int KC = decltype(k_)::value;
          const int Kn = KC ? KC : K;
          float wr[KC ? KC * KC : 1];
          if (KC) {
#pragma unroll
            for (int t = 0; t < KC * KC; ++t) wr[t] = w[-t];
          }
#pragma unroll
          for (int ky = 0; ky < Kn; ++ky)
#pragma unroll
            for (int kx = 0; kx < Kn; ++kx) {
              float* a = o + ky * Wi + kx;
              const float v = *a;
              *a = fmaf(d, KC ? wr[ky * KC + kx] : w[-(ky * Kn + kx)], v);
              asm volatile("" ::: "memory");
            }
        };
        switch (K) {
          case 2: taps(IC<2>{}); break;
          case 3: taps(IC<3>{}); break;
          case 4: taps(IC<4>{}); break;
          case 5: taps(IC<5>{}); break;
          default: taps(IC<0>{}); break;
        }
      }
    }
  }
  __syncthreads();
}

// ---- BP through a convolutional layer, pull form (Sec. 3.3), for the own input maps ------------------
// Neuron (r, c) of input map i collects, over every output map j that reads map i, the deltas of
// the output neurons whose receptive field covers it (the four inequalities of Sec. 3.3), each
// times its weight (old value).  Written as FP's mirror image: the deltas of a chunk of output
// maps are put at their places (y (S+1) + K-1, x (S+1) + K-1) in maps of (Hi+K-1) x (Wi+K-1) zeros
// -- only pooling winners are non-zero -- and correlated with the filters rotated by 180 degrees;
// a tap that has no output neuron then meets a zero and the loop has no branches.  The zero maps
// are kept zero between uses: after a chunk the winners' places are cleared again.
// delta_below[p] = pulled sum * f'(y_below[p]).
template <int ID>
__device__ __forceinline__ bool flow_pull(const Rt& rt, int l, const float* dall, const int* yxall, unsigned int tag) {
  DECL_SPEC(Z, rt);
  const ConvSpec& C = Z.conv[l];
  const ConvSpec& Cb = Z.conv[l - 1];
  float* lds = rt.lds;
  const int tid = threadIdx.x;
  const JobStat S = pull_job(Z, l);
  const JobDyn D = rt.sh->pull[l];
  const int nb = D.n_maps;
  float* dd = lds + Z.o_scratch;
  float* part = lds + Z.o_part;
  const int Mo = C.Mo, HW = C.Hp * C.Wp, stride = C.S + 1, Km1 = C.K - 1;
  const int Wd = S.Wi, HWd = S.map_sz;
  const int chunk = C.pull_chunk;
  const int H = C.pull_shares;
  const bool full = C.full_table != 0 && H == 1;  // (a share's entries are found through its list)
  const int* cnt = (const int*)(lds + S.cnt);
  // output maps this rank's entries lie among: all of them, or, for a share, from its first entry to its last
  int j_lo = 0, j_hi = Mo;
  if (H > 1) {
    const int* bj0 = (const int*)(lds + S.idx);
    const int ne = cnt[0];
    j_lo = ne > 0 ? bj0[0] : 0;
    j_hi = ne > 0 ? bj0[ne - 1] + 1 : 0;
  }
  const int tot = nb * S.Ho * S.Wo;
  const FDiv dHW(HW);
  const int slots = uni_of<ID>(C.pull_slots);
  const float* sums = slots > 0 ? dd : part;    // planes of partial sums [n_sums][tot]
  const int n_sums = slots > 0 ? slots : D.R;
  if (slots > 0) {
    pull_winners<ID>(rt, l, dall, yxall, dd, slots, nb);
  } else {
  if (Z.arena_shared) {  // the arena has held other things since the last pull: the delta maps start from zeros
    for (int x = tid; x < Z.scratch_floats; x += WG) dd[x] = 0.f;
    __syncthreads();
  }
  DSTAMP(120);
  job_dispatch<false>(S.variant, [&](auto k_, auto sw_, auto th_, auto) {
    constexpr int K = decltype(k_)::value, SW = decltype(sw_)::value, TH = decltype(th_)::value;
    for (int pass = 0; pass < D.passes; ++pass) {
      const Lane ln = lane_get(S, D, lds, pass);
      float acc[TH * SW];
#pragma unroll
      for (int i = 0; i < TH * SW; ++i) acc[i] = 0.f;
      int e_next = 0;
      for (int j0 = j_lo; j0 < j_hi; j0 += chunk) {
        const int n = min(chunk, j_hi - j0);
        for (int x = tid; x < n * HW; x += WG) {
          const int c = dHW.div(x), q = x - c * HW;
          const int yx = yxall[(j0 + c) * HW + q];
          dd[c * HWd + ((yx >> 16) * stride + Km1) * Wd + (yx & 0xffff) * stride + Km1] = dall[(j0 + c) * HW + q];
        }
        __syncthreads();
        if (j0 == j_lo) DSTAMP(121);
        if (ln.on) {
          // entries of the lane's input map whose output map lies in [j0, j0 + n): the list is
          // sorted, this chunk's start is the last chunk's end, its end is found by bisection
          int e_lo = j0, e_hi = j0 + n;
          if (!full && n == j_hi - j_lo) {  // one chunk holds every map: the whole list, nothing to look for
            e_lo = 0;
            e_hi = cnt[ln.am];
          } else if (!full) {
            const int* bj = (const int*)(lds + S.idx) + ln.am * S.w_pitch;
            e_lo = e_next;
            int lo = e_lo, hi = cnt[ln.am];
            while (lo < hi) {
              const int mid = (lo + hi) >> 1;
              if (bj[mid] < j0 + n) lo = mid + 1; else hi = mid;
            }
            e_hi = lo;
            e_next = e_hi;
          }
          if (j0 == j_lo) DSTAMP(122);
          job_mac<K, SW, TH, true, 1>(S, D.R, lds, ln, e_lo, e_hi, j0, acc);
        }
        __syncthreads();
        if (j0 == j_lo) DSTAMP(123);
        for (int x = tid; x < n * HW; x += WG) {
          const int c = dHW.div(x), q = x - c * HW;
          const int yx = yxall[(j0 + c) * HW + q];
          dd[c * HWd + ((yx >> 16) * stride + Km1) * Wd + (yx & 0xffff) * stride + Km1] = 0.f;
        }
        if (j0 + chunk < j_hi) __syncthreads();
      }
      if (Z.stream != 0) __syncthreads();  // the partial sums go where the delta maps lay
      if (ln.on) {
        float* dst = part + (ln.r * nb + ln.am) * (S.Ho * S.Wo) + ln.pix;
#pragma unroll
        for (int ty = 0; ty < TH; ++ty)
#pragma unroll
          for (int i = 0; i < SW; ++i)
            if (ty < ln.nrows && i < ln.ncols) dst[ty * S.Wo + i] = acc[ty * SW + i];
      }
    }
  });
  __syncthreads();
  }
  DSTAMP(124);
  const float* fbelow = lds + Cb.o_dact;   // f' of the own units of the layer below
  float* dbelow = lds + Cb.o_delta;
  if (H == 1) {
    reduce_partials(sums, n_sums, tot, [&](int p, float s) { dbelow[p] = s * fbelow[p]; });
    __syncthreads();
    return true;
  }
  // A shared pull (one map, tot = Hi * Wi sums): the shares beyond the first send their sums to the map's owner,
  // who adds them to its own in the order of the shares and multiplies by the activation derivative.
  const int i = rt.rank % C.Mi, h = rt.rank / C.Mi;
  const FlowConvPtrs& P = rt.sh->ptrs.conv[l];
  gtagged* xp = P.x_part + ((size_t)(tag & 1u) * C.Mi + i) * (H - 1) * tot;
  if (h > 0) {
    reduce_partials(sums, n_sums, tot, [&](int p, float s) { put_f(xp + (size_t)(h - 1) * tot + p, s, tag); });
    __syncthreads();
    return true;
  }
  reduce_partials(sums, n_sums, tot, [&](int p, float s) { dbelow[p] = s; });
  __syncthreads();
  bool ok = true;  // (a lane whose wait gave up goes on to the barrier like the others; the flag tells)
  for (int p0 = 0; p0 < tot; p0 += WG) {
    const int p = p0 + tid;
    float s = p < tot ? dbelow[p] : 0.f;
    if (H == 2) {
      tagged_t w[1];
      ok = fetch_tagged<1>(rt, w, tag, [&](int) { return xp + min(p, tot - 1); });
      s += __uint_as_float((unsigned int)w[0]);
    } else {
      // four shares' words in flight at a time (every batch is a round trip), added in the order of the shares
      for (int h0 = 1; h0 < H && ok; h0 += 4) {
        tagged_t w[4];
        ok = fetch_tagged<4>(rt, w, tag, [&](int u) { return xp + (size_t)(min(h0 + u, H - 1) - 1) * tot + min(p, tot - 1); });
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (h0 + u < H) s += __uint_as_float((unsigned int)w[u]);
      }
    }
    if (ok && p < tot) dbelow[p] = s * fbelow[p];
  }
  __syncthreads();
  return rt.sh->fail == 0;
}

// y[k] = b[k] + sum_m W[k][m] v[m], all in LDS; lane groups of a power of two per row.
__device__ __forceinline__ void flow_matvec(const float* W, const float* b, const float* v, float* y, int n_out, int n_in) {
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
    s = group_sum(s, lpl);
    if (sub == 0 && k < n_out) y[k] = s + b[k];
  }
  __syncthreads();
}

// Sum over the ranks of the partial sums of the first fully connected layer, every rank in the
// same order: lane (k, part) adds the ranks of its part one after the other as their words
// arrive, the parts are then added in order.  y[k] = b[k] + sum.
__device__ __forceinline__ bool flow_reduce_partials(const Rt& rt, const gtagged* xp, int NR, int n1, const float* b,
                                                     float* y, float* dy, float* part, unsigned int tag, bool through_act) {
  const int tid = threadIdx.x;
  const int parts = max(1, min(WG / max(n1, 1), NR));
  const int per = (NR + parts - 1) / parts;
  constexpr int U = 8;
  const FDiv dN(n1);
  for (int k0 = 0; k0 < n1; k0 += WG) {
    const int pi = dN.div(tid), k = k0 + tid - pi * n1;
    const bool on = pi < parts && k < n1;
    if (on) {
      const int r_lo = pi * per, r_hi = min(NR, r_lo + per);
      float s = 0.f;
      for (int r0 = r_lo; r0 < r_hi; r0 += U) {
        tagged_t w[U];
        if (!fetch_tagged<U>(rt, w, tag, [&](int u) { return xp + (size_t)min(r0 + u, r_hi - 1) * n1 + k; })) break;
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (r0 + u < r_hi) s += __uint_as_float((unsigned int)w[u]);
      }
      part[pi * n1 + (k - k0)] = s;
    }
    __syncthreads();
    if (tid < n1 - k0 && tid < WG) {
      const float v = b[k0 + tid] + sum_strided(part, parts, n1, tid);
      y[k0 + tid] = through_act ? f_act_fc(v) : v;
      if (through_act) dy[k0 + tid] = f_dact_pre(v);
    }
    __syncthreads();
    if (n1 <= WG) break;
  }
  return rt.sh->fail == 0;
}

// The same sums when the partial sums are many: output k is added up by rank k mod G alone (a wavefront per
// output, lane l taking the ranks l, l + 64, ...), which sends sum + bias round; every rank gathers the n1 values.
// One more crossing, but n1 words to read per rank instead of NR x n1.
__device__ __forceinline__ bool flow_reduce_owned(const Rt& rt, const gtagged* xp, gtagged* xs, int NR, int n1, int G,
                                                  const float* b, float* y, float* dy, unsigned int tag,
                                                  bool through_act) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nk = n_mine(n1, rt.rank, G);
  for (int a = wave; a < nk; a += WG / 64) {
    const int k = rt.rank + a * G;
    float s = 0.f;
    constexpr int U = 2;
    for (int r0 = 0; r0 < NR; r0 += 64 * U) {
      tagged_t w[U];
      if (r0 + lane < NR) {
        if (!fetch_tagged<U>(rt, w, tag, [&](int u) { return xp + (size_t)min(r0 + lane + 64 * u, NR - 1) * n1 + k; })) break;
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (r0 + lane + 64 * u < NR) s += __uint_as_float((unsigned int)w[u]);
      }
    }
    s = f_wave_sum(s);
    if (lane == 0) put_f(xs + k, s + b[k], tag);
  }
  if (!gather(rt, (unsigned int*)y, xs, n1, tag)) return false;
  if (through_act) {
    for (int k = tid; k < n1; k += WG) {
      const float v = y[k];
      y[k] = f_act_fc(v);
      dy[k] = f_dact_pre(v);
    }
    __syncthreads();
  }
  return rt.sh->fail == 0;
}

// Work out the rank's share of the correlation jobs and fill their lane tables (once per call).
template <int ID>
__device__ __forceinline__ void flow_prepare_jobs(const Rt& rt) {
  Shared& sh = *rt.sh;
  DECL_SPEC(Z, rt);
  const int G = Z.G, rank = rt.rank;
  if (threadIdx.x == 0)
    for_up<ID, 0, FLOW_MAX_CONV>(Z.n_conv, [&](auto lc) {
      const int l = lv(lc);
      sh.fwd[l] = job_dyn(fwd_job(Z, l), n_mine(Z.conv[l].Mo, rank, G));
      if (l >= 1) sh.pull[l] = job_dyn(pull_job(Z, l), n_pull_maps(Z.conv[l].Mi, rank, G, Z.conv[l].pull_shares));
      return true;
    });
  __syncthreads();
  for_up<ID, 0, FLOW_MAX_CONV>(Z.n_conv, [&](auto lc) {
    const int l = lv(lc);
    const JobStat S = fwd_job(Z, l);
    const JobDyn D = sh.fwd[l];
    if (D.n_maps > 0 && S.table >= 0 && D.passes == 1) lane_save(lane_decode(S, D, 0), (int*)(rt.lds + S.table));
    if (l >= 1) {
      const JobStat B = pull_job(Z, l);
      const JobDyn E = sh.pull[l];
      if (E.n_maps > 0 && B.table >= 0 && E.passes == 1) lane_save(lane_decode(B, E, 0), (int*)(rt.lds + B.table));
    }
    return true;
  });
  __syncthreads();
}

#define STAMP(i)                                                                              \
  do {                                                                                        \
    if (stamp) status->stamps[i] = wall_clock64();                                            \
  } while (0)

// ID = 0: any network, the plan is the argument kspec.  ID > 0: the network of StaticSpec<ID>; the host
// launches it only when the plan it made at run time equals that one word for word.
template <int ID>
__global__ void __launch_bounds__(WG) k_resident(const FlowSpec kspec, const FlowPtrs* __restrict__ gptrs,
                                                 StatusDev* status, RunArgs a) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ Shared sh;
  const int tid = threadIdx.x;
  {
    const int stride = ID ? StaticSpec<(ID ? ID : 1)>::value.stride : kspec.stride;
    const int G0 = ID ? StaticSpec<(ID ? ID : 1)>::value.G : kspec.G;
    if (blockIdx.x % stride != 0 || (int)(blockIdx.x / stride) >= G0) return;
    const unsigned int* src = (const unsigned int*)gptrs;
    unsigned int* dst = (unsigned int*)&sh.ptrs;
    for (int i = tid; i < (int)(sizeof(FlowPtrs) / 4); i += WG) dst[i] = src[i];
    if (tid == 0) sh.fail = 0;
    __syncthreads();
  }
  Rt rt;
  // the plan where the launch put it: the kernel's argument block, whose first bytes it is.  (The address of
  // the parameter itself would be that of a copy in each lane's scratch memory.)
  rt.spec = (const FlowSpec*)__builtin_amdgcn_kernarg_segment_ptr();
  DECL_SPEC(Z, rt);
  const FlowPtrs& Q = sh.ptrs;
  const int G = uni_of<ID>(Z.G);
  const int rank = blockIdx.x / uni_of<ID>(Z.stride);
  rt.sh = &sh; rt.status = status; rt.lds = lds; rt.rank = rank; rt.spin_limit = a.spin_limit;
  rt.dbg = false;
  flow_load<ID>(rt);
  flow_prepare_jobs<ID>(rt);

  const int n_conv = uni_of<ID>(Z.n_conv), n_fc = uni_of<ID>(Z.n_fc), n_classes = uni_of<ID>(Z.n_classes);
  const ConvSpec& Cc = Z.conv[n_conv - 1];      // last convolutional layer
  const FlowConvPtrs& Pc = Q.conv[n_conv - 1];
  const FcSpec& L1 = Z.fc[0];                   // first fully connected layer
  const int HWc = uni_of<ID>(Cc.Hp) * uni_of<ID>(Cc.Wp);
  const int ncols = n_mine(uni_of<ID>(Cc.Mo), rank, G) * HWc;  // own columns of the first fully connected layer
  const int n1 = uni_of<ID>(L1.n_out);
  const int NR = uni_of<ID>(Z.n_col_ranks);
  float* part = lds + Z.o_part;
  gfloat* g_out = a.grad_out;
  const float lr = a.lr;

  bool pend = false;  // the previous image left adjustments to do
  bool ship_pend = false;  // streamed plan: the previous image's adjusted filters are on their way to the forward copies
  constexpr int IMG_U = 4;
  const int img_n = uni_of<ID>(Z.conv[0].Mi) * uni_of<ID>(Z.conv[0].Hi) * uni_of<ID>(Z.conv[0].Wi);
  const bool img_ahead = img_n <= IMG_U * WG;
  float img_reg[IMG_U] = {0.f, 0.f, 0.f, 0.f};
  if (img_ahead && a.n_images > 0) {
#pragma unroll
    for (int u = 0; u < IMG_U; ++u)
      if (tid + u * WG < img_n) img_reg[u] = a.images[tid + u * WG];
  }
  for (long long t = 0; t < a.n_images; ++t) {
    const unsigned int tag = a.epoch_base + (unsigned int)t + 1u;
    const unsigned int par = tag & 1u;
    const bool taps = (t == a.n_images - 1);
    // timestamps: the last image but one (the last also stores the parity taps)
    const bool stamp = (a.n_images > 1 ? t == a.n_images - 2 : taps) && rank == 0 && tid == 0;
    rt.dbg = stamp;
    const int label = a.labels ? a.labels[t] : a.label_imm;
    bool train = a.train != 0;
    if (train && (label < 0 || label >= n_classes)) {
      train = false;
      if (rank == 0 && tid == 0) status->bad_label = 1u;
    }

    // ---- AW pieces that may run either in place or during the next image's waits ----
    // first fully connected layer: own columns, and the (replicated) biases
    auto fc1_update = [&]() __attribute__((always_inline)) {
      const FlowFcPtrs& P1 = Q.fc[0];
      float* wc = lds + L1.o_w;
      float* b = lds + L1.o_b;
      const float* d = lds + L1.o_delta;
      const float* vcol = lds + Cc.o_pool;
      const FDiv dN(n1), dHW(HWc);
      for (int x = tid; x < ncols * n1; x += WG) {
        const int c = dN.div(x), k = x - c * n1;
        const float g = d[k] * vcol[c];
        if (g_out) {
          const int am = dHW.div(c), q = c - am * HWc;
          g_out[P1.w_canon + (long long)k * L1.n_in + (long long)(rank + am * G) * HWc + q] = g;
        } else {
          wc[x] = fmaf(-lr, g, wc[x]);
        }
      }
      for (int k = tid; k < n1; k += WG) {
        if (g_out) { if (rank == 0) g_out[P1.b_canon + k] = d[k]; }
        else b[k] = fmaf(-lr, d[k], b[k]);
        if (taps && rank == 0) P1.delta[k] = d[k];  // (the last image is never put off)
      }
    };
    // forward copy of the own maps' filters of conv layer l, and their biases
    // (tagw: the tag of the image the gradient belongs to -- this image's, or the one before when the adjustment was
    // put off; a plan that streams the layer's inputs fetches them again under that tag, chunk by chunk)
    auto wgrad_fwd = [&](auto lc, unsigned int tagw, bool with_weights) __attribute__((always_inline)) {
      const int l = lv(lc);
      const ConvSpec& C = Z.conv[l];
      const FlowConvPtrs& P = Q.conv[l];
      const int K = uni_of<ID>(C.K), KK = K * K, HW = uni_of<ID>(C.Hp) * uni_of<ID>(C.Wp), stride = uni_of<ID>(C.S) + 1,
                Wi = uni_of<ID>(C.Wi), HiWi = uni_of<ID>(C.Hi) * Wi;
      const int nm = sh.fwd[l].n_maps;
      if (nm <= 0) return;
      const float* dl = lds + C.o_delta;
      const int* yx = (const int*)(lds + C.o_yx);
      const int* cidx = (const int*)(lds + C.o_cidx);
      const int* ncf = (const int*)(lds + C.o_ncf);
      const float* in = lds + C.o_in;
      const int pitch = uni_of<ID>(C.max_conn);
      const int per_map = pitch * KK;
      const FDiv dPM(per_map), dKK(KK), dK(K);
      const bool full = C.full_table != 0;
      const int Mi = uni_of<ID>(C.Mi);
      if (!with_weights) {
        // (the filters arrive adjusted from the holders of the pull copies: only the biases are this rank's to do)
      } else if (Z.stream != 0 && l >= 1) {
        gtagged* src = Q.conv[l >= 1 ? l - 1 : 0].x_out;
        const int chunk = C.in_chunk;
        for (int i0 = 0; i0 < Mi; i0 += chunk) {
          const int n = min(chunk, Mi - i0);
          __syncthreads();  // whoever read the arena before is done
          if (!gather_bulk(rt, lds + C.o_in, bulk_data(src, Mi * HiWi, tagw & 1u) + (size_t)i0 * HiWi, n * HiWi,
                           bulk_flags(src, Mi * HiWi, Mi, tagw & 1u) + i0, n, tagw)) return;
          for (int am = 0; am < nm; ++am) {
            // connections of own map am whose input map lies in [i0, i0 + n) (the list is sorted)
            int c_lo = i0, c_hi = min(i0 + n, ncf[am]);
            if (!full) {
              const int* ci = cidx + am * pitch;
              int lo = 0, hi = ncf[am];
              while (lo < hi) { const int mid = (lo + hi) >> 1; if (ci[mid] < i0) lo = mid + 1; else hi = mid; }
              c_lo = lo;
              hi = ncf[am];
              while (lo < hi) { const int mid = (lo + hi) >> 1; if (ci[mid] < i0 + n) lo = mid + 1; else hi = mid; }
              c_hi = lo;
            }
            if (c_hi <= c_lo) continue;
            flow_wgrad(lds + C.o_wf + (am * pitch + c_lo) * KK, (c_hi - c_lo) * KK, HW, stride, Wi,
                       uni_of<ID>(C.wgrad_R_log2), lr, g_out, [&](int wi) {
              const int cc = dKK.div(wi), tt = wi - cc * KK, c = c_lo + cc;
              const int ky = dK.div(tt), kx = tt - ky * K;
              WgradInfo I;
              I.ok = true;
              I.d = dl + am * HW;
              I.yx = yx + am * HW;
              I.in = in + (cidx[am * pitch + c] - i0) * HiWi + ky * Wi + kx;
              I.canon = 0;
              if (g_out) {
                const int j = rank + am * G;
                I.canon = P.w_canon + (long long)((full ? j * Mi : P.csr_ptr[j]) + c) * KK + tt;
              }
              return I;
            });
          }
        }
      } else
      flow_wgrad(lds + C.o_wf, nm * per_map, HW, stride, Wi, uni_of<ID>(C.wgrad_R_log2), lr, g_out, [&](int wi) {
        const int am = dPM.div(wi), rem = wi - am * per_map;
        const int c = dKK.div(rem), tt = rem - c * KK;
        const int ky = dK.div(tt), kx = tt - ky * K;
        WgradInfo I;
        I.ok = c < ncf[am];
        I.d = dl + am * HW;
        I.yx = yx + am * HW;
        I.in = in + cidx[am * pitch + c] * HiWi + ky * Wi + kx;
        I.canon = 0;
        if (g_out) {
          const int j = rank + am * G;
          I.canon = P.w_canon + (long long)((full ? j * Mi : P.csr_ptr[j]) + c) * KK + tt;
        }
        return I;
      });
      const int wave = tid >> 6, lane = tid & 63;
      for (int am = wave; am < nm; am += WG / 64) {
        float s = 0.f;
        for (int q = lane; q < HW; q += 64) s += dl[am * HW + q];
        s = f_wave_sum(s);
        if (lane == 0) {
          if (g_out) g_out[P.b_canon + rank + am * G] = s;
          else lds[C.o_bf + am] = fmaf(-lr, s, lds[C.o_bf + am]);
        }
      }
      __syncthreads();
    };
    // pull copy of the filters of conv layer l that read the own maps of the layer below (stored
    // rotated); own_in = those maps' pooled outputs, [n_own_below][Hi*Wi]
    auto wgrad_pull = [&](auto lc, const float* own_in) __attribute__((always_inline)) {
      const int l = lv(lc);
      const ConvSpec& C = Z.conv[l];
      const int K = uni_of<ID>(C.K), KK = K * K, HW = uni_of<ID>(C.Hp) * uni_of<ID>(C.Wp), stride = uni_of<ID>(C.S) + 1,
                Wi = uni_of<ID>(C.Wi), HiWi = uni_of<ID>(C.Hi) * Wi;
      const int nb = sh.pull[l].n_maps;
      if (nb <= 0) return;
      const float* dall = lds + Z.o_dall;
      const int* yxall = (const int*)(lds + Z.o_yxall);
      const int* bj = (const int*)(lds + C.o_bj);
      const int* ncb = (const int*)(lds + C.o_ncb);
      const int pitch = uni_of<ID>(C.back_pitch);
      const int per_map = pitch * KK;
      const FDiv dPM(per_map), dKK(KK), dK(K);
      flow_wgrad(lds + C.o_wb, nb * per_map, HW, stride, Wi, uni_of<ID>(C.wgrad_R_log2), lr, (gfloat*)nullptr,
                 [&](int wi) {
                   const int ab = dPM.div(wi), rem = wi - ab * per_map;
                   const int e = dKK.div(rem), tt = KK - 1 - (rem - e * KK);
                   const int ky = dK.div(tt), kx = tt - ky * K;
                   const int j = bj[ab * pitch + e];
                   WgradInfo I;
                   I.ok = e < ncb[ab];
                   I.d = dall + j * HW;
                   I.yx = yxall + j * HW;
                   I.in = own_in + ab * HiWi + ky * Wi + kx;
                   I.canon = 0;
                   return I;
                 });
      __syncthreads();
    };
    // Put off what no other rank and no later step of this image waits for: the adjustments of the
    // conv layers' forward copies (above the first layer) and of the first FC layer run while the
    // next image's inputs of that layer are on their way, the pull copy of the second conv layer
    // while the first FC layer's partial sums are.  Same arithmetic on the same values, only later.
    // Streamed plans adjust every filter above the first layer once, in the pull copy (whose holder has the deltas
    // of all output maps at hand and the input map in its own LDS), and send the new values to the rank that holds
    // the forward copy: entry (j, i) goes to its place in row j of the table, tap order turned back.
    auto ship_rows = [&](auto lc, unsigned int tagw) __attribute__((always_inline)) {
      const int l = lv(lc);
      const ConvSpec& C = Z.conv[l];
      const FlowConvPtrs& P = Q.conv[l];
      const int KK = C.K * C.K, pitch = C.back_pitch, Mi = C.Mi;
      const int nb = sh.pull[l].n_maps;
      const float* wb = lds + C.o_wb;
      const int* ncb = (const int*)(lds + C.o_ncb);
      const bool full = C.full_table != 0;
      if (!full) {  // sparse table: tagged words to their places in table order
        const FDiv dKK(KK);
        gtagged* dst = P.x_w + (size_t)(tagw & 1u) * ((size_t)P.csr_ptr[C.Mo] * KK);
        for (int ab = 0; ab < nb; ++ab) {
          const int i = rank + ab * G, ne = ncb[ab], eb = P.csc_ptr[i];
          for (int x = tid; x < ne * KK; x += WG) {
            const int e = dKK.div(x), t = x - e * KK;
            put_f(dst + (size_t)P.csc_slot[eb + e] * KK + (KK - 1 - t), wb[(ab * pitch + e) * KK + t], tagw);
          }
        }
        return;
      }
      // full table: the filters of input map i as plain floats [i][j][K*K rounded up to a multiple of 4], stored 128
      // bits a lane so that a wavefront writes whole cache lines (a written-through store of one word is a memory
      // transaction of its own: sent word by word these were most of the bytes the kernel wrote); then the map's flag
      const int KKp = (KK + 3) & ~3, U4 = KKp >> 2, Mo = C.Mo;
      const int n_w = Mi * Mo * KKp;
      gfloat* data = bulk_data(P.x_w, n_w, tagw & 1u);
      const FDiv dU4(U4);
      for (int ab = 0; ab < nb; ++ab) {
        const int i = rank + ab * G;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)(data + (size_t)i * Mo * KKp), 0, Mo * KKp * 4, 0x00020000);
        for (int x = tid; x < Mo * U4; x += WG) {
          const int e = dU4.div(x), u = x - e * U4;   // (entry e of a full table is output map e)
          f4v v;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int t = 4 * u + c;   // natural tap t lies at KK-1-t of the rotated copy
            v[c] = t < KK ? wb[(ab * pitch + e) * KK + (KK - 1 - t)] : 0.f;
          }
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4v, v), rs, (e * KKp + 4 * u) * 4, 0, 16 /* device scope */);
        }
      }
      stores_done();
      __syncthreads();
      guint* fl = bulk_flags(P.x_w, n_w, Mi, tagw & 1u);
      for (int ab = tid; ab < nb; ab += WG) __hip_atomic_store(fl + rank + ab * G, tagw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto take_rows = [&](auto lc, unsigned int tagw) __attribute__((always_inline)) -> bool {
      const int l = lv(lc);
      const ConvSpec& C = Z.conv[l];
      const FlowConvPtrs& P = Q.conv[l];
      const int KK = C.K * C.K, Mi = C.Mi;
      const int nm = sh.fwd[l].n_maps;
      const int* ncf = (const int*)(lds + C.o_ncf);
      const bool full = C.full_table != 0;
      const gtagged* src0 = P.x_w + (size_t)(tagw & 1u) * (full ? (size_t)C.Mo * Mi : (size_t)P.csr_ptr[C.Mo]) * KK;
      for (int am = 0; am < nm; ++am) {
        const int j = rank + am * G;
        unsigned int* dst = (unsigned int*)(lds + C.o_wf + am * C.max_conn * KK);
        if (!full) {
          if (!gather(rt, dst, src0 + (size_t)P.csr_ptr[j] * KK, ncf[am] * KK, tagw)) return false;
          continue;
        }
        // full table: row j is spread over the runs of the Mi input maps, one padded filter in each; wait for every
        // map's flag (once, for all own maps), then pick the row out, 128 bits a lane
        const int KKp = (KK + 3) & ~3, U4 = KKp >> 2;
        const int n_w = Mi * C.Mo * KKp;
        if (am == 0) {
          const guint* fl = bulk_flags(P.x_w, n_w, Mi, tagw & 1u);
          for (int m = tid; m < Mi; m += WG) {
            unsigned int spins = 0;
            while (__hip_atomic_load(fl + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tagw)
              if (!poll_again(rt, spins)) break;
          }
          __syncthreads();
          if (sh.fail) return false;
        }
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)bulk_data(P.x_w, n_w, tagw & 1u), 0, n_w * 4, 0x00020000);
        const FDiv dU4(U4);
        float* wrow = (float*)dst;
        for (int x = tid; x < Mi * U4; x += WG) {
          const int c = dU4.div(x), u = x - c * U4;
          const u4v raw = __builtin_amdgcn_raw_buffer_load_b128(rs, ((c * C.Mo + j) * KKp + 4 * u) * 4, 0, 16 /* device scope */);
          const f4v v = __builtin_bit_cast(f4v, raw);
#pragma unroll
          for (int cc = 0; cc < 4; ++cc)
            if (4 * u + cc < KK) wrow[c * KK + 4 * u + cc] = v[cc];
        }
      }
      __syncthreads();
      return sh.fail == 0;
    };
    const bool defer = Z.defer != 0 && !taps && !g_out && train;
    STAMP(0);
    {  // the image: a small one was fetched into registers while the previous image was being worked on
      const gfloat* img = a.images + t * a.image_stride;
      float* in = lds + Z.conv[0].o_in;
      if (img_ahead) {
#pragma unroll
        for (int u = 0; u < IMG_U; ++u)
          if (tid + u * WG < img_n) in[tid + u * WG] = img_reg[u];
      } else {
        for (int x = tid; x < img_n; x += WG) in[x] = img[x];
      }
      __syncthreads();
      if (img_ahead && t + 1 < a.n_images) {
#pragma unroll
        for (int u = 0; u < IMG_U; ++u)
          if (tid + u * WG < img_n) img_reg[u] = img[a.image_stride + tid + u * WG];
      }
    }
    STAMP(1);
    // ---- FP, convolutional layers ----
    if (!for_up<ID, 0, FLOW_MAX_CONV>(n_conv, [&](auto lc) {
          const int l = lv(lc);
          const ConvSpec& C = Z.conv[l];
          gtagged* src = nullptr;
          if (l >= 1) {
            if (pend) {
              if (l == 1) DSTAMP(90);
              if (l == n_conv - 1) fc1_update();
              if (Z.stream == 0) wgrad_fwd(lc, tag - 1u, true);
              if (l == 1) DSTAMP(91);
            }
            if (Z.stream != 0 && ship_pend && !take_rows(lc, tag - 1u)) return false;
            const int nw = C.Mi * C.Hi * C.Wi;
            src = Q.conv[l >= 1 ? l - 1 : 0].x_out;
            if (Z.stream == 0) {
              if (!gather(rt, (unsigned int*)(lds + C.o_in), src + (size_t)par * nw, nw, tag)) return false;
              src = nullptr;
            }
          }
          STAMP(2 + 2 * l);
          const int nm = sh.fwd[l].n_maps;
          if (nm > 0) {
            if (!flow_conv_fwd<ID>(rt, l, src, tag)) return false;
            flow_pool<ID>(rt, l, nm, tag, taps);
          }
          STAMP(3 + 2 * l);
          return true;
        }))
      return;
    // ---- FP, first fully connected layer: partial sums over the own columns, exchanged ----
    {
      const float* wc = lds + L1.o_w;
      const float* vcol = lds + Cc.o_pool;
      if (rank < NR) {
        gtagged* xp = Q.xp + ((size_t)par * NR + rank) * n1;
        for (int k = tid; k < n1; k += WG) {
          float s = 0.f;
          for (int c0 = 0; c0 < ncols; c0 += 8) {
            float wv[8], vv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const int c = min(c0 + u, ncols - 1);
              wv[u] = wc[c * n1 + k];
              vv[u] = vcol[c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (c0 + u < ncols) s = fmaf(wv[u], vv[u], s);
          }
          put_f(xp + k, s, tag);
        }
      }
      STAMP(30);
      if (pend) {
        DSTAMP(92);
        if (Z.stream == 0) wgrad_pull(IC<1>{}, lds + Z.o_prev);
        DSTAMP(93);
        pend = false;
      }
      ship_pend = false;
      float* y = lds + L1.o_act;
      if (Z.fc1_owned) {
        if (!flow_reduce_owned(rt, Q.xp + (size_t)par * NR * n1, Q.xsum + (size_t)par * n1, NR, n1, G, lds + L1.o_b, y,
                               lds + L1.o_dact, tag, !L1.is_output)) return;
      } else if (!flow_reduce_partials(rt, Q.xp + (size_t)par * NR * n1, NR, n1, lds + L1.o_b, y, lds + L1.o_dact, part, tag, !L1.is_output)) return;
      STAMP(31);
    }
    // ---- FP, remaining fully connected layers: every rank computes all of them ----
    if (!for_up<ID, 1, FLOW_MAX_FC>(n_fc, [&](auto fc_) {
      const int f = lv(fc_);
      const FcSpec& L = Z.fc[f];
      float* y = lds + L.o_act;
      if (L.by_cols) {
        // a layer too large to hold whole: partial sums over the own columns, added up by every rank
        const int n_out = uni_of<ID>(L.n_out), n_in = uni_of<ID>(L.n_in);
        const int NQ = min(G, n_in), nq = n_mine(n_in, rank, G);
        const float* wq = lds + L.o_w;
        const float* v = lds + Z.fc[f >= 1 ? f - 1 : 0].o_act;
        const FlowFcPtrs& PL = Q.fc[f];
        if (rank < NQ) {
          gtagged* xq = PL.x_part + ((size_t)par * NQ + rank) * n_out;
          for (int k = tid; k < n_out; k += WG) {
            float s = 0.f;
            for (int c = 0; c < nq; ++c) s = fmaf(wq[c * n_out + k], v[rank + c * G], s);
            put_f(xq + k, s, tag);
          }
        }
        return flow_reduce_partials(rt, PL.x_part + (size_t)par * NQ * n_out, NQ, n_out, lds + L.o_b, y, lds + L.o_dact,
                                    part, tag, true);
      }
      flow_matvec(lds + L.o_w, lds + L.o_b, lds + Z.fc[f >= 1 ? f - 1 : 0].o_act, y, uni_of<ID>(L.n_out), uni_of<ID>(L.n_in));
      if (!L.is_output) {
        float* dy = lds + L.o_dact;
        for (int k = tid; k < L.n_out; k += WG) {
          const float v = y[k];
          y[k] = f_act_fc(v);
          dy[k] = f_dact_pre(v);
        }
        __syncthreads();
      }
      return true;
    })) return;
    STAMP(32);
    // soft-max, cross-entropy error, output delta  delta_k = p_k - [k == label].  With at most 64
    // classes every wavefront works them out for itself (lane k holds class k), so nobody waits
    // for a broadcast: the output layer's BP below reads delta_k straight from its own wave.
    float dreg = 0.f;
    const FcSpec& Lo = Z.fc[n_fc - 1];
    const FlowFcPtrs& Po = Q.fc[n_fc - 1];
    const int N = n_classes;
    const bool wave_softmax = N <= 64;
    const bool tanh_out = uni_of<ID>(Z.out_units) == 1;
    {
      float* y = lds + Lo.o_act;
      float* d = lds + Lo.o_delta;
      // only the wavefronts whose lanes the output layer's BP below gives work need the deltas: the others
      // would repeat the same instructions on the same four SIMDs and slow those down
      const int soft_lanes = (max(n_fc >= 2 ? uni_of<ID>(Lo.n_in) : 1, N) + 63) & ~63;
      if (wave_softmax && tid < soft_lanes) {
        const int k = tid & 63;
        const float yk = (k < N) ? y[k] : -INFINITY;
        // exponential, reciprocal and logarithm of the hardware (relative error about 1e-7 each): this chain of
        // dependent operations is walked by one wavefront while every other one waits
        const float mx = f_wave_max(yk);
        const float e = (k < N) ? __builtin_amdgcn_exp2f(1.44269504088896340736f * (yk - mx)) : 0.f;
        // the label's delta p - 1 = -(sum of the other classes' exponentials) / z: summed apart from the
        // label's own term, so that a confident net (p -> 1) loses no digits of it
        const float zo = f_wave_sum(k == label ? 0.f : e);
        const float e_lab = lane_f(e, uni(label) & 63);
        const float z = zo + ((label >= 0 && label < N) ? e_lab : 0.f);
        const float rz = __builtin_amdgcn_rcpf(z);
        float p = e * rz;
        dreg = (k == label) ? -zo * rz : p;
        float err = 0.f;
        if (tanh_out) {  // scaled-tanh outputs, squared error against targets +1 / -1
          p = (k < N) ? f_act_fc(yk) : 0.f;
          const float dev = (k < N) ? p - (k == label ? 1.f : -1.f) : 0.f;
          dreg = (k < N) ? dev * f_dact_pre(yk) : 0.f;
          err = 0.5f * f_wave_sum(dev * dev);
        }
        if (tid < N) {
          if (rank == 0) {
            if (a.probs_out) a.probs_out[t * n_classes + k] = p;
            if (train && tanh_out && k == 0) status->loss = err;
            if (train && !tanh_out && k == label) status->loss = -0.69314718055994530942f * __builtin_amdgcn_logf(p);
          }
          if (taps || n_fc == 1) d[k] = dreg;
          if (taps && rank == 0) Po.act[k] = p;
        }
      }
      if (wave_softmax) {
        if (n_fc == 1) __syncthreads();  // the first FC layer's BP reads the deltas from LDS
      } else {
        if (tid < 64 && tanh_out) {
          float err = 0.f;
          for (int k = tid; k < N; k += 64) {
            const float p = f_act_fc(y[k]);
            const float dev = p - (k == label ? 1.f : -1.f);
            d[k] = dev * f_dact_pre(y[k]);
            y[k] = p;
            err = fmaf(dev, dev, err);
            if (rank == 0) {
              if (a.probs_out) a.probs_out[t * n_classes + k] = p;
              if (taps) Po.act[k] = p;
            }
          }
          err = f_wave_sum(err);
          if (rank == 0 && train && tid == 0) status->loss = 0.5f * err;
        } else if (tid < 64) {
          float mx = -INFINITY;
          for (int k = tid; k < N; k += 64) mx = fmaxf(mx, y[k]);
          mx = f_wave_max(mx);
          float zo = 0.f;
          for (int k = tid; k < N; k += 64) zo += (k == label) ? 0.f : expf(y[k] - mx);
          zo = f_wave_sum(zo);
          const float z = zo + ((label >= 0 && label < N) ? expf(y[max(label, 0)] - mx) : 0.f);
          for (int k = tid; k < N; k += 64) {
            const float p = expf(y[k] - mx) / z;
            d[k] = (k == label) ? -zo / z : p;
            y[k] = p;
            if (rank == 0) {
              if (a.probs_out) a.probs_out[t * n_classes + k] = p;
              if (train && k == label) status->loss = -logf(p);
              if (taps) Po.act[k] = p;
            }
          }
        }
        __syncthreads();
      }
    }
    if (taps && rank == 0)
      for_up<ID, 0, FLOW_MAX_FC>(n_fc - 1, [&](auto fc_) {
        const int f = lv(fc_);
        for (int k = tid; k < Z.fc[f].n_out; k += WG) Q.fc[f].act[k] = lds[Z.fc[f].o_act + k];
        return true;
      });
    STAMP(33);
    if (!train) continue;

    // ---- BP + AW, fully connected layers behind the first (every rank, same arithmetic) ----
    if (!for_down<ID, 1, FLOW_MAX_FC>(n_fc, [&](auto fc_) {
      const int f = lv(fc_);
      const FcSpec& L = Z.fc[f];
      const FlowFcPtrs& PL = Q.fc[f];
      float* W = lds + L.o_w;
      float* b = lds + L.o_b;
      const float* d = lds + L.o_delta;
      const float* v = lds + Z.fc[f >= 1 ? f - 1 : 0].o_act;
      const float* fprev = lds + Z.fc[f >= 1 ? f - 1 : 0].o_dact;
      float* dprev = lds + Z.fc[f >= 1 ? f - 1 : 0].o_delta;
      const int n_in = uni_of<ID>(L.n_in), n_out = uni_of<ID>(L.n_out);
      const bool from_reg = wave_softmax && f == n_fc - 1;
      if (L.by_cols) {
        // own columns: a wavefront per column works out the delta of the unit below, adjusts the column and
        // sends the delta to everybody
        const int nq = n_mine(n_in, rank, G);
        const int wave = tid >> 6, lane = tid & 63;
        for (int c = wave; c < nq; c += WG / 64) {
          const int m = rank + c * G;
          const float vm = v[m];
          float g = 0.f;
          for (int k = lane; k < n_out; k += 64) {
            const float wv = W[c * n_out + k], dk = d[k];
            g = fmaf(wv, dk, g);
            if (g_out) g_out[PL.w_canon + (long long)k * n_in + m] = dk * vm;
            else W[c * n_out + k] = fmaf(-lr, dk * vm, wv);
          }
          g = f_wave_sum(g);
          if (lane == 0) put_f(PL.x_dprev + (size_t)par * n_in + m, g * fprev[m], tag);
        }
        for (int k = tid; k < n_out; k += WG) {
          const float dk = d[k];
          if (g_out) { if (rank == 0) g_out[PL.b_canon + k] = dk; }
          else b[k] = fmaf(-lr, dk, b[k]);
          if (taps && rank == 0) PL.delta[k] = dk;
        }
        return gather(rt, (unsigned int*)dprev, PL.x_dprev + (size_t)par * n_in, n_in, tag);
      }
      for (int m = tid; m < n_in; m += WG) {
        const float vm = v[m];
        float g = 0.f;
        for (int k0 = 0; k0 < n_out; k0 += 4) {
          float wv[4], dv[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int k = min(k0 + u, n_out - 1);
            wv[u] = W[k * n_in + m];
            dv[u] = from_reg ? lane_f(dreg, k) : d[k];
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int k = k0 + u;
            if (k < n_out) {
              g = fmaf(wv[u], dv[u], g);
              if (g_out) { if (rank == 0) g_out[PL.w_canon + (long long)k * n_in + m] = dv[u] * vm; }
              else W[k * n_in + m] = fmaf(-lr, dv[u] * vm, wv[u]);
            }
          }
        }
        dprev[m] = g * fprev[m];
      }
      for (int k = tid; k < n_out; k += WG) {
        const float dk = from_reg ? dreg : d[k];   // tid < 64 here: lane k of wave 0
        if (g_out) { if (rank == 0) g_out[PL.b_canon + k] = dk; }
        else b[k] = fmaf(-lr, dk, b[k]);
        if (taps && rank == 0) PL.delta[k] = dk;
      }
      __syncthreads();
      return true;
    })) return;
    STAMP(34);
    {  // ---- BP + AW, first fully connected layer: own columns ----
      const float* wc = lds + L1.o_w;
      const float* d = lds + L1.o_delta;
      const float* fcol = lds + Cc.o_dact;
      float* dconv = lds + Cc.o_delta;
      const int* yxc = (const int*)(lds + Cc.o_yx);
      const int Moc = uni_of<ID>(Cc.Mo);
      const int wave = tid >> 6, lane = tid & 63;
      const FDiv dHW(HWc);
      for (int c = wave; c < ncols; c += WG / 64) {
        float s = 0.f;
        for (int k = lane; k < n1; k += 64) s = fmaf(wc[c * n1 + k], d[k], s);
        s = f_wave_sum(s);
        if (lane == 0) {
          const float dc = s * fcol[c];
          dconv[c] = dc;
          const int am = dHW.div(c), q = c - am * HWc;
          const size_t o = (size_t)(rank + am * G) * HWc + q;
          if (n_conv >= 2) {  // the layer below pulls through these: on their way at once
            put_f(Pc.x_delta + (size_t)par * Moc * HWc + o, dc, tag);
            put_i(Pc.x_yx + (size_t)par * Moc * HWc + o, yxc[c], tag);
          }
          if (taps) Pc.delta[o] = dc;
        }
      }
      __syncthreads();
      if (!defer) fc1_update();
    }
    STAMP(35);
    // ---- BP + AW, convolutional layers, top down ----
    if (!for_down<ID, 0, FLOW_MAX_CONV>(n_conv, [&](auto lc) {
      const int l = lv(lc);
      const ConvSpec& C = Z.conv[l];
      const FlowConvPtrs& P = Q.conv[l];
      const int HW = uni_of<ID>(C.Hp) * uni_of<ID>(C.Wp), HiWi = uni_of<ID>(C.Hi) * uni_of<ID>(C.Wi), Mo = uni_of<ID>(C.Mo);
      const int nm = sh.fwd[l].n_maps;
      const float* dl = lds + C.o_delta;
      const int* yx = (const int*)(lds + C.o_yx);
      if (l < n_conv - 1 && (l >= 1 || taps)) {  // (the last layer's went out with the first FC layer's BP)
        const FDiv dHW(HW);
        for (int x = tid; x < nm * HW; x += WG) {
          const int am = dHW.div(x), q = x - am * HW;
          const size_t o = (size_t)(rank + am * G) * HW + q;
          if (l >= 1) {
            put_f(P.x_delta + (size_t)par * Mo * HW + o, dl[x], tag);
            put_i(P.x_yx + (size_t)par * Mo * HW + o, yx[x], tag);
          }
          if (taps) P.delta[o] = dl[x];
        }
      }
      STAMP(40 + 4 * l);
      // streamed plan: the filters above the first layer are adjusted once, by the holders of the pull copies, who
      // send them on (ship_rows below); the gradient tap still works them out here, from the inputs fetched again
      if (Z.stream != 0 && l >= 1) wgrad_fwd(lc, tag, g_out != nullptr);
      else if (!(defer && l >= 1)) wgrad_fwd(lc, tag, true);
      STAMP(41 + 4 * l);
      if (l >= 1) {
        const int nb = sh.pull[l].n_maps;
        if (nb > 0) {
          float* dall = lds + Z.o_dall;
          int* yxall = (int*)(lds + Z.o_yxall);
          if (!gather2(rt, (unsigned int*)dall, P.x_delta + (size_t)par * Mo * HW, (unsigned int*)yxall,
                       P.x_yx + (size_t)par * Mo * HW, Mo * HW, tag))
            return false;
          STAMP(42 + 4 * l);
          if (!flow_pull<ID>(rt, l, dall, yxall, tag)) return false;
          STAMP(43 + 4 * l);
          // the pooled maps of the layer below that the pull copy's adjustment needs: the own ones, or, for a
          // share of another rank's map, that map among this layer's inputs
          const int Hs = uni_of<ID>(C.pull_shares), Mi = uni_of<ID>(C.Mi);
          const float* own = (Hs > 1 && rank >= Mi) ? lds + C.o_in + (rank % Mi) * HiWi
                                                    : lds + Z.conv[l >= 1 ? l - 1 : 0].o_pool;
          if (Z.stream != 0) {
            if (!g_out) {
              if (l == 1) DSTAMP(125);
              const int K = C.K;
              if (K >= 2 && K <= 5) {
                const bool full = C.full_table != 0;
                gtagged* xw = full ? nullptr : P.x_w + (size_t)par * ((size_t)P.csr_ptr[Mo] * (K * K));
                auto go = [&](auto k_) __attribute__((always_inline)) {
                  flow_wgrad_entries<decltype(k_)::value>(lds + C.o_wb, (const int*)(lds + C.o_bj), (const int*)(lds + C.o_ncb),
                      nb, C.back_pitch, lds + Z.o_dall, (const int*)(lds + Z.o_yxall), HW, own, HiWi, C.Wi, C.S + 1, lr, Mi, Mo,
                      rank, G, full, P.csc_ptr, P.csc_slot, xw, tag, rt);
                };
                switch (K) {
                  case 2: go(IC<2>{}); break;
                  case 3: go(IC<3>{}); break;
                  case 4: go(IC<4>{}); break;
                  default: go(IC<5>{}); break;
                }
                if (l == 1) DSTAMP(126);
                __syncthreads();
                if (full) ship_rows(lc, tag);
              } else {
                wgrad_pull(lc, own);
                ship_rows(lc, tag);
              }
              if (l == 1) DSTAMP(127);
            }
          } else if (defer && l == 1) {
            // the pull copy is adjusted during the next image's wait; the next FP overwrites the
            // pooled maps it needs, so they are set aside
            float* prev = lds + Z.o_prev;
            for (int x = tid; x < nb * HiWi; x += WG) prev[x] = own[x];
          } else if (!g_out) {
            wgrad_pull(lc, own);
          }
        }
      }
      return true;
    }))
      return;
    STAMP(70);
    pend = defer;
    // streamed plan: the forward copies take their adjusted filters at the next image's FP -- or now, after the
    // last image of the call (the copies go back to global memory below)
    ship_pend = Z.stream != 0 && !g_out;
    if (ship_pend && taps) {
      if (!for_up<ID, 1, FLOW_MAX_CONV>(n_conv, [&](auto lc) { return take_rows(lc, tag); })) return;
      ship_pend = false;
    }
  }
  if (!g_out && a.train) flow_store<ID>(rt);
}

#ifdef CNN355_SPECIAL_HEADER
// ---- this file compiled for one network alone: its kernel and its plan, nothing else -------------------
template __global__ void k_resident<FLOW_SPECIAL_ID>(const FlowSpec, const FlowPtrs* __restrict__, StatusDev*, RunArgs);
extern "C" __device__ __attribute__((used)) const FlowSpec cnn355_special_plan = StaticSpec<FLOW_SPECIAL_ID>::value;
}  // namespace cnn355
#else

template <int ID>
static hipError_t launch_resident_id(int grid, size_t lds_bytes, hipStream_t stream, const FlowSpec& spec,
                                     const FlowPtrs* d_ptrs, StatusDev* d_status, const RunArgs& a) {
  hipError_t e = hipFuncSetAttribute((const void*)k_resident<ID>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  RunArgs args = a;
  FlowSpec plan = spec;
  void* params[] = {(void*)&plan, (void*)&d_ptrs, (void*)&d_status, (void*)&args};
  return hipLaunchCooperativeKernel((const void*)k_resident<ID>, dim3(grid), dim3(WG), params, (unsigned int)lds_bytes, stream);
}

// static_id: 0 = the kernel for any network; k > 0 = the one compiled for StaticSpec<k> (the caller
// has checked that the plan equals it)
hipError_t launch_resident(int static_id, int grid, size_t lds_bytes, hipStream_t stream, const FlowSpec& spec,
                           const FlowPtrs* d_ptrs, StatusDev* d_status, const RunArgs& a) {
  switch (static_id) {
    case 1: return launch_resident_id<1>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
    case 2: return launch_resident_id<2>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
    case 3: return launch_resident_id<3>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
    case 4: return launch_resident_id<4>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
    case 5: return launch_resident_id<5>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
    default: return launch_resident_id<0>(grid, lds_bytes, stream, spec, d_ptrs, d_status, a);
  }
}

// ---- measurement aids: what one crossing between compute units, and one kernel launch, cost ------------
// One round = every rank stores `words` tagged words and then fetches the words of all G ranks (the exchange
// the resident kernel does between layers), `rounds` times; rank 0 stamps the clock before the first round
// after a warm-up round and after the last.
__global__ void __launch_bounds__(WG) k_crossing_probe(tagged_t* buf_, int G, int stride, int words, int rounds,
                                                       unsigned int epoch_base, unsigned int spin_limit,
                                                       StatusDev* status) {
  __shared__ Shared sh;
  gtagged* buf = (gtagged*)buf_;
  if (blockIdx.x % stride != 0 || (int)(blockIdx.x / stride) >= G) return;
  const int rank = blockIdx.x / stride, tid = threadIdx.x;
  if (tid == 0) sh.fail = 0;
  __syncthreads();
  Rt rt;
  rt.dbg = false; rt.spec = nullptr; rt.sh = &sh; rt.status = status; rt.lds = nullptr; rt.rank = rank;
  rt.spin_limit = spin_limit;
  const int n = G * words;
  unsigned int acc = 0;
  for (int e = 0; e <= rounds; ++e) {
    if (e == 1 && rank == 0 && tid == 0) status->stamps[0] = wall_clock64();
    const unsigned int tag = epoch_base + (unsigned int)e + 1u;
    gtagged* b = buf + (size_t)(tag & 1u) * n;
    for (int x = tid; x < words; x += WG) put_f(b + (size_t)rank * words + x, (float)x, tag);
    for (int base = 0; base < n; base += 4 * WG) {
      tagged_t w[4];
      if (!fetch_tagged<4>(rt, w, tag, [&](int u) { return b + min(base + tid + u * WG, n - 1); })) break;
      acc += (unsigned int)w[0] ^ (unsigned int)w[3];
    }
    __syncthreads();
    if (sh.fail) return;
  }
  if (rank == 0 && tid == 0) status->stamps[1] = wall_clock64();
  if (acc == 0x12345u) status->stamps[2] = acc;
}
hipError_t launch_crossing_probe(int G, int stride, hipStream_t stream, tagged_t* buf, int words, int rounds,
                                 unsigned int epoch_base, unsigned int spin_limit, StatusDev* d_status) {
  void* params[] = {(void*)&buf, (void*)&G, (void*)&stride, (void*)&words, (void*)&rounds, (void*)&epoch_base,
                    (void*)&spin_limit, (void*)&d_status};
  return hipLaunchCooperativeKernel((const void*)k_crossing_probe, dim3(G * stride), dim3(WG), params, 0, stream);
}
__global__ void k_empty(StatusDev* status) {
  if (status == nullptr) __builtin_trap();
}
hipError_t launch_empty(hipStream_t stream, StatusDev* d_status) {
  hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, stream, d_status);
  return hipGetLastError();
}

// which compiled-in network, if any, has exactly this plan
int resident_static_id(const FlowSpec& z) {
  if (__builtin_memcmp(&z, &StaticSpec<1>::value, sizeof(FlowSpec)) == 0) return 1;
  if (__builtin_memcmp(&z, &StaticSpec<2>::value, sizeof(FlowSpec)) == 0) return 2;
  if (__builtin_memcmp(&z, &StaticSpec<3>::value, sizeof(FlowSpec)) == 0) return 3;
  if (__builtin_memcmp(&z, &StaticSpec<4>::value, sizeof(FlowSpec)) == 0) return 4;
  if (__builtin_memcmp(&z, &StaticSpec<5>::value, sizeof(FlowSpec)) == 0) return 5;
  return 0;
}

}  // namespace cnn355
#endif  // CNN355_SPECIAL_HEADER
